// Attention for the three cases of Table 2: SigLIP multi-head attention per view (head dim 72),
// prefix attention with 8 query heads sharing one key/value head (head dim 256, no mask inside
// the prefix), and the action expert's attention over [cached prefix keys ; own 64 keys] with the
// state/action block mask.
//
// Keys and values arrive already in MFMA fragment order (written that way by the QKV GEMM's
// epilogue), so every operand fetch is one coalesced 16-byte-per-lane read from L2.
//
// One block of 8 waves owns 32 query rows of one head.  The kernels of this pass are short and
// bound by memory round trips, not by arithmetic, so the block is organised to need one round
// trip when the prefix has at most 8 chunks of 32 keys: at entry every wave issues its loads of Q
// (to LDS), of the key fragments of "its" prefix chunks (chunk index = wave, wave + 8, ...), of
// the value fragments of "its" 32-wide slice of the head dimension, and the block copies the
// (at most two) key chunks of the second segment - the action expert's own 64 keys - to LDS, so
// that waves 0 and 1 can score them without a second trip to memory.
//   phase 1  S^T = K Q^T per chunk (keys x queries): a lane owns one query row, so max and sum
//            are per-lane scalars; the probabilities in the accumulator registers are, without
//            any data movement, B-operand fragments of the second product and go to LDS as such;
//   phase 2  O^T = V^T P^T: wave w accumulates head-dimension slice w over ALL chunks, reading
//            the probability fragments of every wave from LDS.  No cross-wave merge of O.
// The softmax uses the exact row maximum (two LDS exchanges), so results do not depend on the
// chunk-to-wave assignment.
#include "pi0_internal.h"

#include "attention_body.h"

template <int DQK, int NVB, int MAXR, int VRING, int CPW>
__global__ __launch_bounds__(512) void attention_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  attention_body<DQK, NVB, MAXR, VRING, CPW>(p, LaunchCtx::from_block_idx(), smem_raw);
}

// The vision case cut for two resident blocks per compute unit (4 waves per SIMD: at most 128 registers, which a value
// ring of 2 chunks gives without spilling): the 384 blocks of 3 views then run in one round instead of one and a half,
// and a block's shorter ring is covered by its neighbour.  Same order of every sum, so the same bits.
template <int VRING>
__global__ __launch_bounds__(512, 4) void attention_vision2_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  attention_body<80, 3, 1, VRING, 0>(p, LaunchCtx::from_block_idx(), smem_raw);
}

template <int DQK>
static int attn_smem(int ntot) { return 3 * (DQK / 16) * 1024 + 2 * ATT_WAVES * 32 * 4 + ntot * 2048; }

#define ATTN_VARIANTS(X) \
  X(256, 8, 1, 8, 10)    \
  X(256, 8, 2, 8, 0)     \
  X(256, 8, 4, 8, 0)     \
  X(80, 3, 1, 8, 0)

hipError_t attention_init_attributes() {
#define X(DQK, NVB, MAXR, VRING, CPW)                                                                              \
  {                                                                                                           \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<DQK, NVB, MAXR, VRING, CPW>), \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, attn_smem<DQK>(8 * MAXR + 2)); \
    if (e != hipSuccess) return e;                                                                            \
  }
  ATTN_VARIANTS(X)
#undef X
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_vision2_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             attn_smem<80>(8));
}

hipError_t launch_attention(hipStream_t s, const AttnParams& p) {
  if (p.q == nullptr || p.k0 == nullptr || p.v0 == nullptr || p.out == nullptr) return hipErrorInvalidValue;
  if (p.Tq <= 0 || p.heads <= 0 || p.chunks0 <= 0 || p.valid0 <= 0 || p.valid0 > p.chunks0 * 32) return hipErrorInvalidValue;
  if (p.q_head_stride % 512 != 0 || p.out_ld % 16 != 0 || p.head_dim % 4 != 0 || p.out_ld < p.heads * p.head_dim) return hipErrorInvalidValue;
  if (p.chunks1 != 0 && (p.k1 == nullptr || p.v1 == nullptr)) return hipErrorInvalidValue;
  if (p.chunks1 != 0 && p.chunks1 != 2) return hipErrorInvalidValue;
  if (p.suffix_mask && p.Tq > 32 * p.chunks1) return hipErrorInvalidValue;
  int n0 = p.chunks0;
  if (p.view_tokens > 0) {
    if (p.view_tokens % 32 != 0 || p.Tq % p.view_tokens != 0 || p.chunks0 * 32 != p.Tq) return hipErrorInvalidValue;
    n0 = p.view_tokens / 32;
  }
  if (p.key_splits > 1) {   // keys of segment 0 shared out over gridDim.z blocks, merged by the consumer
    if (p.view_tokens > 0 || p.ml_out == nullptr || p.chunks_per_split < 1 || p.key_splits > 8) return hipErrorInvalidValue;
    if ((p.key_splits - 1) * p.chunks_per_split >= p.chunks0 || p.key_splits * p.chunks_per_split < p.chunks0) return hipErrorInvalidValue;
    if (p.out_split_stride < (size_t)((p.Tq + 31) / 32) * 32 * p.out_ld) return hipErrorInvalidValue;
    n0 = p.chunks_per_split;
  } else if (p.key_splits != 0 && p.key_splits != 1) {
    return hipErrorInvalidValue;
  }
  const int ntot = n0 + p.chunks1;
  if (n0 > 32) return hipErrorInvalidValue;   // at most 1024 keys in segment 0 per query row
  if (p.v_split != 0 && p.v_split != 1 && ((p.v_split != 2 && p.v_split != 4 && p.v_split != 8) || p.head_dim != 256)) return hipErrorInvalidValue;
  const int vs = p.v_split > 1 ? p.v_split : 1;
  dim3 grid(((p.Tq + 31) / 32) * vs, p.heads, p.key_splits > 1 ? p.key_splits : 1);
  if (p.pf.blocks != 0) {   // warm-up blocks as extra grid rows
    const PrefetchDesc& d = p.pf;
    if (d.blocks < 0 || d.blocks % 16 != 0 || d.blocks > 1024 || d.sink == nullptr || d.blocks % (int)grid.x != 0) return hipErrorInvalidValue;
    for (int r = 0; r < 3; r++) {
      if (d.ptr[r] == nullptr) continue;
      if (d.tiles[r] <= 0 || d.tile16[r] <= 0 || (reinterpret_cast<uintptr_t>(d.ptr[r]) & 15) != 0) return hipErrorInvalidValue;
      if ((long)((d.tiles[r] + 7) / 8) * d.tile16[r] > 0x7fffffffL) return hipErrorInvalidValue;
    }
    grid.y += d.blocks / grid.x;
  }
  if (p.head_dim == 256) {
    if (n0 <= 8) attention_kernel<256, 8, 1, 8, 10><<<grid, dim3(512), attn_smem<256>(ntot), s>>>(p);
    else if (n0 <= 16) attention_kernel<256, 8, 2, 8, 0><<<grid, dim3(512), attn_smem<256>(ntot), s>>>(p);
    else attention_kernel<256, 8, 4, 8, 0><<<grid, dim3(512), attn_smem<256>(ntot), s>>>(p);
  } else if (p.head_dim <= 80 && p.head_dim > 64) {
    if (n0 > 8 || p.chunks1 != 0) return hipErrorInvalidValue;
    if (grid.x * grid.y > 256 && p.pf.blocks == 0) attention_vision2_kernel<2><<<grid, dim3(512), attn_smem<80>(ntot), s>>>(p);
    else attention_kernel<80, 3, 1, 8, 0><<<grid, dim3(512), attn_smem<80>(ntot), s>>>(p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
