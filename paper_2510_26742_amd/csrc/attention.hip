// Attention for the three cases of Table 2: SigLIP multi-head attention per view (head dim 72),
// prefix attention with 8 query heads sharing one key/value head (head dim 256, no mask inside
// the prefix), and the action expert's attention over [cached prefix keys ; own 64 keys] with the
// state/action block mask.
//
// Keys and values arrive already in MFMA fragment order (written that way by the QKV GEMM's
// epilogue), so every operand fetch is one coalesced 16-byte-per-lane read from L2 and the kernel
// needs no LDS staging.  Per 32-key chunk a wave computes S^T = K Q^T (keys x queries) so that a
// lane owns one query row: the running max / sum of the online softmax are per-lane scalars, and
// the probabilities in the accumulator registers are, without any data movement, the B operand
// of O^T = V^T P^T.  The four waves of a block take every fourth chunk of the same 32 query rows
// and merge their partial results through LDS in a fixed order.
#include "pi0_internal.h"

#define NEG_BIG (-1.0e30f)

template <int DQK, int NVB>
__global__ __launch_bounds__(256) void attention_kernel(AttnParams p) {
  constexpr int S16 = DQK / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* mw = reinterpret_cast<float*>(smem_raw);          // [4][32]
  float* lw = mw + 4 * 32;                                 // [4][32]
  float* ored = lw + 4 * 32;                               // [3][NVB][16][64]

  const int lane = threadIdx.x & 63;
  const int w = threadIdx.x >> 6;
  const int lq = lane & 31;
  const int lh = lane >> 5;
  const int tile = blockIdx.x;
  const int head = blockIdx.y;
  const int row = tile * 32 + lq;
  const bool row_ok = row < p.Tq;

  // query fragments (B operand): lane (query lq, half lh) holds d = 16 s + 8 lh .. + 8
  bf16x8 qf[S16];
#pragma unroll
  for (int s = 0; s < S16; s++) {
    if (row_ok) {
      qf[s] = *reinterpret_cast<const bf16x8*>(p.q + (size_t)row * p.q_ld + head * p.q_head_stride + s * 16 + lh * 8);
    } else {
#pragma unroll
      for (int j = 0; j < 8; j++) qf[s][j] = (bf16)0.0f;
    }
  }

  int cbeg0 = 0, n0 = p.chunks0;
  if (p.view_tokens > 0) {
    const int view = (tile * 32) / p.view_tokens;
    cbeg0 = view * (p.view_tokens >> 5);
    n0 = p.view_tokens >> 5;
  }
  const int ntot = n0 + p.chunks1;
  const bf16* kbase0 = p.k0 + (size_t)head * p.kv_head_stride0;
  const bf16* vbase0 = p.v0 + (size_t)head * p.v_head_stride0;

  f32x16 o[NVB];
#pragma unroll
  for (int vb = 0; vb < NVB; vb++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[vb][r] = 0.f;
  float m_run = NEG_BIG, l_run = 0.f;

  for (int ci = w; ci < ntot; ci += 4) {
    const bool seg1 = ci >= n0;
    const int chunk = seg1 ? (ci - n0) : (cbeg0 + ci);
    const bf16* kf = (seg1 ? p.k1 : kbase0) + (size_t)chunk * S16 * 512 + lane * 8;
    const bf16* vf = (seg1 ? p.v1 : vbase0) + (size_t)chunk * NVB * 1024 + lane * 8;
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; r++) sacc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < S16; s++) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(kf + (size_t)s * 512);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], sacc, 0, 0, 0);
    }
    // mask + online softmax (lane = query row; registers = keys 8*(r/4) + 4*lh + r%4)
    float sv[16];
    bool ok[16];
    float cmax = NEG_BIG;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int kk = 8 * (r >> 2) + 4 * lh + (r & 3);
      const int key = chunk * 32 + kk;
      bool valid;
      if (!seg1) {
        valid = key < p.valid0;
      } else {
        valid = p.suffix_mask ? (row == 0 ? key == 0 : true) : true;
      }
      ok[r] = valid;
      sv[r] = sacc[r] * p.scale;
      if (valid) cmax = fmaxf(cmax, sv[r]);
    }
    cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
    const float m_new = fmaxf(m_run, cmax);
    const float alpha = __expf(m_run - m_new);
    float psum = 0.f;
    float pr[16];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      pr[r] = ok[r] ? __expf(sv[r] - m_new) : 0.f;
      psum += pr[r];
    }
    psum += __shfl_xor(psum, 32, 64);
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int vb = 0; vb < NVB; vb++)
#pragma unroll
      for (int r = 0; r < 16; r++) o[vb][r] *= alpha;
    bf16x8 pb[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
      for (int j = 0; j < 8; j++) pb[s2][j] = (bf16)pr[8 * s2 + j];
#pragma unroll
    for (int vb = 0; vb < NVB; vb++) {
#pragma unroll
      for (int s2 = 0; s2 < 2; s2++) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(vf + (size_t)(vb * 2 + s2) * 512);
        o[vb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[s2], o[vb], 0, 0, 0);
      }
    }
  }

  // merge the four waves
  if (lh == 0) {
    mw[w * 32 + lq] = m_run;
    lw[w * 32 + lq] = l_run;
  }
  __syncthreads();
  float m_all = NEG_BIG;
#pragma unroll
  for (int i = 0; i < 4; i++) m_all = fmaxf(m_all, mw[i * 32 + lq]);
  float l_all = 0.f;
#pragma unroll
  for (int i = 0; i < 4; i++) l_all += lw[i * 32 + lq] * __expf(mw[i * 32 + lq] - m_all);
  const float f = __expf(m_run - m_all) / l_all;
#pragma unroll
  for (int vb = 0; vb < NVB; vb++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[vb][r] *= f;
  if (w > 0) {
#pragma unroll
    for (int vb = 0; vb < NVB; vb++)
#pragma unroll
      for (int r = 0; r < 16; r++) ored[(((size_t)(w - 1) * NVB + vb) * 16 + r) * 64 + lane] = o[vb][r];
  }
  __syncthreads();
  if (w != 0 || !row_ok) return;
#pragma unroll
  for (int i = 1; i < 4; i++)
#pragma unroll
    for (int vb = 0; vb < NVB; vb++)
#pragma unroll
      for (int r = 0; r < 16; r++) o[vb][r] += ored[(((size_t)(i - 1) * NVB + vb) * 16 + r) * 64 + lane];
#pragma unroll
  for (int vb = 0; vb < NVB; vb++) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int d = vb * 32 + 8 * i + 4 * lh;
      if (d < p.head_dim) {
        const bf16x4 ob = {(bf16)o[vb][4 * i], (bf16)o[vb][4 * i + 1], (bf16)o[vb][4 * i + 2], (bf16)o[vb][4 * i + 3]};
        *reinterpret_cast<bf16x4*>(p.out + (size_t)row * p.out_ld + head * p.head_dim + d) = ob;
      }
    }
  }
}

template <int NVB>
static constexpr int attn_smem() { return (2 * 4 * 32 + 3 * NVB * 16 * 64) * 4; }

hipError_t attention_init_attributes() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<256, 8>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, attn_smem<8>());
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<80, 3>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, attn_smem<3>());
}

hipError_t launch_attention(hipStream_t s, const AttnParams& p) {
  if (p.q == nullptr || p.k0 == nullptr || p.v0 == nullptr || p.out == nullptr) return hipErrorInvalidValue;
  if (p.Tq <= 0 || p.heads <= 0 || p.chunks0 <= 0 || p.valid0 <= 0 || p.valid0 > p.chunks0 * 32) return hipErrorInvalidValue;
  if (p.q_ld % 8 != 0 || p.q_head_stride % 8 != 0 || p.out_ld % 4 != 0 || p.head_dim % 4 != 0) return hipErrorInvalidValue;
  if (p.chunks1 != 0 && (p.k1 == nullptr || p.v1 == nullptr)) return hipErrorInvalidValue;
  if (p.chunks1 < 0 || p.chunks1 > 2) return hipErrorInvalidValue;
  if (p.suffix_mask && p.Tq > 32 * p.chunks1) return hipErrorInvalidValue;
  if (p.view_tokens > 0) {
    if (p.view_tokens % 32 != 0 || p.Tq % p.view_tokens != 0 || p.chunks0 * 32 != p.Tq) return hipErrorInvalidValue;
  }
  dim3 grid((p.Tq + 31) / 32, p.heads, 1);
  if (p.head_dim == 256) {
    constexpr int smem = attn_smem<8>();
    attention_kernel<256, 8><<<grid, dim3(256), smem, s>>>(p);
  } else if (p.head_dim <= 80 && p.head_dim > 64) {
    constexpr int smem = attn_smem<3>();
    attention_kernel<80, 3><<<grid, dim3(256), smem, s>>>(p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
