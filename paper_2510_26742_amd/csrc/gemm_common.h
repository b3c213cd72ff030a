// Pieces of the GEMM family that more than one translation unit needs: the fused epilogues of Table 2's rows
// and the bodies of the action expert's skinny GEMMs, which run both as per-operation launches and inside the
// persistent kernel of the denoise loop (exec_ctx.h).
#pragma once
#include "pi0_internal.h"
#include "exec_ctx.h"
#include <type_traits>

__device__ __forceinline__ float gelu_tanh_f(float x) {
  // 0.5 x (1 + tanh u) = x * sigmoid(2u) = x / (1 + exp(-2u)); hardware exp2 and reciprocal
  const float u2 = -1.5957691216057308f * (x + 0.044715f * x * x * x);
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(1.4426950408889634f * u2));
}

// Sum over groups of 8 adjacent lanes with DPP (no LDS traffic): xor 1, xor 2 inside quads, then
// the mirror inside each half row pairs quad 0 with quad 1.  Every lane of the group gets the sum.
__device__ __forceinline__ float sum8_dpp(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true));
  return v;
}

__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int j = 0; j < 8; j++) z[j] = (bf16)0.0f;
  return z;
}

// Activation matrices that feed a GEMM are stored in MFMA B-fragment order ("XF" layout):
// element (row m, column k) of a matrix padded to kc16*16 columns lives at
//   ((m/32 * kc16 + k/16) * 64 + ((k%16)/8)*32 + m%32) * 8 + k%8,
// i.e. the 32-token x 16-k fragment (m/32, k/16) is 1 KiB of consecutive memory, lane-major.
// Producers write it from their accumulator layout in 8-byte pieces that coalesce to 512-byte
// runs; consumers copy fragments to LDS (or registers) with fully contiguous accesses, and LDS
// fragment reads run at the full 128 B/clk (a padded row-major tile only reaches half of that).
__device__ __forceinline__ size_t xf_index(int m, int k, int kc16) {
  return ((size_t)(m >> 5) * kc16 + (k >> 4)) * 512 + (((k & 15) >> 3) * 32 + (m & 31)) * 8 + (k & 7);
}

// Operands of the epilogue that come from memory (bias, column sums, residual / RoPE table, gain),
// loaded ahead of time: a kernel calls epilogue_preload as early as it knows its (tile, row), so
// that the round trip overlaps the main loop instead of following it.
// slot j holds the operands of the tile's step I0 + j of the wave that asked for steps I0 .. I1 - 1
struct EpiOps {
  f32x4 bias[4], colsum[4], aux[4], gain[4];
};

// Steps I0 .. I1-1 of the tile's four 8-feature steps (all of them unless a kernel shares a tile's epilogue out
// over several waves; the residual epilogue's row statistics need the whole tile, the GeGLU one whole pairs).
// DEP selects what is fetched: 1 = only what blocks of the operation before produced (the residual rows), 0 = only
// constants (bias, column sums, gain, RoPE table), 2 = both.  A persistent kernel asks for the constants before it
// waits for its inputs and for the rest after.
template <int PRO, int EPI, int I0 = 0, int I1 = 4, int DEP = 2, class Cx = LaunchCtx>
__device__ __forceinline__ void epilogue_preload(const GemmParams& p, int nt, int m, int lh, EpiOps& o, const Cx& cx = Cx{}) {
  if (EPI == EPI_PARTIAL) return;
#pragma unroll
  for (int i = I0; i < I1; i++) {
    const int n4 = nt * 32 + 8 * i + 4 * lh;
    if (DEP != 1) {
      if (PRO == PRO_LN) o.colsum[i - I0] = *reinterpret_cast<const f32x4*>(p.colsum + n4);
      if (p.bias != nullptr) o.bias[i - I0] = *reinterpret_cast<const f32x4*>(p.bias + n4);
    }
    if (EPI == EPI_RESID) {
      if (n4 < p.n_valid) {
        if (DEP != 0 && p.resid != nullptr) {
          const int rr = p.resid_mod > 0 ? (m % p.resid_mod) : m;
          o.aux[i - I0] = cx.ld(reinterpret_cast<const f32x4*>(p.resid + (size_t)rr * p.ldo + n4));
        }
        if (DEP != 1 && p.gain != nullptr) o.gain[i - I0] = *reinterpret_cast<const f32x4*>(p.gain + n4);
      }
    } else if (EPI == EPI_QKV) {
      if (DEP != 1 && p.rope != nullptr && n4 < p.q_cols + p.k_cols) {
        const int nl = n4 < p.q_cols ? n4 : n4 - p.q_cols;
        const int i0 = (nl & 255) >> 1;
        o.aux[i - I0] = *reinterpret_cast<const f32x4*>(p.rope + ((size_t)(p.pos0 + m) * 128 + i0) * 2);
      }
    } else if (EPI == EPI_EULER) {
      // the x values this lane updates, with the other inputs (read inside the epilogue they cost one round trip per
      // step of the tile, each behind the stores of the step before: 4.7 of the out-projection's 7.2 us)
      if (DEP != 0 && m >= 1 && n4 < p.n_valid) {
        const float* xp = p.out_f32 + (size_t)(m - 1) * p.ldo + n4;
        f32x4 xv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; j++) {
          if (n4 + j < p.n_valid) xv[j] = cx.ld(xp + j);
        }
        o.aux[i - I0] = xv;
      }
    }
  }
}

// One 32-token x 32-feature accumulator tile -> memory.  `acc` is the MFMA accumulator of the
// calling lane (token = lane % 32, features nt*32 + 8*(r/4) + 4*(lane/32) + r%4), `m` the global
// row, (s_sum, s_sq) the row's sum and sum of squares over the true k columns.
template <int PRO, int EPI, int I0 = 0, int I1 = 4, class Cx = LaunchCtx>
__device__ __forceinline__ void epilogue_tile(const GemmParams& p, const f32x16& acc, int nt, int m, int lh,
                                              float s_sum, float s_sq, int zsplit, const EpiOps& ops, const Cx& cx = Cx{}) {
  static_assert(EPI != EPI_RESID || (I0 == 0 && I1 == 4), "row statistics are taken over the whole tile");
  static_assert(EPI != EPI_GEGLU || (I0 % 2 == 0 && I1 % 2 == 0), "gate / up steps are stored in pairs");
  const float inv_k = 1.0f / (float)p.k_true;
  {
    float rs = 1.f, mu = 0.f;
    float st_a = 0.f, st_b = 0.f;   // EPI_RESID: sum / sum of squares of this lane's fp32 outputs
    unsigned geglu_keep = 0u;       // EPI_GEGLU: the products of the even step, until the odd step pairs them
    if (PRO == PRO_RMS) {
      rs = rsqrtf(s_sq * inv_k + 1e-6f);
    } else if (PRO == PRO_LN) {
      mu = s_sum * inv_k;
      float var = s_sq * inv_k - mu * mu;
      rs = rsqrtf(fmaxf(var, 0.f) + 1e-6f);
    }
#pragma unroll
    for (int i = I0; i < I1; i++) {
      const int n4 = nt * 32 + 8 * i + 4 * lh;
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; j++) v[j] = acc[4 * i + j];
      if (EPI == EPI_PARTIAL) {
        f32x4 o = {v[0], v[1], v[2], v[3]};
        cx.st(reinterpret_cast<f32x4*>(p.out_f32 + ((size_t)zsplit * p.M + m) * p.ldo + n4), o);
        continue;
      }
      if (PRO == PRO_RMS) {
#pragma unroll
        for (int j = 0; j < 4; j++) v[j] *= rs;
      } else if (PRO == PRO_LN) {
        const f32x4 cs = ops.colsum[i - I0];
#pragma unroll
        for (int j = 0; j < 4; j++) v[j] = rs * (v[j] - mu * cs[j]);
      }
      if (p.bias != nullptr) {
        const f32x4 bb = ops.bias[i - I0];
#pragma unroll
        for (int j = 0; j < 4; j++) v[j] += bb[j];
      }
      if (EPI == EPI_RESID) {
        if (n4 < p.n_valid) {
          if (p.resid != nullptr) {
            const f32x4 r4 = ops.aux[i - I0];
#pragma unroll
            for (int j = 0; j < 4; j++) v[j] += r4[j];
          }
          const int mo = m + p.row_offset;
          f32x4 o = {v[0], v[1], v[2], v[3]};
          cx.st(reinterpret_cast<f32x4*>(p.out_f32 + (size_t)mo * p.ldo + n4), o);
#pragma unroll
          for (int j = 0; j < 4; j++) {
            st_a += v[j];
            st_b += v[j] * v[j];
          }
          if (p.gain != nullptr) {
            const f32x4 g4 = ops.gain[i - I0];
#pragma unroll
            for (int j = 0; j < 4; j++) v[j] *= g4[j];
          }
          bf16x4 ob = {(bf16)v[0], (bf16)v[1], (bf16)v[2], (bf16)v[3]};
          cx.st(reinterpret_cast<bf16x4*>(p.out_bf16 + xf_index(mo, n4, p.ldo2 >> 4)), ob);
        }
      } else if (EPI == EPI_BF16) {
        if (n4 < p.n_valid) {
          if (p.act == ACT_GELU) {
#pragma unroll
            for (int j = 0; j < 4; j++) v[j] = gelu_tanh_f(v[j]);
          }
          bf16x4 ob = {(bf16)v[0], (bf16)v[1], (bf16)v[2], (bf16)v[3]};
          cx.st(reinterpret_cast<bf16x4*>(p.out_bf16 + xf_index(m, n4, p.ldo >> 4)), ob);
        }
      } else if (EPI == EPI_GEGLU) {
        // this lane's two products of step i; steps are paired (0,1), (2,3): the lane halves swap one
        // pair each, so that a lane stores 4 consecutive columns (8 bytes) and the two halves together
        // fill whole 16-byte pieces of the XF layout
        const bf16x2 ob = {(bf16)(gelu_tanh_f(v[0]) * v[1]), (bf16)(gelu_tanh_f(v[2]) * v[3])};
        const unsigned mine = __builtin_bit_cast(unsigned, ob);
        if ((i & 1) == 0) {
          geglu_keep = mine;
        } else {
          const unsigned give = lh ? geglu_keep : mine;            // half 0 gives step i, half 1 gives step i-1
          const unsigned got = (unsigned)__shfl_xor((int)give, 32, 64);
          const unsigned lo = lh ? got : geglu_keep;                 // half 0: own i-1, partner's i-1
          const unsigned hi = lh ? mine : got;                       // half 1: partner's i, own i
          const int col = nt * 16 + 4 * (i - 1) + 4 * lh;            // (n4 >> 1) of step i-1 for half 0, +4 for half 1
          const uint2 o2 = {lo, hi};
          cx.st(reinterpret_cast<uint2*>(p.out_bf16 + xf_index(m, col, p.ldo >> 4)), o2);
        }
      } else if (EPI == EPI_EULER) {
        if (m >= 1 && n4 < p.n_valid) {
          float* xp = p.out_f32 + (size_t)(m - 1) * p.ldo + n4;
          const f32x4 xv = ops.aux[i - I0];   // x before the update, fetched with the other inputs
#pragma unroll
          for (int j = 0; j < 4; j++) {
            if (n4 + j < p.n_valid) cx.st(xp + j, xv[j] + p.dt * v[j]);
          }
        }
      } else if (EPI == EPI_QKV) {
        const int S16 = p.dqk_pad >> 4;
        const int key = m;
        const int kc = key >> 5, kk = key & 31;
        if (n4 < p.q_cols + p.k_cols) {
          const bool is_q = n4 < p.q_cols;
          const int nl = is_q ? n4 : n4 - p.q_cols;
          if (p.rope != nullptr) {
            // packed head layout: row 2i = dim i, row 2i+1 = dim i + 128
            const int head = nl >> 8;
            const int i0 = (nl & 255) >> 1;          // even
            const f32x4 c4 = ops.aux[i - I0];   // cos i0, sin i0, cos i0+1, sin i0+1
            const float lo0 = v[0] * c4[0] - v[1] * c4[1], hi0 = v[1] * c4[0] + v[0] * c4[1];
            const float lo1 = v[2] * c4[2] - v[3] * c4[3], hi1 = v[3] * c4[2] + v[2] * c4[3];
            const bf16x2 lo = {(bf16)lo0, (bf16)lo1};
            const bf16x2 hi = {(bf16)hi0, (bf16)hi1};
            {
              bf16* dst = (is_q ? p.out_bf16 + ((size_t)head * p.q_mbs + kc) * S16 * 512 : p.kfrag + ((size_t)kc * S16) * 512) +
                          kk * 8;
              const int d0 = i0, d1 = i0 + 128;
              cx.st(reinterpret_cast<bf16x2*>(dst + (size_t)(d0 >> 4) * 512 + ((d0 & 15) >> 3) * 256 + (d0 & 7)), lo);
              cx.st(reinterpret_cast<bf16x2*>(dst + (size_t)(d1 >> 4) * 512 + ((d1 & 15) >> 3) * 256 + (d1 & 7)), hi);
            }
          } else {
            const int head = nl / p.head_dim;
            const int d = nl - head * p.head_dim;    // multiple of 4
            const bf16x4 ob = {(bf16)v[0], (bf16)v[1], (bf16)v[2], (bf16)v[3]};
            {
              bf16* dst = (is_q ? p.out_bf16 + ((size_t)head * p.q_mbs + kc) * S16 * 512
                                : p.kfrag + ((size_t)head * p.kv_chunks + kc) * S16 * 512) + kk * 8;
              cx.st(reinterpret_cast<bf16x4*>(dst + (size_t)(d >> 4) * 512 + ((d & 15) >> 3) * 256 + (d & 7)), ob);
            }
          }
        } else {
          const int nl = n4 - p.q_cols - p.k_cols;
          const int head = nl / p.head_dim;
          const int d = nl - head * p.head_dim;
          if (head < p.kv_heads) {
            const int s2 = kk >> 4, g = (kk & 15) >> 3, hh = (kk & 7) >> 2, jp = kk & 3;
            bf16* dst = p.vfrag + (((size_t)head * p.kv_chunks + kc) * p.nvb) * 1024 + s2 * 512 + hh * 256 + 4 * g + jp;
#pragma unroll
            for (int j = 0; j < 4; j++) {
              const int dd = d + j;
              cx.st(dst + (size_t)(dd >> 5) * 1024 + (dd & 31) * 8, (bf16)v[j]);
            }
          }
        }
      }
    }
    if (EPI == EPI_RESID && p.stat_out != nullptr) {
      // partial row statistics over this tile's 32 columns: [n tile][stat_rows (64 if not given)][2]
      st_a += __shfl_xor(st_a, 32, 64);
      st_b += __shfl_xor(st_b, 32, 64);
      if (lh == 0) {
        float* dst = p.stat_out + ((size_t)nt * (p.stat_rows > 0 ? p.stat_rows : 64) + m + p.row_offset) * 2;
        cx.st(reinterpret_cast<float2*>(dst), make_float2(st_a, st_b));
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Skinny GEMM (at most 64 tokens): the action expert's projections.  These kernels move a few MB
// of weights each and are bound by memory round trips, so a block issues ALL of its loads at entry
// and waits once.  One block = one 32-feature tile, 8 waves splitting a k range of at most 1024;
// wave w owns k16 steps w*8 .. w*8+7 and reads exactly the activation fragments of those steps
// (both 32-token blocks) from the XF layout straight into registers: no LDS staging, no barrier
// before the MFMAs.  Partial tiles and partial row statistics are summed through LDS in wave order
// (deterministic); waves 0 and 1 finish one 32-token tile each.
// ------------------------------------------------------------------------------------------------
#define SK_WAVES 8
#define SK_KMAX 1024

// MS = 1: the two 32-token blocks go to separate blocks (gridDim.z = 2), which halves the activation
// bytes per CU; used where the launch would otherwise leave most CUs idle (the expert's QKV).
// Steps I0 .. I1-1 of one token block's tile: the 8 waves' partial tiles [wave][token block][step][lane][4] are
// added in wave order, then the epilogue runs on those steps.
template <int PRO, int EPI, int I0, int I1, class Cx>
__device__ __forceinline__ void skinny_finish(const GemmParams& p, const float* red, int mb /* slot */, int lane, int nt, int ml, int lh,
                                              float ssum, float ssq, const EpiOps& ops, const Cx& cx) {
  f32x16 sum;
#pragma unroll
  for (int r = 0; r < 16; r++) sum[r] = 0.f;
#pragma unroll
  for (int ww = 0; ww < SK_WAVES; ww++)
#pragma unroll
    for (int q = I0; q < I1; q++) {
      const f32x4 v4 = *reinterpret_cast<const f32x4*>(red + ((((size_t)ww * 2 + mb) * 4 + q) * 64 + lane) * 4);
#pragma unroll
      for (int j = 0; j < 4; j++) sum[4 * q + j] += v4[j];
    }
  if (ml < p.M) epilogue_tile<PRO, EPI, I0, I1>(p, sum, nt, ml, lh, ssum, ssq, cx.by, ops, cx);
}

// the epilogue operands of finishing wave piece fpc (a tile's four 8-feature steps are shared out over PIECES waves)
template <int PRO, int EPI, int PIECES, int DEP, class Cx>
__device__ __forceinline__ void skinny_preload(const GemmParams& p, int nt, int mrow, int lh, int fpc, EpiOps& ops, const Cx& cx) {
  if constexpr (PIECES == 1) epilogue_preload<PRO, EPI, 0, 4, DEP>(p, nt, mrow, lh, ops, cx);
  else if constexpr (PIECES == 2) {
    if (fpc == 0) epilogue_preload<PRO, EPI, 0, 2, DEP>(p, nt, mrow, lh, ops, cx);
    else epilogue_preload<PRO, EPI, 2, 4, DEP>(p, nt, mrow, lh, ops, cx);
  } else {
    if (fpc == 0) epilogue_preload<PRO, EPI, 0, 1, DEP>(p, nt, mrow, lh, ops, cx);
    else if (fpc == 1) epilogue_preload<PRO, EPI, 1, 2, DEP>(p, nt, mrow, lh, ops, cx);
    else if (fpc == 2) epilogue_preload<PRO, EPI, 2, 3, DEP>(p, nt, mrow, lh, ops, cx);
    else epilogue_preload<PRO, EPI, 3, 4, DEP>(p, nt, mrow, lh, ops, cx);
  }
}

template <int PRO, int EPI, int MS, class Cx>
__device__ __forceinline__ void gemm_skinny_body(const GemmParams p, const Cx cx, unsigned char* smem_raw) {
  // MS = 0: one feature tile, both token blocks; 1: one feature tile, one token block (cx.bz); 2: two adjacent feature
  // tiles (2 cx.bx, 2 cx.bx + 1), one token block (cx.bz) - half the activation bytes of MS = 0 behind the wait of a
  // persistent kernel, where the weights have been requested before it.  A "slot" is a (token block, tile) of the block.
  constexpr int NMB = MS == 0 ? 2 : 1;         // token blocks per block
  constexpr int NTL = MS == 2 ? 2 : 1;         // feature tiles per block
  constexpr int NSLOT = NMB * NTL;
  float* red = reinterpret_cast<float*>(smem_raw);                 // [8 waves][2 slots][16][64]
  const int t = cx.tid();
  const int lane = t & 63;
  const int w = t >> 6;
  const int lq = lane & 31;
  const int lh = lane >> 5;
  if (!Cx::kPersistent) {
    if (cx.bx >= p.n_tiles) {   // warm-up block (only launched with gridDim.y == 1)
      if (cx.bz == 0) prefetch_role(p.pf, cx.bx - p.n_tiles);
      return;
    }
    if (p.progress != nullptr && t == 0 && cx.bx == 0 && cx.by == 0 && cx.bz == 0)
      __hip_atomic_store(p.progress, p.progress_value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  const int nt = NTL * cx.bx;   // first feature tile of the block
  const int k_pad = p.W.k_pad;
  const int kbeg = cx.by * p.k_per_split;
  const int kend = min(kbeg + p.k_per_split, k_pad);
  const int n16 = (kend - kbeg) >> 4;          // k16 steps of this block (<= 64)
  const int KC16 = k_pad >> 4;
  const int XKC16 = p.ldx >> 4;

  // row statistics of the input: parts partial sums per row (1, or one per 32-column tile of the
  // producer); wave w adds parts w, w+8, ... for row `lane`, the epilogue adds the 8 wave sums
  float* sstat8 = red + SK_WAVES * 2 * 16 * 64 + 128;   // [8 waves][64][2]
  bf16x8 wf[NTL][8], xf[NMB][8];
  const bf16* wbase = p.W.w + ((size_t)nt * KC16 + (kbeg >> 4)) * 512 + lane * 8;   // tile j: + j * KC16 * 512
  const bf16* xbase = p.X + (size_t)(kbeg >> 4) * 512 + lane * 8;
  const int mb_last = p.M > 32 ? 1 : 0;        // last token block (clamps when M <= 32)
  const int mb_first = MS ? min(cx.bz, mb_last) : 0;   // global index of local token block 0
  // The tile of a token block is finished by PIECES waves, each taking 4 / PIECES of its four 8-feature steps
  // (finishing wave f: token block f / PIECES, piece f % PIECES): the sum over the 8 waves' partial tiles and the
  // epilogue arithmetic are the tail of the launch, and one wave alone took 3.8 k cycles over them for the QKV
  // epilogue (2.2 k for GeGLU)
  constexpr int PIECES = EPI == EPI_QKV ? 4 : EPI == EPI_GEGLU ? 2 : 1;
  constexpr int NFIN = NSLOT * PIECES;
  static_assert(NFIN <= SK_WAVES, "finishing waves");
  EpiOps ops;
  const int fslot = w / PIECES, fpc = w % PIECES;   // finishing wave f: slot f / PIECES, piece f % PIECES
  const int fmb = NTL == 1 ? fslot : 0;             // its token block (local) ...
  const int fnt = nt + (NTL == 1 ? 0 : fslot);      // ... and feature tile
  const int mrow = (mb_first + fmb) * 32 + lq;   // the row this lane finishes if w < NFIN
  if (Cx::kPersistent) {
    // constants first (weights, then the epilogue's vectors); the inputs are requested once they exist
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const int st = min(w * 8 + i, n16 - 1);
#pragma unroll
      for (int j = 0; j < NTL; j++) wf[j][i] = *reinterpret_cast<const bf16x8*>(wbase + ((size_t)j * KC16 + st) * 512);
    }
    if (w < NFIN && mrow < p.M) skinny_preload<PRO, EPI, PIECES, 0>(p, fnt, mrow, lh, fpc, ops, cx);
    cx.wait_inputs();
  }
  // statistics partials: issued ahead of the operand loads (same round trip), clamped and unconditional
  float2 sp[8];
  if (PRO != PRO_NONE) {
#pragma unroll
    for (int jj = 0; jj < 8; jj++) {
      const int j = min(w + SK_WAVES * jj, p.rowstat_parts - 1);
      sp[jj] = cx.ld_bulk(reinterpret_cast<const float2*>(p.rowstat + ((size_t)j * 64 + lane) * 2));
    }
  }
#pragma unroll
  for (int i = 0; i < 8; i++) {
    const int st = min(w * 8 + i, n16 - 1);    // clamped: steps beyond the range are never used
    if (!Cx::kPersistent) {
#pragma unroll
      for (int j = 0; j < NTL; j++) wf[j][i] = *reinterpret_cast<const bf16x8*>(wbase + ((size_t)j * KC16 + st) * 512);
    }
#pragma unroll
    for (int mb = 0; mb < NMB; mb++)
      xf[mb][i] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(xbase + ((size_t)min(mb_first + mb, mb_last) * XKC16 + st) * 512));
  }
  // operands of the epilogue, in the same round trip
  if (w < NFIN && mrow < p.M) {
    if (Cx::kPersistent) skinny_preload<PRO, EPI, PIECES, 1>(p, fnt, mrow, lh, fpc, ops, cx);
    else skinny_preload<PRO, EPI, PIECES, 2>(p, fnt, mrow, lh, fpc, ops, cx);
  }
  f32x16 acc[NSLOT];   // slot = token block (NTL == 1) or feature tile (NTL == 2)
#pragma unroll
  for (int sl = 0; sl < NSLOT; sl++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[sl][r] = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++) {
    if (w * 8 + i < n16) {
#pragma unroll
      for (int sl = 0; sl < NSLOT; sl++)
        acc[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[NTL == 1 ? 0 : sl][i], xf[NTL == 1 ? sl : 0][i], acc[sl], 0, 0, 0);
    }
  }
#pragma unroll
  for (int sl = 0; sl < NSLOT; sl++)
#pragma unroll
    for (int q = 0; q < 4; q++) {   // 16-byte pieces: [wave][slot][q][lane][4]
      const f32x4 v4 = {acc[sl][4 * q], acc[sl][4 * q + 1], acc[sl][4 * q + 2], acc[sl][4 * q + 3]};
      *reinterpret_cast<f32x4*>(red + ((((size_t)w * 2 + sl) * 4 + q) * 64 + lane) * 4) = v4;
    }
  cx.mark(1);   // operands arrived, products done
  if (PRO != PRO_NONE) {
    float pa = 0.f, pb = 0.f;
#pragma unroll
    for (int jj = 0; jj < 8; jj++) {
      if (w + SK_WAVES * jj < p.rowstat_parts) {
        pa += sp[jj].x;
        pb += sp[jj].y;
      }
    }
    sstat8[(w * 64 + lane) * 2] = pa;
    sstat8[(w * 64 + lane) * 2 + 1] = pb;
  }
  __syncthreads();
  cx.mark(2);   // partial tiles of all waves in LDS
  if (w >= NFIN) return;
  if (MS && cx.bz > mb_last) return;   // M <= 32: the second block of a split launch has nothing to store
  const int ml = mrow;
  float ssum = 0.f, ssq = 0.f;
  if (PRO != PRO_NONE) {   // statistics of the lane's own row: the 8 waves' partial sums, in wave order
#pragma unroll
    for (int ww = 0; ww < SK_WAVES; ww++) {
      ssum += sstat8[(ww * 64 + ml) * 2];
      ssq += sstat8[(ww * 64 + ml) * 2 + 1];
    }
  }
  if constexpr (PIECES == 1) skinny_finish<PRO, EPI, 0, 4>(p, red, fslot, lane, fnt, ml, lh, ssum, ssq, ops, cx);
  else if constexpr (PIECES == 2) {
    if (fpc == 0) skinny_finish<PRO, EPI, 0, 2>(p, red, fslot, lane, fnt, ml, lh, ssum, ssq, ops, cx);
    else skinny_finish<PRO, EPI, 2, 4>(p, red, fslot, lane, fnt, ml, lh, ssum, ssq, ops, cx);
  } else {
    if (fpc == 0) skinny_finish<PRO, EPI, 0, 1>(p, red, fslot, lane, fnt, ml, lh, ssum, ssq, ops, cx);
    else if (fpc == 1) skinny_finish<PRO, EPI, 1, 2>(p, red, fslot, lane, fnt, ml, lh, ssum, ssq, ops, cx);
    else if (fpc == 2) skinny_finish<PRO, EPI, 2, 3>(p, red, fslot, lane, fnt, ml, lh, ssum, ssq, ops, cx);
    else skinny_finish<PRO, EPI, 3, 4>(p, red, fslot, lane, fnt, ml, lh, ssum, ssq, ops, cx);
  }
}

template <int PRO, int EPI, int MS = 0>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_skinny_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  gemm_skinny_body<PRO, EPI, MS>(p, LaunchCtx::from_block_idx(), smem_raw);
}

// Skinny GEMM over the whole k range on 16-feature x 16-token tiles (mfma_f32_16x16x32_bf16): the
// expert's O and down projections.  A launch lasts as long as its busiest CU needs to pull its
// operands, and a CU sustains only ~60-100 GB/s, so the 64 x 1024 output is cut into 256 blocks
// (one per CU) of 16 x 16: each block reads 16 weight rows and 16 token rows over all of k, half of
// what a 32 x 32 tile needs, and every CU takes part.  The 16-row operand of one 32-k step is two
// half fragments of the 32 x 16 fragment order (weights and XF activations alike): lane (g, i),
// g = lane / 16, i = lane % 16, takes the 16 bytes of row i at k = 32 j + 8 g .. + 7, i.e. piece
// ((g & 1) * 32 + 16 * (tile & 1) + i) of fragment 2 j + (g >> 1); every lane of every load is
// used.  8 waves split k; NS steps per wave, all loads issued at once; fixed-order LDS reduction;
// wave 0 adds the residual, writes fp32, the gain-scaled bf16 copy and per-tile row statistics.
// Accumulator: lane -> token lane % 16, features 4 * (lane / 16) + r.
template <int NS, class Cx>
__device__ __forceinline__ void gemm_skinny16_body(const GemmParams p, const Cx cx, unsigned char* smem_raw) {
  float (*red)[64][4] = reinterpret_cast<float (*)[64][4]>(smem_raw);   // [SK_WAVES][64][4]
  const int t = cx.tid();
  const int lane = t & 63;
  const int w = t >> 6;
  const int li = lane & 15;
  const int lg = lane >> 4;
  const int ntiles16 = p.n_tiles * 2;
  if (!Cx::kPersistent) {
    if (cx.bx >= ntiles16) {   // warm-up block; rank = linear block index (mod 8)
      prefetch_role(p.pf, cx.bx - ntiles16 + cx.by * ((int)gridDim.x - ntiles16));
      return;
    }
  }
  const int nt16 = cx.bx;
  const int mt16 = cx.by;
  const int KC16 = p.W.k_pad >> 4;
  const int XKC16 = p.ldx >> 4;
  const int piece_w = ((lg & 1) * 32 + (nt16 & 1) * 16 + li) * 8;
  const int piece_x = ((lg & 1) * 32 + (mt16 & 1) * 16 + li) * 8;
  const bf16* wbase = p.W.w + ((size_t)(nt16 >> 1) * KC16 + (size_t)w * NS * 2 + (lg >> 1)) * 512 + piece_w;
  const bf16* xbase = p.X + ((size_t)(mt16 >> 1) * XKC16 + (size_t)w * NS * 2 + (lg >> 1)) * 512 + piece_x;
  bf16x8 wf[NS], xf[NS];
  const int m = mt16 * 16 + li;
  // operands of the epilogue (wave 0): the constants with the weights, the residual rows with the inputs
  const int n4 = nt16 * 16 + 4 * lg;
  const bool live = w == 0 && m < p.M && n4 < p.n_valid;
  f32x4 rv = {0.f, 0.f, 0.f, 0.f}, gv = {1.f, 1.f, 1.f, 1.f}, bv = {0.f, 0.f, 0.f, 0.f};
  if (Cx::kPersistent) {   // constants before the wait
#pragma unroll
    for (int j = 0; j < NS; j++) wf[j] = *reinterpret_cast<const bf16x8*>(wbase + (size_t)j * 1024);
    if (live) {
      if (p.gain != nullptr) gv = *reinterpret_cast<const f32x4*>(p.gain + n4);
      if (p.bias != nullptr) bv = *reinterpret_cast<const f32x4*>(p.bias + n4);
    }
    cx.wait_inputs();
  }
#pragma unroll
  for (int j = 0; j < NS; j++) {
    if (!Cx::kPersistent) wf[j] = *reinterpret_cast<const bf16x8*>(wbase + (size_t)j * 1024);
    xf[j] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(xbase + (size_t)j * 1024));
  }
  // X given as attention shares over disjoint key ranges (k = 8 heads x 256, so wave w holds exactly
  // head w).  Share z carries its normalised output and (max, sum) of its exponentials; the merged
  // row is sum_z c_z x_z with c_z = l_z exp(m_z - max m) / sum over shares.  The product is linear
  // in x and a lane of the accumulator belongs to one token, so every share is multiplied on its
  // own and the 4 accumulator values per lane are combined with the lane's c_z: no element-wise
  // merge of the operand fragments.
  f32x4 acc_merged = {0.f, 0.f, 0.f, 0.f};
  const bool merge = NS == 8 && p.xsplits > 1;
  if (NS == 8 && p.xsplits > 1) {
    const int nz = p.xsplits;             // 2 .. 4, uniform
    bf16x8 xo[3][NS];
    float2 ml[4];
    const int mrow = min(m, 63);
    ml[0] = cx.ld_bulk(reinterpret_cast<const float2*>(p.xsplit_ml + ((size_t)w * 64 + mrow) * 2));
#pragma unroll
    for (int z = 1; z < 4; z++) {
      if (z < nz) {
#pragma unroll
        for (int j = 0; j < NS; j++) xo[z - 1][j] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(xbase + (size_t)z * p.xsplit_stride + (size_t)j * 1024));
        ml[z] = cx.ld_bulk(reinterpret_cast<const float2*>(p.xsplit_ml + (((size_t)z * SK_WAVES + w) * 64 + mrow) * 2));
      }
    }
    float mx = ml[0].x;
#pragma unroll
    for (int z = 1; z < 4; z++) {
      if (z < nz) mx = fmaxf(mx, ml[z].x);
    }
    float c[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f;
#pragma unroll
    for (int z = 0; z < 4; z++) {
      if (z < nz) {
        c[z] = ml[z].y * __expf(ml[z].x - mx);
        den += c[z];
      }
    }
    const float rden = 1.0f / den;
#pragma unroll
    for (int z = 0; z < 4; z++) c[z] *= rden;
#pragma unroll
    for (int z = 0; z < 4; z++) {
      if (z < nz) {
        f32x4 az = {0.f, 0.f, 0.f, 0.f}, az1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NS; j += 2) {
          az = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j], z == 0 ? xf[j] : xo[z == 0 ? 0 : z - 1][j], az, 0, 0, 0);
          az1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j + 1], z == 0 ? xf[j + 1] : xo[z == 0 ? 0 : z - 1][j + 1], az1, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; r++) acc_merged[r] += c[z] * (az[r] + az1[r]);
      }
    }
  }
  // operands of the epilogue (wave 0), behind the operand loads
  if (live) {
    if (p.resid != nullptr) rv = cx.ld(reinterpret_cast<const f32x4*>(p.resid + (size_t)m * p.ldo + n4));
    if (!Cx::kPersistent) {
      if (p.gain != nullptr) gv = *reinterpret_cast<const f32x4*>(p.gain + n4);
      if (p.bias != nullptr) bv = *reinterpret_cast<const f32x4*>(p.bias + n4);
    }
  }
  f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  if (!merge) {
#pragma unroll
    for (int j = 0; j < NS; j += 2) {
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j], xf[j], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j + 1], xf[j + 1], acc1, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; r++) acc0[r] += acc1[r];
  } else {
    acc0 = acc_merged;
  }
  *reinterpret_cast<f32x4*>(&red[w][lane][0]) = acc0;
  __syncthreads();
  if (w != 0) return;
  float v[4];
  {
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ww = 0; ww < SK_WAVES; ww++) a += *reinterpret_cast<const f32x4*>(&red[ww][lane][0]);
#pragma unroll
    for (int r = 0; r < 4; r++) v[r] = a[r] + bv[r] + rv[r];
  }
  float st_a = 0.f, st_b = 0.f;
  const int mo = m + p.row_offset;
  if (live) {
    const f32x4 o = {v[0], v[1], v[2], v[3]};
    cx.st(reinterpret_cast<f32x4*>(p.out_f32 + (size_t)mo * p.ldo + n4), o);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      st_a += v[r];
      st_b += v[r] * v[r];
    }
    const bf16x4 ob = {(bf16)(v[0] * gv[0]), (bf16)(v[1] * gv[1]), (bf16)(v[2] * gv[2]), (bf16)(v[3] * gv[3])};
    cx.st(reinterpret_cast<bf16x4*>(p.out_bf16 + xf_index(mo, n4, p.ldo2 >> 4)), ob);
  }
  if (p.stat_out != nullptr) {   // partial row statistics over this tile's 16 columns: [16-column tile][64 rows][2]
    st_a += __shfl_xor(st_a, 16, 64);
    st_b += __shfl_xor(st_b, 16, 64);
    st_a += __shfl_xor(st_a, 32, 64);
    st_b += __shfl_xor(st_b, 32, 64);
    if (lg == 0 && m < p.M) {
      float* dst = p.stat_out + ((size_t)nt16 * 64 + mo) * 2;
      cx.st(reinterpret_cast<float2*>(dst), make_float2(st_a, st_b));
    }
  }
}

template <int NS>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_skinny16_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem16[SK_WAVES * 64 * 4 * 4];
  gemm_skinny16_body<NS>(p, LaunchCtx::from_block_idx(), smem16);
}

