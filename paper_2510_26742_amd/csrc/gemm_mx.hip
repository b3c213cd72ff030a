// Reduced-precision variant of the prefix feed-forward GEMMs (gate||up with the GeGLU epilogue, down as
// split-K partials) on MXFP8 operands: FP8 E4M3 elements with one power-of-two scale per 32 consecutive
// k, multiplied by mfma_scale_f32_32x32x64_f8f6f4, which applies the block scales in hardware.  The
// paper only names 8-bit multiplication as a direction (Section 9.1); the format and where the rounding
// happens are choices of this build.
//
// Same plan as the bf16 tall kernel with two feature tiles per wave: block = 128 tokens x 256 features,
// 4 waves x 2 feature tiles; the activation chunk (128 tokens x 64 k = 8 KiB) is staged through LDS, the
// weights go straight to registers; one MFMA covers a whole 64-k chunk, so a chunk is 8 MFMAs per wave.
// Four register stages in flight; the scales of four chunks are one dword per lane, fetched one group
// of four chunks ahead.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pi0_internal.h"

namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int MX_MB = 4;       // 32-token blocks per tile
constexpr int MX_WN = 4;       // waves
constexpr int MX_NT = 2;       // feature tiles per wave
constexpr int MX_D = 4;        // register stages (= chunks per scale group)
constexpr int MX_NP = MX_MB * 2 / MX_WN;          // 1 KiB activation pieces staged per wave per chunk
constexpr int MX_SMEM = 2 * MX_MB * 2048;         // two buffers of MB fragments

__device__ __forceinline__ i32x8 cat(const i32x4& lo, const i32x4& hi) {
  i32x8 r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return r;
}

__device__ __forceinline__ float gelu_tanh_mx(float x) {
  // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3)
  const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  return x * __builtin_amdgcn_rcpf(1.0f + exp2f(-2.885390081777927f * u));
}

// OCC = blocks per CU the register budget is cut for: with more blocks than CUs, two resident blocks hide each
// other's waits (measured -16 % at 512 / 768 tokens, at the price of a few spilled registers); with one block per
// CU the full register file is the better use (+20 % the other way at 256 tokens).
template <int EPI, int OCC>
__global__ __launch_bounds__(64 * MX_WN) __attribute__((amdgpu_waves_per_eu(OCC, OCC))) void gemm_mx_kernel(MxGemmParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char xs[];     // [2][MB * 2][1024]
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wn = t >> 6;
  const int lq = lane & 31;
  const int lh = lane >> 5;

  const int n_tiles = p.n_pad >> 5;
  const int nblocks_n = n_tiles / (MX_WN * MX_NT);
  const int id = blockIdx.x;
  const int slot = id >> 3;
  const int nb = (id & 7) + 8 * (slot / p.m_tiles);      // the blocks that share a weight panel run on one XCD
  const int mt = slot % p.m_tiles;
  if (nb >= nblocks_n) return;
  const int m0 = mt * (MX_MB * 32);
  const int nt0 = (nb * MX_WN + wn) * MX_NT;

  const int KC64 = p.k_pad >> 6;
  const int XKC64 = p.ldx >> 6;
  const int kbeg = blockIdx.y * p.k_per_split;
  const int kend = min(kbeg + p.k_per_split, p.k_pad);
  const int NC = (kend - kbeg) >> 6;                      // multiple of 4 (host)
  const int NG = NC >> 2;
  const int mb_last = (p.M - 1) >> 5;

  // operand addresses: a 1 KiB piece pair is lane-contiguous (16 bytes per lane)
  const unsigned char* xsrc[MX_NP];
#pragma unroll
  for (int i = 0; i < MX_NP; i++) {
    const int f = wn + MX_WN * i;                         // piece pair f = mb * 2 + half
    const int mbg = min((m0 >> 5) + (f >> 1), mb_last);
    xsrc[i] = p.X8 + ((size_t)mbg * XKC64 + (kbeg >> 6)) * 2048 + (f & 1) * 1024 + lane * 16;
  }
  const unsigned char* wsrc[MX_NT];
  const unsigned char* wscl[MX_NT];
#pragma unroll
  for (int j = 0; j < MX_NT; j++) {
    wsrc[j] = p.W8 + ((size_t)(nt0 + j) * KC64 + (kbeg >> 6)) * 2048 + lane * 16;
    wscl[j] = p.WS + (((size_t)(nt0 + j) * (KC64 >> 2) + (kbeg >> 8)) * 64 + lane) * 4;
  }
  const unsigned char* xscl[MX_MB];
#pragma unroll
  for (int mb = 0; mb < MX_MB; mb++) {
    const int mbg = min((m0 >> 5) + mb, mb_last);
    xscl[mb] = p.XS + (((size_t)mbg * (XKC64 >> 2) + (kbeg >> 8)) * 64 + lane) * 4;
  }

  i32x4 xr[MX_D][MX_NP];
  i32x4 wr[MX_D][MX_NT][2];
#define MX_ISSUE(c, u)                                                                              \
  {                                                                                                 \
    const int cc_ = min((c), NC - 1);                                                               \
    _Pragma("unroll") for (int i = 0; i < MX_NP; i++)                                               \
      xr[u][i] = *reinterpret_cast<const i32x4*>(xsrc[i] + (size_t)cc_ * 2048);                     \
    _Pragma("unroll") for (int j = 0; j < MX_NT; j++) {                                             \
      wr[u][j][0] = *reinterpret_cast<const i32x4*>(wsrc[j] + (size_t)cc_ * 2048);                  \
      wr[u][j][1] = *reinterpret_cast<const i32x4*>(wsrc[j] + (size_t)cc_ * 2048 + 1024);           \
    }                                                                                               \
  }
#define MX_STORE(u, buf)                                                                            \
  {                                                                                                 \
    _Pragma("unroll") for (int i = 0; i < MX_NP; i++)                                               \
      *reinterpret_cast<i32x4*>(xs + ((size_t)(buf) * MX_MB * 2 + wn + MX_WN * i) * 1024 + lane * 16) = xr[u][i]; \
  }

  f32x16 acc[MX_NT][MX_MB];
#pragma unroll
  for (int j = 0; j < MX_NT; j++)
#pragma unroll
    for (int mb = 0; mb < MX_MB; mb++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[j][mb][r] = 0.f;

#pragma unroll
  for (int u = 0; u < MX_D; u++) MX_ISSUE(u, u)
  int sw_c[MX_NT], sx_c[MX_MB], sw_n[MX_NT], sx_n[MX_MB];
#pragma unroll
  for (int j = 0; j < MX_NT; j++) sw_c[j] = *reinterpret_cast<const int*>(wscl[j]);
#pragma unroll
  for (int mb = 0; mb < MX_MB; mb++) sx_c[mb] = *reinterpret_cast<const int*>(xscl[mb]);
  MX_STORE(0, 0)
  __syncthreads();

  int cur = 0;
  for (int g = 0; g < NG; g++) {
    const int gn = min(g + 1, NG - 1);                    // next group's scales (clamped on the last group)
#pragma unroll
    for (int j = 0; j < MX_NT; j++) sw_n[j] = *reinterpret_cast<const int*>(wscl[j] + (size_t)gn * 256);
#pragma unroll
    for (int mb = 0; mb < MX_MB; mb++) sx_n[mb] = *reinterpret_cast<const int*>(xscl[mb] + (size_t)gn * 256);
    // one chunk: u is the register stage and also selects the chunk's byte of the scale dwords (an immediate)
#define MX_CHUNK(u)                                                                                              \
    {                                                                                                            \
      const int c = g * MX_D + (u);                                                                              \
      const unsigned char* xb = xs + (size_t)cur * MX_MB * 2048 + lane * 16;                                     \
      _Pragma("unroll") for (int mb = 0; mb < MX_MB; mb++) {                                                     \
        const i32x4 blo = *reinterpret_cast<const i32x4*>(xb + (size_t)(mb * 2) * 1024);                         \
        const i32x4 bhi = *reinterpret_cast<const i32x4*>(xb + (size_t)(mb * 2 + 1) * 1024);                     \
        const i32x8 bq = cat(blo, bhi);                                                                          \
        _Pragma("unroll") for (int j = 0; j < MX_NT; j++)                                                        \
          acc[j][mb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(cat(wr[u][j][0], wr[u][j][1]), bq,        \
                                                                      acc[j][mb], 0, 0, (u), sw_c[j], (u), sx_c[mb]); \
      }                                                                                                          \
      MX_ISSUE(c + MX_D, u)                                                                                      \
      MX_STORE(((u) + 1) % MX_D, cur ^ 1)                                                                        \
      __syncthreads();                                                                                           \
      cur ^= 1;                                                                                                  \
    }
    MX_CHUNK(0)
    MX_CHUNK(1)
    MX_CHUNK(2)
    MX_CHUNK(3)
#undef MX_CHUNK
#pragma unroll
    for (int j = 0; j < MX_NT; j++) sw_c[j] = sw_n[j];
#pragma unroll
    for (int mb = 0; mb < MX_MB; mb++) sx_c[mb] = sx_n[mb];
  }
#undef MX_ISSUE
#undef MX_STORE

  // ---- epilogue: lane -> token lq of each 32-token block, features nt * 32 + 8 * (r / 4) + 4 * lh + r % 4 ----
  if (EPI == MX_EPI_PARTIAL) {
#pragma unroll
    for (int mb = 0; mb < MX_MB; mb++) {
      const int m = m0 + mb * 32 + lq;
      if (m < p.M) {
#pragma unroll
        for (int j = 0; j < MX_NT; j++)
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const int n4 = (nt0 + j) * 32 + 8 * i + 4 * lh;
            const f32x4 o = {acc[j][mb][4 * i], acc[j][mb][4 * i + 1], acc[j][mb][4 * i + 2], acc[j][mb][4 * i + 3]};
            *reinterpret_cast<f32x4*>(p.out_f32 + ((size_t)blockIdx.y * p.M + m) * p.ldo + n4) = o;
          }
      }
    }
  } else {
    // RMS statistics of the rows, then gelu(gate) * up of neighbouring accumulator pairs: the wave's two tiles
    // give 32 consecutive product columns = one scale block of the down projection's input
    float2 rst[MX_MB];
#pragma unroll
    for (int mb = 0; mb < MX_MB; mb++)
      rst[mb] = *reinterpret_cast<const float2*>(p.rowstat + 2 * (size_t)min(m0 + mb * 32 + lq, p.M - 1));
    const float inv_k = 1.0f / (float)p.k_true;
    const int OKC64 = p.ldo8 >> 6;
#pragma unroll
    for (int mb = 0; mb < MX_MB; mb++) {
      const int m = m0 + mb * 32 + lq;
      const float rs = rsqrtf(rst[mb].y * inv_k + 1e-6f);
      float pr[MX_NT][8];        // products 4 i + 2 lh + {0, 1} of tile j at [j][2 i + {0, 1}]
      float amax = 0.f;
#pragma unroll
      for (int j = 0; j < MX_NT; j++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const float g0 = acc[j][mb][4 * i] * rs, u0 = acc[j][mb][4 * i + 1] * rs;
          const float g1 = acc[j][mb][4 * i + 2] * rs, u1 = acc[j][mb][4 * i + 3] * rs;
          pr[j][2 * i] = gelu_tanh_mx(g0) * u0;
          pr[j][2 * i + 1] = gelu_tanh_mx(g1) * u1;
          amax = fmaxf(amax, fmaxf(fabsf(pr[j][2 * i]), fabsf(pr[j][2 * i + 1])));
        }
      amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
      const int code = mx_scale_code(amax);
      const float inv = mx_inv_scale(code);
      const int mbg = (m0 >> 5) + mb;
#pragma unroll
      for (int j = 0; j < MX_NT; j++) {
        const int col0 = (nt0 + j) * 16;                 // first of the tile's 16 product columns
        unsigned char* frag = p.out8 + ((size_t)mbg * OKC64 + (col0 >> 6)) * 2048 + ((size_t)((col0 & 63) >> 4) * 32 + lq) * 16;
#pragma unroll
        for (int ip = 0; ip < 2; ip++) {
          // steps 2 ip and 2 ip + 1: half 0 ends up with the four columns of step 2 ip, half 1 with those of step 2 ip + 1
          const unsigned e_even = mx_encode2(pr[j][4 * ip], pr[j][4 * ip + 1], inv);
          const unsigned e_odd = mx_encode2(pr[j][4 * ip + 2], pr[j][4 * ip + 3], inv);
          const unsigned give = lh ? e_even : e_odd;
          const unsigned got = (unsigned)__shfl_xor((int)give, 32, 64);
          const unsigned word = lh ? (got | (e_odd << 16)) : (e_even | (got << 16));
          if (m < p.M) *reinterpret_cast<unsigned*>(frag + 8 * ip + 4 * lh) = word;
        }
      }
      if (lh == 0 && m < p.M) {
        const int chunk = (nt0 * 16) >> 6, b = ((nt0 * 16) & 63) >> 5;
        p.out_scales[(((size_t)mbg * (OKC64 >> 2) + (chunk >> 2)) * 64 + b * 32 + lq) * 4 + (chunk & 3)] = (unsigned char)code;
      }
    }
  }
}

}  // namespace

hipError_t gemm_mx_init_attributes() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mx_kernel<MX_EPI_PARTIAL, 1>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, MX_SMEM);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mx_kernel<MX_EPI_GEGLU, 1>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, MX_SMEM);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mx_kernel<MX_EPI_GEGLU, 2>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, MX_SMEM);
}

hipError_t launch_gemm_mx(hipStream_t s, int epi, const MxGemmParams& p, int z_splits) {
  // everything the kernel's indexing assumes
  if (p.X8 == nullptr || p.XS == nullptr || p.W8 == nullptr || p.WS == nullptr || p.M <= 0 || z_splits < 1) return hipErrorInvalidValue;
  if (p.n_pad % 256 != 0 || p.k_pad % 256 != 0 || p.ldx % 256 != 0 || p.ldx < p.k_pad) return hipErrorInvalidValue;
  if (p.k_per_split <= 0 || p.k_per_split % 256 != 0 || (long)p.k_per_split * z_splits < p.k_pad) return hipErrorInvalidValue;
  if ((long)p.k_per_split * (z_splits - 1) >= p.k_pad) return hipErrorInvalidValue;     // no empty slice
  if (p.m_tiles < 1 || p.m_tiles * MX_MB * 32 < p.M) return hipErrorInvalidValue;
  if (epi == MX_EPI_PARTIAL) {
    if (p.out_f32 == nullptr || p.ldo < p.n_pad || p.ldo % 4 != 0) return hipErrorInvalidValue;
  } else if (epi == MX_EPI_GEGLU) {
    if (z_splits != 1 || p.rowstat == nullptr || p.out8 == nullptr || p.out_scales == nullptr || p.k_true <= 0) return hipErrorInvalidValue;
    if (p.ldo8 % 256 != 0 || p.ldo8 < p.n_pad / 2) return hipErrorInvalidValue;
  } else {
    return hipErrorInvalidValue;
  }
  const int nblocks_n = (p.n_pad >> 5) / (MX_WN * MX_NT);
  const dim3 grid(8 * ((nblocks_n + 7) / 8) * p.m_tiles, z_splits);
  if (epi == MX_EPI_PARTIAL) gemm_mx_kernel<MX_EPI_PARTIAL, 1><<<grid, dim3(64 * MX_WN), MX_SMEM, s>>>(p);
  else if (nblocks_n * p.m_tiles > 256) gemm_mx_kernel<MX_EPI_GEGLU, 2><<<grid, dim3(64 * MX_WN), MX_SMEM, s>>>(p);
  else gemm_mx_kernel<MX_EPI_GEGLU, 1><<<grid, dim3(64 * MX_WN), MX_SMEM, s>>>(p);
  return hipGetLastError();
}
