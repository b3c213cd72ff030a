// Attainable-peak micro-benchmarks: what this one device sustains on the two resources that bound
// the forward pass (Section 5.1 of the paper prices every GEMM by memory bandwidth or by matrix
// throughput).  A streaming read of a large buffer gives the HBM figure, a register-resident
// loop of independent bf16 MFMAs gives the matrix figure.  Both are reported beside the published
// peaks, so that a roofline fraction can be read against either.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "pi0_internal.h"

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int PEAK_THREADS = 256;
constexpr int READ_BLOCKS = 2048;      // 8 blocks per compute unit
constexpr int MFMA_BLOCKS = 512;       // 2 blocks of 4 waves per compute unit: 2 waves per SIMD
constexpr int MFMA_ACC = 4;            // independent accumulators per wave
constexpr unsigned NEVER = 0x9e3779b9u;

// Every lane xor-folds what it reads and compares the fold with a constant: the store below is
// practically never taken, but the loads cannot be removed.  A plain grid-stride loop (consecutive
// lanes on consecutive 16-byte words, the whole grid one contiguous front moving through the
// buffer) measured fastest here: 6.4-6.5 TB/s against 5.0-5.7 TB/s for variants that keep several
// loads per lane in flight a whole grid apart, and the same on zeros as on random words.
__global__ __launch_bounds__(PEAK_THREADS) void peak_read_kernel(const u32x4* buf, size_t n16, unsigned* sink) {
  const size_t stride = (size_t)gridDim.x * PEAK_THREADS;
  u32x4 f = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * PEAK_THREADS + threadIdx.x; i < n16; i += stride) f ^= buf[i];
  const unsigned fold = f[0] ^ f[1] ^ f[2] ^ f[3];
  if (fold == NEVER) sink[0] = fold;
}

// What the caches deliver to the compute units: every block reads one of eight slices over and over (the blocks of
// a die share a slice), 8 loads of 16 bytes in flight per lane.
__global__ __launch_bounds__(512) void peak_cache_kernel(const u32x4* buf, size_t n16_slice, int iters, unsigned* sink) {
  const u32x4* p = buf + (size_t)(blockIdx.x & 7) * n16_slice;
  u32x4 f = {0u, 0u, 0u, 0u};
  for (int it = 0; it < iters; it++) {
    for (size_t i = threadIdx.x; i < n16_slice; i += 8 * 512) {
      u32x4 v[8];
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const size_t idx = i + (size_t)j * 512;
        v[j] = p[idx < n16_slice ? idx : n16_slice - 1];
      }
#pragma unroll
      for (int j = 0; j < 8; j++) f ^= v[j];
    }
    asm volatile("" ::: "memory");   // the next pass reads again
  }
  const unsigned fold = f[0] ^ f[1] ^ f[2] ^ f[3];
  if (fold == NEVER) sink[0] = fold;
}

// Operands and accumulators never leave the registers.  The operands are small non-zero values
// that differ per lane (a matrix pipe fed with zeros draws less power and clocks higher than one
// fed with data).
__global__ __launch_bounds__(PEAK_THREADS) void peak_mfma_kernel(int iters, unsigned* sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; j++) {
    a[j] = (__bf16)((float)(((lane * 7 + j * 3) & 15) - 8) * 0.0625f + 0.03125f);
    b[j] = (__bf16)((float)(((lane * 5 + j * 11) & 15) - 7) * 0.0625f - 0.03125f);
  }
  f32x16 acc[MFMA_ACC];
#pragma unroll
  for (int q = 0; q < MFMA_ACC; q++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[q][r] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int q = 0; q < MFMA_ACC; q++) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < MFMA_ACC; q++)
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc[q][r];
  if (__builtin_bit_cast(unsigned, s) == NEVER) sink[0] = NEVER;
}

// the shader's cycle counter (moves with the clock the power management currently grants) and the constant
// 100 MHz counter, read back to back by one lane.  The cycle counters of the eight dies do not start together
// (two samples taken on different dies gave "3.2 GHz"), and a one-block launch lands on any die: so the launch has
// 256 one-wave blocks and only those on die 0, shader engine 0 write the pair (several may: they differ by well
// under a microsecond).
__global__ void clock_pair_kernel(long long* out) {
  const unsigned xcc = (unsigned)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7u;    // XCC_ID, bits 3:0
  const unsigned se = (unsigned)__builtin_amdgcn_s_getreg(4 | (13 << 6) | (2 << 11)) & 7u;     // HW_ID, SE_ID bits 15:13
  if (xcc != 0u || se != 0u || threadIdx.x != 0) return;
  out[0] = (long long)__builtin_amdgcn_s_memtime();
  out[1] = (long long)wall_clock64();
}

}  // namespace

extern "C" int pi0_clock_sample(long long* d_out, void* hip_stream) {
  if (d_out == nullptr || (reinterpret_cast<uintptr_t>(d_out) & 7) != 0) return PI0_EINVAL;
  clock_pair_kernel<<<256, 64, 0, reinterpret_cast<hipStream_t>(hip_stream)>>>(d_out);
  return hipGetLastError() == hipSuccess ? PI0_OK : PI0_EHIP;
}

extern "C" int pi0_peak_bench(int kind, const void* d_buf, size_t bytes, int iters, int reps, unsigned* d_sink,
                              double* h_result, void* hip_stream) {
  if (d_sink == nullptr || h_result == nullptr || reps < 1 || reps > 1000) return PI0_EINVAL;
  if (kind == PI0_PEAK_HBM_READ) {
    if (d_buf == nullptr || bytes < 16 || (bytes & 15) != 0 || (reinterpret_cast<uintptr_t>(d_buf) & 15) != 0) return PI0_EINVAL;
  } else if (kind == PI0_PEAK_MFMA_BF16) {
    if (iters < 1 || iters > (1 << 22)) return PI0_EINVAL;
  } else if (kind == PI0_PEAK_CACHE_READ) {
    if (d_buf == nullptr || bytes < 65536 || (bytes & 127) != 0 || (reinterpret_cast<uintptr_t>(d_buf) & 15) != 0) return PI0_EINVAL;
    if (iters < 1 || iters > (1 << 20)) return PI0_EINVAL;
  } else {
    return PI0_EINVAL;
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) {
    // one untimed launch first (code upload, clocks), then `reps` timed ones
    for (int r = -1; r < reps && e == hipSuccess; r++) {
      if (r == 0) e = hipEventRecord(e0, s);
      if (e != hipSuccess) break;
      if (kind == PI0_PEAK_HBM_READ)
        peak_read_kernel<<<dim3(READ_BLOCKS), dim3(PEAK_THREADS), 0, s>>>(reinterpret_cast<const u32x4*>(d_buf), bytes / 16, d_sink);
      else if (kind == PI0_PEAK_CACHE_READ)
        peak_cache_kernel<<<dim3(256), dim3(512), 0, s>>>(reinterpret_cast<const u32x4*>(d_buf), bytes / 128, iters, d_sink);
      else
        peak_mfma_kernel<<<dim3(MFMA_BLOCKS), dim3(PEAK_THREADS), 0, s>>>(iters, d_sink);
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) {
      const double sec = (double)ms * 1e-3 / reps;
      if (sec <= 0.0) {
        e = hipErrorUnknown;
      } else if (kind == PI0_PEAK_HBM_READ) {
        *h_result = (double)bytes / sec * 1e-9;                                  // GB/s
      } else if (kind == PI0_PEAK_CACHE_READ) {
        *h_result = 256.0 * (double)iters * (double)(bytes / 8) / sec * 1e-9;    // GB/s into the compute units
      } else {
        const double flops = (double)MFMA_BLOCKS * (PEAK_THREADS / 64) * (double)iters * MFMA_ACC * (2.0 * 32 * 32 * 16);
        *h_result = flops / sec * 1e-12;                                         // TFLOP/s
      }
    }
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  return e == hipSuccess ? PI0_OK : PI0_EHIP;
}

// One read-ahead kernel over a caller's buffer, alone on the stream: the buffer is cut into `layers` equal
// slices (one range per layer), the kernel walks steps * layers of them at the pace d_progress allows.
extern "C" int pi0_read_ahead_probe(const void* d_buf, size_t bytes, int layers, int steps, int lead, const int* d_progress,
                                    long long wait_ticks, int blocks, unsigned* d_sink, double* h_ms, void* hip_stream) {
  if (d_buf == nullptr || d_progress == nullptr || d_sink == nullptr || h_ms == nullptr) return PI0_EINVAL;
  if (layers < 1 || layers > 4096 || steps < 1 || steps > 4096 || lead < 1 || wait_ticks < 1 || blocks < 1 || blocks > 1024)
    return PI0_EINVAL;
  if ((reinterpret_cast<uintptr_t>(d_buf) & 15) != 0 || bytes < (size_t)layers * 16 || bytes % ((size_t)layers * 16) != 0 ||
      bytes / layers >= ((size_t)1 << 31))
    return PI0_EINVAL;
  ReadAheadParams p;
  memset(&p, 0, sizeof(p));
  p.base[0] = reinterpret_cast<const unsigned char*>(d_buf);
  p.layer_stride[0] = bytes / layers;
  p.n16[0] = (unsigned)(bytes / layers / 16);
  p.layers = layers; p.steps = steps; p.lead = lead;
  p.progress = d_progress;
  p.wait_ticks = wait_ticks;
  p.sink = d_sink;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) e = hipEventRecord(e0, s);
  if (e == hipSuccess) e = launch_read_ahead(s, p, blocks, 256, 4);
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  if (e == hipSuccess) *h_ms = (double)ms;
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  return e == hipSuccess ? PI0_OK : PI0_EHIP;
}
