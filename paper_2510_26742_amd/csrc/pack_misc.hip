// Load-time weight packing (the graph simplifications of Section 3.2 applied to the weights) and
// the small non-GEMM kernels of the pass (patch extraction, prompt embedding, state token,
// folded action/time embedding of Table 2 rows 1x32x1024 and 63x32x1024).
#include "pi0_internal.h"
#include "embed_bodies.h"

// ------------------------------------------------------------------------------------------------
// packed row n -> (source matrix, source column); returns false for padding rows
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ bool map_row(const PackSrc& s, int n, int& which, int& col) {
  if (n >= s.n_true) return false;
  if (s.rowmap == ROWMAP_PAIR) {
    which = n & 1;
    col = n >> 1;
    return true;
  }
  if (s.rowmap == ROWMAP_ROPE_QKV) {
    const int qc = s.q_heads * 256;
    if (n < qc + 256) {
      const bool is_q = n < qc;
      const int nl = is_q ? n : n - qc;
      const int head = nl >> 8, pp = nl & 255;
      const int d = (pp >> 1) + 128 * (pp & 1);
      which = is_q ? 0 : 1;
      col = head * 256 + d;
      return true;
    }
    which = 2;
    col = n - qc - 256;
    return true;
  }
  int c = n;
  for (int i = 0; i < 3; i++) {
    if (c < s.cols[i]) {
      which = i;
      col = c;
      return true;
    }
    c -= s.cols[i];
  }
  return false;
}

__device__ __forceinline__ float k_scale(const PackSrc& s, int k) {
  if (s.kscale == KSCALE_GAIN) return (float)s.gain[k];
  if (s.kscale == KSCALE_ONE_PLUS) return 1.0f + (float)s.gain[k];
  return 1.0f;
}

// one thread per 16-byte fragment piece: (n-tile, k-step, lane)
__global__ __launch_bounds__(256) void pack_weights_kernel(PackSrc s, bf16* dst, int n_pad, int k_pad) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t total = (size_t)(n_pad >> 5) * (k_pad >> 4) * 64;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const size_t f = idx >> 6;
  const int kc = (int)(f % (size_t)(k_pad >> 4));
  const int nt = (int)(f / (size_t)(k_pad >> 4));
  const int n = nt * 32 + (lane & 31);
  const int k0 = kc * 16 + (lane >> 5) * 8;
  int which = 0, col = 0;
  const bool live = map_row(s, n, which, col);
  bf16x8 out;
#pragma unroll
  for (int j = 0; j < 8; j++) {
    const int k = k0 + j;
    float v = 0.f;
    if (live && k < s.K) v = (float)s.src[which][(size_t)k * s.cols[which] + col];
    out[j] = (bf16)v;
  }
  *reinterpret_cast<bf16x8*>(dst + idx * 8) = out;
}

hipError_t launch_pack_weights(hipStream_t st, const PackSrc& s, bf16* dst, int n_pad, int k_pad) {
  if (n_pad % 32 != 0 || k_pad % 64 != 0 || s.n_true > n_pad || s.K > k_pad || dst == nullptr) return hipErrorInvalidValue;
  const size_t total = (size_t)(n_pad >> 5) * (k_pad >> 4) * 64;
  hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s, dst, n_pad, k_pad);
  return hipGetLastError();
}

// MXFP8 copy of a weight matrix: one thread per (n-tile, 64-k fragment, lane); lane (b, i) quantises the 32
// values of row i in k block b of the fragment (one scale) and writes the block's two 16-byte pieces.
__global__ __launch_bounds__(256) void pack_weights_mx_kernel(PackSrc s, unsigned char* dst, unsigned char* scales, int n_pad,
                                                              int k_pad) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int kc64 = k_pad >> 6;
  const size_t total = (size_t)(n_pad >> 5) * kc64 * 64;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  const size_t f = idx >> 6;
  const int kc = (int)(f % (size_t)kc64);
  const int nt = (int)(f / (size_t)kc64);
  const int i = lane & 31, b = lane >> 5;
  const int n = nt * 32 + i;
  const int k0 = kc * 64 + b * 32;
  int which = 0, col = 0;
  const bool live = map_row(s, n, which, col);
  float v[32];
  float amax = 0.f;
#pragma unroll
  for (int j = 0; j < 32; j++) {
    const int k = k0 + j;
    v[j] = (live && k < s.K) ? (float)s.src[which][(size_t)k * s.cols[which] + col] : 0.f;
    amax = fmaxf(amax, fabsf(v[j]));
  }
  const int code = mx_scale_code(amax);
  const float inv = mx_inv_scale(code);
  unsigned w[8];
#pragma unroll
  for (int j = 0; j < 8; j++) w[j] = mx_encode2(v[4 * j], v[4 * j + 1], inv) | (mx_encode2(v[4 * j + 2], v[4 * j + 3], inv) << 16);
  unsigned char* frag = dst + f * 2048;
  *reinterpret_cast<uint4*>(frag + ((size_t)(2 * b) * 32 + i) * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  *reinterpret_cast<uint4*>(frag + ((size_t)(2 * b + 1) * 32 + i) * 16) = make_uint4(w[4], w[5], w[6], w[7]);
  scales[(((size_t)nt * (kc64 >> 2) + (kc >> 2)) * 64 + lane) * 4 + (kc & 3)] = (unsigned char)code;
}

hipError_t launch_pack_weights_mx(hipStream_t st, const PackSrc& s, unsigned char* dst, unsigned char* scales, int n_pad, int k_pad) {
  if (n_pad % 32 != 0 || k_pad % 256 != 0 || s.n_true > n_pad || s.K > k_pad || dst == nullptr || scales == nullptr)
    return hipErrorInvalidValue;
  const size_t total = (size_t)(n_pad >> 5) * (k_pad >> 6) * 64;
  hipLaunchKernelGGL(pack_weights_mx_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s, dst, scales, n_pad, k_pad);
  return hipGetLastError();
}

// colsum[n] = sum_k gain_k * W[k][col]   (the activations reach the GEMM already scaled by gain_k)
// bias_out[n] = sum_k ln_bias[k] * W[k][col] + bias_src[which][col]
struct FoldArgs {
  PackSrc s;
  const bf16* ln_bias;
  const bf16* bias_src[3];
  float* colsum;
  float* bias_out;
  int n_pad;
};
__global__ __launch_bounds__(256) void fold_vectors_kernel(FoldArgs a) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= a.n_pad) return;
  int which = 0, col = 0;
  const bool live = map_row(a.s, n, which, col);
  float cs = 0.f, bo = 0.f;
  if (live) {
    if (a.colsum != nullptr || a.ln_bias != nullptr) {
      for (int k = 0; k < a.s.K; k++) {
        const float w = (float)a.s.src[which][(size_t)k * a.s.cols[which] + col];
        cs += w * k_scale(a.s, k);
        if (a.ln_bias != nullptr) bo += (float)a.ln_bias[k] * w;
      }
    }
    if (a.bias_src[which] != nullptr) bo += (float)a.bias_src[which][col];
  }
  if (a.colsum != nullptr) a.colsum[n] = cs;
  if (a.bias_out != nullptr) a.bias_out[n] = bo;
}

hipError_t launch_fold_vectors(hipStream_t st, const PackSrc& s, const bf16* ln_bias, const bf16* const bias_src[3],
                               float* colsum, float* bias_out, int n_pad) {
  if (n_pad <= 0 || s.n_true > n_pad) return hipErrorInvalidValue;
  FoldArgs a;
  a.s = s;
  a.ln_bias = ln_bias;
  for (int i = 0; i < 3; i++) a.bias_src[i] = bias_src ? bias_src[i] : nullptr;
  a.colsum = colsum;
  a.bias_out = bias_out;
  a.n_pad = n_pad;
  hipLaunchKernelGGL(fold_vectors_kernel, dim3((n_pad + 255) / 256), dim3(256), 0, st, a);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void bf16_to_f32_kernel(const bf16* src, float* dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = (float)src[i];
}
hipError_t launch_bf16_to_f32(hipStream_t st, const bf16* src, float* dst, size_t n) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src, dst, n);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void gain_vector_kernel(const bf16* src, float* dst, int n, float add) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = (float)src[i] + add;
}
hipError_t launch_gain_vector(hipStream_t st, const bf16* src, float* dst, int n, int one_plus) {
  if (n <= 0 || src == nullptr || dst == nullptr) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gain_vector_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src, dst, n, one_plus ? 1.0f : 0.0f);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void copy_u16_kernel(const uint16_t* src, uint16_t* dst, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) dst[i] = src[i];
}
hipError_t launch_copy_bf16(hipStream_t st, const bf16* src, bf16* dst, size_t n) {
  if (n == 0) return hipSuccess;
  const unsigned blocks = (unsigned)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL(copy_u16_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<const uint16_t*>(src),
                     reinterpret_cast<uint16_t*>(dst), n);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void copy_f32_kernel(const float* src, float* dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
hipError_t launch_copy_f32(hipStream_t st, const float* src, float* dst, size_t n) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src, dst, n);
  return hipGetLastError();
}

// bytes must be a multiple of 16, dst 16-byte aligned
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* dst, size_t n16) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  const uint4 z = {0u, 0u, 0u, 0u};
  for (; i < n16; i += stride) dst[i] = z;
}
hipError_t launch_fill_zero(hipStream_t st, void* dst, size_t bytes) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(dst) & 15) != 0) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const unsigned blocks = (unsigned)((n16 + 255) / 256 < 16384 ? (n16 + 255) / 256 : 16384);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<uint4*>(dst), n16);
  return hipGetLastError();
}

// Folded action/time encoder (Section 3.2): rows r < A:  W_fold[r][n] = sum_j wa[r][j] * wt1[j][n];
// rows r = A + k: bias_k[n] = sum_j ba[j] * wt1[j][n] + sum_j tau_k[j] * wt1[X + j][n] + bt1[n].
__global__ __launch_bounds__(256) void time_fold_kernel(const bf16* wa, const bf16* ba, const bf16* wt1, const bf16* bt1,
                                                        const float* tau, int A, int X, int steps, float* wfold,
                                                        float* bias_tab) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int r = blockIdx.y;
  if (n >= X) return;
  float acc = 0.f;
  if (r < A) {
    for (int j = 0; j < X; j++) acc += (float)wa[(size_t)r * X + j] * (float)wt1[(size_t)j * X + n];
    wfold[(size_t)r * X + n] = acc;
  } else {
    const int k = r - A;
    for (int j = 0; j < X; j++) acc += (float)ba[j] * (float)wt1[(size_t)j * X + n];
    for (int j = 0; j < X; j++) acc += tau[(size_t)k * X + j] * (float)wt1[(size_t)(X + j) * X + n];
    bias_tab[(size_t)k * X + n] = acc + (float)bt1[n];
  }
}
hipError_t launch_time_fold(hipStream_t st, const bf16* wa, const bf16* ba, const bf16* wt1, const bf16* bt1,
                            const float* tau, int action_dim, int X, int steps, float* wfold, float* bias_tab) {
  hipLaunchKernelGGL(time_fold_kernel, dim3((X + 255) / 256, action_dim + steps), dim3(256), 0, st, wa, ba, wt1, bt1, tau,
                     action_dim, X, steps, wfold, bias_tab);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// images [V][img][img][3] fp32 -> patch vectors bf16, XF layout with ld padded columns, vector
// order (dy, dx, c); columns >= patch*patch*3 are left untouched (zero from load time).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void patchify_kernel(const float* images, int n_views, int img, int patch, bf16* out,
                                                       int ld) {
  const int per_side = img / patch;
  const int T = per_side * per_side;
  const int pd = patch * patch * 3;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)n_views * T * pd) return;
  const int e = (int)(idx % pd);
  const int tok = (int)(idx / pd);
  const int v = tok / T, tt = tok % T;
  const int py = tt / per_side, px = tt % per_side;
  const int c = e % 3, dx = (e / 3) % patch, dy = e / (3 * patch);
  const float val = images[(((size_t)v * img + (py * patch + dy)) * img + (px * patch + dx)) * 3 + c];
  out[xf_index(tok, e, ld >> 4)] = (bf16)val;
}
hipError_t launch_patchify(hipStream_t st, const float* images, int n_views, int img, int patch, bf16* out, int ld) {
  const int per_side = img / patch;
  const size_t total = (size_t)n_views * per_side * per_side * patch * patch * 3;
  if (ld < patch * patch * 3 || ld % 16 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(patchify_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, images, n_views, img, patch,
                     out, ld);
  return hipGetLastError();
}

// prompt rows: out[row0 + i][:] = scale * table[clamp(ids[i])][:]
__global__ __launch_bounds__(256) void embed_prompt_kernel(const int32_t* ids, int n, const bf16* table, int vocab, int E,
                                                           float scale, float* out_f32, bf16* out_bf16, int row0) {
  const int i = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (i >= n || c >= E) return;
  int id = ids[i];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);   // out-of-range ids are clamped, never read out of bounds
  const float v = scale * (float)table[(size_t)id * E + c];
  out_f32[(size_t)(row0 + i) * E + c] = v;
  out_bf16[xf_index(row0 + i, c, E >> 4)] = (bf16)v;
}
hipError_t launch_embed_prompt(hipStream_t st, const int32_t* ids, int n, const bf16* table, int vocab, int E, float scale,
                               float* out_f32, bf16* out_bf16, int row0) {
  if (n <= 0) return hipSuccess;
  if (ids == nullptr || table == nullptr || vocab <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(embed_prompt_kernel, dim3((E + 255) / 256, n), dim3(256), 0, st, ids, n, table, vocab, E, scale,
                     out_f32, out_bf16, row0);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void state_token_kernel(StateTokenArgs a) {
  state_token_body(a, LaunchCtx::from_block_idx());
}
hipError_t launch_state_token(hipStream_t st, const float* state, int state_dim, const float* ws, const float* bs, int X,
                              float* out, int* progress) {
  if (state_dim < 1 || state_dim > 32) return hipErrorInvalidValue;
  hipLaunchKernelGGL(state_token_kernel, dim3((X + 255) / 256), dim3(256), 0, st, StateTokenArgs{state, state_dim, ws, bs, X, out, progress});
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Read-ahead kernel of the action expert (the prefetch-across-synchronisation-points idea of
// Section 5.2, as a kernel of its own beside the compute launches instead of extra blocks inside
// them).  It runs on a second stream for the whole denoise loop and reads the weights and cache
// slices of layer-step i (i = step * layers + layer) once the compute stream has started
// layer-step i - lead + 1, which it learns from a counter the QKV launch of every layer stores.
// The loads only pull the bytes into the memory-side cache; their values are xor-folded into a
// word compared with a constant so they cannot be elided, and no result depends on them.
// Every wait is bounded: a block that does not see the counter move within `wait_ticks` of the
// 100 MHz wall clock stops reading ahead altogether and exits (so a machine that runs the two
// streams one after the other only loses that one wait).  A block that finds the compute stream
// already past layer-step i skips that slice, so a kernel that has fallen behind catches up and
// the join at the end of the loop never waits for reads nobody needs any more.
// ------------------------------------------------------------------------------------------------
// Register budget: the expert's compute launches keep two waves of up to 224 registers on every SIMD, so a
// wave of this kernel only fits beside them with at most 64 (asked for through the occupancy attribute).
template <int RA_DEPTH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8, 8))) void read_ahead_kernel(ReadAheadParams p) {
  __shared__ int s_go;
  const unsigned tid = blockIdx.x * blockDim.x + threadIdx.x;
  const unsigned nth = gridDim.x * blockDim.x;
  unsigned acc = 0;
  const int total = p.steps * p.layers;
  for (int i = 0; i < total; i++) {
    // thread 0 decides for the block: 1 read slice i, 2 skip it (the compute stream is already past layer-step
    // i, so its bytes would come too late: a read-ahead kernel that has fallen behind catches up instead of
    // holding the join back), 0 give up (the counter did not move within the bound)
    const int need = i + 1 - p.lead;
    if (threadIdx.x == 0) {
      int seen = __hip_atomic_load(p.progress, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      int go = 1;
      if (seen < need) {
        const long long t0 = wall_clock64();
        while ((seen = __hip_atomic_load(p.progress, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) < need) {
          if (wall_clock64() - t0 > p.wait_ticks) {
            go = 0;
            break;
          }
          __builtin_amdgcn_s_sleep(16);
        }
      }
      if (go && seen >= i + 2) go = 2;
      s_go = go;
    }
    __syncthreads();
    const int go = s_go;
    __syncthreads();
    if (go == 0) break;
    if (go == 2) continue;
    const int layer = i % p.layers;
    // The layer's ranges as one virtual range of `total` bytes (below 4 GiB, checked by the host), walked in batches
    // of RA_DEPTH loads per lane: the word at virtual offset v lies in the last range r with cum[r] <= v.  Offsets past
    // the end are clamped to the last word (a repeated load, no branch).
    const unsigned char* lbase[RA_REGIONS];
    unsigned cum[RA_REGIONS + 1];
    cum[0] = 0u;
#pragma unroll
    for (int r = 0; r < RA_REGIONS; r++) {
      lbase[r] = p.base[r] + (size_t)layer * p.layer_stride[r];
      cum[r + 1] = cum[r] + p.n16[r] * 16u;
    }
    const unsigned total = cum[RA_REGIONS];
    for (unsigned o0 = tid * 16u; o0 < total; o0 += RA_DEPTH * nth * 16u) {
      // overtaken in the middle of the layer: leave the rest of it (every lane of the wave reads the same word)
      if (o0 != tid * 16u && __hip_atomic_load(p.progress, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= i + 2) break;
      uint4 v[RA_DEPTH];
#pragma unroll
      for (int k = 0; k < RA_DEPTH; k++) {
        const unsigned vo = min(o0 + (unsigned)k * nth * 16u, total - 16u);
        const unsigned char* ptr = lbase[0] + vo;
#pragma unroll
        for (int r = 1; r < RA_REGIONS; r++) {
          if (vo >= cum[r]) ptr = lbase[r] + (vo - cum[r]);
        }
        v[k] = *reinterpret_cast<const uint4*>(ptr);
      }
#pragma unroll
      for (int k = 0; k < RA_DEPTH; k++) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
  }
  if (acc == 0x9e3779b9u) p.sink[tid & 1023] = acc;
}
hipError_t launch_read_ahead(hipStream_t st, const ReadAheadParams& p, int blocks, int threads, int depth) {
  if (blocks < 1 || blocks > 4096 || (threads != 64 && threads != 128 && threads != 256) || p.progress == nullptr ||
      p.sink == nullptr || p.lead < 1 || p.layers < 1 || p.steps < 1 || p.wait_ticks < 1)
    return hipErrorInvalidValue;
  size_t words = 0;
  for (int r = 0; r < RA_REGIONS; r++) words += p.n16[r];
  if (words == 0 || words >= ((size_t)1 << 27)) return hipErrorInvalidValue;   // byte offsets over a whole layer are 32-bit in the kernel
  for (int r = 0; r < RA_REGIONS; r++) {
    if (p.n16[r] != 0 && (p.base[r] == nullptr || (reinterpret_cast<uintptr_t>(p.base[r]) & 15) != 0 || p.layer_stride[r] % 16 != 0))
      return hipErrorInvalidValue;
  }
  switch (depth) {
#define X(D) case D: hipLaunchKernelGGL(read_ahead_kernel<D>, dim3(blocks), dim3(threads), 0, st, p); break;
    X(1) X(2) X(3) X(4) X(5) X(6) X(8)
#undef X
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void action_embed_kernel(ActionEmbedArgs a) {
  action_embed_body(a, LaunchCtx::from_block_idx());
}
hipError_t launch_action_embed(hipStream_t st, const float* x, int chunk, int action_dim, const float* wfold,
                               const float* bias_k, int X, bf16* z, const float* state_tok, float* y_f32, bf16* y_bf16,
                               const float* gain, float* stat_parts) {
  if (X % 32 != 0 || gain == nullptr || stat_parts == nullptr) return hipErrorInvalidValue;
  hipLaunchKernelGGL(action_embed_kernel, dim3((X + 255) / 256, chunk + 1), dim3(256), 0, st,
                     ActionEmbedArgs{x, chunk, action_dim, wfold, bias_k, X, z, state_tok, y_f32, y_bf16, gain, stat_parts});
  return hipGetLastError();
}

// natural-order fp32 dump of one layer's fragment-ordered key / value cache (head dim 256)
__global__ __launch_bounds__(256) void unpack_kv_kernel(const bf16* kfrag, const bf16* vfrag, int P, float* k_out,
                                                        float* v_out) {
  const int d = threadIdx.x;
  const int key = blockIdx.x;
  if (key >= P) return;
  const int kc = key >> 5, kk = key & 31;
  const size_t ka = ((size_t)kc * 16 + (d >> 4)) * 512 + (((d & 15) >> 3) * 32 + kk) * 8 + (d & 7);
  k_out[(size_t)key * 256 + d] = (float)kfrag[ka];
  const int s2 = kk >> 4, g = (kk & 15) >> 3, hh = (kk & 7) >> 2, jp = kk & 3;
  const size_t va = ((((size_t)kc * 8 + (d >> 5)) * 2 + s2) * 64 + hh * 32 + (d & 31)) * 8 + 4 * g + jp;
  v_out[(size_t)key * 256 + d] = (float)vfrag[va];
}
hipError_t launch_unpack_kv(hipStream_t st, const bf16* kfrag, const bf16* vfrag, int P, float* k_out, float* v_out) {
  hipLaunchKernelGGL(unpack_kv_kernel, dim3(P), dim3(256), 0, st, kfrag, vfrag, P, k_out, v_out);
  return hipGetLastError();
}
