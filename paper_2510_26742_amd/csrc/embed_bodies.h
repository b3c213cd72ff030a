// Bodies of the action expert's two small non-GEMM operations (Table 2 rows 1x32x1024 and 63x32x1024), templated
// on the execution context so that they run as launches of their own and inside the persistent kernel of the
// denoise loop (exec_ctx.h).  Work item = (256 columns, row); threads beyond 256 of a wider block idle.
#pragma once
#include "gemm_common.h"

struct StateTokenArgs {
  const float* state; int sd; const float* ws; const float* bs; int X;
  float* out;
  int* progress;   // per-operation launches only: pace counter of the read-ahead kernel, reset here
};

// state token: out[n] = sum_j state[j] * ws[j][n] + bs[n]   (Table 2 row 1x32x1024)
template <class Cx>
__device__ __forceinline__ void state_token_body(const StateTokenArgs a, const Cx cx) {
  const int tx = cx.tid();
  if (tx >= 256) return;
  const int n = cx.bx * 256 + tx;
  // first launch of the action expert: no layer has started yet (read by the read-ahead kernel)
  if (!Cx::kPersistent && n == 0 && a.progress != nullptr) __hip_atomic_store(a.progress, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (n >= a.X) return;
  // all (at most 32) loads issued together (clamped, unconditional), added in index order
  float wv[32], sv[32];
#pragma unroll
  for (int j = 0; j < 32; j++) {
    const int jj = min(j, a.sd - 1);
    wv[j] = a.ws[(size_t)jj * a.X + n];
    sv[j] = a.state[jj];
  }
  float acc = a.bs[n];
#pragma unroll
  for (int j = 0; j < 32; j++) {
    if (j < a.sd) acc += sv[j] * wv[j];
  }
  cx.st(a.out + n, acc);
}

struct ActionEmbedArgs {
  const float* x; int chunk; int A; const float* wfold; const float* bias_k; int X;
  bf16* z; const float* state_tok; float* y_f32; bf16* y_bf16; const float* gain; float* stat_parts;
};

// Table 2 row 63x32x1024 (bias, silu) with the folded weights; also re-seeds suffix row 0 of the
// expert's residual stream with the state token at the start of every Euler step.
// Rows (cx.by) 0 .. chunk-1 -> z[r]; row chunk -> state token copy and zero z[chunk].
// The state row also gets its gain-scaled bf16 copy and, per 32 columns, its (sum, sum of squares) in
// stat_parts[tile][64 rows][2] (row 0), the form the first QKV GEMM of the step reads.
template <class Cx>
__device__ __forceinline__ void action_embed_body(const ActionEmbedArgs a, const Cx cx) {
  const int tx = cx.tid();
  if (tx >= 256) return;
  const int n = cx.bx * 256 + tx;
  const int r = cx.by;
  const int X = a.X, A = a.A, chunk = a.chunk;
  if (n >= X) return;
  if (r < chunk) {
    // all loads of (up to) 32 terms issued together - the x values cross blocks, i.e. come from memory, and a batch
    // that waits for the one before costs a round trip each (4 batches of 8: 3.9 us per operation) - then accumulated
    // in index order
    float acc = a.bias_k[n];
    for (int j0 = 0; j0 < A; j0 += 32) {
      float wv[32], xv[32];
#pragma unroll
      for (int u = 0; u < 32; u++) {
        const int j = min(j0 + u, A - 1);
        xv[u] = cx.ld(a.x + (size_t)r * A + j);
        wv[u] = a.wfold[(size_t)j * X + n];
      }
#pragma unroll
      for (int u = 0; u < 32; u++) {
        if (j0 + u < A) acc += xv[u] * wv[u];
      }
    }
    const float sv = acc / (1.0f + __expf(-acc));
    cx.st(a.z + xf_index(r, n, X >> 4), (bf16)sv);
  } else {
    cx.st(a.z + xf_index(chunk, n, X >> 4), (bf16)0.0f);
    const float s = cx.ld(a.state_tok + n);
    cx.st(a.y_f32 + n, s);
    cx.st(a.y_bf16 + xf_index(0, n, X >> 4), (bf16)(s * a.gain[n]));
    float sa = s, sb = s * s;     // X is a multiple of 32: a 32-lane group is here completely or not at all
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
      sa += __shfl_xor(sa, off, 64);
      sb += __shfl_xor(sb, off, 64);
    }
    if ((tx & 31) == 0) cx.st(reinterpret_cast<float2*>(a.stat_parts + (size_t)(n >> 5) * 128), make_float2(sa, sb));
  }
}
