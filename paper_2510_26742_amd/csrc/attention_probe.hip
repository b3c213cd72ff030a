// Test entry point: the attention kernels of the pass (Table 2: SigLIP attention per view, prefix attention with a
// shared key/value head, the expert's attention over [prefix cache ; own 64 keys] with the state/action block mask) on
// operands given in natural order.  The probe rounds them to bf16, places them in the fragment order that the QKV
// projections write, launches the same kernel variants with the same launch shapes as the pass, and returns the
// outputs in natural order.  It allocates and frees its staging buffers and synchronises: a tool for tests.
#include "pi0_internal.h"

#include <string.h>

namespace {

struct ProbeGeom {
  int heads, kv_heads, head_dim, s16, nvb, Tq, qmb, n0, c0, n1, c1;
};

// q [heads][Tq][d] -> [head][Tq / 32][s16][64][8]; same for keys with their own head count and chunk count
__global__ void probe_pack_qk(const float* src, bf16* dst, int heads, int T, int chunks, int head_dim, int s16) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long total = (long)heads * T * head_dim;
  if (i >= total) return;
  const int d = (int)(i % head_dim);
  const int t = (int)((i / head_dim) % T);
  const int h = (int)(i / ((long)head_dim * T));
  const int kc = t >> 5, kk = t & 31;
  dst[(((size_t)h * chunks + kc) * s16 + (d >> 4)) * 512 + ((d & 15) >> 3) * 256 + kk * 8 + (d & 7)] = (bf16)src[i];
}

// v [heads][T][d] -> [head][T / 32][nvb][2][64][8] (transposed fragments of the second product)
__global__ void probe_pack_v(const float* src, bf16* dst, int heads, int T, int chunks, int head_dim, int nvb) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long total = (long)heads * T * head_dim;
  if (i >= total) return;
  const int d = (int)(i % head_dim);
  const int t = (int)((i / head_dim) % T);
  const int h = (int)(i / ((long)head_dim * T));
  const int kc = t >> 5, kk = t & 31;
  const int s2 = kk >> 4, g = (kk & 15) >> 3, hh = (kk & 7) >> 2, jp = kk & 3;
  dst[(((size_t)h * chunks + kc) * nvb + (d >> 5)) * 1024 + s2 * 512 + hh * 256 + (d & 31) * 8 + 4 * g + jp] = (bf16)src[i];
}

// out (activation fragment order, ld columns) -> [Tq][cols]
__global__ void probe_unpack_out(const bf16* src, float* dst, int Tq, int cols, int ld) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)Tq * cols) return;
  const int col = (int)(i % cols), row = (int)(i / cols);
  dst[i] = (float)src[((size_t)(row >> 5) * (ld >> 4) + (col >> 4)) * 512 + (((col & 15) >> 3) * 32 + (row & 31)) * 8 + (col & 7)];
}

struct DevBuf {
  void* p = nullptr;
  hipError_t alloc_zero(size_t bytes, hipStream_t s) {
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) return e;
    return launch_fill_zero(s, p, bytes);
  }
  ~DevBuf() { if (p) (void)hipFree(p); }
};

}  // namespace

extern "C" int pi0_attention_probe(int heads, int kv_heads, int head_dim, int Tq, int n0, int n1, int view_tokens,
                                   int suffix_mask, int chunks_per_share, int v_split, float scale, const float* d_q,
                                   const float* d_k0, const float* d_v0, const float* d_k1, const float* d_v1,
                                   float* d_out, float* d_ml, void* hip_stream) {
  if (heads < 1 || heads > 64 || (kv_heads != heads && kv_heads != 1) || Tq < 1 || Tq > 1024 || n0 < 1 || n0 > 1024) return PI0_EINVAL;
  if (head_dim != 256 && !(head_dim > 64 && head_dim <= 80 && head_dim % 4 == 0)) return PI0_EINVAL;
  if (n1 != 0 && (n1 != 64 || head_dim != 256 || kv_heads != 1)) return PI0_EINVAL;
  if (d_q == nullptr || d_k0 == nullptr || d_v0 == nullptr || d_out == nullptr || (n1 != 0 && (d_k1 == nullptr || d_v1 == nullptr))) return PI0_EINVAL;
  if (view_tokens != 0 && (view_tokens % 32 != 0 || Tq % view_tokens != 0 || n0 != Tq)) return PI0_EINVAL;
  ProbeGeom g;
  g.heads = heads; g.kv_heads = kv_heads; g.head_dim = head_dim;
  g.s16 = head_dim == 256 ? 16 : 5;
  g.nvb = head_dim == 256 ? 8 : 3;
  g.Tq = Tq; g.qmb = (Tq + 31) / 32;
  g.n0 = n0; g.c0 = (n0 + 31) / 32;
  g.n1 = n1; g.c1 = n1 / 32;
  int shares = 1;
  if (chunks_per_share > 0 && g.c0 > chunks_per_share) {
    shares = (g.c0 + chunks_per_share - 1) / chunks_per_share;
    if (shares > 8 || d_ml == nullptr || view_tokens != 0) return PI0_EINVAL;
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if (attention_init_attributes() != hipSuccess) return PI0_EHIP;
  const int out_ld = ((heads * head_dim + 15) / 16) * 16;
  const size_t out_share = (size_t)g.qmb * 32 * out_ld;
  DevBuf q, k0, v0, k1, v1, out, ml;
  hipError_t e = hipSuccess;
  auto ok = [&](hipError_t x) { if (e == hipSuccess) e = x; return e == hipSuccess; };
  ok(q.alloc_zero((size_t)heads * g.qmb * g.s16 * 512 * sizeof(bf16), s));
  ok(k0.alloc_zero((size_t)kv_heads * g.c0 * g.s16 * 512 * sizeof(bf16), s));
  ok(v0.alloc_zero((size_t)kv_heads * g.c0 * g.nvb * 1024 * sizeof(bf16), s));
  ok(out.alloc_zero(out_share * shares * sizeof(bf16), s));
  if (n1) {
    ok(k1.alloc_zero((size_t)kv_heads * g.c1 * g.s16 * 512 * sizeof(bf16), s));
    ok(v1.alloc_zero((size_t)kv_heads * g.c1 * g.nvb * 1024 * sizeof(bf16), s));
  }
  if (shares > 1) ok(ml.alloc_zero((size_t)shares * heads * g.qmb * 32 * 2 * sizeof(float), s));
  if (e != hipSuccess) return e == hipErrorOutOfMemory ? PI0_ENOMEM : PI0_EHIP;
  auto blocks = [](long n) { return dim3((unsigned)((n + 255) / 256)); };
  probe_pack_qk<<<blocks((long)heads * Tq * head_dim), 256, 0, s>>>(d_q, (bf16*)q.p, heads, Tq, g.qmb, head_dim, g.s16);
  probe_pack_qk<<<blocks((long)kv_heads * n0 * head_dim), 256, 0, s>>>(d_k0, (bf16*)k0.p, kv_heads, n0, g.c0, head_dim, g.s16);
  probe_pack_v<<<blocks((long)kv_heads * n0 * head_dim), 256, 0, s>>>(d_v0, (bf16*)v0.p, kv_heads, n0, g.c0, head_dim, g.nvb);
  if (n1) {
    probe_pack_qk<<<blocks((long)kv_heads * n1 * head_dim), 256, 0, s>>>(d_k1, (bf16*)k1.p, kv_heads, n1, g.c1, head_dim, g.s16);
    probe_pack_v<<<blocks((long)kv_heads * n1 * head_dim), 256, 0, s>>>(d_v1, (bf16*)v1.p, kv_heads, n1, g.c1, head_dim, g.nvb);
  }
  AttnParams a;
  memset(&a, 0, sizeof(a));
  a.q = (const bf16*)q.p; a.q_head_stride = g.qmb * g.s16 * 512;
  a.Tq = Tq; a.heads = heads;
  a.k0 = (const bf16*)k0.p; a.v0 = (const bf16*)v0.p;
  a.chunks0 = g.c0; a.valid0 = n0;
  a.kv_head_stride0 = kv_heads == 1 ? 0 : g.c0 * g.s16 * 512;
  a.v_head_stride0 = kv_heads == 1 ? 0 : g.c0 * g.nvb * 1024;
  if (n1) { a.k1 = (const bf16*)k1.p; a.v1 = (const bf16*)v1.p; a.chunks1 = g.c1; }
  a.view_tokens = view_tokens;
  a.suffix_mask = suffix_mask;
  a.scale = scale;
  a.out = (bf16*)out.p; a.out_ld = out_ld; a.head_dim = head_dim;
  if (shares > 1) {
    a.key_splits = shares;
    a.chunks_per_split = chunks_per_share;
    a.out_split_stride = out_share;
    a.ml_out = (float*)ml.p;
  }
  a.v_split = v_split;
  hipError_t le = launch_attention(s, a);
  if (le == hipErrorInvalidValue) { (void)hipStreamSynchronize(s); return PI0_EINVAL; }
  ok(le);
  for (int z = 0; z < shares && e == hipSuccess; z++)
    probe_unpack_out<<<blocks((long)Tq * heads * head_dim), 256, 0, s>>>((const bf16*)out.p + z * out_share, d_out + (size_t)z * Tq * heads * head_dim,
                                                                          Tq, heads * head_dim, out_ld);
  if (shares > 1 && e == hipSuccess)
    ok(hipMemcpyAsync(d_ml, ml.p, (size_t)shares * heads * g.qmb * 32 * 2 * sizeof(float), hipMemcpyDeviceToDevice, s));
  ok(hipGetLastError());
  ok(hipStreamSynchronize(s));
  return e == hipSuccess ? PI0_OK : PI0_EHIP;
}
