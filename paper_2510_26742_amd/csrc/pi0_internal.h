// Internal declarations shared by the host code and the HIP kernels of the pi0 library.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/pi0_bench.h"

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int round_up(int a, int b) { return ceil_div(a, b) * b; }
static inline size_t round_up_sz(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ------------------------------------------------------------------------------------------
// Packed weight matrix: MFMA "A operand" fragment order.
// Logical matrix W'[n][k] (n = output feature, k = input feature), zero padded to n_pad x k_pad.
// Element (n, k) lives at  ((n/32 * (k_pad/16) + k/16) * 64 + ((k%16)/8)*32 + n%32) * 8 + k%8,
// so one wave reads the 32x16 fragment of n-tile nt, k-step kc as 64 consecutive 16-byte pieces.
// ------------------------------------------------------------------------------------------
struct PackedW {
  const bf16* w;  // fragment-ordered weights
  int n_pad;      // multiple of 32
  int k_pad;      // multiple of 64
};

enum RowMap { ROWMAP_CONCAT = 0, ROWMAP_ROPE_QKV = 1, ROWMAP_PAIR = 2 };
enum KScale { KSCALE_NONE = 0, KSCALE_GAIN = 1, KSCALE_ONE_PLUS = 2 };

// Source description for packing: up to three [K][cols_i] row-major bf16 matrices that are
// concatenated along the output axis (ROWMAP_CONCAT), concatenated with the q and k blocks
// re-ordered so that RoPE partners (d, d + 128) become neighbours (ROWMAP_ROPE_QKV), or
// interleaved pairwise src0/src1 (ROWMAP_PAIR: packed row 2i = src0 col i, 2i+1 = src1 col i).
struct PackSrc {
  const bf16* src[3];
  int cols[3];
  int K;              // true input features
  int n_true;         // true number of packed rows
  int rowmap;
  int kscale;         // per-k gain of the preceding norm: enters the column sums only (the weights stay unscaled,
                      // the gain is applied where the activations are cast to bf16)
  const bf16* gain;   // [K] (KSCALE_GAIN: g, KSCALE_ONE_PLUS: 1 + g)
  int q_heads;        // ROWMAP_ROPE_QKV: number of 256-wide q heads in src0
};

// ------------------------------------------------------------------------------------------
// Cache warm-up blocks.  The expert's kernels are short and each reads weights that were last
// touched one Euler step (600+ MB of traffic) ago, so every kernel starts with HBM-cold misses.
// A launch may therefore carry extra blocks that do no arithmetic: they read the weights (and
// cache slices) of the kernels that follow, which pulls them into the 256 MB memory-side cache;
// the consumer then misses L2 (whose contents do not survive a kernel boundary) but not HBM.
// Regions are given as `tiles` pieces of `tile16` 16-byte words; warm-up block `rank` reads the
// pieces nt = rank % 8 (mod 8), i.e. the ones whose consumer block would run on the same XCD
// under round-robin dispatch (that only matters if a later hardware keeps L2 across launches).
// The values are folded into a word that is compared with a constant, so the loads cannot be
// elided; results of the pass do not depend on them in any way.
// ------------------------------------------------------------------------------------------
struct PrefetchDesc {
  const void* ptr[3];
  int tiles[3];
  int tile16[3];
  int blocks;        // number of warm-up blocks of the launch, multiple of 16 (0 = none)
  unsigned* sink;    // [blocks]
};

static __device__ __forceinline__ void prefetch_role(const PrefetchDesc& d, int rank) {
  const int xcd = rank & 7, sub = rank >> 3, nsub = d.blocks >> 3;
  const int step = nsub * (int)blockDim.x;
  unsigned acc = 0;
#pragma unroll
  for (int r = 0; r < 3; r++) {
    if (d.ptr[r] == nullptr || d.tiles[r] <= xcd) continue;
    const uint4* base = reinterpret_cast<const uint4*>(d.ptr[r]);
    const int t16 = d.tile16[r];
    const int total = ((d.tiles[r] - xcd + 7) >> 3) * t16;
#pragma unroll 4
    for (int i = sub * (int)blockDim.x + (int)threadIdx.x; i < total; i += step) {
      const int j = i / t16;
      const uint4 v = base[(size_t)(xcd + 8 * j) * t16 + (i - j * t16)];
      acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
  }
  if (acc == 0x9e3779b9u) d.sink[rank] = acc;
}

// ------------------------------------------------------------------------------------------
// GEMM:  C^T[n][m] = sum_k W'[n][k] * X[m][k]   (weights are the MFMA A operand, tokens the B
// operand; each lane of the accumulator owns one token and groups of 4 consecutive n).
// ------------------------------------------------------------------------------------------
enum Prologue { PRO_NONE = 0, PRO_RMS = 1, PRO_LN = 2 };
enum Epilogue {
  EPI_PARTIAL = 0,   // fp32 partial sums [z][M][n_pad] for a later split-K reduction
  EPI_RESID = 1,     // out_f32 = acc (+bias) (+resid[row % resid_mod]); bf16 shadow
  EPI_BF16 = 2,      // out_bf16 = act(norm(acc) + bias)
  EPI_QKV = 3,       // q, K, V in the attention kernel's fragment orders (K / V straight into the cache); optional RoPE / bias
  EPI_GEGLU = 4,     // out_bf16[m][n/2] = gelu(gate) * up
  EPI_EULER = 5      // x[m-1][n] += dt * (norm(acc) + bias), rows m >= 1
};
enum Act { ACT_NONE = 0, ACT_GELU = 1, ACT_SILU = 2 };

struct GemmParams {
  const bf16* X;      // activations in XF layout with ldx (padded) columns, ldx >= k_pad, pad columns zero
  int ldx;
  int M;              // valid rows
  PackedW W;
  int n_tiles;        // n_pad / 32
  int k_per_split;    // k range of one blockIdx.z slice, multiple of 64 * WK
  int k_true;         // divisor of the row statistics
  int m_tiles;        // number of MB*32 row tiles
  int m_split;        // TILE_SKINNY QKV: 1 = one block per (feature tile, 32-token block)
  int* progress;      // TILE_SKINNY: when set, the launch stores progress_value there on entry (read-ahead kernel's pace)
  int progress_value;
  // statistics / affine
  const float* bias;    // [n_pad] or null
  const float* colsum;  // [n_pad], PRO_LN only: sum_k W'[n][k]
  const float* rowstat; // (sum, sum of squares) of the fp32 residual rows, PRO_RMS / PRO_LN: [rows][2] for the tall
                        // kernels; [rowstat_parts][64][2] partial sums for the skinny kernel
  int rowstat_parts;    // tall kernels: 0 / 1 = rowstat holds whole-row sums, > 1 = [rowstat_parts][stat_rows][2] partial sums
  float* stat_out;      // EPI_RESID: partial row statistics of the output per 32-column tile, [n tile][stat_rows][2], or null
  int stat_rows;        // rows per plane of stat_out (producer) / of a partial rowstat (tall consumer); 0 = 64
  const float* gain;    // EPI_RESID: per-column scale of the bf16 shadow (gain of the norm that follows), or null
  // outputs
  float* out_f32;     // EPI_RESID / EPI_PARTIAL / EPI_EULER
  bf16* out_bf16;     // EPI_RESID shadow (XF), EPI_BF16 (XF), EPI_GEGLU (XF), EPI_QKV q (fragment order per head)
  int ldo;            // leading dimension of out_f32; padded columns of the XF output of EPI_BF16 / EPI_GEGLU
  int ldo2;           // padded columns of the XF shadow in EPI_RESID
  int n_valid;        // columns >= n_valid are not stored (EPI_RESID / EPI_BF16 / EPI_EULER)
  const float* resid; // EPI_RESID: residual input [*][ldo] or null
  int resid_mod;      // row index of resid taken modulo this (0 = no modulo)
  int row_offset;     // EPI_RESID: output row = m + row_offset
  int act;
  // EPI_QKV
  bf16* kfrag;        // key fragments
  bf16* vfrag;        // value fragments (transposed)
  const float* rope;  // [pos][128][2] (cos, sin) or null
  int pos0;           // position of row 0
  int q_cols;         // packed rows belonging to q  (heads * head_dim)
  int k_cols;         // packed rows belonging to k
  int head_dim;       // true head dim (72 or 256)
  int dqk_pad;        // head dim padded for QK^T (80 or 256)
  int nvb;            // value blocks of 32 (3 or 8)
  int kv_heads;       // 16 (vision) or 1
  int kv_chunks;      // key chunks (of 32) per head in kfrag / vfrag
  int q_mbs;          // 32-token blocks per head in the fragment-ordered q buffer
  // EPI_EULER
  float dt;
  // TILE_SKINNY16 with k = heads * 256: X is given as xsplits attention shares (each ldx-padded, xsplit_stride
  // elements apart) with their (row maximum, sum) pairs xsplit_ml[((z * 8 + head) * 64 + row) * 2]; the
  // kernel merges them while loading (0 / 1 = X is a plain matrix)
  int xsplits;
  size_t xsplit_stride;
  const float* xsplit_ml;
  // warm-up blocks for later launches (skinny tiles only)
  PrefetchDesc pf;
};

// Tile configuration ids (template instantiations that exist)
enum GemmTile {
  TILE_BIG = 0,     // 256 tokens x 128 features per block (4 waves), 3 register stages in flight
  TILE_MID = 1,     // 64 tokens x 128 features per block (4 waves), 6 register stages in flight
  TILE_SKINNY = 2,  // <= 64 tokens, one 32-feature tile per block, 8 waves split k <= 1024, loads issued at once
  TILE_SKINNY_FULLK = 3,  // <= 64 tokens, k = 2048 or 4096 in one block per (feature tile, 32-token block), residual epilogue
  TILE_SKINNY16 = 4,      // same on 16-feature x 16-token tiles (mfma 16x16x32): 256 blocks for the expert's O / down
  TILE_SMALL = 5,         // 64 tokens x 64 features per block (2 waves), 6 stages: small GEMMs of the vision tower
  // two feature tiles per wave: an activation fragment read from LDS feeds two MFMAs (prefix gate||up / down only)
  TILE_WIDE = 6,          // 256 tokens x 256 features per block (4 waves x 2 feature tiles), 2 stages
  TILE_WIDE128 = 7,       // 128 tokens x 256 features per block, 3 stages
  TILE_ENTRY = 8,         // 64 tokens x 32 / 64 features per block, k <= 2048 split over 8 waves, every load issued at entry
  TILE_SQ128 = 9,         // 128 tokens x 128 features per block (4 waves), 5 stages: the mid-size GEMMs at three views
  TILE_T192 = 10,         // 192 tokens x 256 features per block, 2 stages: 768 tokens in four tiles
  TILE_MID2 = 11          // 64 tokens x 128 features as TILE_MID, cut for two resident blocks per compute unit
};

// ------------------------------------------------------------------------------------------
// MXFP8 (OCP Microscaling: FP8 E4M3 elements, one power-of-two E8M0 scale per 32 consecutive k) operands
// of the reduced-precision prefix feed-forward GEMMs.  A 32-row x 64-k fragment is 2 KiB:
//   [piece k/16 (4)][row (32)][16 bytes]
// which is what mfma_scale_f32_32x32x64_f8f6f4 takes when lane (h, i) loads pieces h and h + 2 of row i
// (two 16-byte loads, each contiguous over the wave).  Fragments are ordered [row block][k / 64].  The scale
// of (row i, 32-k block b of a fragment) is supplied to the MFMA by lane b * 32 + i, so scales are stored as
// one dword per lane for four consecutive fragments: [row block][k / 256][lane (64)][fragment % 4].
// ------------------------------------------------------------------------------------------
static __device__ __forceinline__ int mx_scale_code(float amax) {   // floor(log2 amax) - 8 + 127, clamped at 0
  const int ef = (int)((__builtin_bit_cast(unsigned, amax) >> 23) & 0xffu);
  return ef > 8 ? ef - 8 : 0;
}
static __device__ __forceinline__ float mx_inv_scale(int code) {    // 2^(127 - code), exact
  return __builtin_bit_cast(float, (unsigned)(254 - code) << 23);
}
// two values scaled, saturated at +-448 (the conversion alone would give NaN beyond 464) and rounded to nearest
// even E4M3: codes in bits 0..7 and 8..15
static __device__ __forceinline__ unsigned mx_encode2(float a, float b, float inv) {
  a = fminf(fmaxf(a * inv, -448.f), 448.f);
  b = fminf(fmaxf(b * inv, -448.f), 448.f);
  return (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xffffu;
}

struct MxGemmParams {
  const unsigned char* X8;   // activations, MX fragment order, ldx (multiple of 256) k columns, rows padded to 32
  const unsigned char* XS;   // their scales
  int ldx;
  int M;                     // valid rows
  const unsigned char* W8;   // weights, MX fragment order [n / 32][k / 64]
  const unsigned char* WS;   // their scales [n / 32][k / 256][64][4]
  int n_pad, k_pad;          // n_pad multiple of 256, k_pad multiple of 256
  int m_tiles;               // 128-row tiles
  int k_per_split;           // multiple of 256
  int k_true;                // divisor of the row statistics (GEGLU epilogue: RMS)
  const float* rowstat;      // [rows][2] whole-row (sum, sum of squares) of the fp32 input rows
  float* out_f32;            // partial epilogue: [split][M][ldo]
  int ldo;
  unsigned char* out8;       // GeGLU epilogue: gelu(gate) * up in MX fragment order, ldo8 (multiple of 256) columns
  unsigned char* out_scales;
  int ldo8;
};
enum MxEpi { MX_EPI_PARTIAL = 0, MX_EPI_GEGLU = 1 };
// 128 x 256 block tiles; grid = (n_pad / 256 rounded up to 8) x m_tiles blocks, z_splits in y
hipError_t launch_gemm_mx(hipStream_t s, int epi, const MxGemmParams& p, int z_splits);
hipError_t gemm_mx_init_attributes();
// weights -> MX fragments + scales (same row maps as launch_pack_weights)
hipError_t launch_pack_weights_mx(hipStream_t s, const PackSrc& src, unsigned char* dst, unsigned char* scales, int n_pad, int k_pad);

hipError_t launch_gemm(hipStream_t s, int tile, int pro, int epi, const GemmParams& p, int z_splits);
int gemm_rows_per_tile(int tile);
hipError_t gemm_init_attributes();

// Split-K reduction: out[m][n] = sum_z part[z][m][n] (+bias[n]) (+resid[m % resid_mod][n]); bf16 shadow in XF
// layout; (sum, sum sq) of each output row.
struct ReduceParams {
  const float* part;  // [Z][M][ldp]
  int Z, M, N, ldp;
  const float* bias;
  const float* resid;
  int resid_mod;      // row index of resid taken modulo this (0 = no modulo)
  float* stat_out;    // [rows][2] or null
  const float* gain;  // per-column scale of the bf16 shadow (gain of the norm that follows), or null
  float* out_f32;
  bf16* out_bf16;     // XF layout with ldo2 padded columns
  int ldo, ldo2;
  unsigned char* out8;         // optional MXFP8 copy of the gain-scaled row (N multiple of 256) in MX fragment order, or null
  unsigned char* out8_scales;
};
hipError_t launch_splitk_reduce(hipStream_t s, const ReduceParams& p);
// stat_out[m] = (sum, sum sq) of fp32 row m of x; out_xf = bf16(x * gain) in XF layout with k_pad columns
hipError_t launch_row_stats(hipStream_t s, const float* x, int ld, int M, int K, int k_pad, const float* gain, bf16* out_xf,
                            float* stat_out);
// dst[i] = src[i] (+1 if one_plus): fp32 gain vectors of the norms
hipError_t launch_gain_vector(hipStream_t s, const bf16* src, float* dst, int n, int one_plus);

// ------------------------------------------------------------------------------------------
// Attention over fragment-ordered keys / values.
// Key fragments:   [head][chunk][s = d/16][lane = ((d%16)/8)*32 + key%32][d%8]
// Value fragments: [head][chunk][vb = d/32][s2 = (key%32)/16][lane = ((key%8)/4)*32 + d%32]
//                  [j = ((key%16)/8)*4 + key%4]
// ------------------------------------------------------------------------------------------
struct AttnParams {
  const bf16* q;       // fragment order [head][ceil(Tq/32)][dqk/16][64][8]; q_head_stride elements per head
  int q_head_stride;
  int Tq;              // query rows per head
  int heads;
  const bf16* k0;      // first key segment (prefix cache or the layer's own keys)
  const bf16* v0;
  int chunks0;         // chunks in segment 0 (per head)
  int valid0;          // valid keys in segment 0 (keys >= valid0 are masked)
  int kv_head_stride0; // elements between heads in k0 (0 = shared head); v uses v_head_stride0
  int v_head_stride0;
  const bf16* k1;      // optional second segment (the suffix's own keys), 0 or 2 chunks
  const bf16* v1;
  int chunks1;
  int view_tokens;     // > 0: query row m only sees keys of its own view [m/vt*vt, +vt)
  int suffix_mask;     // 1: row 0 sees only key 0 of segment 1; other rows see all of segment 1
  float scale;
  bf16* out;           // XF layout, out_ld padded columns; head h at columns h * head_dim ..
  int out_ld;
  int head_dim;        // 72 or 256
  // keys of segment 0 shared out over key_splits blocks per (query tile, head) (0 / 1 = off): share z
  // takes chunks [z * chunks_per_split, ...), the last one also segment 1; each share writes its own
  // normalised output at out + z * out_split_stride and (row maximum, sum of exponentials) at
  // ml_out[((z * heads + head) * ceil32(Tq) + row) * 2]; the consumer merges them
  int key_splits;
  int chunks_per_split;
  size_t out_split_stride;
  float* ml_out;
  int v_split;         // head dim 256 only: 2 / 4 / 8 blocks per (query tile, head), each with 1 / v_split of the value slices (0 / 1 = off)
  PrefetchDesc pf;     // warm-up blocks for later launches
};
hipError_t launch_attention(hipStream_t s, const AttnParams& p);
hipError_t attention_init_attributes();

// ------------------------------------------------------------------------------------------
// small kernels
// ------------------------------------------------------------------------------------------
hipError_t launch_pack_weights(hipStream_t s, const PackSrc& src, bf16* dst, int n_pad, int k_pad);
// colsum[n] = sum_k gain_k * W[k][col] in fp32; bias_out[n] = sum_k ln_bias[k]*W[k][col] + bias_cat[n]
hipError_t launch_fold_vectors(hipStream_t s, const PackSrc& src, const bf16* ln_bias, const bf16* const bias_src[3],
                               float* colsum, float* bias_out, int n_pad);
hipError_t launch_bf16_to_f32(hipStream_t s, const bf16* src, float* dst, size_t n);
hipError_t launch_copy_bf16(hipStream_t s, const bf16* src, bf16* dst, size_t n);
hipError_t launch_fill_zero(hipStream_t s, void* dst, size_t bytes);
// W_fold[r][n] (r < action_dim) and bias table rows (r = action_dim + step)
hipError_t launch_time_fold(hipStream_t s, const bf16* wa, const bf16* ba, const bf16* wt1, const bf16* bt1,
                            const float* tau, int action_dim, int X, int steps, float* wfold, float* bias_tab);

hipError_t launch_patchify(hipStream_t s, const float* images, int n_views, int img, int patch, bf16* out, int ld);
hipError_t launch_embed_prompt(hipStream_t s, const int32_t* ids, int n, const bf16* table, int vocab, int E, float scale,
                               float* out_f32, bf16* out_bf16, int row0);
hipError_t launch_state_token(hipStream_t s, const float* state, int state_dim, const float* ws, const float* bs, int X,
                              float* out, int* progress);
// read-ahead kernel of the action expert: per layer RA_REGIONS byte ranges (weights of the four GEMMs, the
// layer's slice of the key and of the value cache), region r of layer l at base[r] + l * layer_stride[r]
enum { RA_REGIONS = 6 };
struct ReadAheadParams {
  const unsigned char* base[RA_REGIONS];
  size_t layer_stride[RA_REGIONS];   // bytes, multiples of 16
  unsigned n16[RA_REGIONS];          // 16-byte words per layer (0 = region unused)
  int layers, steps;
  int lead;                          // layer-steps read ahead of the compute stream (>= 1)
  const int* progress;               // number of layer-steps the compute stream has started
  long long wait_ticks;              // bound of one wait, 100 MHz wall-clock ticks
  unsigned* sink;                    // [1024]
};
hipError_t launch_read_ahead(hipStream_t s, const ReadAheadParams& p, int blocks, int threads, int depth);
// z = silu(x @ W_fold + bias_k) -> bf16 [64][X] (row chunk.. zero);  Y row 0 = state token
hipError_t launch_action_embed(hipStream_t s, const float* x, int chunk, int action_dim, const float* wfold,
                               const float* bias_k, int X, bf16* z, const float* state_tok, float* y_f32, bf16* y_bf16,
                               const float* gain, float* stat_parts);
hipError_t launch_copy_f32(hipStream_t s, const float* src, float* dst, size_t n);
// natural-order dump of fragment-ordered caches (debug taps)
hipError_t launch_unpack_kv(hipStream_t s, const bf16* kfrag, const bf16* vfrag, int P, float* k_out, float* v_out);
