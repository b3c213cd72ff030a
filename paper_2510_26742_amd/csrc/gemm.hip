// bf16 MFMA GEMM family for gfx950 with fused prologue statistics and epilogues.
//
// Orientation: the packed weights are the MFMA A operand (32 output features x 16 k per
// fragment, read straight from HBM in fragment order, one coalesced 1 KiB read per wave), the
// activations are the B operand (32 tokens x 16 k, staged through LDS).  The accumulator of
// v_mfma_f32_32x32x16_bf16 then holds C^T: lane l owns token (l % 32) and, in register r, output
// feature 8*(r/4) + 4*(l/32) + r%4.  Per-token quantities (norm statistics, RoPE position) are
// per-lane scalars and partner features (RoPE pairs, gate/up pairs) sit in neighbouring
// registers of one lane, so every epilogue of Table 2 (bias, residual, activation, RMS / LN applied
// after accumulation as in Section 4.4, RoPE of Section 3.2, gated MLP of Section 4.2) is lane-local.
#include "pi0_internal.h"


#include "gemm_common.h"

// Tall GEMM (256 .. 816 tokens): the vision tower and the prefix transformer.
// Block = WN waves, each owning NT adjacent 32-feature tiles, all sharing one MB*32-token activation
// tile that is staged through LDS in chunks of 64 k (4 fragments per 32-token block, copied 1 KiB at
// a time from the XF layout, so global reads, LDS writes and LDS reads are all contiguous).  A
// "stage" is the block's activation chunk plus each wave's 4 * NT weight fragments.  D stages are kept
// in flight in registers and every stage is issued the same distance ahead of its use:
// vector-memory loads complete in issue order, so a weight prefetch issued far ahead does not
// help if the activation load behind which it queues is only one chunk ahead.
#define STAT_PARTS_MAX 64   // most partial-statistics planes a tall kernel accepts (2048 columns / 32)
// NT > 1: every wave owns NT adjacent feature tiles, so that an activation fragment read from LDS
// feeds NT MFMAs (with NT = 1 and 32-feature wave tiles the LDS read rate, one 1 KiB fragment per
// MFMA per wave, is exactly the LDS peak, and the matrix pipe cannot be kept busy).
// OCC = 2: cut for two resident blocks per compute unit (two waves per SIMD, at most 256 registers): launches with a
// few more blocks than compute units then run in one round, and a block's cold start and epilogue overlap its neighbour's loop.
template <int MB, int WN, int D, int PRO, int EPI, int NT = 1, int OCC = 1>
__global__ __launch_bounds__(64 * WN) __attribute__((amdgpu_waves_per_eu(OCC, OCC))) void gemm_kernel(GemmParams p) {
  constexpr int ROWS = MB * 32;
  constexpr int NFR = MB * 4;             // fragments per chunk
  constexpr int NP = NFR / WN;            // fragments staged per wave per chunk
  static_assert(NFR % WN == 0, "staging must tile the fragments");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* xs = reinterpret_cast<bf16*>(smem_raw);                                        // [2][NFR][64][8]

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wn = t >> 6;

  // XCD-aware tile order: consecutive block ids go to different XCDs (separate L2s), so the
  // m-tiles that share one weight panel are given ids with equal (id % 8).
  const int nblocks_n = (p.n_tiles + WN * NT - 1) / (WN * NT);
  const int id = blockIdx.x;
  const int slot = id >> 3;
  const int nb = (id & 7) + 8 * (slot / p.m_tiles);
  const int mt = slot % p.m_tiles;
  if (nb >= nblocks_n) return;
  const int m0 = mt * ROWS;
  const int nt = (nb * WN + wn) * NT;          // first of the wave's NT feature tiles (n_tiles is a multiple of NT)
  const bool wave_active = nt < p.n_tiles;

  const int k_pad = p.W.k_pad;
  const int kbeg = blockIdx.y * p.k_per_split;
  const int kend = min(kbeg + p.k_per_split, k_pad);
  const int NC = (kend - kbeg + 63) >> 6;
  const int KC16 = k_pad >> 4;
  const int XKC16 = p.ldx >> 4;
  const int mb_last = (p.M - 1) >> 5;

  // Staging: fragment f = wn + WN*i of the chunk, f = mb*4 + s.  All loads are unconditional
  // (block index clamped into the valid range) so that the loop body is straight-line code: the
  // compiler then keeps exact per-register wait counts and really leaves D stages in flight.
  // Token blocks beyond M re-read the last block (their outputs are never stored), chunks beyond
  // the last re-read the last chunk (never computed).
  bf16x8 xr[D][NP];
  bf16x8 wr[D][NT][4];
  const bf16* xfrag[NP];
#pragma unroll
  for (int i = 0; i < NP; i++) {
    const int f = wn + WN * i;
    const int mbg = min((m0 >> 5) + (f >> 2), mb_last);
    xfrag[i] = p.X + ((size_t)mbg * XKC16 + (kbeg >> 4) + (f & 3)) * 512 + lane * 8;
  }
  const bf16* wbase = p.W.w + ((size_t)(wave_active ? nt : 0) * KC16 + (kbeg >> 4)) * 512 + lane * 8;
  const size_t wtile = (size_t)KC16 * 512;     // elements between adjacent feature tiles

#define ISSUE_STAGE(c, u)                                                                             \
  {                                                                                                   \
    const int cc_ = min((c), NC - 1);                                                                 \
    _Pragma("unroll") for (int i = 0; i < NP; i++)                                                    \
      xr[u][i] = *reinterpret_cast<const bf16x8*>(xfrag[i] + (size_t)cc_ * 2048);                     \
    _Pragma("unroll") for (int j_ = 0; j_ < NT; j_++)                                                 \
      _Pragma("unroll") for (int s_ = 0; s_ < 4; s_++)                                                \
        wr[u][j_][s_] = *reinterpret_cast<const bf16x8*>(wbase + j_ * wtile + (size_t)(cc_ * 4 + s_) * 512); \
  }
#define STORE_STAGE(u, buf)                                                                           \
  {                                                                                                   \
    _Pragma("unroll") for (int i = 0; i < NP; i++)                                                    \
      *reinterpret_cast<bf16x8*>(xs + (((size_t)(buf) * NFR + wn + WN * i) * 64 + lane) * 8) = xr[u][i]; \
  }

  f32x16 acc[NT][MB];
#pragma unroll
  for (int j = 0; j < NT; j++)
#pragma unroll
    for (int mb = 0; mb < MB; mb++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[j][mb][r] = 0.f;

#pragma unroll
  for (int u = 0; u < D; u++) ISSUE_STAGE(u, u)
  // Row statistics given as partial sums (the producer was a GEMM over the whole k range that left
  // one sum per 32-column tile): thread (g, row) adds planes g * pg .. g * pg + pg - 1 of its row.
  // The loads are issued together behind the first stages (no extra round trip) and the SG group
  // sums per row are kept in LDS until the epilogue adds them, always in the same order.
  constexpr int SG = (64 * WN) / ROWS > 0 ? (64 * WN) / ROWS : 1;      // thread groups per row
  constexpr int SPG = STAT_PARTS_MAX / SG;                             // planes per group, at most
  static_assert(ROWS <= 64 * WN, "one thread per row at least");
  float2* sstat = reinterpret_cast<float2*>(smem_raw + 2 * NFR * 1024);   // [SG][ROWS]
  if (PRO != PRO_NONE && p.rowstat_parts > 1) {
    const int row = t % ROWS, g = t / ROWS;
    const int pg = (p.rowstat_parts + SG - 1) / SG;
    const size_t rowg = (size_t)min(m0 + row, p.M - 1);
    float2 v[SPG];
#pragma unroll
    for (int jj = 0; jj < SPG; jj++) {
      const int j = min(g * pg + min(jj, pg - 1), p.rowstat_parts - 1);   // clamped, unconditional
      v[jj] = *reinterpret_cast<const float2*>(p.rowstat + 2 * ((size_t)j * p.stat_rows + rowg));
    }
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int jj = 0; jj < SPG; jj++) {
      if (jj < pg && g * pg + jj < p.rowstat_parts) {
        a += v[jj].x;
        b += v[jj].y;
      }
    }
    if (g < SG) sstat[g * ROWS + row] = make_float2(a, b);
  }
  STORE_STAGE(0, 0)
  __syncthreads();

  const int lq = lane & 31;
  const int lh = lane >> 5;
  int cur = 0;
  // One chunk: 4 k16 steps of MB MFMAs against the wave's weight fragments wr[u][*]; the B
  // fragments of step s+1 are read from LDS while the MFMAs of step s run.  With one wave per SIMD
  // nothing else overlaps memory instructions with the matrix pipe, so the main loop asks the
  // scheduler for an explicit interleave: behind every MFMA one LDS read (next step's operands),
  // one of the 12 global loads of the stage issued this iteration, or one of the LDS writes of
  // the next chunk.
#define COMPUTE_CHUNK(u)                                                                              \
  {                                                                                                   \
    const bf16* xb_ = xs + ((size_t)cur * NFR * 64 + lane) * 8;                                       \
    bf16x8 bq_[2][MB];                                                                                \
    _Pragma("unroll") for (int mb = 0; mb < MB; mb++)                                                 \
      bq_[0][mb] = *reinterpret_cast<const bf16x8*>(xb_ + (size_t)(mb * 4) * 512);                    \
    _Pragma("unroll") for (int s = 0; s < 4; s++) {                                                   \
      if (s < 3) {                                                                                    \
        _Pragma("unroll") for (int mb = 0; mb < MB; mb++)                                             \
          bq_[(s + 1) & 1][mb] = *reinterpret_cast<const bf16x8*>(xb_ + (size_t)(mb * 4 + s + 1) * 512); \
      }                                                                                               \
      _Pragma("unroll") for (int mb = 0; mb < MB; mb++)                                               \
        _Pragma("unroll") for (int j_ = 0; j_ < NT; j_++)                                             \
          acc[j_][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[u][j_][s], bq_[s & 1][mb], acc[j_][mb], 0, 0, 0); \
    }                                                                                                 \
  }
  int c0 = 0;
  for (; c0 + D <= NC; c0 += D) {
#pragma unroll
    for (int u = 0; u < D; u++) {
      const int c = c0 + u;
      COMPUTE_CHUNK(u)
      ISSUE_STAGE(c + D, u)
      STORE_STAGE((u + 1) % D, cur ^ 1)
      // ---- requested instruction order (masks: 0x008 MFMA, 0x100 LDS read, 0x200 LDS write, 0x020 VMEM read)
      __builtin_amdgcn_sched_group_barrier(0x100, MB, 0);
      if (NT == 1) {
#pragma unroll
        for (int i = 0; i < MB; i++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < MB; i++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if (i < NP + 4 - MB) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < MB; i++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < MB; i++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (i < NP) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
      } else {
        // NT MFMAs per LDS read; the NP + 4 NT global loads of the new stage behind the first ones
        // of steps 0..2, the NP LDS writes of the next chunk inside step 3
#pragma unroll
        for (int st = 0; st < 3; st++) {
#pragma unroll
          for (int i = 0; i < MB; i++) {
            __builtin_amdgcn_sched_group_barrier(0x008, NT, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (st * MB + i < NP + 4 * NT) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          }
        }
#pragma unroll
        for (int i = 0; i < MB; i++) {
          __builtin_amdgcn_sched_group_barrier(0x008, NT, 0);
          if (i < NP) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
      }
      __syncthreads();
      cur ^= 1;
    }
  }
  // tail: fewer than D chunks left, same steps with guards
#pragma unroll
  for (int u = 0; u < D - 1; u++) {
    const int c = c0 + u;
    if (c < NC) {
      COMPUTE_CHUNK(u)
      STORE_STAGE((u + 1) % D, cur ^ 1)
      __syncthreads();
      cur ^= 1;
    }
  }
#undef COMPUTE_CHUNK
#undef ISSUE_STAGE
#undef STORE_STAGE

  // ---- epilogue --------------------------------------------------------------------------------
  // row statistics (from the kernel that produced the residual stream) of all token blocks in one
  // round trip, rows clamped into range
  float2 rst[MB];
  if (PRO != PRO_NONE) {
    if (p.rowstat_parts <= 1) {
#pragma unroll
      for (int mb = 0; mb < MB; mb++)
        rst[mb] = *reinterpret_cast<const float2*>(p.rowstat + 2 * (size_t)min(m0 + mb * 32 + lq, p.M - 1));
    } else {
      // partial statistics were added up at entry (see above): one sum per thread group in LDS
#pragma unroll
      for (int mb = 0; mb < MB; mb++) {
        float a = 0.f, b = 0.f;
#pragma unroll
        for (int g = 0; g < SG; g++) {
          const float2 v = sstat[g * ROWS + mb * 32 + lq];
          a += v.x;
          b += v.y;
        }
        rst[mb] = make_float2(a, b);
      }
    }
  }
  if (!wave_active) return;
#pragma unroll
  for (int mb = 0; mb < MB; mb++) {
    const int ml = mb * 32 + lq;
    const int m = m0 + ml;
    if (m < p.M) {
      float ssum = 0.f, ssq = 0.f;
      if (PRO != PRO_NONE) {
        ssum = rst[mb].x;
        ssq = rst[mb].y;
      }
#pragma unroll
      for (int j = 0; j < NT; j++) {
        EpiOps ops;
        epilogue_preload<PRO, EPI>(p, nt + j, m, lh, ops);
        epilogue_tile<PRO, EPI>(p, acc[j][mb], nt + j, m, lh, ssum, ssq, blockIdx.y, ops);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// "Entry" GEMM: the skinny kernels' plan (every load of the block issued at entry, one wait, no
// LDS staging) for the O projections of the vision tower (k = 1152) and of the prefix at one view
// (k = 2048).  As split-K partial GEMMs these need a reduction launch behind them; as one tall
// GEMM over the whole k range they spend their time on consecutive memory round trips (18 or 32
// chunks at 6 in flight).  Here one block = 64 tokens x NT feature tiles; 8 waves split the k16
// steps (at most EN_SPW each) and hold their slice of both operands in registers, so the block
// pays one round trip, and the residual epilogue runs in the same launch.  Partial tiles meet in
// LDS, one 32-token block at a time, and are added in wave order; wave mb * NT + j finishes tile
// (mb, j).  Input row statistics (unused by the residual epilogue) would be whole-row sums.
// ------------------------------------------------------------------------------------------------
template <int PRO, int EPI, int NT, int EN_SPW>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_entry_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* red = reinterpret_cast<float*>(smem_raw);                 // [8 waves][NT][4][64][4]
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int w = t >> 6;
  const int lq = lane & 31;
  const int lh = lane >> 5;
  // die-aware order: consecutive block ids go to different dies (an L2 each), so the token blocks that share one
  // weight panel are given ids with equal (id % 8) and fetch it from memory once
  // (measured: vision QKV, 8 MB of weights, 10.8 -> 10.1 us and 3.7 x -> 1 x of its bytes from memory; the O projections
  // with one feature tile per block lose 0.3 us, so they keep the plain two-dimensional grid)
  int nb = (int)blockIdx.x, mt = (int)blockIdx.y;
  if (NT > 1) {
    const int nblocks_n = (p.n_tiles + NT - 1) / NT;
    const int slot = (int)blockIdx.x >> 3;
    nb = ((int)blockIdx.x & 7) + 8 * (slot / p.m_tiles);
    mt = slot % p.m_tiles;
    if (nb >= nblocks_n) return;
  }
  const int nt0 = nb * NT;
  const int m0 = mt * 64;
  const int KC16 = p.W.k_pad >> 4;
  const int XKC16 = p.ldx >> 4;
  const int spw = (KC16 + SK_WAVES - 1) / SK_WAVES;        // host picks the instantiation with spw <= EN_SPW
  const int s_beg = w * spw, s_end = min(s_beg + spw, KC16);
  const int mb_last = (p.M - 1) >> 5;
  bf16x8 wf[NT][EN_SPW], xf[2][EN_SPW];
#pragma unroll
  for (int i = 0; i < EN_SPW; i++) {
    const int st = min(s_beg + i, KC16 - 1);   // clamped: steps beyond the wave's range are never used
#pragma unroll
    for (int j = 0; j < NT; j++)
      wf[j][i] = *reinterpret_cast<const bf16x8*>(p.W.w + ((size_t)min(nt0 + j, p.n_tiles - 1) * KC16 + st) * 512 + lane * 8);
#pragma unroll
    for (int mb = 0; mb < 2; mb++)
      xf[mb][i] = *reinterpret_cast<const bf16x8*>(p.X + ((size_t)min((m0 >> 5) + mb, mb_last) * XKC16 + st) * 512 + lane * 8);
  }
  const int fin_mb = w / NT, fin_j = w - fin_mb * NT;
  const bool finisher = w < 2 * NT && nt0 + fin_j < p.n_tiles;
  const int mrow = m0 + fin_mb * 32 + lq;
  f32x16 acc[2][NT];
#pragma unroll
  for (int mb = 0; mb < 2; mb++)
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mb][j][r] = 0.f;
#pragma unroll
  for (int i = 0; i < EN_SPW; i++) {
    if (s_beg + i < s_end) {
#pragma unroll
      for (int mb = 0; mb < 2; mb++)
#pragma unroll
        for (int j = 0; j < NT; j++) acc[mb][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j][i], xf[mb][i], acc[mb][j], 0, 0, 0);
    }
  }
  // The finishing waves fetch what their epilogue needs once the operand registers are free; the
  // round trip overlaps the reduction through LDS.
  EpiOps ops;
  float2 rst = make_float2(0.f, 0.f);
  if (finisher && mrow < p.M) {
    if (PRO != PRO_NONE) rst = *reinterpret_cast<const float2*>(p.rowstat + 2 * (size_t)mrow);
    epilogue_preload<PRO, EPI>(p, nt0 + fin_j, mrow, lh, ops);
  }
  f32x16 sum;
#pragma unroll
  for (int r = 0; r < 16; r++) sum[r] = 0.f;
#pragma unroll
  for (int mb = 0; mb < 2; mb++) {
    if (mb) __syncthreads();   // the readers of the first round are done
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const f32x4 v4 = {acc[mb][j][4 * q], acc[mb][j][4 * q + 1], acc[mb][j][4 * q + 2], acc[mb][j][4 * q + 3]};
        *reinterpret_cast<f32x4*>(red + ((((size_t)w * NT + j) * 4 + q) * 64 + lane) * 4) = v4;
      }
    __syncthreads();
    if (fin_mb == mb && w < 2 * NT) {
#pragma unroll
      for (int ww = 0; ww < SK_WAVES; ww++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const f32x4 v4 = *reinterpret_cast<const f32x4*>(red + ((((size_t)ww * NT + fin_j) * 4 + q) * 64 + lane) * 4);
#pragma unroll
          for (int jj = 0; jj < 4; jj++) sum[4 * q + jj] += v4[jj];
        }
    }
  }
  if (finisher && mrow < p.M) epilogue_tile<PRO, EPI>(p, sum, nt0 + fin_j, mrow, lh, rst.x, rst.y, 0, ops);
}

// Skinny GEMM over the whole k range with the residual epilogue (the expert's O and down
// projections, k = 2048 / 4096): one block per (32-feature tile, 32-token block), 8 waves each
// owning 1/8 of k in NB batches of 16 k16 steps.  No split across blocks, so the residual add, the
// bf16 shadow and the per-tile row statistics are done here and no reduction kernel follows.
template <int NB>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_skinny_fullk_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* red = reinterpret_cast<float*>(smem_raw);                 // [8 waves][16][64]
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int w = t >> 6;
  const int lq = lane & 31;
  const int lh = lane >> 5;
  if ((int)blockIdx.x >= p.n_tiles) {   // warm-up block; rank = linear block index (mod 8)
    prefetch_role(p.pf, (int)blockIdx.x - p.n_tiles + (int)blockIdx.y * ((int)gridDim.x - p.n_tiles));
    return;
  }
  const int nt = blockIdx.x;
  const int mb = blockIdx.y;
  const int KC16 = p.W.k_pad >> 4;
  const int XKC16 = p.ldx >> 4;
  const int spw = 16 * NB;                     // steps per wave; host guarantees KC16 == 8 * spw
  const bf16* wbase = p.W.w + ((size_t)nt * KC16 + (size_t)w * spw) * 512 + lane * 8;
  const bf16* xbase = p.X + ((size_t)mb * XKC16 + (size_t)w * spw) * 512 + lane * 8;
  // two accumulators: consecutive MFMAs do not wait for each other
  f32x16 acc, acc1;
#pragma unroll
  for (int r = 0; r < 16; r++) acc[r] = 0.f, acc1[r] = 0.f;
  EpiOps ops;
  const int m = mb * 32 + lq;
#pragma unroll
  for (int b = 0; b < NB; b++) {
    bf16x8 wf[16], xf[16];
#pragma unroll
    for (int i = 0; i < 16; i++) {
      wf[i] = *reinterpret_cast<const bf16x8*>(wbase + (size_t)(b * 16 + i) * 512);
      xf[i] = *reinterpret_cast<const bf16x8*>(xbase + (size_t)(b * 16 + i) * 512);
    }
    // operands of the epilogue (wave 0 runs it), behind the first batch of operand loads
    if (b == 0 && w == 0 && m < p.M) epilogue_preload<PRO_NONE, EPI_RESID>(p, nt, m, lh, ops);
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[i], acc, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i + 1], xf[i + 1], acc1, 0, 0, 0);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; r++) red[((size_t)w * 16 + r) * 64 + lane] = acc[r] + acc1[r];
  __syncthreads();
  if (w != 0) return;
  f32x16 sum;
#pragma unroll
  for (int r = 0; r < 16; r++) sum[r] = 0.f;
#pragma unroll
  for (int ww = 0; ww < SK_WAVES; ww++)
#pragma unroll
    for (int r = 0; r < 16; r++) sum[r] += red[((size_t)ww * 16 + r) * 64 + lane];
  if (m < p.M) epilogue_tile<PRO_NONE, EPI_RESID>(p, sum, nt, m, lh, 0.f, 0.f, 0, ops);
}

static constexpr int skinny_smem_bytes() { return (SK_WAVES * 2 * 16 * 64 + 128 + SK_WAVES * 128) * 4; }

// ------------------------------------------------------------------------------------------------
// two staging buffers of MB * 4 fragments, then one (sum, sum of squares) pair per thread
template <int MB, int WN>
static constexpr int smem_bytes_for() {
  return 2 * (MB * 4) * 1024 + 64 * WN * 8;
}

int gemm_rows_per_tile(int tile) {
  switch (tile) {
    case TILE_BIG: return 256;
    case TILE_MID: return 64;
    case TILE_SKINNY: return 64;
    case TILE_SKINNY_FULLK: return 64;
    case TILE_SKINNY16: return 64;
    case TILE_SMALL: return 64;
    case TILE_WIDE: return 256;
    case TILE_WIDE128: return 128;
    case TILE_ENTRY: return 64;
    case TILE_SQ128: return 128;
    case TILE_T192: return 192;
    case TILE_MID2: return 64;
    default: return -1;
  }
}

template <int MB, int WN, int D, int PRO, int EPI, int NT, int OCC = 1>
static hipError_t launch_one(hipStream_t s, const GemmParams& p, int z) {
  if (p.n_tiles % NT != 0) return hipErrorInvalidValue;
  const int nblocks_n = (p.n_tiles + WN * NT - 1) / (WN * NT);
  dim3 grid(8 * ((nblocks_n + 7) / 8) * p.m_tiles, z, 1);
  dim3 block(64 * WN, 1, 1);
  constexpr int smem = smem_bytes_for<MB, WN>();
  gemm_kernel<MB, WN, D, PRO, EPI, NT, OCC><<<grid, block, smem, s>>>(p);
  return hipGetLastError();
}

template <int MB, int WN, int D, int PRO, int EPI, int NT, int OCC = 1>
static hipError_t set_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<MB, WN, D, PRO, EPI, NT, OCC>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes_for<MB, WN>());
}

// The instantiations that exist.  X(tile id, MB, WN, D, PRO, EPI, NT)
#define TALL_EPIS(X, T, MB, WN, D)    \
  X(T, MB, WN, D, PRO_NONE, EPI_RESID, 1)   \
  X(T, MB, WN, D, PRO_NONE, EPI_PARTIAL, 1) \
  X(T, MB, WN, D, PRO_LN, EPI_QKV, 1)       \
  X(T, MB, WN, D, PRO_LN, EPI_BF16, 1)      \
  X(T, MB, WN, D, PRO_LN, EPI_RESID, 1)     \
  X(T, MB, WN, D, PRO_RMS, EPI_QKV, 1)      \
  X(T, MB, WN, D, PRO_RMS, EPI_GEGLU, 1)
#define GEMM_VARIANTS(X)           \
  TALL_EPIS(X, TILE_BIG, 8, 4, 3)  \
  TALL_EPIS(X, TILE_MID, 2, 4, 6)   \
  TALL_EPIS(X, TILE_SMALL, 2, 2, 6) \
  TALL_EPIS(X, TILE_SQ128, 4, 4, 5) \
  X(TILE_WIDE, 8, 4, 2, PRO_RMS, EPI_GEGLU, 2)   \
  X(TILE_WIDE, 8, 4, 2, PRO_NONE, EPI_PARTIAL, 2) \
  X(TILE_WIDE128, 4, 4, 3, PRO_RMS, EPI_GEGLU, 2)   \
  X(TILE_WIDE128, 4, 4, 3, PRO_NONE, EPI_PARTIAL, 2) \
  X(TILE_T192, 6, 4, 3, PRO_RMS, EPI_GEGLU, 2)   \
  X(TILE_T192, 6, 4, 2, PRO_NONE, EPI_PARTIAL, 2)

// ... and those cut for two resident blocks per compute unit: 64 x 128 tiles, 6 stages
#define TALL_EPIS2(X, T, MB, WN, D)    \
  X(T, MB, WN, D, PRO_NONE, EPI_RESID, 1, 2)   \
  X(T, MB, WN, D, PRO_NONE, EPI_PARTIAL, 1, 2) \
  X(T, MB, WN, D, PRO_LN, EPI_QKV, 1, 2)       \
  X(T, MB, WN, D, PRO_LN, EPI_BF16, 1, 2)      \
  X(T, MB, WN, D, PRO_LN, EPI_RESID, 1, 2)     \
  X(T, MB, WN, D, PRO_RMS, EPI_QKV, 1, 2)
#define GEMM_VARIANTS2(X) TALL_EPIS2(X, TILE_MID2, 2, 4, 6)

// X(PRO, EPI, feature tiles per block, k16 steps per wave), ascending steps: vision O (k = 1152), prefix O
// (k = 2048), vision QKV (k = 1152, 64 x 64 tiles)
#define ENTRY_VARIANTS(X)       \
  X(PRO_NONE, EPI_RESID, 1, 9)  \
  X(PRO_NONE, EPI_RESID, 1, 16) \
  X(PRO_LN, EPI_QKV, 2, 9)
static constexpr int entry_smem_bytes(int nt) { return SK_WAVES * nt * 16 * 64 * 4; }

#define SKINNY_VARIANTS(X)      \
  X(PRO_NONE, EPI_RESID)        \
  X(PRO_NONE, EPI_PARTIAL)      \
  X(PRO_RMS, EPI_QKV)           \
  X(PRO_RMS, EPI_GEGLU)         \
  X(PRO_RMS, EPI_EULER)

hipError_t gemm_init_attributes() {
#define X(PRO, EPI)                                                                                              \
  {                                                                                                              \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_skinny_kernel<PRO, EPI>),             \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, skinny_smem_bytes());         \
    if (e != hipSuccess) return e;                                                                               \
  }
  SKINNY_VARIANTS(X)
#undef X
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_skinny_kernel<PRO_RMS, EPI_QKV, 1>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, skinny_smem_bytes());
    if (e != hipSuccess) return e;
  }
#define X(PRO, EPI, NT, SPW)                                                                                     \
  {                                                                                                              \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_entry_kernel<PRO, EPI, NT, SPW>),     \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, entry_smem_bytes(NT));        \
    if (e != hipSuccess) return e;                                                                               \
  }
  ENTRY_VARIANTS(X)
#undef X
#define X(T, MB, WN, D, PRO, EPI, NT)                                 \
  {                                                                   \
    hipError_t e = set_attr<MB, WN, D, PRO, EPI, NT>();               \
    if (e != hipSuccess) return e;                                    \
  }
  GEMM_VARIANTS(X)
#undef X
#define X(T, MB, WN, D, PRO, EPI, NT, OCC)                            \
  {                                                                   \
    hipError_t e = set_attr<MB, WN, D, PRO, EPI, NT, OCC>();          \
    if (e != hipSuccess) return e;                                    \
  }
  GEMM_VARIANTS2(X)
#undef X
  return hipSuccess;
}

// every region of a warm-up descriptor must be given completely; the caller guarantees that
// [ptr, ptr + tiles * tile16 * 16) is readable device memory
static bool prefetch_ok(const PrefetchDesc& d) {
  if (d.blocks == 0) return true;
  if (d.blocks < 0 || d.blocks % 16 != 0 || d.blocks > 1024 || d.sink == nullptr) return false;
  for (int r = 0; r < 3; r++) {
    if (d.ptr[r] == nullptr) continue;
    if (d.tiles[r] <= 0 || d.tile16[r] <= 0 || (reinterpret_cast<uintptr_t>(d.ptr[r]) & 15) != 0) return false;
    if ((long)((d.tiles[r] + 7) / 8) * d.tile16[r] > 0x7fffffffL) return false;
  }
  return true;
}

hipError_t launch_gemm(hipStream_t s, int tile, int pro, int epi, const GemmParams& p, int z_splits) {
  // Host-side shape checks: everything the kernel's indexing assumes.
  if (!prefetch_ok(p.pf)) return hipErrorInvalidValue;
  if (p.pf.blocks != 0 && ((tile != TILE_SKINNY && tile != TILE_SKINNY_FULLK && tile != TILE_SKINNY16) || z_splits != 1)) return hipErrorInvalidValue;
  if (p.X == nullptr || p.W.w == nullptr || p.M <= 0 || z_splits < 1) return hipErrorInvalidValue;
  if (p.W.k_pad % 64 != 0 || p.W.n_pad % 32 != 0 || p.n_tiles * 32 != p.W.n_pad) return hipErrorInvalidValue;
  if (p.ldx < p.W.k_pad || p.ldx % 16 != 0) return hipErrorInvalidValue;   // X is in XF layout with ldx padded columns
  if (p.k_per_split % 64 != 0 || (long)p.k_per_split * z_splits < p.W.k_pad) return hipErrorInvalidValue;
  if (pro != PRO_NONE && (z_splits != 1 || p.rowstat == nullptr)) return hipErrorInvalidValue;
  if (epi != EPI_PARTIAL && z_splits != 1) return hipErrorInvalidValue;
  if (p.m_tiles < 1) return hipErrorInvalidValue;
  if (tile == TILE_BIG || tile == TILE_MID || tile == TILE_SMALL || tile == TILE_WIDE || tile == TILE_WIDE128 || tile == TILE_T192 || tile == TILE_ENTRY || tile == TILE_MID2) {
    // partial row statistics: planes of stat_rows rows, every row a block touches inside a plane
    if (pro != PRO_NONE && p.rowstat_parts > 1 && (p.stat_rows < p.M || p.rowstat_parts > STAT_PARTS_MAX)) return hipErrorInvalidValue;
    if (epi == EPI_RESID && p.stat_out != nullptr && p.stat_rows < p.M + p.row_offset) return hipErrorInvalidValue;
  }
  if (tile == TILE_SKINNY16) {
    // 16 x 16 tiles over the whole k range: k = 8 waves x NS steps x 32
    const int kc16 = p.W.k_pad >> 4;
    if (p.M > 64 || pro != PRO_NONE || epi != EPI_RESID || z_splits != 1 || (kc16 != 128 && kc16 != 256)) return hipErrorInvalidValue;
    if (p.out_f32 == nullptr || p.out_bf16 == nullptr || p.ldo % 4 != 0 || p.ldo2 % 16 != 0) return hipErrorInvalidValue;
    if (p.xsplits > 1 && (kc16 != 128 || p.xsplits > 4 || p.xsplit_ml == nullptr || p.xsplit_stride < (size_t)64 * p.ldx))
      return hipErrorInvalidValue;
    const int my = (p.M + 15) / 16;
    if (p.pf.blocks != 0 && (p.pf.blocks % my != 0 || (p.n_tiles * 2) % 8 != 0 || ((p.n_tiles * 2 + p.pf.blocks / my) * my) % 8 != 0))
      return hipErrorInvalidValue;
    const dim3 grid(p.n_tiles * 2 + (p.pf.blocks != 0 ? p.pf.blocks / my : 0), my);
    if (kc16 == 128) gemm_skinny16_kernel<8><<<grid, dim3(64 * SK_WAVES), 0, s>>>(p);
    else gemm_skinny16_kernel<16><<<grid, dim3(64 * SK_WAVES), 0, s>>>(p);
    return hipGetLastError();
  }
  if (tile == TILE_ENTRY) {
    // 64 tokens x NT feature tiles per block, the k16 steps split over 8 waves, at most EN_SPW each
    const int kc16 = p.W.k_pad >> 4;
    const int spw = (kc16 + SK_WAVES - 1) / SK_WAVES;
    if (z_splits != 1 || p.m_tiles * 64 < p.M) return hipErrorInvalidValue;
    if (pro != PRO_NONE && p.rowstat_parts > 1) return hipErrorInvalidValue;   // whole-row statistics only
    if (epi == EPI_RESID && (p.out_f32 == nullptr || p.out_bf16 == nullptr)) return hipErrorInvalidValue;
#define X(PRO, EPI, NT, SPW)                                                                                   \
  if (pro == PRO && epi == EPI && spw <= SPW) {                                                                \
    gemm_entry_kernel<PRO, EPI, NT, SPW><<<NT > 1 ? dim3(8 * (((p.n_tiles + NT - 1) / NT + 7) / 8) * p.m_tiles) : dim3(p.n_tiles, p.m_tiles), dim3(64 * SK_WAVES), \
                                           entry_smem_bytes(NT), s>>>(p);                                      \
    return hipGetLastError();                                                                                  \
  }
    ENTRY_VARIANTS(X)
#undef X
    return hipErrorInvalidValue;
  }
  if (tile == TILE_SKINNY_FULLK) {
    const int kc16 = p.W.k_pad >> 4;
    if (p.M > 64 || pro != PRO_NONE || epi != EPI_RESID || z_splits != 1 || (kc16 != 128 && kc16 != 256)) return hipErrorInvalidValue;
    if (p.pf.blocks != 0 && ((p.M + 31) / 32 != 2 || p.n_tiles % 8 != 0)) return hipErrorInvalidValue;
    const dim3 grid(p.n_tiles + p.pf.blocks / 2, (p.M + 31) / 32);
    if (kc16 == 128) gemm_skinny_fullk_kernel<1><<<grid, dim3(64 * SK_WAVES), SK_WAVES * 16 * 64 * 4, s>>>(p);
    else gemm_skinny_fullk_kernel<2><<<grid, dim3(64 * SK_WAVES), SK_WAVES * 16 * 64 * 4, s>>>(p);
    return hipGetLastError();
  }
  if (tile == TILE_SKINNY) {
    if (pro != PRO_NONE && (p.rowstat_parts < 1 || p.rowstat_parts > 8 * SK_WAVES)) return hipErrorInvalidValue;
    if (p.M > 64 || p.m_tiles != 1 || p.k_per_split > SK_KMAX || p.k_per_split % 16 != 0) return hipErrorInvalidValue;
    if (p.m_split) {   // one block per (feature tile, 32-token block)
      if (pro != PRO_RMS || epi != EPI_QKV || z_splits != 1) return hipErrorInvalidValue;
      gemm_skinny_kernel<PRO_RMS, EPI_QKV, 1><<<dim3(p.n_tiles + p.pf.blocks, 1, 2), dim3(64 * SK_WAVES), skinny_smem_bytes(), s>>>(p);
      return hipGetLastError();
    }
#define X(PRO, EPI)                                                                                          \
  if (pro == PRO && epi == EPI) {                                                                            \
    gemm_skinny_kernel<PRO, EPI><<<dim3(p.n_tiles + p.pf.blocks, z_splits), dim3(64 * SK_WAVES), skinny_smem_bytes(), s>>>(p); \
    return hipGetLastError();                                                                                \
  }
    SKINNY_VARIANTS(X)
#undef X
    return hipErrorInvalidValue;
  }
#define X(T, MB, WN, D, PRO, EPI, NT)                                          \
  if (tile == T && pro == PRO && epi == EPI) {                                  \
    if (p.m_tiles * MB * 32 < p.M) return hipErrorInvalidValue;                 \
    return launch_one<MB, WN, D, PRO, EPI, NT>(s, p, z_splits);                 \
  }
  GEMM_VARIANTS(X)
#undef X
#define X(T, MB, WN, D, PRO, EPI, NT, OCC)                                     \
  if (tile == T && pro == PRO && epi == EPI) {                                  \
    if (p.m_tiles * MB * 32 < p.M) return hipErrorInvalidValue;                 \
    return launch_one<MB, WN, D, PRO, EPI, NT, OCC>(s, p, z_splits);            \
  }
  GEMM_VARIANTS2(X)
#undef X
  return hipErrorInvalidValue;
}

// ------------------------------------------------------------------------------------------------
// split-K reduction (fixed summation order -> run-to-run bitwise determinism)
// ------------------------------------------------------------------------------------------------
// One block per output row.  Besides the fp32 sum it writes the row's (sum, sum of squares) and the
// bf16 copy that the next GEMM reads, in XF layout.  The copy is scaled per column by the gain of
// the normalisation that follows (g for LayerNorm, 1 + g for RMSNorm): the affine part of the norm
// is folded into the activation cast, so the weights stay the checkpoint's bf16 values, and the
// row statistics are applied after accumulation by the consumer (Sections 3.2 and 4.4).
__global__ __launch_bounds__(512) void splitk_reduce_kernel(ReduceParams p) {
  __shared__ float sred[2][8];
  const int m = blockIdx.x;
  const int ro = m;
  float sa = 0.f, sb = 0.f;
  for (int n = threadIdx.x * 4; n < p.N; n += 2048) {   // one pass for rows of up to 2048 columns
    // bias and residual first, so that their round trip overlaps the partial sums
    f32x4 extra = {0.f, 0.f, 0.f, 0.f};
    if (p.bias != nullptr) extra = *reinterpret_cast<const f32x4*>(p.bias + n);
    f32x4 rv = {0.f, 0.f, 0.f, 0.f};
    if (p.resid != nullptr) {
      const int rr = p.resid_mod > 0 ? (m % p.resid_mod) : m;
      rv = *reinterpret_cast<const f32x4*>(p.resid + (size_t)rr * p.ldo + n);
    }
    f32x4 gv = {1.f, 1.f, 1.f, 1.f};
    if (p.gain != nullptr) gv = *reinterpret_cast<const f32x4*>(p.gain + n);
    // partial sums in batches of 8 loads in flight (clamped, unconditional), added in slice order
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    for (int z0 = 0; z0 < p.Z; z0 += 8) {
      f32x4 v[8];
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const int z = min(z0 + j, p.Z - 1);
        v[j] = *reinterpret_cast<const f32x4*>(p.part + ((size_t)z * p.M + m) * p.ldp + n);
      }
#pragma unroll
      for (int j = 0; j < 8; j++) {
        if (z0 + j < p.Z) a += v[j];
      }
    }
    a += extra;    // same order of additions as ever: partial sums, bias, residual
    a += rv;
    *reinterpret_cast<f32x4*>(p.out_f32 + (size_t)ro * p.ldo + n) = a;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      sa += a[j];
      sb += a[j] * a[j];
    }
    a *= gv;
    const bf16x4 ob = {(bf16)a[0], (bf16)a[1], (bf16)a[2], (bf16)a[3]};
    *reinterpret_cast<bf16x4*>(p.out_bf16 + xf_index(ro, n, p.ldo2 >> 4)) = ob;
    if (p.out8 != nullptr) {
      // MXFP8 copy of the same gain-scaled values: 8 threads hold one 32-column scale block (N is a multiple of
      // 256, so a block's threads are all inside the loop)
      float amax = fmaxf(fmaxf(fabsf(a[0]), fabsf(a[1])), fmaxf(fabsf(a[2]), fabsf(a[3])));
      amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
      amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
      amax = fmaxf(amax, __shfl_xor(amax, 4, 64));
      const int code = mx_scale_code(amax);
      const float inv = mx_inv_scale(code);
      const unsigned word = mx_encode2(a[0], a[1], inv) | (mx_encode2(a[2], a[3], inv) << 16);
      const int kc64 = p.N >> 6, kc = n >> 6;
      unsigned char* frag = p.out8 + ((size_t)(ro >> 5) * kc64 + kc) * 2048;
      *reinterpret_cast<unsigned*>(frag + ((size_t)((n & 63) >> 4) * 32 + (ro & 31)) * 16 + (n & 15)) = word;
      if ((threadIdx.x & 7) == 0)
        p.out8_scales[(((size_t)(ro >> 5) * (kc64 >> 2) + (kc >> 2)) * 64 + ((n & 63) >> 5) * 32 + (ro & 31)) * 4 + (kc & 3)] =
            (unsigned char)code;
    }
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    sa += __shfl_xor(sa, off, 64);
    sb += __shfl_xor(sb, off, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    sred[0][threadIdx.x >> 6] = sa;
    sred[1][threadIdx.x >> 6] = sb;
  }
  __syncthreads();
  if (threadIdx.x == 0 && p.stat_out != nullptr) {
    float ta = 0.f, tb = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) {
      ta += sred[0][i];
      tb += sred[1][i];
    }
    p.stat_out[2 * ro] = ta;
    p.stat_out[2 * ro + 1] = tb;
  }
}

hipError_t launch_splitk_reduce(hipStream_t s, const ReduceParams& p) {
  if (p.N % 4 != 0 || p.ldp < p.N || p.ldo < p.N || p.ldo2 < p.N || p.ldo2 % 16 != 0 || p.M <= 0 || p.Z < 1) return hipErrorInvalidValue;
  if (p.out8 != nullptr && (p.N % 256 != 0 || p.out8_scales == nullptr)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)p.M), dim3(512), 0, s, p);
  return hipGetLastError();
}

// Row statistics and gain-scaled bf16 XF copy of fp32 residual rows that were not produced by a
// GEMM epilogue or the reduction kernel (prefix embeddings, first suffix tokens of a step).
__global__ __launch_bounds__(256) void row_stats_kernel(const float* x, int ld, int K, const float* gain, bf16* out_xf,
                                                        int kc16, float* stat_out) {
  __shared__ float sred[2][4];
  const int m = blockIdx.x;
  float sa = 0.f, sb = 0.f;
  for (int k = threadIdx.x * 8; k < K; k += 2048) {
    f32x4 v0 = *reinterpret_cast<const f32x4*>(x + (size_t)m * ld + k);
    f32x4 v1 = *reinterpret_cast<const f32x4*>(x + (size_t)m * ld + k + 4);
#pragma unroll
    for (int j = 0; j < 4; j++) {
      sa += v0[j] + v1[j];
      sb += v0[j] * v0[j] + v1[j] * v1[j];
    }
    if (gain != nullptr) {
      v0 *= *reinterpret_cast<const f32x4*>(gain + k);
      v1 *= *reinterpret_cast<const f32x4*>(gain + k + 4);
    }
    const bf16x8 o = {(bf16)v0[0], (bf16)v0[1], (bf16)v0[2], (bf16)v0[3], (bf16)v1[0], (bf16)v1[1], (bf16)v1[2], (bf16)v1[3]};
    *reinterpret_cast<bf16x8*>(out_xf + xf_index(m, k, kc16)) = o;
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    sa += __shfl_xor(sa, off, 64);
    sb += __shfl_xor(sb, off, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    sred[0][threadIdx.x >> 6] = sa;
    sred[1][threadIdx.x >> 6] = sb;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    stat_out[2 * m] = sred[0][0] + sred[0][1] + sred[0][2] + sred[0][3];
    stat_out[2 * m + 1] = sred[1][0] + sred[1][1] + sred[1][2] + sred[1][3];
  }
}

hipError_t launch_row_stats(hipStream_t s, const float* x, int ld, int M, int K, int k_pad, const float* gain, bf16* out_xf,
                            float* stat_out) {
  if (x == nullptr || out_xf == nullptr || stat_out == nullptr || M <= 0 || K % 8 != 0 || ld % 4 != 0 || ld < K ||
      k_pad % 16 != 0 || K > k_pad)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(row_stats_kernel, dim3((unsigned)M), dim3(256), 0, s, x, ld, K, gain, out_xf, k_pad >> 4, stat_out);
  return hipGetLastError();
}
