// Body of the attention kernels (see attention.hip for the plan), templated on the execution context so that the
// action expert's attention also runs inside the persistent kernel of the denoise loop (exec_ctx.h).
#pragma once
#include "pi0_internal.h"
#include "exec_ctx.h"

#define NEG_BIG (-1.0e30f)
#define ATT_WAVES 8

// MAXR: key rounds per wave over segment 0 (8 * MAXR chunks = 256 * MAXR keys); VRING: value
// chunks in flight per wave.
// CPW > 0 (needs MAXR == 1 and NVB == 8): phase 2 is shared out over all 8 waves instead of one wave per value slice.
// With nslice value slices in the block, the waves form G = 8 / nslice groups; wave (slice, group g) multiplies the
// chunks g, g + G, ... of [segment 0 ; segment 1] (at most CPW of them, held in registers: no ring, no second round
// trip), the G partial outputs of a slice meet in LDS and are added in group order.  The dependent chain of a wave
// drops from 2 x (all chunks) to 2 x CPW products.
template <int DQK, int NVB, int MAXR, int VRING, int CPW, class Cx>
__device__ __forceinline__ void attention_body(const AttnParams p, const Cx cx, unsigned char* smem_raw) {
  constexpr int S16 = DQK / 16;
  constexpr bool PVG = CPW > 0;
  static_assert(!PVG || (MAXR == 1 && NVB == ATT_WAVES), "chunk groups: one key round, 8 value slices");
  constexpr bool DUAL = MAXR == 1;             // second accumulators (register room permitting)
  constexpr int QB = (MAXR == 1 && S16 % 8 == 0) ? 8 : 1;   // Q fragments read from LDS per batch (register room permitting)
  constexpr int NPQ = 32 * DQK / 8;            // 16-byte pieces of the Q tile
  constexpr int QP = (NPQ + 511) / 512;        // pieces per thread
  constexpr int NPK1 = 2 * S16 * 64;           // 16-byte pieces of the two segment-1 key chunks
  constexpr int KP1 = (NPK1 + 511) / 512;
  bf16* qs = reinterpret_cast<bf16*>(smem_raw);                               // [S16][64][8]
  bf16* k1s = qs + S16 * 512;                                                 // [2][S16][64][8]
  float* mw = reinterpret_cast<float*>(k1s + 2 * S16 * 512);                  // [8][32]
  float* lw = mw + ATT_WAVES * 32;                                            // [8][32]
  bf16* pf = reinterpret_cast<bf16*>(lw + ATT_WAVES * 32);                    // [ntot][2][64][8]

  const int t = cx.tid();
  const int lane = t & 63;
  const int w = t >> 6;
  const int lq = lane & 31;
  const int lh = lane >> 5;
  if (!Cx::kPersistent) {
    if (cx.by >= p.heads) {   // warm-up block; rank = linear block index (mod 8)
      if (cx.bz == 0) prefetch_role(p.pf, cx.bx + (int)gridDim.x * (cx.by - p.heads));
      return;
    }
  }
  // v_split > 1: the head dimension of the values (and of the output) is shared out over v_split blocks per
  // (query tile, head); each repeats phase 1 on all keys and runs phase 2 on its NVB / v_split slices only
  const int vs = p.v_split > 1 ? p.v_split : 1;
  const int tile = cx.bx / vs;
  const int vpart = cx.bx - tile * vs;
  const int nslice = NVB / vs;                 // value slices (waves of phase 2) of this block
  const int pv_groups = PVG ? ATT_WAVES / nslice : 1;   // G
  const int pv_g = PVG ? w / nslice : 0;                // this wave's group
  const int slice = vpart * nslice + (PVG ? w - pv_g * nslice : w);   // the slice this wave accumulates
  const int head = cx.by;
  const int row = tile * 32 + lq;
  const bool row_ok = row < p.Tq;

  int cbeg0 = 0, n0 = p.chunks0;
  if (p.view_tokens > 0) {
    const int view = (tile * 32) / p.view_tokens;
    cbeg0 = view * (p.view_tokens >> 5);
    n0 = p.view_tokens >> 5;
  }
  int n1 = p.chunks1;
  if (p.key_splits > 1) {   // this block's share of segment 0; the last share also takes segment 1
    cbeg0 = cx.bz * p.chunks_per_split;
    n0 = min(p.chunks_per_split, p.chunks0 - cbeg0);
    if (cx.bz != p.key_splits - 1) n1 = 0;
  }
  const bf16* kbase0 = p.k0 + ((size_t)head * p.kv_head_stride0 + (size_t)cbeg0 * S16 * 512) + lane * 8;
  const bf16* vbase0 = p.v0 + ((size_t)head * p.v_head_stride0 + (size_t)cbeg0 * NVB * 1024);
  const bf16* vslice0 = vbase0 + slice * 1024 + lane * 8;   // this wave's slice of the value fragments of segment 0

  // ---- issue every load of the first round (unconditional, clamped addresses) -----------------
  // Keys and values of segment 0 are constants of a persistent kernel (the prefix cache): requested before the
  // wait for this operation's inputs (Q and the second segment, which the QKV projection before produced).
  const bf16* qsrc = p.q + (size_t)head * p.q_head_stride + (size_t)tile * S16 * 512;
  bf16x8 qreg[QP];
  bf16x8 k1reg[KP1];
  bf16x8 kf[S16];
  bf16x8 vf[PVG ? CPW * 2 : VRING * 2];      // ring over the chunks of segment 0 (chunk groups: this wave's chunks)
  bf16x8 vs1[PVG ? 1 : 4];                   // the (at most two) chunks of segment 1 (chunk groups: they are in vf)
  const bool pv_wave = PVG ? true : w < nslice;
  auto load_seg0 = [&]() {
    const bf16* kp0 = kbase0 + (size_t)min(w, n0 - 1) * S16 * 512;
#pragma unroll
    for (int s = 0; s < S16; s++) kf[s] = *reinterpret_cast<const bf16x8*>(kp0 + (size_t)s * 512);
    if (PVG) {
#pragma unroll
      for (int j = 0; j < (PVG ? CPW : 0); j++) {   // chunks beyond segment 0: a valid address, replaced or unused later
        const bf16* vp = vslice0 + (size_t)min(pv_g + j * pv_groups, n0 - 1) * NVB * 1024;
        vf[2 * j] = *reinterpret_cast<const bf16x8*>(vp);
        vf[2 * j + 1] = *reinterpret_cast<const bf16x8*>(vp + 512);
      }
    } else if (pv_wave) {
#pragma unroll
      for (int c = 0; c < VRING; c++) {
        const bf16* vp = vslice0 + (size_t)min(c, n0 - 1) * NVB * 1024;
        vf[2 * c] = *reinterpret_cast<const bf16x8*>(vp);
        vf[2 * c + 1] = *reinterpret_cast<const bf16x8*>(vp + 512);
      }
    }
  };
  if (Cx::kPersistent) {
    load_seg0();
    cx.wait_inputs();
  }
#pragma unroll
  for (int i = 0; i < QP; i++) qreg[i] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(qsrc + (size_t)min(t + i * 512, NPQ - 1) * 8));
  if (n1 > 0) {
#pragma unroll
    for (int i = 0; i < KP1; i++)
      k1reg[i] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(p.k1 + (size_t)min(t + i * 512, n1 * S16 * 64 - 1) * 8));
    if (!PVG && pv_wave) {
#pragma unroll
      for (int c = 0; c < 2; c++) {
        const bf16* vp = p.v1 + (size_t)min(c, n1 - 1) * NVB * 1024 + slice * 1024 + lane * 8;
        vs1[2 * c] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(vp));
        vs1[2 * c + 1] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(vp + 512));
      }
    }
  }
  if (!Cx::kPersistent) load_seg0();
  if (PVG && n1 > 0) {   // this wave's chunks that fall into segment 1 (after load_seg0, whose placeholders they replace)
#pragma unroll
    for (int j = 0; j < (PVG ? CPW : 0); j++) {
      const int c = pv_g + j * pv_groups - n0;
      if (c >= 0 && c < n1) {
        const bf16* vp = p.v1 + (size_t)c * NVB * 1024 + slice * 1024 + lane * 8;
        vf[2 * j] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(vp));
        vf[2 * j + 1] = cx.ld_bulk(reinterpret_cast<const bf16x8*>(vp + 512));
      }
    }
  }
#pragma unroll
  for (int i = 0; i < QP; i++) {
    const int pc = t + i * 512;
    if (pc < NPQ) *reinterpret_cast<bf16x8*>(qs + (size_t)pc * 8) = qreg[i];
  }
  if (n1 > 0) {
#pragma unroll
    for (int i = 0; i < KP1; i++) {
      const int pc = t + i * 512;
      if (pc < NPK1) *reinterpret_cast<bf16x8*>(k1s + (size_t)pc * 8) = k1reg[i];
    }
  }
  __syncthreads();
  cx.mark(1);   // Q and the second segment's keys are in LDS

  // ---- phase 1: scores of this wave's chunks ------------------------------------------------
  float sv[MAXR][16];
  float sv1[16];
  float m_loc = NEG_BIG;
#pragma unroll
  for (int r = 0; r < MAXR; r++) {
    const int ci = w + ATT_WAVES * r;
    if (ci < n0) {
      const bool more = ci + ATT_WAVES < n0;
      const bf16* kn = kbase0 + (size_t)min(ci + ATT_WAVES, n0 - 1) * S16 * 512;
      f32x16 sacc, sacc1;      // two accumulators where registers allow: a dependent MFMA waits ~64 clocks
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[e] = 0.f, sacc1[e] = 0.f;
      // the Q fragments come from LDS in batches of QB reads issued together: a read that is only
      // issued when its MFMA is next costs a full LDS round trip per step
#pragma unroll
      for (int s0 = 0; s0 < S16; s0 += QB) {
        bf16x8 qb[QB];
#pragma unroll
        for (int j = 0; j < QB; j++) qb[j] = *reinterpret_cast<const bf16x8*>(qs + ((size_t)(s0 + j) * 64 + lane) * 8);
#pragma unroll
        for (int j = 0; j < QB; j++) {
          const int s = s0 + j;
          const bf16x8 a = kf[s];
          if (r + 1 < MAXR && more) kf[s] = *reinterpret_cast<const bf16x8*>(kn + (size_t)s * 512);
          if (DUAL && (s & 1)) sacc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb[j], sacc1, 0, 0, 0);
          else sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb[j], sacc, 0, 0, 0);
        }
      }
      if (DUAL) {
#pragma unroll
        for (int e = 0; e < 16; e++) sacc[e] += sacc1[e];
      }
#pragma unroll
      for (int e = 0; e < 16; e++) {
        const int key = (cbeg0 + ci) * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
        sv[r][e] = key < p.valid0 ? sacc[e] * p.scale : NEG_BIG;
        m_loc = fmaxf(m_loc, sv[r][e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; e++) sv[r][e] = NEG_BIG;
    }
  }
  const bool seg1_wave = w < n1;             // waves 0 and 1 score the second segment from LDS
  if (seg1_wave) {
    f32x16 sacc, sacc1;
#pragma unroll
    for (int e = 0; e < 16; e++) sacc[e] = 0.f, sacc1[e] = 0.f;
#pragma unroll
    for (int s0 = 0; s0 < S16; s0 += 4) {
      bf16x8 ka[4], qb[4];
#pragma unroll
      for (int j = 0; j < 4; j++) {
        if (s0 + j < S16) {
          ka[j] = *reinterpret_cast<const bf16x8*>(k1s + (((size_t)w * S16 + s0 + j) * 64 + lane) * 8);
          qb[j] = *reinterpret_cast<const bf16x8*>(qs + ((size_t)(s0 + j) * 64 + lane) * 8);
        }
      }
#pragma unroll
      for (int j = 0; j < 4; j++) {
        if (s0 + j < S16) {
          if (DUAL && (j & 1)) sacc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[j], qb[j], sacc1, 0, 0, 0);
          else sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[j], qb[j], sacc, 0, 0, 0);
        }
      }
    }
    if (DUAL) {
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[e] += sacc1[e];
    }
#pragma unroll
    for (int e = 0; e < 16; e++) {
      const int key = w * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
      const bool valid = p.suffix_mask ? (row == 0 ? key == 0 : true) : true;
      sv1[e] = valid ? sacc[e] * p.scale : NEG_BIG;
      m_loc = fmaxf(m_loc, sv1[e]);
    }
  }
  m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, 64));
  if (lh == 0) mw[w * 32 + lq] = m_loc;
  __syncthreads();
  cx.mark(2);   // scores done
  float m_all = NEG_BIG;
#pragma unroll
  for (int i = 0; i < ATT_WAVES; i++) m_all = fmaxf(m_all, mw[i * 32 + lq]);
  float l_loc = 0.f;
  auto emit = [&](const float* svals, int slot) {   // probabilities -> B-operand fragments in LDS
    float pr[16];
#pragma unroll
    for (int e = 0; e < 16; e++) {
      pr[e] = svals[e] > 0.5f * NEG_BIG ? __expf(svals[e] - m_all) : 0.f;   // masked keys: exactly 0
      l_loc += pr[e];
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      bf16x8 pb;
#pragma unroll
      for (int j = 0; j < 8; j++) pb[j] = (bf16)pr[8 * s2 + j];
      *reinterpret_cast<bf16x8*>(pf + ((size_t)(slot * 2 + s2) * 64 + lane) * 8) = pb;
    }
  };
#pragma unroll
  for (int r = 0; r < MAXR; r++) {
    const int ci = w + ATT_WAVES * r;
    if (ci < n0) emit(sv[r], ci);
  }
  if (seg1_wave) emit(sv1, n0 + w);
  l_loc += __shfl_xor(l_loc, 32, 64);
  if (lh == 0) lw[w * 32 + lq] = l_loc;
  __syncthreads();
  cx.mark(3);   // probabilities in LDS
  if (!pv_wave) return;

  // ---- phase 2: this wave's 32-wide slice of the head dimension over all chunks --------------
  f32x16 o, o1;
#pragma unroll
  for (int e = 0; e < 16; e++) o[e] = 0.f, o1[e] = 0.f;
  // Segment 0: one ring of VRING chunks per round: the probability fragments of the whole round are read
  // from LDS up front (clamped, unconditional), chunks beyond the end multiply zeros; the value
  // fragments of the next round are requested (whole round, one uniform branch) as the registers
  // of this round are consumed.  Then the chunks of segment 1, whose value fragments came with Q.
  const bf16x8 zero8v = {(bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f};
  if (PVG) {
    const int ntot = n0 + n1;
    bf16x8 bpg[PVG ? 2 * CPW : 1];   // the probability fragments of this wave's chunks, read together (clamped, unconditional)
#pragma unroll
    for (int j = 0; j < (PVG ? CPW : 0); j++) {
      const int c = min(pv_g + j * pv_groups, ntot - 1);
      bpg[2 * j] = *reinterpret_cast<const bf16x8*>(pf + ((size_t)(c * 2) * 64 + lane) * 8);
      bpg[2 * j + 1] = *reinterpret_cast<const bf16x8*>(pf + ((size_t)(c * 2 + 1) * 64 + lane) * 8);
    }
#pragma unroll
    for (int j = 0; j < (PVG ? CPW : 0); j++) {
      if (pv_g + j * pv_groups < ntot) {   // uniform per wave
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[2 * j], bpg[2 * j], o, 0, 0, 0);
        o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[2 * j + 1], bpg[2 * j + 1], o1, 0, 0, 0);
      }
    }
  } else {
    for (int c0 = 0; c0 < n0; c0 += VRING) {
      bf16x8 bp[2 * VRING];
  #pragma unroll
      for (int cc = 0; cc < VRING; cc++) {
        const int c = min(c0 + cc, n0 - 1);
  #pragma unroll
        for (int s2 = 0; s2 < 2; s2++)
          bp[2 * cc + s2] = *reinterpret_cast<const bf16x8*>(pf + ((size_t)(c * 2 + s2) * 64 + lane) * 8);
      }
      const bool more_round = c0 + VRING < n0;
  #pragma unroll
      for (int cc = 0; cc < VRING; cc++) {
        const bool live = c0 + cc < n0;
  #pragma unroll
        for (int s2 = 0; s2 < 2; s2++) {
          const bf16x8 a = vf[2 * cc + s2];
          if (more_round) vf[2 * cc + s2] = *reinterpret_cast<const bf16x8*>(vslice0 + (size_t)min(c0 + cc + VRING, n0 - 1) * NVB * 1024 + (size_t)s2 * 512);
          if (DUAL && s2) o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, live ? bp[2 * cc + s2] : zero8v, o1, 0, 0, 0);
          else o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, live ? bp[2 * cc + s2] : zero8v, o, 0, 0, 0);
        }
      }
    }
    if (n1 > 0) {
  #pragma unroll
      for (int cc = 0; cc < 2; cc++) {
        const bool live = cc < n1;
        const int c = n0 + min(cc, n1 - 1);
  #pragma unroll
        for (int s2 = 0; s2 < 2; s2++) {
          const bf16x8 bpv = *reinterpret_cast<const bf16x8*>(pf + ((size_t)(c * 2 + s2) * 64 + lane) * 8);
          if (DUAL && s2) o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vs1[2 * cc + s2], live ? bpv : zero8v, o1, 0, 0, 0);
          else o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vs1[2 * cc + s2], live ? bpv : zero8v, o, 0, 0, 0);
        }
      }
    }
  }
  if (DUAL) {
#pragma unroll
    for (int e = 0; e < 16; e++) o[e] += o1[e];
  }
  cx.mark(4);   // P V done
  float l_all = 0.f;
#pragma unroll
  for (int i = 0; i < ATT_WAVES; i++) l_all += lw[i * 32 + lq];
  const float inv = 1.0f / l_all;
  if (PVG && pv_groups > 1) {
    // the groups' partial outputs meet in LDS (over Q and the keys of segment 1, which phase 1 is done with):
    // [wave][4][64][4] floats; wave (slice, g) then finishes the pieces i = g, g + G, .. of its slice
    float* red = reinterpret_cast<float*>(smem_raw);
    static_assert(3 * S16 * 1024 >= ATT_WAVES * 4096 || !PVG, "partial outputs fit over Q and the keys of segment 1");
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const f32x4 v4 = {o[4 * i], o[4 * i + 1], o[4 * i + 2], o[4 * i + 3]};
      *reinterpret_cast<f32x4*>(red + (((size_t)w * 4 + i) * 64 + lane) * 4) = v4;
    }
    __syncthreads();
    const int sl = w - pv_g * nslice;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if ((i % pv_groups) == pv_g % 4 && pv_g < 4) {   // uniform per wave
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
        for (int gg = 0; gg < pv_groups; gg++) {
          const f32x4 v4 = *reinterpret_cast<const f32x4*>(red + (((size_t)(gg * nslice + sl) * 4 + i) * 64 + lane) * 4);
          sum[0] += v4[0]; sum[1] += v4[1]; sum[2] += v4[2]; sum[3] += v4[3];
        }
        o[4 * i] = sum[0]; o[4 * i + 1] = sum[1]; o[4 * i + 2] = sum[2]; o[4 * i + 3] = sum[3];
      }
    }
  }
  if (!row_ok) return;
  if (p.ml_out != nullptr && w == 0 && lh == 0 && vpart == 0) {   // (row maximum, sum) of this share, for the consumer's merge
    float* dst = p.ml_out + ((((size_t)cx.bz * p.heads + head) * ((p.Tq + 31) >> 5) * 32) + row) * 2;
    cx.st(reinterpret_cast<float2*>(dst), make_float2(m_all, l_all));
  }
  bf16* outp = p.out + (size_t)cx.bz * p.out_split_stride;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    if (PVG && pv_groups > 1 && !((i % pv_groups) == pv_g % 4 && pv_g < 4)) continue;   // another wave's piece
    const int d = slice * 32 + 8 * i + 4 * lh;
    if (d < p.head_dim) {
      const bf16x4 ob = {(bf16)(o[4 * i] * inv), (bf16)(o[4 * i + 1] * inv), (bf16)(o[4 * i + 2] * inv),
                         (bf16)(o[4 * i + 3] * inv)};
      const int col = head * p.head_dim + d;
      cx.st(reinterpret_cast<bf16x4*>(outp + ((size_t)(row >> 5) * (p.out_ld >> 4) + (col >> 4)) * 512 +
                                      (((col & 15) >> 3) * 32 + (row & 31)) * 8 + (col & 7)), ob);
    }
  }
}


template <int DQK>
static constexpr int attn_smem_bytes(int ntot) { return 3 * (DQK / 16) * 1024 + 2 * ATT_WAVES * 32 * 4 + ntot * 2048; }
