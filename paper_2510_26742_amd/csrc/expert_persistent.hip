// The action expert's whole denoise loop as ONE persistent kernel (Section 5.2 of the paper: software barriers
// in place of kernel boundaries, operands requested across the synchronisation points; Section 6.2 names the
// persistent megakernel as the way to take the expert's per-kernel overhead out).
//
// 256 blocks of 8 waves, one per compute unit, walk the operation list of Table 2's action-expert rows - state
// token; per Euler step the folded action/time embedding and its second linear layer; per layer QKV + RoPE,
// attention over [prefix cache ; own keys], O projection + residual, gate||up GeGLU, down + residual; final norm,
// output projection and the Euler update - with one grid barrier between consecutive operations.  Every operation
// is the same body that the per-operation launches run (gemm_common.h, attention_body.h, embed_bodies.h), cut
// into the same work items, so the results agree with that path bit for bit; a block takes the work items
// block index, block index + 256, ... of each operation and then arrives at the barrier.
// What the persistent form buys: a body requests its weights (constant during the kernel, ordinary loads) and
// the other constants BEFORE it waits for the operation before to complete everywhere, so the weights' trip
// from HBM overlaps the barrier; and there is no dispatch, no cold instruction / argument fetch, no end-of-kernel
// cache write-back per operation.  What it costs: data that crosses blocks must be written through to memory
// and read past the per-die L2 (exec_ctx.h), and a barrier costs two dependent atomics plus a poll.
#include "attention_body.h"
#include "expert_loop.h"

namespace {

constexpr int PK_THREADS = 512;

// Reading ahead inside the loop.  The expert's weights (623 MB) cycle through the 256 MB memory-side cache once per Euler
// step, so an operation's weight request - issued when the operation before ends - goes all the way to HBM (the same loop
// run on one layer's weights throughout, i.e. from that cache, is 0.46 ms faster).  The attention has 64 items for 256
// blocks: the blocks without one use the time to read the weights that the following operations will ask for, which puts
// them into the memory-side cache.  Part `part` of `nparts` of [base, base + bytes): 16 bytes per lane, 8 loads in flight
// (4 finish too late, 16 disturb the working blocks' loads more than they gain: same-box A/B 5.47 / 5.42 / 5.48 ms);
// the values are folded into a word that is stored only if it equals a constant, so no result depends on them.
__device__ __forceinline__ unsigned read_ahead_part(const void* base, size_t bytes, int part, int nparts, int tid, unsigned fold) {
  const size_t n16 = bytes >> 4;
  const size_t per = (n16 + (size_t)nparts - 1) / (size_t)nparts;
  const size_t beg = (size_t)part * per;
  const size_t end = beg + per < n16 ? beg + per : n16;
  const u32x4_t* p = reinterpret_cast<const u32x4_t*>(base);
  for (size_t i = beg + (size_t)tid; i < end; i += 8 * PK_THREADS) {
    u32x4_t v[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const size_t idx = i + (size_t)j * PK_THREADS;
      v[j] = p[idx < end ? idx : end - 1];   // clamped, unconditional
    }
#pragma unroll
    for (int j = 0; j < 8; j++) fold ^= v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
  }
  return fold;
}

template <class F>
__device__ __forceinline__ void for_items(int n_items, F&& f) {
  bool first = true;
  for (int it = (int)blockIdx.x; it < n_items; it += (int)gridDim.x) {
    if (!first) __syncthreads();   // shared memory of the item before is free
    f(it);
    first = false;
  }
}

// The parameter block lives in device memory and every operation reads its own part afresh: taken by value, the
// operations' pointers and sizes stay live across the whole loop and the kernel spills hundreds of registers.
__device__ __forceinline__ const ExpertLoopParams& fresh(const ExpertLoopParams* p) {
  asm volatile("" : "+s"(p));   // nothing read through the pointer before this point is reused after it
  return *p;
}

__global__ void expert_loop_params_kernel(ExpertLoopParams P, ExpertLoopParams* dst) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *dst = P;
}

__global__ __launch_bounds__(PK_THREADS) void expert_loop_kernel(const ExpertLoopParams* __restrict__ Pg) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  GridBarrier bar;
  const ExpertLoopParams& P = *Pg;
  bar.init(P.sync, P.spin_limit);
  PersistCtx cx;
  cx.arena = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(P.arena), 0, (int)P.arena_bytes, 0x00020000);
  cx.arena_base = P.arena;
  cx.bar = &bar;
  cx.bx = cx.by = cx.bz = 0;
  cx.thread = (int)threadIdx.x;
  long long* const trace = P.trace;
  const int trace_ops = P.trace_ops;
  int opi = 0;
  // timeline, 8 samples per (operation, block): 0 at the start of an operation, 1 by the barrier when the wait ends,
  // 2 after the body, 3 after arrive, 4 .. 7 by the body itself (cx.mark)
  auto op_begin = [&]() {
    if (trace != nullptr && opi < trace_ops) {
      long long* slot = trace + ((size_t)opi * gridDim.x + blockIdx.x) * 8;
      bar.trace = slot + 1;
      if (threadIdx.x == 0) { slot[0] = (long long)wall_clock64(); slot[1] = slot[4] = slot[5] = slot[6] = slot[7] = 0; }
    } else {
      bar.trace = nullptr;
    }
  };
  auto op_end = [&]() {
    long long* slot = trace != nullptr && opi < trace_ops ? trace + ((size_t)opi * gridDim.x + blockIdx.x) * 8 : nullptr;
    if (slot != nullptr && threadIdx.x == 0) slot[2] = (long long)wall_clock64();
    bar.trace = nullptr;
    bar.arrive();
    if (slot != nullptr && threadIdx.x == 0) slot[3] = (long long)wall_clock64();
    opi++;
  };
  auto item = [&](int bx, int by, int bz) {
    PersistCtx c = cx;
    c.bx = bx; c.by = by; c.bz = bz;
    int t = (int)threadIdx.x;
    asm volatile("" : "+v"(t));
    c.thread = t;
    return c;
  };

  op_begin();
  // ---- C0: state token; x <- noise ---------------------------------------------------------------
  for_items((P.stok.X + 255) / 256, [&](int it) { state_token_body(P.stok, item(it, 0, 0)); });
  if ((int)blockIdx.x == (int)gridDim.x - 1) {
    for (int i = threadIdx.x; i < P.x_elems; i += PK_THREADS) cx.st(P.emb.x_rw + i, P.noise[i]);
  }
  op_end();

  const int emb_cols = (P.emb.a.X + 255) / 256;
  const int steps = P.steps, layers = P.layers;
  for (int k = 0; k < steps; k++) {
    op_begin();
    {  // ---- C1: folded action/time embedding + SiLU; suffix row 0 <- state token ----------------
      ActionEmbedArgs a = fresh(Pg).emb.a;
      a.bias_k += (size_t)k * a.X;
      bool waited = false;
      for_items(emb_cols * (a.chunk + 1), [&](int it) {
        if (!waited) { bar.wait(); waited = true; }
        action_embed_body(a, item(it % emb_cols, it / emb_cols, 0));
      });
      op_end();
    }
    op_begin();
    // ---- C2: second linear of the action/time MLP -> suffix rows 1 .. chunk --------------------------
    {
      const GemmParams t = fresh(Pg).tout;
      for_items(t.n_tiles * 2, [&](int it) { gemm_skinny_body<PRO_NONE, EPI_RESID, 1>(t, item(it % t.n_tiles, 0, it / t.n_tiles), smem_raw); });
    }
    op_end();
    for (int l = 0; l < layers; l++) {
      op_begin();
      {  // ---- C3: RMS -> QKV, RoPE at positions P .. P + 63 -------------------------------------
        const ExpertLoopParams& F = fresh(Pg);
        GemmParams q = F.qkv;
        q.W.w += (size_t)l * F.w_stride;
        char* slot = F.ring + (size_t)(k * layers + l) * F.ring_stride;
        q.out_bf16 = reinterpret_cast<bf16*>(slot + F.r_q);
        q.kfrag = reinterpret_cast<bf16*>(slot + F.r_k);
        q.vfrag = reinterpret_cast<bf16*>(slot + F.r_v);
        if (l == 0) {   // input: the step's embedding (two operations wrote its rows)
          q.rowstat_parts = F.parts_first;
          for_items(q.n_tiles * 2, [&](int it) { gemm_skinny_body<PRO_RMS, EPI_QKV, 1>(q, item(it % q.n_tiles, 0, it / q.n_tiles), smem_raw); });
        } else {
          q.rowstat_parts = F.parts_rest;
          q.X = reinterpret_cast<const bf16*>(slot - F.ring_stride + F.r_yb_d);
          q.rowstat = reinterpret_cast<const float*>(slot - F.ring_stride + F.r_st_d);
          for_items(q.n_tiles * 2, [&](int it) {
            gemm_skinny_body<PRO_RMS, EPI_QKV, 1>(q, item(it % q.n_tiles, 0, it / q.n_tiles).template as<true>(), smem_raw);
          });
        }
        if ((int)blockIdx.x >= q.n_tiles * 2 && (F.read_ahead & 48)) {   // no item: what the attention and O of this layer read
          const int tid = item(0, 0, 0).thread;
          const int part = (int)blockIdx.x - q.n_tiles * 2, nparts = (int)gridDim.x - q.n_tiles * 2;
          unsigned fold = 0;
          if (F.read_ahead & 32) {   // this layer's slices of the prefix cache
            const size_t cache_bytes = (size_t)F.att.chunks0 * 32 * 256 * 2;
            fold = read_ahead_part(F.att.k0 + (size_t)l * F.kcache_stride, cache_bytes, part, nparts, tid, fold);
            fold = read_ahead_part(F.att.v0 + (size_t)l * F.vcache_stride, cache_bytes, part, nparts, tid, fold);
          }
          if (F.read_ahead & 16) fold = read_ahead_part(F.o.W.w + (size_t)l * F.w_stride, (size_t)F.o.n_tiles * 64 * F.o.W.k_pad, part, nparts, tid, fold);
          if (fold == 0x9e3779b9u) F.sync[GB_SINK] = fold;
        }
        op_end();
      }
      op_begin();
      {  // ---- C4 + C5: scores, block mask, softmax, PV over [cache ; own keys] ---------------------
        const ExpertLoopParams& F = fresh(Pg);
        AttnParams a = F.att;
        a.k0 += (size_t)l * F.kcache_stride;
        a.v0 += (size_t)l * F.vcache_stride;
        char* slot = F.ring + (size_t)(k * layers + l) * F.ring_stride;
        a.q = reinterpret_cast<const bf16*>(slot + F.r_q);
        a.k1 = reinterpret_cast<const bf16*>(slot + F.r_k);
        a.v1 = reinterpret_cast<const bf16*>(slot + F.r_v);
        a.out = reinterpret_cast<bf16*>(slot + F.r_attn);
        if (a.ml_out != nullptr) a.ml_out = reinterpret_cast<float*>(slot + F.r_ml);
        const int att_gx = F.att_gx, att_gxy = F.att_gx * a.heads;
        for_items(F.att_items, [&](int it) {
          attention_body<256, 8, 1, 6, 5>(a, item(it % att_gx, (it % att_gxy) / att_gx, it / att_gxy).template as<true>(), smem_raw);
        });
        if ((int)blockIdx.x >= F.att_items && F.read_ahead != 0) {   // no item: read ahead (constants only, no wait needed)
          const int part = (int)blockIdx.x - F.att_items, nparts = (int)gridDim.x - F.att_items;
          const int ln = l + 1 < layers ? l + 1 : 0;
          const int tid = item(0, 0, 0).thread;
          unsigned fold = 0;
          if (F.read_ahead & 1) fold = read_ahead_part(F.gu.W.w + (size_t)l * F.w_stride, (size_t)F.gu.n_tiles * 64 * F.gu.W.k_pad, part, nparts, tid, fold);
          if (F.read_ahead & 2) fold = read_ahead_part(F.dn.W.w + (size_t)l * F.w_stride, (size_t)F.dn.n_tiles * 64 * F.dn.W.k_pad, part, nparts, tid, fold);
          if (F.read_ahead & 4) fold = read_ahead_part(F.qkv.W.w + (size_t)ln * F.w_stride, (size_t)F.qkv.n_tiles * 64 * F.qkv.W.k_pad, part, nparts, tid, fold);
          if (F.read_ahead & 8) fold = read_ahead_part(F.o.W.w + (size_t)ln * F.w_stride, (size_t)F.o.n_tiles * 64 * F.o.W.k_pad, part, nparts, tid, fold);
          if (fold == 0x9e3779b9u) F.sync[GB_SINK] = fold;
        }
        op_end();
      }
      op_begin();
      {  // ---- C6: O projection + residual ------------------------------------------------------
        const ExpertLoopParams& F = fresh(Pg);
        GemmParams o = F.o;
        o.W.w += (size_t)l * F.w_stride;
        o.gain = F.g_mlp0 + (size_t)l * F.gain_stride;
        char* slot = F.ring + (size_t)(k * layers + l) * F.ring_stride;
        o.X = reinterpret_cast<const bf16*>(slot + F.r_attn);
        if (o.xsplits > 1) o.xsplit_ml = reinterpret_cast<const float*>(slot + F.r_ml);
        o.out_bf16 = reinterpret_cast<bf16*>(slot + F.r_yb_o);
        o.stat_out = reinterpret_cast<float*>(slot + F.r_st_o);
        const int nx = o.n_tiles * 2;
        for_items(nx * F.m16, [&](int it) { gemm_skinny16_body<8>(o, item(it % nx, it / nx, 0).template as<true>(), smem_raw); });
        op_end();
      }
      op_begin();
      {  // ---- C7: RMS -> gate||up, fused gate -----------------------------------------------------
        const ExpertLoopParams& F = fresh(Pg);
        GemmParams g = F.gu;
        g.W.w += (size_t)l * F.w_stride;
        char* slot = F.ring + (size_t)(k * layers + l) * F.ring_stride;
        g.X = reinterpret_cast<const bf16*>(slot + F.r_yb_o);
        g.rowstat = reinterpret_cast<const float*>(slot + F.r_st_o);
        g.out_bf16 = reinterpret_cast<bf16*>(slot + F.r_mid);
        // two feature tiles x one token block per item: the same sums as one tile x both token blocks, half the
        // activation bytes per block behind the wait
        const int pairs = g.n_tiles / 2;
        for_items(pairs * 2, [&](int it) { gemm_skinny_body<PRO_RMS, EPI_GEGLU, 2>(g, item(it % pairs, 0, it / pairs).template as<true>(), smem_raw); });
        op_end();
      }
      op_begin();
      {  // ---- C8: down + residual -----------------------------------------------------------------
        const ExpertLoopParams& F = fresh(Pg);
        GemmParams d = F.dn;
        d.W.w += (size_t)l * F.w_stride;
        d.gain = l + 1 < F.layers ? F.g_attn0 + (size_t)(l + 1) * F.gain_stride : F.g_final;
        char* slot = F.ring + (size_t)(k * layers + l) * F.ring_stride;
        d.X = reinterpret_cast<const bf16*>(slot + F.r_mid);
        d.out_bf16 = reinterpret_cast<bf16*>(slot + F.r_yb_d);
        d.stat_out = reinterpret_cast<float*>(slot + F.r_st_d);
        const int nx = d.n_tiles * 2;
        if (F.dn_ns == 16) for_items(nx * F.m16, [&](int it) { gemm_skinny16_body<16>(d, item(it % nx, it / nx, 0).template as<true>(), smem_raw); });
        else for_items(nx * F.m16, [&](int it) { gemm_skinny16_body<8>(d, item(it % nx, it / nx, 0).template as<true>(), smem_raw); });
        op_end();
      }
    }
    op_begin();
    // ---- C9: final RMS -> out-projection (+bias), Euler update x <- x + dt * v ----------------------
    {
      const ExpertLoopParams& F = fresh(Pg);
      GemmParams u = F.outp;
      char* slot = F.ring + (size_t)(k * layers + layers - 1) * F.ring_stride;
      u.X = reinterpret_cast<const bf16*>(slot + F.r_yb_d);
      u.rowstat = reinterpret_cast<const float*>(slot + F.r_st_d);
      // one item per (feature tile, token block): half the activation bytes per block
      for_items(u.n_tiles * 2, [&](int it) { gemm_skinny_body<PRO_RMS, EPI_EULER, 1>(u, item(it % u.n_tiles, 0, it / u.n_tiles).template as<true>(), smem_raw); });
    }
    op_end();
  }
}

}  // namespace

int expert_loop_smem_bytes() {
  const int sk = (SK_WAVES * 2 * 16 * 64 + 128 + SK_WAVES * 128) * 4;
  const int at = attn_smem_bytes<256>(8 + 2);
  return sk > at ? sk : at;
}

hipError_t expert_loop_init_attributes() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&expert_loop_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             expert_loop_smem_bytes());
}

hipError_t expert_loop_max_blocks_per_cu(int* out) {
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(out, reinterpret_cast<const void*>(&expert_loop_kernel), PK_THREADS,
                                                      expert_loop_smem_bytes());
}

// Host-side checks of everything the kernel's indexing assumes; the caller has zeroed the barrier words.
hipError_t launch_expert_loop(hipStream_t s, const ExpertLoopParams& P, ExpertLoopParams* d_params, int blocks) {
  if (d_params == nullptr || (reinterpret_cast<uintptr_t>(d_params) & 15) != 0) return hipErrorInvalidValue;
  if (blocks < 1 || blocks > 1024 || P.sync == nullptr || P.arena == nullptr || P.arena_bytes == 0 || P.spin_limit == 0)
    return hipErrorInvalidValue;
  if (P.layers < 1 || P.steps < 1 || P.x_elems < 1 || P.noise == nullptr || P.emb.x_rw == nullptr)
    return hipErrorInvalidValue;
  // every buffer that blocks exchange lies inside the arena (offsets are 32-bit)
  auto in_arena = [&](const void* p, size_t bytes) {
    const char* c = reinterpret_cast<const char*>(p);
    return p != nullptr && c >= P.arena && c + bytes <= P.arena + P.arena_bytes;
  };
  const GemmParams* gs[6] = {&P.qkv, &P.o, &P.gu, &P.dn, &P.tout, &P.outp};
  for (const GemmParams* g : gs) {
    if (g->X == nullptr || g->W.w == nullptr || g->M < 1 || g->M > 64 || g->W.k_pad % 64 != 0 || g->n_tiles * 32 != g->W.n_pad)
      return hipErrorInvalidValue;
    if (g->ldx < g->W.k_pad || g->ldx % 16 != 0 || !in_arena(g->X, (size_t)64 * g->ldx * 2)) return hipErrorInvalidValue;
    if (g->pf.blocks != 0 || g->progress != nullptr) return hipErrorInvalidValue;
  }
  const GemmParams* sk[4] = {&P.qkv, &P.gu, &P.tout, &P.outp};   // 32-feature tiles, k <= 1024 split over 8 waves
  for (const GemmParams* g : sk) {
    if (g->k_per_split != g->W.k_pad || g->W.k_pad > SK_KMAX || g->m_tiles != 1) return hipErrorInvalidValue;
  }
  if (P.read_ahead < 0 || P.read_ahead > 63) return hipErrorInvalidValue;
  if (P.gu.n_tiles % 2 != 0 || P.gu.M <= 32) return hipErrorInvalidValue;   // gate||up: pairs of feature tiles, two token blocks
  if (P.qkv.rowstat == nullptr || P.gu.rowstat == nullptr || P.outp.rowstat == nullptr) return hipErrorInvalidValue;
  if (P.parts_first < 1 || P.parts_first > 8 * SK_WAVES || P.parts_rest < 1 || P.parts_rest > 8 * SK_WAVES) return hipErrorInvalidValue;
  if (P.gu.rowstat_parts < 1 || P.gu.rowstat_parts > 8 * SK_WAVES || P.outp.rowstat_parts < 1 || P.outp.rowstat_parts > 8 * SK_WAVES)
    return hipErrorInvalidValue;
  if (!in_arena(P.qkv.rowstat, (size_t)8 * SK_WAVES * 64 * 8)) return hipErrorInvalidValue;
  if (P.qkv.rope == nullptr || P.qkv.out_bf16 == nullptr || P.qkv.kfrag == nullptr || P.qkv.vfrag == nullptr) return hipErrorInvalidValue;
  const GemmParams* s16[2] = {&P.o, &P.dn};   // 16 x 16 tiles over the whole k range
  for (const GemmParams* g : s16) {
    const int kc16 = g->W.k_pad >> 4;
    if ((kc16 != 128 && kc16 != 256) || g->out_f32 == nullptr || g->out_bf16 == nullptr || g->resid == nullptr || g->ldo % 4 != 0 ||
        g->ldo2 % 16 != 0 || g->stat_out == nullptr)
      return hipErrorInvalidValue;
  }
  if ((P.o.W.k_pad >> 4) != 128 || P.dn_ns != ((P.dn.W.k_pad >> 4) == 256 ? 16 : 8) || P.m16 != (P.o.M + 15) / 16) return hipErrorInvalidValue;
  if (P.o.xsplits > 1 && (P.o.xsplits > 4 || P.o.xsplit_ml == nullptr || P.o.xsplit_stride < (size_t)64 * P.o.ldx)) return hipErrorInvalidValue;
  // attention: head dim 256, at most 8 prefix chunks per share, the suffix's own 2 chunks as second segment
  const AttnParams& a = P.att;
  if (a.q == nullptr || a.k0 == nullptr || a.v0 == nullptr || a.k1 == nullptr || a.v1 == nullptr || a.out == nullptr) return hipErrorInvalidValue;
  if (a.head_dim != 256 || a.Tq != 64 || a.chunks1 != 2 || a.heads < 1 || a.chunks0 < 1 || a.valid0 < 1 || a.valid0 > a.chunks0 * 32)
    return hipErrorInvalidValue;
  const int shares = a.key_splits > 1 ? a.key_splits : 1;
  const int n0 = shares > 1 ? a.chunks_per_split : a.chunks0;
  if (n0 < 1 || n0 > 8 || shares > 4 || (shares > 1 && (a.ml_out == nullptr || (shares - 1) * a.chunks_per_split >= a.chunks0 ||
                                                        shares * a.chunks_per_split < a.chunks0)))
    return hipErrorInvalidValue;
  const int vs = a.v_split > 1 ? a.v_split : 1;
  // value slices in groups of waves: at most 5 chunks of [segment 0 ; segment 1] per wave
  if (vs != 2 && vs != 4 && vs != 8) return hipErrorInvalidValue;
  if ((n0 + 2 + vs - 1) / vs > 5) return hipErrorInvalidValue;
  if (P.att_gx != 2 * vs || P.att_items != 2 * vs * a.heads * shares || a.pf.blocks != 0) return hipErrorInvalidValue;
  if (!in_arena(a.q, 2) || !in_arena(a.k1, 2) || !in_arena(a.v1, 2) || !in_arena(a.out, 2)) return hipErrorInvalidValue;
  if (P.emb.a.X % 32 != 0 || P.emb.a.gain == nullptr || P.emb.a.stat_parts == nullptr || P.emb.a.x != P.emb.x_rw) return hipErrorInvalidValue;
  if (!in_arena(P.emb.x_rw, (size_t)P.x_elems * 4) || !in_arena(P.stok.out, (size_t)P.stok.X * 4)) return hipErrorInvalidValue;
  if (P.stok.sd < 1 || P.stok.sd > 32) return hipErrorInvalidValue;
  if (P.ring == nullptr || P.ring_stride % 256 != 0 || !in_arena(P.ring, P.ring_stride * (size_t)P.layers * P.steps)) return hipErrorInvalidValue;
  if (P.r_mid >= P.ring_stride || P.r_attn >= P.ring_stride) return hipErrorInvalidValue;
  hipLaunchKernelGGL(expert_loop_params_kernel, dim3(1), dim3(64), 0, s, P, d_params);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(expert_loop_kernel, dim3(blocks), dim3(PK_THREADS), expert_loop_smem_bytes(), s, d_params);
  return hipGetLastError();
}
