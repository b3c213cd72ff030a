// Host side of the pi0 library: geometry checks, workspace layout, load-time packing, the kernel
// sequence of one inference (Table 2 of the paper, top to bottom) and its HIP-graph capture/replay
// (Section 3.1: record the kernel stream once, replay it with constant kernels and pointers).
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <new>
#include <vector>

#include "expert_loop.h"
#include "pi0_internal.h"

namespace {

struct Dims {
  int T, PD, PDp, Dv, Hv, hdv, Fv, Fv_np, Fv_kp;
  int E, H, F, X, Fx;
  int S, A, SD, steps;
  int maxI, maxP, maxPc, maxpos;
  int Lv, Ll, Le;
};

bool derive_dims(const pi0_config& c, Dims& d) {
  if (c.vis_layers < 1 || c.llm_layers < 2 || c.exp_layers != c.llm_layers) return false;
  if (c.patch < 1 || c.img_size < c.patch || c.img_size % c.patch != 0) return false;
  d.T = (c.img_size / c.patch) * (c.img_size / c.patch);
  if (d.T % 32 != 0 || d.T > 256) return false;   // vision attention: one view's keys in one round of 8 chunks
  d.PD = c.patch * c.patch * 3;
  d.PDp = round_up(d.PD, 64);
  d.Dv = c.vis_width;
  d.Hv = c.vis_heads;
  if (d.Dv < 64 || d.Dv % 64 != 0 || d.Hv < 1 || d.Dv % d.Hv != 0) return false;
  d.hdv = d.Dv / d.Hv;
  if (d.hdv % 4 != 0 || d.hdv <= 64 || d.hdv > 80) return false;
  d.Fv = c.vis_mlp;
  if (d.Fv < 32 || d.Fv % 4 != 0) return false;
  d.Fv_np = round_up(d.Fv, 32);
  d.Fv_kp = round_up(d.Fv, 64);
  d.E = c.llm_width;
  d.H = c.llm_q_heads;
  d.F = c.llm_mlp;
  d.X = c.exp_width;
  d.Fx = c.exp_mlp;
  if (c.head_dim != 256 || d.H < 1 || d.H > 64) return false;
  if (d.E < 64 || d.E % 64 != 0 || d.F < 64 || d.F % 64 != 0) return false;
  if (d.X < 64 || d.X % 64 != 0 || d.Fx < 64 || d.Fx % 64 != 0) return false;
  if (c.chunk + 1 != 64) return false;
  d.S = 64;
  d.A = c.action_dim;
  d.SD = c.state_dim;
  if (d.A < 1 || d.A > 32 || d.SD < 1 || d.SD > 32) return false;
  d.steps = c.steps;
  if (d.steps < 1 || d.steps > 1000) return false;
  if (c.max_views < 1 || c.max_views > 8 || c.max_prompt < 0 || c.max_prompt > 4096) return false;
  if (c.vocab < 0) return false;
  d.maxI = c.max_views * d.T;
  d.maxP = d.maxI + c.max_prompt;
  if (d.maxP > 1024) return false;   // prefix / expert attention: at most 32 key chunks per query row
  d.maxPc = ceil_div(d.maxP, 32);
  d.maxpos = d.maxPc * 32 + d.S;
  d.Lv = c.vis_layers;
  d.Ll = c.llm_layers;
  d.Le = c.exp_layers;
  return true;
}

// ---- canonical blob layout (element offsets), in the order documented in pi0.h -------------------
struct BlobVis { size_t ln1g, ln1b, wq, bq, wk, bk, wv, bv, wo, bo, ln2g, ln2b, w1, b1, w2, b2; };
struct BlobTr { size_t g_attn, wq, wk, wv, wo, g_mlp, wg, wu, wd; };
struct BlobLayout {
  size_t patch_w, patch_b, pos;
  std::vector<BlobVis> vis;
  size_t lnfg, lnfb, proj_w, proj_b;
  size_t embed;
  std::vector<BlobTr> llm, exp;
  size_t state_w, state_b, ain_w, ain_b, tin_w, tin_b, tout_w, tout_b, g_final, out_w, out_b;
  size_t total;
};

struct Cursor {
  size_t off = 0;
  size_t take(size_t n) {
    size_t o = off;
    off += round_up_sz(n, 128);
    return o;
  }
};

void blob_layout(const pi0_config& c, const Dims& d, BlobLayout& b) {
  Cursor cur;
  b.patch_w = cur.take((size_t)d.PD * d.Dv);
  b.patch_b = cur.take(d.Dv);
  b.pos = cur.take((size_t)d.T * d.Dv);
  b.vis.resize(d.Lv);
  for (int l = 0; l < d.Lv; l++) {
    BlobVis& v = b.vis[l];
    v.ln1g = cur.take(d.Dv); v.ln1b = cur.take(d.Dv);
    v.wq = cur.take((size_t)d.Dv * d.Dv); v.bq = cur.take(d.Dv);
    v.wk = cur.take((size_t)d.Dv * d.Dv); v.bk = cur.take(d.Dv);
    v.wv = cur.take((size_t)d.Dv * d.Dv); v.bv = cur.take(d.Dv);
    v.wo = cur.take((size_t)d.Dv * d.Dv); v.bo = cur.take(d.Dv);
    v.ln2g = cur.take(d.Dv); v.ln2b = cur.take(d.Dv);
    v.w1 = cur.take((size_t)d.Dv * d.Fv); v.b1 = cur.take(d.Fv);
    v.w2 = cur.take((size_t)d.Fv * d.Dv); v.b2 = cur.take(d.Dv);
  }
  b.lnfg = cur.take(d.Dv); b.lnfb = cur.take(d.Dv);
  b.proj_w = cur.take((size_t)d.Dv * d.E); b.proj_b = cur.take(d.E);
  b.embed = 0;
  if (c.vocab > 0) b.embed = cur.take((size_t)c.vocab * d.E);
  auto tr = [&](std::vector<BlobTr>& v, int L, int W, int M) {
    v.resize(L);
    for (int l = 0; l < L; l++) {
      BlobTr& t = v[l];
      t.g_attn = cur.take(W);
      t.wq = cur.take((size_t)W * d.H * 256); t.wk = cur.take((size_t)W * 256); t.wv = cur.take((size_t)W * 256);
      t.wo = cur.take((size_t)d.H * 256 * W);
      t.g_mlp = cur.take(W);
      t.wg = cur.take((size_t)W * M); t.wu = cur.take((size_t)W * M); t.wd = cur.take((size_t)M * W);
    }
  };
  tr(b.llm, d.Ll, d.E, d.F);
  tr(b.exp, d.Le, d.X, d.Fx);
  b.state_w = cur.take((size_t)d.SD * d.X); b.state_b = cur.take(d.X);
  b.ain_w = cur.take((size_t)d.A * d.X); b.ain_b = cur.take(d.X);
  b.tin_w = cur.take((size_t)2 * d.X * d.X); b.tin_b = cur.take(d.X);
  b.tout_w = cur.take((size_t)d.X * d.X); b.tout_b = cur.take(d.X);
  b.g_final = cur.take(d.X);
  b.out_w = cur.take((size_t)d.X * d.A); b.out_b = cur.take(d.A);
  b.total = cur.off;
}

// ---- workspace layout (byte offsets) ----------------------------------------------------------------
struct PW { size_t w; int n_pad, k_pad; size_t colsum, bias; };   // packed weight + optional vectors
struct WsVis { PW qkv, o, up, down; };
struct WsTr { PW qkv, o, gu, down; size_t gu8 = 0, gu8s = 0, down8 = 0, down8s = 0; };   // *8 / *8s: MXFP8 copy and its scales (prefix only)
struct WsLayout {
  PW patch; size_t pos;
  std::vector<WsVis> vis;
  PW proj;
  size_t embed;
  std::vector<WsTr> llm, exp;
  size_t state_w, state_b, wfold, bias_tab, tau;
  PW tout, outp;
  size_t rope;
  std::vector<size_t> g_v1, g_v2, g_l1, g_l2, g_e1, g_e2;   // fp32 gain vectors of the norms (g or 1 + g)
  size_t g_vf, g_ef;
  size_t act_begin;   // everything from here on is zero-filled at load time
  size_t st_images, st_ids, st_state, st_noise, xa;
  size_t xpatch, vh, vh_b, vq, vk, vv, vattn, vmid, part;
  size_t lx, lx_b, lq, kcache, vcache, lattn, lmid;
  size_t stok, z, y, y_b, eq, ek, ev, eattn, eml, emid;
  size_t vstat, lstat, estat, estat_parts, pf_sink, vstat_parts, lstat_parts, progress;
  size_t es_begin, es_end;           // the expert's scratch block [es_begin, es_end)
  size_t esync, eparams;             // persistent denoise kernel: barrier words, parameter block
  size_t ering, ering_slot;          // ... its ring of per-layer-step activation buffers, bytes per slot
  unsigned r_yb_o, r_st_o, r_yb_d, r_st_d, r_q, r_k, r_v, r_attn, r_ml, r_mid;   // byte offsets inside a slot
  size_t lx8, lx8s, lmid8, lmid8s;   // MXFP8 copies of the prefix feed-forward inputs
  bool mx_ok = false;                // the prefix feed-forward shapes fit the MXFP8 kernels (multiples of 256)
  size_t total;
  size_t kcache_layer, vcache_layer;   // bytes per layer
  size_t kcache_slot, vcache_slot;     // bytes per cache copy (two copies: double buffering for pi0_stream_frame)
  size_t epart;                        // split-K partial sums of the expert (separate from the prefix's)
  int zmax;
};

struct WsCursor {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off += round_up_sz(bytes, 256);
    return o;
  }
};

const int SK_KMAX_HOST = 1024;   // widest contraction of the expert's 32-feature skinny kernels
const int PK_BLOCKS = 256;   // blocks of the persistent denoise kernel
const int Z_MAX = 32;   // upper bound on split-K slices (sizes the partial-sum buffer)

void ws_layout(const pi0_config& c, const Dims& d, WsLayout& w) {
  WsCursor cur;
  auto pw = [&](int n_true, int k_true, bool colsum, bool bias) {
    PW p;
    p.n_pad = round_up(n_true, 32);
    p.k_pad = round_up(k_true, 64);
    p.w = cur.take((size_t)p.n_pad * p.k_pad * 2);
    p.colsum = colsum ? cur.take((size_t)p.n_pad * 4) : 0;
    p.bias = bias ? cur.take((size_t)p.n_pad * 4) : 0;
    return p;
  };
  w.patch = pw(d.Dv, d.PD, false, true);
  w.pos = cur.take((size_t)d.T * d.Dv * 4);
  w.vis.resize(d.Lv);
  for (int l = 0; l < d.Lv; l++) {
    w.vis[l].qkv = pw(3 * d.Dv, d.Dv, true, true);
    w.vis[l].o = pw(d.Dv, d.Dv, false, true);
    w.vis[l].up = pw(d.Fv, d.Dv, true, true);
    w.vis[l].down = pw(d.Dv, d.Fv, false, true);
  }
  w.proj = pw(d.E, d.Dv, true, true);
  w.embed = c.vocab > 0 ? cur.take((size_t)c.vocab * d.E * 2) : 0;
  w.llm.resize(d.Ll);
  for (int l = 0; l < d.Ll; l++) {
    const bool last = l == d.Ll - 1;
    w.llm[l].qkv = pw(last ? 512 : (d.H + 2) * 256, d.E, false, false);
    if (!last) {
      w.llm[l].o = pw(d.E, d.H * 256, false, false);
      w.llm[l].gu = pw(2 * d.F, d.E, false, false);
      w.llm[l].down = pw(d.E, d.F, false, false);
    } else {
      w.llm[l].o = PW{0, 0, 0, 0, 0};
      w.llm[l].gu = w.llm[l].o;
      w.llm[l].down = w.llm[l].o;
    }
  }
  w.mx_ok = d.E % 256 == 0 && d.F % 256 == 0;
  if (w.mx_ok) {
    for (int l = 0; l + 1 < d.Ll; l++) {
      w.llm[l].gu8 = cur.take((size_t)2 * d.F * d.E);
      w.llm[l].gu8s = cur.take((size_t)2 * d.F * d.E / 32);
      w.llm[l].down8 = cur.take((size_t)d.E * d.F);
      w.llm[l].down8s = cur.take((size_t)d.E * d.F / 32);
    }
  }
  w.exp.resize(d.Le);
  for (int l = 0; l < d.Le; l++) {
    w.exp[l].qkv = pw((d.H + 2) * 256, d.X, false, false);
    w.exp[l].o = pw(d.X, d.H * 256, false, false);
    w.exp[l].gu = pw(2 * d.Fx, d.X, false, false);
    w.exp[l].down = pw(d.X, d.Fx, false, false);
  }
  w.state_w = cur.take((size_t)d.SD * d.X * 4);
  w.state_b = cur.take((size_t)d.X * 4);
  w.wfold = cur.take((size_t)d.A * d.X * 4);
  w.bias_tab = cur.take((size_t)d.steps * d.X * 4);
  w.tau = cur.take((size_t)d.steps * d.X * 4);
  w.tout = pw(d.X, d.X, false, true);
  w.outp = pw(d.A, d.X, false, true);
  w.rope = cur.take((size_t)d.maxpos * 128 * 2 * 4);
  w.g_v1.resize(d.Lv); w.g_v2.resize(d.Lv);
  for (int l = 0; l < d.Lv; l++) { w.g_v1[l] = cur.take((size_t)d.Dv * 4); w.g_v2[l] = cur.take((size_t)d.Dv * 4); }
  w.g_vf = cur.take((size_t)d.Dv * 4);
  w.g_l1.resize(d.Ll); w.g_l2.resize(d.Ll);
  for (int l = 0; l < d.Ll; l++) { w.g_l1[l] = cur.take((size_t)d.E * 4); w.g_l2[l] = cur.take((size_t)d.E * 4); }
  w.g_e1.resize(d.Le); w.g_e2.resize(d.Le);
  for (int l = 0; l < d.Le; l++) { w.g_e1[l] = cur.take((size_t)d.X * 4); w.g_e2[l] = cur.take((size_t)d.X * 4); }
  w.g_ef = cur.take((size_t)d.X * 4);
  // ---- activations ----
  w.act_begin = cur.off;
  w.st_images = cur.take((size_t)c.max_views * c.img_size * c.img_size * 3 * 4);
  w.st_ids = cur.take((size_t)(c.max_prompt > 0 ? c.max_prompt : 1) * 4);
  w.xpatch = cur.take((size_t)d.maxI * d.PDp * 2);
  w.vh = cur.take((size_t)d.maxI * d.Dv * 4);
  w.vh_b = cur.take((size_t)d.maxI * d.Dv * 2);
  w.vq = cur.take((size_t)d.Hv * (d.maxI / 32) * 5 * 512 * 2);
  w.vk = cur.take((size_t)d.Hv * (d.maxI / 32) * 5 * 512 * 2);
  w.vv = cur.take((size_t)d.Hv * (d.maxI / 32) * 3 * 1024 * 2);
  w.vattn = cur.take((size_t)d.maxI * d.Dv * 2);
  w.vmid = cur.take((size_t)d.maxI * d.Fv_kp * 2);
  w.zmax = Z_MAX;
  {
    size_t a = (size_t)w.zmax * d.maxI * round_up(d.Dv, 32) * 4;
    size_t b = (size_t)w.zmax * d.maxP * d.E * 4;
    w.part = cur.take(a > b ? a : b);
  }
  w.lx = cur.take((size_t)d.maxP * d.E * 4);
  w.lx_b = cur.take((size_t)d.maxPc * 32 * d.E * 2);
  w.lq = cur.take((size_t)d.H * d.maxPc * 16 * 512 * 2);
  w.kcache_layer = (size_t)d.maxPc * 16 * 512 * 2;
  w.vcache_layer = (size_t)d.maxPc * 8 * 1024 * 2;
  w.kcache_slot = round_up_sz(w.kcache_layer * d.Ll, 256);
  w.vcache_slot = round_up_sz(w.vcache_layer * d.Ll, 256);
  w.kcache = cur.take(w.kcache_slot * 2);
  w.vcache = cur.take(w.vcache_slot * 2);
  w.lattn = cur.take((size_t)d.maxPc * 32 * d.H * 256 * 2);
  w.lmid = cur.take((size_t)d.maxPc * 32 * d.F * 2);
  // ---- scratch of the action expert's per-operation launches: one contiguous block, so that it can also live
  // in the library's static device array (pi0_denoise_static) ----
  w.es_begin = cur.off;
  w.st_state = cur.take((size_t)d.SD * 4);
  w.st_noise = cur.take((size_t)c.chunk * d.A * 4);
  w.xa = cur.take((size_t)c.chunk * d.A * 4);
  w.stok = cur.take((size_t)d.X * 4);
  w.z = cur.take((size_t)64 * d.X * 2);
  w.y = cur.take((size_t)64 * d.X * 4);
  w.y_b = cur.take((size_t)64 * d.X * 2);
  w.eq = cur.take((size_t)d.H * 2 * 16 * 512 * 2);
  w.ek = cur.take((size_t)2 * 16 * 512 * 2);
  w.ev = cur.take((size_t)2 * 8 * 1024 * 2);
  w.eattn = cur.take((size_t)4 * 64 * d.H * 256 * 2);   // up to 4 key shares
  w.eml = cur.take((size_t)4 * d.H * 64 * 2 * 4);
  w.emid = cur.take((size_t)64 * d.Fx * 2);
  w.estat = cur.take((size_t)64 * 2 * 4);
  w.estat_parts = cur.take((size_t)(d.X / 16) * 64 * 2 * 4);
  w.pf_sink = cur.take(1024 * 4);
  w.progress = cur.take(256);
  {
    const int kmax = d.H * 256 > d.Fx ? d.H * 256 : d.Fx;
    w.epart = cur.take((size_t)ceil_div(round_up(kmax, 64), 1024) * 64 * round_up(d.X, 32) * 4);
  }
  w.es_end = cur.off;
  w.vstat = cur.take((size_t)d.maxI * 2 * 4);
  w.lstat = cur.take((size_t)d.maxPc * 32 * 2 * 4);
  w.lx8 = cur.take((size_t)d.maxPc * 32 * d.E);
  w.lx8s = cur.take((size_t)d.maxPc * 32 * d.E / 32 + 256);
  w.lmid8 = cur.take((size_t)d.maxPc * 32 * d.F);
  w.lmid8s = cur.take((size_t)d.maxPc * 32 * d.F / 32 + 256);
  w.vstat_parts = cur.take((size_t)(d.Dv / 32) * d.maxI * 2 * 4);                     // [32-column tile][maxI][2]
  w.lstat_parts = cur.take((size_t)(d.E / 32) * d.maxPc * 32 * 2 * 4);                // [32-column tile][maxPc * 32][2]
  w.esync = cur.take((size_t)GB_WORDS * 4);
  w.eparams = cur.take(sizeof(ExpertLoopParams));
  {  // one slot per (Euler step, expert layer): the same buffers as stok .. emid above, each 256-byte aligned
    WsCursor sl;
    w.r_yb_o = (unsigned)sl.take((size_t)64 * d.X * 2);
    w.r_st_o = (unsigned)sl.take((size_t)(d.X / 16) * 64 * 2 * 4);
    w.r_yb_d = (unsigned)sl.take((size_t)64 * d.X * 2);
    w.r_st_d = (unsigned)sl.take((size_t)(d.X / 16) * 64 * 2 * 4);
    w.r_q = (unsigned)sl.take((size_t)d.H * 2 * 16 * 512 * 2);
    w.r_k = (unsigned)sl.take((size_t)2 * 16 * 512 * 2);
    w.r_v = (unsigned)sl.take((size_t)2 * 8 * 1024 * 2);
    w.r_attn = (unsigned)sl.take((size_t)4 * 64 * d.H * 256 * 2);
    w.r_ml = (unsigned)sl.take((size_t)4 * d.H * 64 * 2 * 4);
    w.r_mid = (unsigned)sl.take((size_t)64 * d.Fx * 2);
    w.ering_slot = sl.off;
    w.ering = cur.take(w.ering_slot * (size_t)d.steps * d.Le);
  }
  w.total = cur.off;
}

struct GraphKey {
  int kind, n_views, n_prompt, slot_w, slot_r, precision, read_ahead;
  bool operator<(const GraphKey& o) const {
    if (kind != o.kind) return kind < o.kind;
    if (precision != o.precision) return precision < o.precision;
    if (n_views != o.n_views) return n_views < o.n_views;
    if (n_prompt != o.n_prompt) return n_prompt < o.n_prompt;
    if (slot_w != o.slot_w) return slot_w < o.slot_w;
    if (read_ahead != o.read_ahead) return read_ahead < o.read_ahead;
    return slot_r < o.slot_r;
  }
};
enum { KIND_PREFILL = 0, KIND_DENOISE = 1, KIND_INFER = 2 };

}  // namespace

// Per-shape tile choices (Section 4.1 of the paper tunes tiles per GEMM shape; these are the
// gfx950 counterparts).  Overridable for tuning runs through pi0_tune,
// e.g. "vis=1,lqkv=1,lgu=0,vo=1,vd=1,lo=0,ld=0,zvo=6,zlo=8,zld=16".
struct Tune {
  int vis = TILE_MID;     // vision patch / projector (and QKV / up unless overridden below)
  int vqkv = -1, vup = -1; // vision QKV / up tile (-1: QKV on the entry kernel up to 256 tokens, else same as vis)
  int lqkv = -1;          // prefix QKV (-1: 64 x 64 tiles up to 256 tokens, 64 x 128 beyond)
  int lgu = -1;           // prefix gate||up (-1: 128, 192 or 256 tokens x 256 features, whichever fills the 256 CUs at the least cost)
  int vo = TILE_MID, vd = -1, lo = -1, ld = TILE_WIDE128;   // split-K partial GEMMs: vision O / down, prefix O / down
  int zvo = -1, zlo = -1, zld = -1, zvd = -1;   // -1: chosen from the number of tokens (measured optima at 1 / 2 / 3 views)
  // warm-up blocks carried by the expert's launches (0 = none): QKV, attention, O, down.  Used instead of the read-ahead
  // kernel below with ras=0
  int pfq = 64, pfa = 64, pfo = 128, pfd = 128;
  int qms = 1;            // expert QKV: token blocks on separate blocks (160 instead of 80)
  int ksplit = 1;         // expert attention: key shares for prefixes beyond kcps chunks
  int kcps = 8;
  // expert attention: the 8 value slices of a (query tile, head) shared out over this many blocks, each repeating the
  // scores (-1: 4 with one key share, 2 with several; measured -0.2 ms of denoise.  The prefix attention gains nothing)
  int avs = -1;
  int ae16 = 1;           // expert O / down on 16 x 16 tiles (256 blocks) instead of 32 x 32 (64 blocks)
  // O projections as one launch over the whole k range (TILE_ENTRY: residual epilogue in the GEMM, no partial
  // buffer, no reduction launch): vision O, prefix O.  -1: up to 256 tokens (measured: -0.06 ms at one view,
  // nothing or a loss beyond, where the blocks' operand reads add up to more than the reduction launch costs)
  int fko = -1, fkl = -1;
  // read-ahead for the expert as one kernel on a second stream beside the compute launches: number of its
  // blocks (0 = warm-up blocks inside the launches instead, see pfq .. pfd), layer-steps it runs ahead,
  // threads per block, loads in flight per lane.  Measured optimum: one 4-wave block per CU (a second wave
  // per SIMD no longer fits beside the compute kernels' registers), 6 loads in flight (more reads the
  // layer in a shorter burst that disturbs the compute launches, fewer arrives late), one layer ahead.
  int ras = 256, ral = 1, rat = 256, rad = 6;
  // the whole denoise loop as one persistent kernel with grid barriers (1) or one launch per operation (0)
  int pdn = 1;
  // ... in which the blocks without an attention item read ahead (bits: gate||up, down, next layer's QKV, next layer's O; 16: this layer's O by the blocks
  // without a QKV item)
  int pra = 39;
  // two-stream frames: blocks of the persistent loop beside the prefill (0: per-operation launches).  A resident block
  // of the loop holds a whole compute unit, so its grid decides how the chip is shared between the two streams
  int psb = -1;           // -1: from the number of prefix tokens (frame_loop_blocks)
};

struct pi0_ctx {
  pi0_config cfg;
  Tune tune;
  Dims d;
  BlobLayout bl;
  WsLayout wl;
  unsigned char* ws = nullptr;
  bool loaded = false;
  bool attrs_set = false;
  int device = -1;                     // device the weights were loaded on
  unsigned char* static_scratch = nullptr;   // that device's copy of the library's static scratch array
  long long* loop_trace = nullptr;     // optional timeline buffer of the persistent denoise kernel (pi0_set_loop_trace)
  int loop_trace_ops = 0;
  bool pk_ok = false;                  // the device can hold the persistent denoise kernel's 256 blocks at once
  bool graph_mode = true;
  int precision = PI0_PRECISION_BF16;   // PI0_PRECISION_MXFP8_PREFIX_MLP: prefix gate||up / down on MXFP8 operands
  int cur_views = 0, cur_prompt = 0;   // shape of the valid prefill (0 views = none)
  int cur_slot = 0;                    // cache copy that holds it
  hipEvent_t ev_prefill[2] = {nullptr, nullptr};   // pi0_stream_frame: copy s was written / last read
  hipEvent_t ev_denoise[2] = {nullptr, nullptr};
  hipStream_t ra_stream = nullptr;                 // read-ahead kernel of the expert (created on first use)
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  int last_hip = 0;
  std::map<GraphKey, hipGraphExec_t> graphs;
  std::vector<float> h_rope, h_tau;
};

namespace {

// Launch recorder: either launches or only counts.
struct OpTimer {
  std::vector<hipEvent_t> ev;   // pairs (before, after)
  std::vector<int> cls;
};
struct Run {
  pi0_ctx* c;
  hipStream_t s;
  bool count_only;
  int launches = 0;
  hipError_t err = hipSuccess;
  int slot_w = 0, slot_r = 0;   // cache copy the prefill writes / the denoise reads
  bool read_ahead = true;       // expert: read ahead of the compute launches (read-ahead kernel on a second stream, or warm-up
                                // blocks inside the launches with pi0_tune "ras=0"); false: neither
  int cls = PI0_OP_MISC;        // class of the launches that follow
  OpTimer* timer = nullptr;     // when set, every RUN / RUN_GEMM launch is bracketed by an event pair
  bool persistent_ok = false;   // the denoise loop may run as one persistent kernel (plain pi0_denoise / pi0_infer calls)
  int persist_blocks = 0;       // its grid (0: one block per compute unit)
  unsigned char* ebase = nullptr;   // where the expert's scratch block lives minus its workspace offset (null: in the workspace)
  bool ok() const { return err == hipSuccess; }
  void did(hipError_t e) {
    launches++;
    if (err == hipSuccess && e != hipSuccess) err = e;
  }
  void mark() {
    if (timer == nullptr || err != hipSuccess) return;
    hipEvent_t e;
    hipError_t r = hipEventCreate(&e);
    if (r == hipSuccess) {
      timer->ev.push_back(e);
      r = hipEventRecord(e, s);
    }
    if (r != hipSuccess) err = r;
  }
  void before() { mark(); }
  void after() {
    mark();
    if (timer != nullptr) timer->cls.push_back(cls);
  }
};

template <typename T>
T* at(pi0_ctx* c, size_t off) { return reinterpret_cast<T*>(c->ws + off); }
// a buffer of the expert's scratch block (workspace offsets es_begin .. es_end): in the workspace, or wherever r.ebase points
template <typename T>
T* ex(const Run& r, size_t off) {
  return reinterpret_cast<T*>(reinterpret_cast<uintptr_t>(r.ebase != nullptr ? r.ebase : r.c->ws) + off);
}

PackedW packed(pi0_ctx* c, const PW& p) {
  PackedW w;
  w.w = at<bf16>(c, p.w);
  w.n_pad = p.n_pad;
  w.k_pad = p.k_pad;
  return w;
}

GemmParams gp_base(pi0_ctx* c, const PW& pw, const bf16* X, int ldx, int M, int tile, int k_true) {
  const int rows_per_tile = gemm_rows_per_tile(tile);
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.X = X;
  p.ldx = ldx;
  p.M = M;
  p.W = packed(c, pw);
  p.n_tiles = pw.n_pad / 32;
  p.k_per_split = pw.k_pad;
  p.k_true = k_true;
  p.m_tiles = ceil_div(M, rows_per_tile);
  p.n_valid = pw.n_pad;
  return p;
}

#define RUN_GEMM(r, tile, pro, epi, p, z) \
  do { if ((r).count_only) (r).launches++; else if ((r).ok()) { (r).before(); (r).did(launch_gemm((r).s, tile, pro, epi, p, z)); (r).after(); } } while (0)
#define RUN(r, call) \
  do { if ((r).count_only) (r).launches++; else if ((r).ok()) { (r).before(); (r).did(call); (r).after(); } } while (0)

// split-K GEMM into the partial buffer followed by the fixed-order reduction with bias/residual
void gemm_splitk_resid(Run& r, const PW& pw, const bf16* X, int ldx, int M, int k_true, int z, int k_per_split,
                       const float* bias, float* resid_io, bf16* shadow, int n_true, int tile, float* stat_out,
                       const float* gain, const float* resid_in = nullptr, int resid_mod = 0, bool no_resid = false,
                       bool expert_scratch = false, unsigned char* out8 = nullptr, unsigned char* out8_scales = nullptr) {
  pi0_ctx* c = r.c;
  if (z > Z_MAX) z = Z_MAX;
  if ((long)k_per_split * z < pw.k_pad) k_per_split = round_up(ceil_div(pw.k_pad, z), 64);
  GemmParams p = gp_base(c, pw, X, ldx, M, tile, k_true);
  p.k_per_split = k_per_split;
  p.out_f32 = expert_scratch ? ex<float>(r, c->wl.epart) : at<float>(c, c->wl.part);
  p.ldo = pw.n_pad;
  RUN_GEMM(r, tile, PRO_NONE, EPI_PARTIAL, p, z);
  const int cls_gemm = r.cls;
  r.cls = PI0_OP_REDUCE;
  ReduceParams q;
  q.part = p.out_f32;
  q.Z = z; q.M = M; q.N = n_true; q.ldp = pw.n_pad;
  q.bias = bias;
  q.resid = no_resid ? nullptr : (resid_in ? resid_in : resid_io);
  q.resid_mod = resid_mod;
  q.stat_out = stat_out;
  q.gain = gain;
  q.out_f32 = resid_io;
  q.out_bf16 = shadow;
  q.ldo = n_true; q.ldo2 = n_true;
  q.out8 = out8; q.out8_scales = out8_scales;
  RUN(r, launch_splitk_reduce(r.s, q));
  r.cls = cls_gemm;
}

// the same operation as one GEMM over the whole k range: bias / residual / gain-scaled shadow in the
// GEMM's epilogue, row statistics left as one partial sum per 32-column tile in parts[n tile][stat_rows][2]
void gemm_fullk_resid(Run& r, const PW& pw, const bf16* X, int ldx, int M, int k_true, const float* bias, float* resid_io,
                      bf16* shadow, int n_true, float* parts, int stat_rows, const float* gain, int tile = TILE_ENTRY) {
  GemmParams p = gp_base(r.c, pw, X, ldx, M, tile, k_true);
  p.bias = bias;
  p.resid = resid_io;
  p.out_f32 = resid_io;
  p.out_bf16 = shadow;
  p.ldo = n_true; p.ldo2 = n_true; p.n_valid = n_true;
  p.gain = gain;
  p.stat_out = parts;
  p.stat_rows = stat_rows;
  RUN_GEMM(r, tile, PRO_NONE, EPI_RESID, p, 1);
}

struct Taps {
  float* base = nullptr;
  size_t off = 0;
  void put(Run& r, const float* src, size_t n) {
    if (base == nullptr) return;
    if (!r.count_only && r.ok()) r.did(launch_copy_f32(r.s, src, base + off, n));
    off += n;
  }
};

void run_prefill(Run& r, int n_views, int n_prompt, Taps* taps) {
  pi0_ctx* c = r.c;
  const Dims& d = c->d;
  const WsLayout& w = c->wl;
  const Tune& T = c->tune;
  const int I = n_views * d.T, P = I + n_prompt;
  // A0: patches -> tokens (+bias, +position embedding)
  r.cls = PI0_OP_MISC;
  RUN(r, launch_patchify(r.s, at<float>(c, w.st_images), n_views, c->cfg.img_size, c->cfg.patch, at<bf16>(c, w.xpatch), d.PDp));
  r.cls = PI0_OP_VIS_PATCH;
  gemm_splitk_resid(r, w.patch, at<bf16>(c, w.xpatch), d.PDp, I, d.PD, 1, w.patch.k_pad, at<float>(c, w.patch.bias),
                    at<float>(c, w.vh), at<bf16>(c, w.vh_b), d.Dv, T.vis, at<float>(c, w.vstat), at<float>(c, w.g_v1[0]),
                    at<float>(c, w.pos), d.T);
  const int vchunks = I / 32;
  const int zvo = T.zvo > 0 ? T.zvo : (I <= 256 ? 3 : I <= 512 ? 2 : 1);
  const int tvd = T.vd >= 0 ? T.vd : (I <= 256 ? TILE_MID : TILE_SQ128);
  const int zvd = T.zvd > 0 ? T.zvd : (I <= 512 ? 4 : 2);
  // one view: the QKV GEMM has too few 64 x 128 tiles for 256 CUs; 64 x 64 tiles with every load issued at entry
  // two and three views: 128 x 128 tiles need fewer operand bytes per CU than 64 x 128 once they still fill the chip
  const int tqkv = T.vqkv >= 0 ? T.vqkv : (I <= 256 ? TILE_ENTRY : I <= 512 ? T.vis : TILE_MID2);   // 3 views: 324 blocks, two per CU
  const int tup = T.vup >= 0 ? T.vup : (I <= 256 ? T.vis : TILE_SQ128);
  const bool fko = T.fko >= 0 ? T.fko != 0 : I <= 256;
  for (int l = 0; l < d.Lv; l++) {
    const WsVis& L = w.vis[l];
    {  // A1: LN -> QKV (+bias), keys/values straight into attention fragment order
      GemmParams p = gp_base(c, L.qkv, at<bf16>(c, w.vh_b), d.Dv, I, tqkv, d.Dv);
      p.bias = at<float>(c, L.qkv.bias);
      p.colsum = at<float>(c, L.qkv.colsum);
      p.rowstat = at<float>(c, w.vstat);
      p.out_bf16 = at<bf16>(c, w.vq);
      p.q_mbs = vchunks;
      p.kfrag = at<bf16>(c, w.vk);
      p.vfrag = at<bf16>(c, w.vv);
      p.rope = nullptr;
      p.q_cols = d.Dv; p.k_cols = d.Dv;
      p.head_dim = d.hdv; p.dqk_pad = 80; p.nvb = 3; p.kv_heads = d.Hv; p.kv_chunks = vchunks;
      r.cls = PI0_OP_VIS_QKV;
      RUN_GEMM(r, tqkv, PRO_LN, EPI_QKV, p, 1);
    }
    {  // A2: attention inside each view
      AttnParams a;
      memset(&a, 0, sizeof(a));
      a.q = at<bf16>(c, w.vq); a.q_head_stride = vchunks * 5 * 512;
      a.Tq = I; a.heads = d.Hv;
      a.k0 = at<bf16>(c, w.vk); a.v0 = at<bf16>(c, w.vv);
      a.chunks0 = vchunks; a.valid0 = I;
      a.kv_head_stride0 = vchunks * 5 * 512; a.v_head_stride0 = vchunks * 3 * 1024;
      a.view_tokens = d.T;
      a.scale = 1.0f / sqrtf((float)d.hdv);
      a.out = at<bf16>(c, w.vattn); a.out_ld = d.Dv; a.head_dim = d.hdv;
      r.cls = PI0_OP_VIS_ATTN;
      RUN(r, launch_attention(r.s, a));
    }
    // A3: O-projection + bias + residual
    r.cls = PI0_OP_VIS_O;
    if (fko)
      gemm_fullk_resid(r, L.o, at<bf16>(c, w.vattn), d.Dv, I, d.Dv, at<float>(c, L.o.bias), at<float>(c, w.vh),
                       at<bf16>(c, w.vh_b), d.Dv, at<float>(c, w.vstat_parts), d.maxI, at<float>(c, w.g_v2[l]),
                       I <= 256 ? TILE_ENTRY : T.vo);
    else
      gemm_splitk_resid(r, L.o, at<bf16>(c, w.vattn), d.Dv, I, d.Dv, zvo, round_up(ceil_div(L.o.k_pad, zvo), 64),
                        at<float>(c, L.o.bias), at<float>(c, w.vh), at<bf16>(c, w.vh_b), d.Dv, T.vo, at<float>(c, w.vstat),
                        at<float>(c, w.g_v2[l]));
    {  // A4: LN -> up (+bias, GELU)
      GemmParams p = gp_base(c, L.up, at<bf16>(c, w.vh_b), d.Dv, I, tup, d.Dv);
      p.bias = at<float>(c, L.up.bias);
      p.colsum = at<float>(c, L.up.colsum);
      p.rowstat = at<float>(c, w.vstat);
      if (fko) { p.rowstat = at<float>(c, w.vstat_parts); p.rowstat_parts = L.o.n_pad / 32; p.stat_rows = d.maxI; }
      p.out_bf16 = at<bf16>(c, w.vmid);
      p.ldo = d.Fv_kp; p.n_valid = L.up.n_pad; p.act = ACT_GELU;
      r.cls = PI0_OP_VIS_UP;
      RUN_GEMM(r, tup, PRO_LN, EPI_BF16, p, 1);
    }
    // A5: down (+bias, residual)
    r.cls = PI0_OP_VIS_DOWN;
    gemm_splitk_resid(r, L.down, at<bf16>(c, w.vmid), d.Fv_kp, I, d.Fv, zvd, round_up(ceil_div(L.down.k_pad, zvd), 64),
                      at<float>(c, L.down.bias), at<float>(c, w.vh), at<bf16>(c, w.vh_b), d.Dv, tvd, at<float>(c, w.vstat),
                      at<float>(c, l + 1 < d.Lv ? w.g_v1[l + 1] : w.g_vf));
    if (taps) taps->put(r, at<float>(c, w.vh), (size_t)I * d.Dv);
  }
  {  // A6: final LN -> projector (+bias) = prefix image embeddings
    GemmParams p = gp_base(c, w.proj, at<bf16>(c, w.vh_b), d.Dv, I, T.vis, d.Dv);
    p.bias = at<float>(c, w.proj.bias);
    p.colsum = at<float>(c, w.proj.colsum);
    p.rowstat = at<float>(c, w.vstat);
    p.out_f32 = at<float>(c, w.lx);
    p.out_bf16 = at<bf16>(c, w.lx_b);
    p.ldo = d.E; p.ldo2 = d.E; p.n_valid = d.E;
    r.cls = PI0_OP_VIS_PROJ;
    RUN_GEMM(r, T.vis, PRO_LN, EPI_RESID, p, 1);
    r.cls = PI0_OP_MISC;
  }
  if (taps) taps->put(r, at<float>(c, w.lx), (size_t)I * d.E);
  if (n_prompt > 0) {  // B0: prompt embeddings after the image tokens
    RUN(r, launch_embed_prompt(r.s, at<int32_t>(c, w.st_ids), n_prompt, at<bf16>(c, w.embed), c->cfg.vocab, d.E,
                               sqrtf((float)d.E), at<float>(c, w.lx), at<bf16>(c, w.lx_b), I));
  }
  RUN(r, launch_row_stats(r.s, at<float>(c, w.lx), d.E, P, d.E, d.E, at<float>(c, w.g_l1[0]), at<bf16>(c, w.lx_b),
                          at<float>(c, w.lstat)));
  const int pchunks = ceil_div(P, 32);
  const int tlqkv = T.lqkv >= 0 ? T.lqkv : (P <= 256 ? TILE_SMALL : P <= 512 ? TILE_MID : TILE_MID2);   // 3 views: 30.0 -> 25.3 us
  const int tlo = T.lo >= 0 ? T.lo : (P <= 512 ? TILE_MID : TILE_SQ128);
  const int zlo = T.zlo > 0 ? T.zlo : (P <= 256 ? 4 : 2);
  const bool mx = c->precision == PI0_PRECISION_MXFP8_PREFIX_MLP;
  // reduced precision: the GeGLU epilogue takes whole-row statistics, so the O projection keeps its reduction launch
  const bool fkl = mx ? false : (T.fkl >= 0 ? T.fkl != 0 : P <= 256);
  // gate||up: 128 blocks of 256 features per token tile of 128, 192 or 256 tokens.  A block's time goes with its
  // height, so a choice costs height x rounds on 256 compute units; take the cheapest, the taller tile on ties
  // (fewer operand bytes per CU and flop).  256 / 512 / 768 / 816 tokens -> 128 / 256 / 192 / 256.
  const int gu_cols = ceil_div(w.llm[0].gu.n_pad, 256);
  int tlgu = T.lgu;
  if (tlgu < 0) {
    const int heights[3] = {128, 192, 256}, ids[3] = {TILE_WIDE128, TILE_T192, TILE_WIDE};
    int best = 0;
    for (int i = 0; i < 3; i++) {
      const int cost = heights[i] * ceil_div(ceil_div(P, heights[i]) * gu_cols, 256);
      if (tlgu < 0 || cost <= best) { best = cost; tlgu = ids[i]; }
    }
  }
  // down: as many k slices as keep all blocks in one round (measured optima 16 / 8 / 5 at 256 / 512 / 768 tokens)
  const int down_tiles = ceil_div(P, gemm_rows_per_tile(T.ld)) * ceil_div(w.llm[0].down.n_pad, T.ld == TILE_WIDE || T.ld == TILE_WIDE128 || T.ld == TILE_T192 ? 256 : 128);
  const int zld = T.zld > 0 ? T.zld : std::max(1, std::min(16, 256 / std::max(1, down_tiles)));
  for (int l = 0; l < d.Ll; l++) {
    const WsTr& L = w.llm[l];
    const bool last = l == d.Ll - 1;
    bf16* kc = reinterpret_cast<bf16*>(c->ws + w.kcache + (size_t)r.slot_w * w.kcache_slot + (size_t)l * w.kcache_layer);
    bf16* vc = reinterpret_cast<bf16*>(c->ws + w.vcache + (size_t)r.slot_w * w.vcache_slot + (size_t)l * w.vcache_layer);
    {  // B1: RMS -> QKV, RoPE, keys/values into the cache (last layer: keys/values only)
      GemmParams p = gp_base(c, L.qkv, at<bf16>(c, w.lx_b), d.E, P, tlqkv, d.E);
      p.rowstat = at<float>(c, w.lstat);
      p.out_bf16 = at<bf16>(c, w.lq);
      p.q_mbs = pchunks;
      p.kfrag = kc; p.vfrag = vc;
      p.rope = at<float>(c, w.rope);
      p.pos0 = 0;
      p.q_cols = last ? 0 : d.H * 256; p.k_cols = 256;
      p.head_dim = 256; p.dqk_pad = 256; p.nvb = 8; p.kv_heads = 1; p.kv_chunks = d.maxPc;
      r.cls = PI0_OP_LLM_QKV;
      RUN_GEMM(r, tlqkv, PRO_RMS, EPI_QKV, p, 1);
    }
    if (last) break;
    {  // B2: attention, whole prefix visible
      AttnParams a;
      memset(&a, 0, sizeof(a));
      a.q = at<bf16>(c, w.lq); a.q_head_stride = pchunks * 16 * 512;
      a.Tq = P; a.heads = d.H;
      a.k0 = kc; a.v0 = vc; a.chunks0 = pchunks; a.valid0 = P;
      a.scale = 1.0f / 16.0f;
      a.out = at<bf16>(c, w.lattn); a.out_ld = d.H * 256; a.head_dim = 256;
      r.cls = PI0_OP_LLM_ATTN;
      RUN(r, launch_attention(r.s, a));
    }
    // B3: O-projection + residual
    r.cls = PI0_OP_LLM_O;
    if (fkl)
      gemm_fullk_resid(r, L.o, at<bf16>(c, w.lattn), d.H * 256, P, d.H * 256, nullptr, at<float>(c, w.lx), at<bf16>(c, w.lx_b),
                       d.E, at<float>(c, w.lstat_parts), d.maxPc * 32, at<float>(c, w.g_l2[l]), P <= 256 ? TILE_ENTRY : tlo);
    else
      gemm_splitk_resid(r, L.o, at<bf16>(c, w.lattn), d.H * 256, P, d.H * 256, zlo,
                        round_up(ceil_div(L.o.k_pad, zlo), 64), nullptr, at<float>(c, w.lx), at<bf16>(c, w.lx_b), d.E, tlo,
                        at<float>(c, w.lstat), at<float>(c, w.g_l2[l]), nullptr, 0, false, false,
                        mx ? c->ws + w.lx8 : nullptr, mx ? c->ws + w.lx8s : nullptr);   // MXFP8 copy for gate||up
    if (mx) {
      // B4 / B5 on MXFP8 operands: x * (1 + g) was quantised per 32 columns by the O projection's reduction, gate||up
      // quantises the GeGLU product in its epilogue, down goes as split-K partials into the usual reduction
      r.cls = PI0_OP_LLM_GATEUP;
      MxGemmParams q;
      memset(&q, 0, sizeof(q));
      q.X8 = c->ws + w.lx8; q.XS = c->ws + w.lx8s; q.ldx = d.E; q.M = P;
      q.W8 = c->ws + L.gu8; q.WS = c->ws + L.gu8s; q.n_pad = L.gu.n_pad; q.k_pad = L.gu.k_pad;
      q.m_tiles = ceil_div(P, 128); q.k_per_split = L.gu.k_pad; q.k_true = d.E;
      q.rowstat = at<float>(c, w.lstat);
      q.out8 = c->ws + w.lmid8; q.out_scales = c->ws + w.lmid8s; q.ldo8 = d.F;
      RUN(r, launch_gemm_mx(r.s, MX_EPI_GEGLU, q, 1));
      r.cls = PI0_OP_LLM_DOWN;
      const int zmx = std::max(1, std::min(16, 256 / std::max(1, ceil_div(P, 128) * ceil_div(L.down.n_pad, 256))));
      const int kps = round_up(ceil_div(L.down.k_pad, zmx), 256);
      const int zeff = ceil_div(L.down.k_pad, kps);
      MxGemmParams u;
      memset(&u, 0, sizeof(u));
      u.X8 = c->ws + w.lmid8; u.XS = c->ws + w.lmid8s; u.ldx = d.F; u.M = P;
      u.W8 = c->ws + L.down8; u.WS = c->ws + L.down8s; u.n_pad = L.down.n_pad; u.k_pad = L.down.k_pad;
      u.m_tiles = ceil_div(P, 128); u.k_per_split = kps; u.k_true = d.F;
      u.out_f32 = at<float>(c, w.part); u.ldo = L.down.n_pad;
      RUN(r, launch_gemm_mx(r.s, MX_EPI_PARTIAL, u, zeff));
      r.cls = PI0_OP_REDUCE;
      ReduceParams rq;
      rq.part = u.out_f32;
      rq.Z = zeff; rq.M = P; rq.N = d.E; rq.ldp = L.down.n_pad;
      rq.bias = nullptr;
      rq.resid = at<float>(c, w.lx);
      rq.resid_mod = 0;
      rq.stat_out = at<float>(c, w.lstat);
      rq.gain = at<float>(c, w.g_l1[l + 1]);
      rq.out_f32 = at<float>(c, w.lx);
      rq.out_bf16 = at<bf16>(c, w.lx_b);
      rq.ldo = d.E; rq.ldo2 = d.E;
      rq.out8 = nullptr; rq.out8_scales = nullptr;
      RUN(r, launch_splitk_reduce(r.s, rq));
      if (taps) taps->put(r, at<float>(c, w.lx), (size_t)P * d.E);
      continue;
    }
    {  // B4: RMS -> gate||up with fused GELU gate
      GemmParams p = gp_base(c, L.gu, at<bf16>(c, w.lx_b), d.E, P, tlgu, d.E);
      p.rowstat = at<float>(c, w.lstat);
      if (fkl) { p.rowstat = at<float>(c, w.lstat_parts); p.rowstat_parts = L.o.n_pad / 32; p.stat_rows = d.maxPc * 32; }
      p.out_bf16 = at<bf16>(c, w.lmid);
      p.ldo = d.F;
      r.cls = PI0_OP_LLM_GATEUP;
      RUN_GEMM(r, tlgu, PRO_RMS, EPI_GEGLU, p, 1);
    }
    // B5: down + residual
    r.cls = PI0_OP_LLM_DOWN;
    gemm_splitk_resid(r, L.down, at<bf16>(c, w.lmid), d.F, P, d.F, zld,
                      round_up(ceil_div(L.down.k_pad, zld), 64), nullptr, at<float>(c, w.lx), at<bf16>(c, w.lx_b),
                      d.E, T.ld, at<float>(c, w.lstat), at<float>(c, w.g_l1[l + 1]));
    if (taps) taps->put(r, at<float>(c, w.lx), (size_t)P * d.E);
  }
  if (taps && taps->base) {
    for (int l = 0; l < d.Ll; l++) {
      bf16* kc = reinterpret_cast<bf16*>(c->ws + w.kcache + (size_t)r.slot_w * w.kcache_slot + (size_t)l * w.kcache_layer);
      bf16* vc = reinterpret_cast<bf16*>(c->ws + w.vcache + (size_t)r.slot_w * w.vcache_slot + (size_t)l * w.vcache_layer);
      float* kout = taps->base + taps->off + (size_t)l * P * 256;
      float* vout = kout + (size_t)d.Ll * P * 256;
      if (!r.count_only && r.ok()) r.did(launch_unpack_kv(r.s, kc, vc, P, kout, vout));
    }
    taps->off += (size_t)2 * d.Ll * P * 256;
  }
}


// The denoise loop as ONE persistent kernel (expert_persistent.hip): the operations' parameters exactly as the
// per-operation launches below fill them for layer 0 / step 0, plus the strides between layers.  Returns false
// (nothing launched) when the shape or the tuning choices are outside what the kernel covers; the caller then
// issues the per-operation launches.
// whether the denoise loop over a prefix of P tokens runs as the persistent kernel: the device holds its blocks, the
// tuning choices are the ones it covers, the per-layer strides are uniform
bool persistent_feasible(const pi0_ctx* c, int P) {
  const Dims& d = c->d;
  const WsLayout& w = c->wl;
  const Tune& T = c->tune;
  if (!T.pdn || !c->pk_ok) return false;
  const int pchunks = ceil_div(P, 32);
  if (!T.ae16 || !T.qms || d.H != 8 || d.X > SK_KMAX_HOST || d.X % 256 != 0) return false;
  const int shares = pchunks > T.kcps ? ceil_div(pchunks, T.kcps) : 1;
  if (T.kcps > 8 || shares > 4 || (shares > 1 && !T.ksplit)) return false;
  const int vs = T.avs > 0 ? T.avs : (shares == 1 ? 4 : 2);
  if (vs != 2 && vs != 4 && vs != 8) return false;   // the kernel's attention keeps at most 5 chunks per wave
  if (ceil_div((shares > 1 ? T.kcps : pchunks) + 2, vs) > 5) return false;
  const WsTr& L0 = w.exp[0];
  if (L0.o.k_pad != 2048 || (L0.down.k_pad != 2048 && L0.down.k_pad != 4096)) return false;
  if (d.Le > 1) {
    const size_t wst = w.exp[1].qkv.w - w.exp[0].qkv.w, gst = w.g_e1[1] - w.g_e1[0];
    for (int l = 1; l < d.Le; l++) {
      const WsTr &A = w.exp[l - 1], &B = w.exp[l];
      if (B.qkv.w - A.qkv.w != wst || B.o.w - A.o.w != wst || B.gu.w - A.gu.w != wst || B.down.w - A.down.w != wst) return false;
      if (w.g_e1[l] - w.g_e1[l - 1] != gst || w.g_e2[l] - w.g_e2[l - 1] != gst) return false;
    }
    if (wst % 2 != 0 || gst % 4 != 0) return false;
  }
  return w.total - w.act_begin < ((size_t)1 << 32);   // offsets inside the arena are 32-bit
}

bool run_denoise_persistent(Run& r, int P) {
  pi0_ctx* c = r.c;
  const Dims& d = c->d;
  const WsLayout& w = c->wl;
  const Tune& T = c->tune;
  if (!r.persistent_ok || r.timer != nullptr || !persistent_feasible(c, P)) return false;
  const int chunk = c->cfg.chunk;
  const int pchunks = ceil_div(P, 32);
  const int shares = pchunks > T.kcps ? ceil_div(pchunks, T.kcps) : 1;
  const WsTr& L0 = w.exp[0];
  const size_t wst = d.Le > 1 ? w.exp[1].qkv.w - w.exp[0].qkv.w : 0, gst = d.Le > 1 ? w.g_e1[1] - w.g_e1[0] : 0;
  const size_t arena_bytes = w.total - w.act_begin;
  if (r.count_only) {
    r.launches += 3;   // barrier words cleared, parameter block written, the loop kernel
    return true;
  }
  if (!r.ok()) return true;
  ExpertLoopParams E;
  memset(&E, 0, sizeof(E));
  float* xa = at<float>(c, w.xa);
  E.stok = StateTokenArgs{at<float>(c, w.st_state), d.SD, at<float>(c, w.state_w), at<float>(c, w.state_b), d.X, at<float>(c, w.stok), nullptr};
  E.emb.a = ActionEmbedArgs{xa, chunk, d.A, at<float>(c, w.wfold), at<float>(c, w.bias_tab), d.X, at<bf16>(c, w.z), at<float>(c, w.stok),
                            at<float>(c, w.y), at<bf16>(c, w.y_b), at<float>(c, w.g_e1[0]), at<float>(c, w.estat_parts)};
  E.emb.x_rw = xa;
  E.noise = at<float>(c, w.st_noise);
  E.x_elems = chunk * d.A;
  E.layers = d.Le;
  E.steps = d.steps;
  E.w_stride = wst / 2;
  E.read_ahead = T.pra;
  E.kcache_stride = w.kcache_layer / 2;
  E.vcache_stride = w.vcache_layer / 2;
  E.g_attn0 = at<float>(c, w.g_e1[0]);
  E.g_mlp0 = at<float>(c, w.g_e2[0]);
  E.g_final = at<float>(c, w.g_ef);
  E.gain_stride = gst / 4;
  {  // C2
    GemmParams p = gp_base(c, w.tout, at<bf16>(c, w.z), d.X, chunk, TILE_SKINNY, d.X);
    p.bias = at<float>(c, w.tout.bias);
    p.out_f32 = at<float>(c, w.y);
    p.out_bf16 = at<bf16>(c, w.y_b);
    p.ldo = d.X; p.ldo2 = d.X; p.n_valid = d.X; p.row_offset = 1;
    p.gain = at<float>(c, w.g_e1[0]);
    p.stat_out = at<float>(c, w.estat_parts);
    E.tout = p;
  }
  E.parts_first = w.tout.n_pad / 32;
  E.parts_rest = L0.down.n_pad / 16;
  {  // C3
    GemmParams p = gp_base(c, L0.qkv, at<bf16>(c, w.y_b), d.X, 64, TILE_SKINNY, d.X);
    p.rowstat = at<float>(c, w.estat_parts);
    p.rowstat_parts = E.parts_first;
    p.out_bf16 = at<bf16>(c, w.eq);
    p.q_mbs = 2;
    p.kfrag = at<bf16>(c, w.ek); p.vfrag = at<bf16>(c, w.ev);
    p.rope = at<float>(c, w.rope);
    p.pos0 = P;
    p.q_cols = d.H * 256; p.k_cols = 256;
    p.head_dim = 256; p.dqk_pad = 256; p.nvb = 8; p.kv_heads = 1; p.kv_chunks = 2;
    p.m_split = 1;
    E.qkv = p;
  }
  {  // C4 + C5
    AttnParams a;
    memset(&a, 0, sizeof(a));
    a.q = at<bf16>(c, w.eq); a.q_head_stride = 2 * 16 * 512;
    a.Tq = 64; a.heads = d.H;
    a.k0 = reinterpret_cast<bf16*>(c->ws + w.kcache + (size_t)r.slot_r * w.kcache_slot);
    a.v0 = reinterpret_cast<bf16*>(c->ws + w.vcache + (size_t)r.slot_r * w.vcache_slot);
    a.chunks0 = pchunks; a.valid0 = P;
    a.k1 = at<bf16>(c, w.ek); a.v1 = at<bf16>(c, w.ev); a.chunks1 = 2;
    a.suffix_mask = 1;
    a.scale = 1.0f / 16.0f;
    a.out = at<bf16>(c, w.eattn); a.out_ld = d.H * 256; a.head_dim = 256;
    if (shares > 1) {
      a.key_splits = shares;
      a.chunks_per_split = T.kcps;
      a.out_split_stride = (size_t)64 * d.H * 256;
      a.ml_out = at<float>(c, w.eml);
    }
    a.v_split = T.avs > 0 ? T.avs : (shares == 1 ? 4 : 2);
    E.att = a;
    E.att_gx = 2 * a.v_split;
    E.att_items = E.att_gx * d.H * shares;
  }
  auto resid = [&](const PW& pw, const bf16* X, int K, const float* gain) {
    GemmParams p = gp_base(c, pw, X, K, 64, TILE_SKINNY16, K);
    p.resid = at<float>(c, w.y);
    p.out_f32 = at<float>(c, w.y);
    p.out_bf16 = at<bf16>(c, w.y_b);
    p.ldo = d.X; p.ldo2 = d.X; p.n_valid = d.X;
    p.stat_out = at<float>(c, w.estat_parts);
    p.gain = gain;
    return p;
  };
  E.o = resid(L0.o, at<bf16>(c, w.eattn), d.H * 256, at<float>(c, w.g_e2[0]));   // C6
  if (shares > 1) {
    E.o.xsplits = shares;
    E.o.xsplit_stride = (size_t)64 * d.H * 256;
    E.o.xsplit_ml = at<float>(c, w.eml);
  }
  {  // C7
    GemmParams p = gp_base(c, L0.gu, at<bf16>(c, w.y_b), d.X, 64, TILE_SKINNY, d.X);
    p.rowstat = at<float>(c, w.estat_parts);
    p.rowstat_parts = L0.o.n_pad / 16;
    p.out_bf16 = at<bf16>(c, w.emid);
    p.ldo = d.Fx;
    E.gu = p;
  }
  E.dn = resid(L0.down, at<bf16>(c, w.emid), d.Fx, at<float>(c, d.Le > 1 ? w.g_e1[1] : w.g_ef));   // C8
  E.m16 = 4;
  E.dn_ns = L0.down.k_pad == 4096 ? 16 : 8;
  {  // C9
    GemmParams p = gp_base(c, w.outp, at<bf16>(c, w.y_b), d.X, 64, TILE_SKINNY, d.X);
    p.rowstat = at<float>(c, w.estat_parts);
    p.rowstat_parts = L0.down.n_pad / 16;
    p.bias = at<float>(c, w.outp.bias);
    p.out_f32 = xa;
    p.ldo = d.A; p.n_valid = d.A; p.dt = -1.0f / (float)d.steps;
    E.outp = p;
  }
  E.ring = reinterpret_cast<char*>(c->ws + w.ering);
  E.ring_stride = w.ering_slot;
  E.r_yb_o = w.r_yb_o; E.r_st_o = w.r_st_o; E.r_yb_d = w.r_yb_d; E.r_st_d = w.r_st_d;
  E.r_q = w.r_q; E.r_k = w.r_k; E.r_v = w.r_v; E.r_attn = w.r_attn; E.r_ml = w.r_ml; E.r_mid = w.r_mid;
  E.sync = at<unsigned>(c, w.esync);
  E.arena = reinterpret_cast<const char*>(c->ws + w.act_begin);
  E.arena_bytes = (unsigned)arena_bytes;
  E.spin_limit = 1u << 20;
  E.trace = c->loop_trace;
  E.trace_ops = c->loop_trace_ops;
  r.cls = PI0_OP_MISC;
  // barrier words restart at zero (the error word, first, stays as it is)
  RUN(r, launch_fill_zero(r.s, at<unsigned>(c, w.esync) + GB_START, (size_t)(GB_WORDS - GB_START) * 4));
  if (r.ok()) {
    r.did(launch_expert_loop(r.s, E, at<ExpertLoopParams>(c, w.eparams), r.persist_blocks > 0 ? r.persist_blocks : PK_BLOCKS));
    r.launches++;   // two launches: parameter block, loop kernel
  }
  return true;
}

void run_denoise(Run& r, int P, Taps* taps) {
  if (taps == nullptr && run_denoise_persistent(r, P)) return;
  pi0_ctx* c = r.c;
  const Dims& d = c->d;
  const WsLayout& w = c->wl;
  const int chunk = c->cfg.chunk;
  const int pchunks = ceil_div(P, 32);
  float* xa = ex<float>(r, w.xa);
  r.cls = PI0_OP_MISC;
  RUN(r, launch_copy_f32(r.s, ex<float>(r, w.st_noise), xa, (size_t)chunk * d.A));
  // C0: state token
  RUN(r, launch_state_token(r.s, ex<float>(r, w.st_state), d.SD, at<float>(c, w.state_w), at<float>(c, w.state_b), d.X,
                            ex<float>(r, w.stok), ex<int>(r, w.progress)));
  const float dt = -1.0f / (float)d.steps;
  size_t tap_step_base = taps ? taps->off : 0;
  // row statistics of the suffix residual stream: where the next RMS-folded GEMM finds them
  const float* stat_ptr = ex<float>(r, w.estat);
  int stat_parts = 1;
  // y += X @ W (expert O / down projection).  k = 2048 or 4096: one kernel with the residual
  // epilogue that also leaves per-tile row statistics; otherwise split-K partials + reduction.
  // warm-up descriptors: each launch reads ahead for the launches that follow it
  auto pf_begin = [&](int blocks) {
    PrefetchDesc f;
    memset(&f, 0, sizeof(f));
    f.blocks = blocks;
    f.sink = ex<unsigned>(r, w.pf_sink);
    return f;
  };
  auto pf_weights = [&](PrefetchDesc& f, int r, const PW& pw) {
    f.ptr[r] = at<bf16>(c, pw.w);
    f.tiles[r] = pw.n_pad / 32;
    f.tile16[r] = pw.k_pad * 4;          // one 32-feature tile = k_pad * 32 bf16
  };
  const int this_slot = r.slot_r;
  auto pf_cache = [&](PrefetchDesc& f, int r, int layer) {
    f.ptr[r] = c->ws + w.kcache + (size_t)this_slot * w.kcache_slot + (size_t)layer * w.kcache_layer;
    f.tiles[r] = pchunks; f.tile16[r] = 1024;   // one key chunk = 16 KiB
    f.ptr[r + 1] = c->ws + w.vcache + (size_t)this_slot * w.vcache_slot + (size_t)layer * w.vcache_layer;
    f.tiles[r + 1] = pchunks; f.tile16[r + 1] = 1024;
  };
  const Tune& T = c->tune;
  // prefixes beyond 256 keys: the attention of the expert is shared out over ceil(chunks / 8) blocks per
  // (query tile, head); needs the 16 x 16 O projection (which merges the shares) and 8 heads of 256
  const int kcps = T.kcps;   // key chunks per share
  const int ksplits = (T.ae16 && T.ksplit && d.H == 8 && pchunks > kcps && ceil_div(pchunks, kcps) <= 4) ? ceil_div(pchunks, kcps) : 1;
  int o_splits = 1;
  // read-ahead kernel on its own stream, forked here and joined after the last Euler step (in a captured graph:
  // a branch beside the chain of compute launches); it replaces the warm-up blocks inside the launches
  bool ras = T.ras > 0 && r.read_ahead;
  for (int l = 1; ras && l < d.Le; l++) {   // one stride between layers for every region
    const WsTr &A = w.exp[l - 1], &B = w.exp[l];
    const size_t st = w.exp[1].qkv.w - w.exp[0].qkv.w;
    ras = B.qkv.w - A.qkv.w == st && B.o.w - A.o.w == st && B.gu.w - A.gu.w == st && B.down.w - A.down.w == st && st % 16 == 0;
  }
  // warm-up blocks inside the launches only where the read-ahead kernel was asked for but is not used (ras=0)
  const bool pfb = r.read_ahead && !ras;
  const int pfq = pfb ? T.pfq : 0, pfa = pfb ? T.pfa : 0, pfo = pfb ? T.pfo : 0, pfd = pfb ? T.pfd : 0;
  if (ras && !r.count_only && r.ok()) {
    ReadAheadParams ra;
    memset(&ra, 0, sizeof(ra));
    const WsTr& L0 = w.exp[0];
    const PW* pws[4] = {&L0.qkv, &L0.o, &L0.gu, &L0.down};
    const int cslot = 4;
    const size_t st = d.Le > 1 ? w.exp[1].qkv.w - w.exp[0].qkv.w : 0;
    for (int i = 0; i < 4; i++) {
      ra.base[i] = c->ws + pws[i]->w;
      ra.layer_stride[i] = st;
      ra.n16[i] = (unsigned)((size_t)pws[i]->n_pad * pws[i]->k_pad * 2 / 16);
    }
    ra.base[cslot] = c->ws + w.kcache + (size_t)this_slot * w.kcache_slot;
    ra.layer_stride[cslot] = w.kcache_layer;
    ra.n16[cslot] = (unsigned)pchunks * 1024;
    ra.base[cslot + 1] = c->ws + w.vcache + (size_t)this_slot * w.vcache_slot;
    ra.layer_stride[cslot + 1] = w.vcache_layer;
    ra.n16[cslot + 1] = (unsigned)pchunks * 1024;
    ra.layers = d.Le; ra.steps = d.steps; ra.lead = T.ral;
    ra.progress = ex<int>(r, w.progress);
    ra.wait_ticks = 50000;   // 0.5 ms
    ra.sink = ex<unsigned>(r, w.pf_sink);
    hipError_t e = c->ra_stream != nullptr ? hipSuccess : hipErrorNotReady;   // made by ensure_read_ahead, outside any capture
    if (e == hipSuccess) e = hipEventRecord(c->ev_fork, r.s);
    if (e == hipSuccess) e = hipStreamWaitEvent(c->ra_stream, c->ev_fork, 0);
    if (e == hipSuccess) e = launch_read_ahead(c->ra_stream, ra, T.ras, T.rat, T.rad);
    if (e == hipSuccess) e = hipEventRecord(c->ev_join, c->ra_stream);
    if (e != hipSuccess) r.err = e;
  }
  auto resid_gemm = [&](const PW& pw, const bf16* X, int K, const float* gain, const PrefetchDesc& pf) {
    if (pw.k_pad == 2048 || pw.k_pad == 4096) {
      const int tile = T.ae16 ? TILE_SKINNY16 : TILE_SKINNY_FULLK;
      GemmParams p = gp_base(c, pw, X, K, 64, tile, K);
      p.resid = ex<float>(r, w.y);
      p.out_f32 = ex<float>(r, w.y);
      p.out_bf16 = ex<bf16>(r, w.y_b);
      p.ldo = d.X; p.ldo2 = d.X; p.n_valid = d.X;
      p.stat_out = ex<float>(r, w.estat_parts);
      p.gain = gain;
      p.pf = pf;
      if (o_splits > 1) {
        p.xsplits = o_splits;
        p.xsplit_stride = (size_t)64 * d.H * 256;
        p.xsplit_ml = ex<float>(r, w.eml);
        o_splits = 1;
      }
      RUN_GEMM(r, tile, PRO_NONE, EPI_RESID, p, 1);
      stat_ptr = ex<float>(r, w.estat_parts);
      stat_parts = T.ae16 ? pw.n_pad / 16 : pw.n_pad / 32;
    } else {
      gemm_splitk_resid(r, pw, X, K, 64, K, ceil_div(pw.k_pad, 1024), 1024, nullptr, ex<float>(r, w.y), ex<bf16>(r, w.y_b),
                        d.X, TILE_SKINNY, ex<float>(r, w.estat), gain, nullptr, 0, false, true);
      stat_ptr = ex<float>(r, w.estat);
      stat_parts = 1;
    }
  };
  for (int k = 0; k < d.steps; k++) {
    // C1: folded action/time embedding, SiLU; suffix row 0 <- state token
    r.cls = PI0_OP_EXP_EMBED;
    RUN(r, launch_action_embed(r.s, xa, chunk, d.A, at<float>(c, w.wfold), at<float>(c, w.bias_tab) + (size_t)k * d.X, d.X,
                               ex<bf16>(r, w.z), ex<float>(r, w.stok), ex<float>(r, w.y), ex<bf16>(r, w.y_b),
                               at<float>(c, w.g_e1[0]), ex<float>(r, w.estat_parts)));
    {  // C2: second linear of the action/time MLP -> suffix rows 1..chunk; gain-scaled copy and per-tile row
       // statistics for the first layer's QKV come out of the same epilogue (row 0: from the kernel above)
      GemmParams p = gp_base(c, w.tout, ex<bf16>(r, w.z), d.X, chunk, TILE_SKINNY, d.X);
      p.bias = at<float>(c, w.tout.bias);
      p.out_f32 = ex<float>(r, w.y);
      p.out_bf16 = ex<bf16>(r, w.y_b);
      p.ldo = d.X; p.ldo2 = d.X; p.n_valid = d.X; p.row_offset = 1;
      p.gain = at<float>(c, w.g_e1[0]);
      p.stat_out = ex<float>(r, w.estat_parts);
      RUN_GEMM(r, TILE_SKINNY, PRO_NONE, EPI_RESID, p, 1);
    }
    stat_ptr = ex<float>(r, w.estat_parts);
    stat_parts = w.tout.n_pad / 32;
    const bool tap_this = taps && (k == 0 || k == d.steps - 1);
    for (int l = 0; l < d.Le; l++) {
      const WsTr& L = w.exp[l];
      bf16* kc = reinterpret_cast<bf16*>(c->ws + w.kcache + (size_t)r.slot_r * w.kcache_slot + (size_t)l * w.kcache_layer);
      bf16* vc = reinterpret_cast<bf16*>(c->ws + w.vcache + (size_t)r.slot_r * w.vcache_slot + (size_t)l * w.vcache_layer);
      {  // C3: RMS -> QKV, RoPE at positions P..P+63
        GemmParams p = gp_base(c, L.qkv, ex<bf16>(r, w.y_b), d.X, 64, TILE_SKINNY, d.X);
        p.rowstat = stat_ptr;
        p.rowstat_parts = stat_parts;
        p.out_bf16 = ex<bf16>(r, w.eq);
        p.q_mbs = 2;
        p.kfrag = ex<bf16>(r, w.ek); p.vfrag = ex<bf16>(r, w.ev);
        p.rope = at<float>(c, w.rope);
        p.pos0 = P;
        p.q_cols = d.H * 256; p.k_cols = 256;
        p.head_dim = 256; p.dqk_pad = 256; p.nvb = 8; p.kv_heads = 1; p.kv_chunks = 2;
        p.m_split = T.qms;
        p.pf = pf_begin(pfq);
        if (ras) { p.progress = ex<int>(r, w.progress); p.progress_value = k * d.Le + l + 1; }
        pf_weights(p.pf, 0, L.o);
        r.cls = PI0_OP_EXP_QKV;
        RUN_GEMM(r, TILE_SKINNY, PRO_RMS, EPI_QKV, p, 1);
      }
      {  // C4 + C5: scores, block mask, softmax, PV over [cache ; own keys]
        AttnParams a;
        memset(&a, 0, sizeof(a));
        a.q = ex<bf16>(r, w.eq); a.q_head_stride = 2 * 16 * 512;
        a.Tq = 64; a.heads = d.H;
        a.k0 = kc; a.v0 = vc; a.chunks0 = pchunks; a.valid0 = P;
        a.k1 = ex<bf16>(r, w.ek); a.v1 = ex<bf16>(r, w.ev); a.chunks1 = 2;
        a.suffix_mask = 1;
        a.scale = 1.0f / 16.0f;
        a.out = ex<bf16>(r, w.eattn); a.out_ld = d.H * 256; a.head_dim = 256;
        if (ksplits > 1) {   // long prefix: key shares over more blocks, merged by the O projection
          a.key_splits = ksplits;
          a.chunks_per_split = kcps;
          a.out_split_stride = (size_t)64 * d.H * 256;
          a.ml_out = ex<float>(r, w.eml);
        }
        a.v_split = T.avs > 0 ? T.avs : (ksplits == 1 ? 4 : 2);
        a.pf = pf_begin(pfa);
        pf_weights(a.pf, 0, L.gu);
        r.cls = PI0_OP_EXP_ATTN;
        RUN(r, launch_attention(r.s, a));
      }
      // C6: O-projection + residual
      {
        PrefetchDesc f = pf_begin(pfo);
        pf_weights(f, 0, L.down);
        r.cls = PI0_OP_EXP_O;
        o_splits = ksplits;
        resid_gemm(L.o, ex<bf16>(r, w.eattn), d.H * 256, at<float>(c, w.g_e2[l]), f);
      }
      {  // C7: RMS -> gate||up, fused gate
        GemmParams p = gp_base(c, L.gu, ex<bf16>(r, w.y_b), d.X, 64, TILE_SKINNY, d.X);
        p.rowstat = stat_ptr;
        p.rowstat_parts = stat_parts;
        p.out_bf16 = ex<bf16>(r, w.emid);
        p.ldo = d.Fx;
        r.cls = PI0_OP_EXP_GATEUP;
        RUN_GEMM(r, TILE_SKINNY, PRO_RMS, EPI_GEGLU, p, 1);
      }
      // C8: down + residual
      {
        // the gate||up launch fills every CU by itself, so the launch after it reads ahead for two
        const int nl = l + 1 < d.Le ? l + 1 : 0;
        PrefetchDesc f = pf_begin(pfd);
        pf_weights(f, 0, w.exp[nl].qkv);
        pf_cache(f, 1, nl);
        r.cls = PI0_OP_EXP_DOWN;
        resid_gemm(L.down, ex<bf16>(r, w.emid), d.Fx, at<float>(c, l + 1 < d.Le ? w.g_e1[l + 1] : w.g_ef), f);
      }
      if (tap_this) {
        // step 0 taps first, last-step taps after them
        const size_t slot = (k == 0 ? 0 : (size_t)d.Le) + l;
        if (taps->base && !r.count_only && r.ok())
          r.did(launch_copy_f32(r.s, ex<float>(r, w.y), taps->base + tap_step_base + slot * 64 * d.X, (size_t)64 * d.X));
      }
    }
    {  // C9: final RMS -> out-projection (+bias), Euler update x <- x + dt * v
      GemmParams p = gp_base(c, w.outp, ex<bf16>(r, w.y_b), d.X, 64, TILE_SKINNY, d.X);
      p.rowstat = stat_ptr;
      p.rowstat_parts = stat_parts;
      p.bias = at<float>(c, w.outp.bias);
      p.out_f32 = xa;
      p.ldo = d.A; p.n_valid = d.A; p.dt = dt;
      r.cls = PI0_OP_EXP_OUT;
      RUN_GEMM(r, TILE_SKINNY, PRO_RMS, EPI_EULER, p, 1);
      r.cls = PI0_OP_MISC;
    }
    if (taps && taps->base && !r.count_only && r.ok()) {
      const size_t xoff = tap_step_base + (size_t)2 * d.Le * 64 * d.X + (size_t)k * chunk * d.A;
      r.did(launch_copy_f32(r.s, xa, taps->base + xoff, (size_t)chunk * d.A));
    }
  }
  if (ras && !r.count_only && r.ok()) {
    const hipError_t e = hipStreamWaitEvent(r.s, c->ev_join, 0);
    if (e != hipSuccess) r.err = e;
  }
  if (taps) taps->off = tap_step_base + (size_t)2 * d.Le * 64 * d.X + (size_t)d.steps * chunk * d.A;
}

// inputs -> static staging buffers (replayed graphs read constant addresses)
struct CopySeg { const uint32_t* src; uint32_t* dst; unsigned n; };
struct CopyArgs { CopySeg seg[4]; };
__global__ __launch_bounds__(256) void copy_segments_kernel(CopyArgs a) {
  const CopySeg s = a.seg[blockIdx.y];
  for (unsigned i = blockIdx.x * 256 + threadIdx.x; i < s.n; i += gridDim.x * 256) s.dst[i] = s.src[i];
}

hipError_t stage_inputs(pi0_ctx* c, hipStream_t s, const float* images, int n_views, const int32_t* ids, int n_prompt,
                        const float* state, const float* noise, unsigned char* ebase = nullptr) {
  Run where{c, s, false};   // only to say where the expert's scratch block is
  where.ebase = ebase;
  CopyArgs a;
  memset(&a, 0, sizeof(a));
  int n = 0;
  if (images) {
    a.seg[n++] = CopySeg{reinterpret_cast<const uint32_t*>(images), at<uint32_t>(c, c->wl.st_images),
                         (unsigned)((size_t)n_views * c->cfg.img_size * c->cfg.img_size * 3)};
  }
  if (ids && n_prompt > 0) {
    a.seg[n++] = CopySeg{reinterpret_cast<const uint32_t*>(ids), at<uint32_t>(c, c->wl.st_ids), (unsigned)n_prompt};
  }
  if (state) a.seg[n++] = CopySeg{reinterpret_cast<const uint32_t*>(state), ex<uint32_t>(where, c->wl.st_state), (unsigned)c->d.SD};
  if (noise) {
    a.seg[n++] = CopySeg{reinterpret_cast<const uint32_t*>(noise), ex<uint32_t>(where, c->wl.st_noise),
                         (unsigned)(c->cfg.chunk * c->d.A)};
  }
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_segments_kernel, dim3(64, n), dim3(256), 0, s, a);
  return hipGetLastError();
}

int fail_hip(pi0_ctx* c, hipError_t e) {
  c->last_hip = (int)e;
  return PI0_EHIP;
}

// stream and events of the read-ahead kernel (not created while a stream is being captured)
hipError_t ensure_read_ahead(pi0_ctx* c) {
  if (c->tune.ras <= 0) return hipSuccess;
  hipError_t e = hipSuccess;
  if (c->ra_stream == nullptr) e = hipStreamCreateWithFlags(&c->ra_stream, hipStreamNonBlocking);
  if (e == hipSuccess && c->ev_fork == nullptr) e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess && c->ev_join == nullptr) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
  return e;
}

// grid of the persistent denoise loop inside a two-stream frame (0: per-operation launches)
int frame_loop_blocks(const pi0_ctx* c, int P) {
  if (c->tune.psb >= 0) return c->tune.psb;
  return P <= 256 ? 160 : P <= 512 ? 128 : P <= 768 ? 96 : 128;   // measured optima at 256 / 512 / 768 / 816 prefix tokens
}

// Runs `kind` either through a cached graph or eagerly.
int execute(pi0_ctx* c, int kind, int n_views, int n_prompt, hipStream_t s, int slot_w = -1, int slot_r = -1, bool read_ahead = true) {
  const int P = n_views * c->d.T + n_prompt;
  if (slot_w < 0) slot_w = c->cur_slot;
  if (slot_r < 0) slot_r = c->cur_slot;
  // the second stream of the read-ahead kernel exists only where the per-operation launches will use it (a stream
  // that is never used still takes one of the process's few hardware queues from the streams that are)
  if (kind != KIND_PREFILL && read_ahead && !persistent_feasible(c, P)) {
    if (const hipError_t e = ensure_read_ahead(c); e != hipSuccess) return fail_hip(c, e);
  }
  auto body = [&](Run& r) {
    if (kind == KIND_PREFILL || kind == KIND_INFER) run_prefill(r, n_views, n_prompt, nullptr);
    if (kind == KIND_DENOISE || kind == KIND_INFER) run_denoise(r, P, nullptr);
  };
  if (!c->graph_mode || s == nullptr) {   // the legacy default stream cannot be captured
    Run r{c, s, false};
    r.slot_w = slot_w;
    r.slot_r = slot_r;
    r.read_ahead = read_ahead;
    // two-stream frames: per-operation launches, or the loop on a part of the chip (the prefill's blocks need compute units too)
    r.persist_blocks = read_ahead ? 0 : frame_loop_blocks(c, P);
    r.persistent_ok = read_ahead || r.persist_blocks > 0;
    body(r);
    return r.ok() ? PI0_OK : fail_hip(c, r.err);
  }
  GraphKey key{kind, n_views, n_prompt, kind == KIND_DENOISE ? 0 : slot_w, kind == KIND_PREFILL ? 0 : slot_r,
               kind == KIND_DENOISE ? 0 : c->precision, kind == KIND_PREFILL ? 0 : (int)read_ahead};
  auto it = c->graphs.find(key);
  if (it == c->graphs.end()) {
    hipError_t e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return fail_hip(c, e);
    Run r{c, s, false};
    r.slot_w = slot_w;
    r.slot_r = slot_r;
    r.read_ahead = read_ahead;
    // two-stream frames: per-operation launches, or the loop on a part of the chip (the prefill's blocks need compute units too)
    r.persist_blocks = read_ahead ? 0 : frame_loop_blocks(c, P);
    r.persistent_ok = read_ahead || r.persist_blocks > 0;
    body(r);
    hipGraph_t g = nullptr;
    e = hipStreamEndCapture(s, &g);
    if (!r.ok() || e != hipSuccess || g == nullptr) {
      if (g) (void)hipGraphDestroy(g);
      return fail_hip(c, r.ok() ? e : r.err);
    }
    hipGraphExec_t ge = nullptr;
    e = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
    (void)hipGraphDestroy(g);
    if (e != hipSuccess) return fail_hip(c, e);
    it = c->graphs.emplace(key, ge).first;
  }
  hipError_t e = hipGraphLaunch(it->second, s);
  return e == hipSuccess ? PI0_OK : fail_hip(c, e);
}

bool check_prefill_args(const pi0_ctx* c, const float* images, int n_views, const int32_t* ids, int n_prompt) {
  if (images == nullptr) return false;
  if (n_views < 1 || n_views > c->cfg.max_views) return false;
  if (n_prompt < 0 || n_prompt > c->cfg.max_prompt) return false;
  if (n_prompt > 0 && (ids == nullptr || c->cfg.vocab <= 0)) return false;
  return true;
}

}  // namespace

// ==================================================================================================
// Static scratch of pi0_denoise_static: the expert's scratch block for callers that cannot provide or allocate
// device memory beyond inputs and outputs at call time.  One copy per device, held until the process ends.  The
// array's name is only a host-side handle; its device address is looked up once per device (with that device
// current) and used everywhere.  Calls that overlap in time on one device share it and would race.
// ==================================================================================================
static __device__ __align__(256) unsigned char scratch[PI0_STATIC_SCRATCH_BYTES];

namespace {
const int MAX_DEVICES = 64;
unsigned char* g_static_scratch[MAX_DEVICES] = {};

// device address of `scratch` on the current device (looked up on first use per device)
hipError_t static_scratch_ptr(int* dev_out, unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (g_static_scratch[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_static_scratch[dev] = reinterpret_cast<unsigned char*>(p);
  }
  *dev_out = dev;
  *out = g_static_scratch[dev];
  return hipSuccess;
}
}  // namespace

// ==================================================================================================
// C ABI
// ==================================================================================================
extern "C" {

const char* pi0_strerror(int code) {
  switch (code) {
    case PI0_OK: return "ok";
    case PI0_EINVAL: return "invalid argument";
    case PI0_ESTATE: return "invalid state (weights not loaded or no valid prefill)";
    case PI0_ENOMEM: return "buffer too small or out of host memory";
    case PI0_EFORMAT: return "weight blob size does not match the configuration";
    case PI0_EHIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

int pi0_create(const pi0_config* cfg, pi0_ctx** out) {
  if (cfg == nullptr || out == nullptr) return PI0_EINVAL;
  Dims d;
  if (!derive_dims(*cfg, d)) return PI0_EINVAL;
  pi0_ctx* c = new (std::nothrow) pi0_ctx();
  if (c == nullptr) return PI0_ENOMEM;
  c->cfg = *cfg;
  c->d = d;
  blob_layout(*cfg, d, c->bl);
  ws_layout(*cfg, d, c->wl);

  // RoPE table (Section 3.2: precomputed): angle = pos * 10000^(-i/128), pairs (i, i+128)
  c->h_rope.resize((size_t)d.maxpos * 128 * 2);
  for (int pos = 0; pos < d.maxpos; pos++) {
    for (int i = 0; i < 128; i++) {
      const double ang = (double)pos * pow(10000.0, -(double)i / 128.0);
      c->h_rope[((size_t)pos * 128 + i) * 2] = (float)cos(ang);
      c->h_rope[((size_t)pos * 128 + i) * 2 + 1] = (float)sin(ang);
    }
  }
  // time encodings of the Euler steps: sin || cos, periods log-spaced from 4e-3 to 4
  c->h_tau.resize((size_t)d.steps * d.X);
  const int half = d.X / 2;
  for (int k = 0; k < d.steps; k++) {
    const double t = 1.0 - (double)k / d.steps;
    for (int j = 0; j < half; j++) {
      const double frac = half > 1 ? (double)j / (half - 1) : 0.0;
      const double period = 4e-3 * pow(4.0 / 4e-3, frac);
      const double ang = 2.0 * M_PI * t / period;
      c->h_tau[(size_t)k * d.X + j] = (float)sin(ang);
      c->h_tau[(size_t)k * d.X + half + j] = (float)cos(ang);
    }
  }
  *out = c;
  return PI0_OK;
}

void pi0_destroy(pi0_ctx* c) {
  if (c == nullptr) return;
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  for (int i = 0; i < 2; i++) {
    if (c->ev_prefill[i]) (void)hipEventDestroy(c->ev_prefill[i]);
    if (c->ev_denoise[i]) (void)hipEventDestroy(c->ev_denoise[i]);
  }
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  if (c->ra_stream) (void)hipStreamDestroy(c->ra_stream);
  delete c;
}

size_t pi0_weights_bytes(const pi0_config* cfg) {
  Dims d;
  if (cfg == nullptr || !derive_dims(*cfg, d)) return 0;
  BlobLayout b;
  blob_layout(*cfg, d, b);
  return b.total * 2;
}

size_t pi0_workspace_bytes(const pi0_config* cfg) {
  Dims d;
  if (cfg == nullptr || !derive_dims(*cfg, d)) return 0;
  WsLayout w;
  ws_layout(*cfg, d, w);
  return w.total;
}

int pi0_tune(pi0_ctx* c, const char* env) {
  if (c == nullptr || env == nullptr) return PI0_EINVAL;
  {
    struct { const char* key; int* dst; int lo, hi; } keys[] = {
        {"vis", &c->tune.vis, 0, 11},   {"lqkv", &c->tune.lqkv, 0, 11}, {"lgu", &c->tune.lgu, 0, 10},
        {"vqkv", &c->tune.vqkv, -1, 11}, {"vup", &c->tune.vup, -1, 11},
        {"vo", &c->tune.vo, 0, 11}, {"vd", &c->tune.vd, 0, 11}, {"lo", &c->tune.lo, 0, 11}, {"ld", &c->tune.ld, 0, 10}, {"zvo", &c->tune.zvo, 1, Z_MAX}, {"zlo", &c->tune.zlo, 1, Z_MAX},
        {"zld", &c->tune.zld, 1, Z_MAX}, {"zvd", &c->tune.zvd, 1, Z_MAX},
        {"pfq", &c->tune.pfq, 0, 1024}, {"pfa", &c->tune.pfa, 0, 1024}, {"pfo", &c->tune.pfo, 0, 1024},
        {"pfd", &c->tune.pfd, 0, 1024}, {"ae16", &c->tune.ae16, 0, 1}, {"ksplit", &c->tune.ksplit, 0, 1}, {"kcps", &c->tune.kcps, 2, 16}, {"qms", &c->tune.qms, 0, 1},
        {"fko", &c->tune.fko, 0, 1}, {"fkl", &c->tune.fkl, 0, 1}, {"ras", &c->tune.ras, 0, 4096}, {"ral", &c->tune.ral, 1, 8}, {"rat", &c->tune.rat, 64, 256}, {"rad", &c->tune.rad, 1, 8 /* 7: no such variant, see below */}, {"avs", &c->tune.avs, 1, 8}, {"pdn", &c->tune.pdn, 0, 1}, {"pra", &c->tune.pra, 0, 63}, {"psb", &c->tune.psb, -1, 256}};
    for (auto& k : keys) {
      const char* f = strstr(env, k.key);
      while (f != nullptr && !((f == env || f[-1] == ',') && f[strlen(k.key)] == '=')) f = strstr(f + 1, k.key);
      if (f != nullptr) {
        const int v = atoi(f + strlen(k.key) + 1);
        if (v >= k.lo && v <= k.hi) *k.dst = v;
      }
    }
    for (int* v : {&c->tune.pfq, &c->tune.pfa, &c->tune.pfo, &c->tune.pfd}) *v &= ~15;
    if (c->tune.rad == 7) c->tune.rad = 6;   // the read-ahead kernel exists with 1 .. 6 and 8 loads in flight
  }
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  c->graphs.clear();
  return PI0_OK;
}

int pi0_loop_trace_ops(const pi0_ctx* c) { return c ? 1 + c->d.steps * (3 + 5 * c->d.Le) : 0; }

int pi0_set_loop_trace(pi0_ctx* c, long long* d_trace, int ops_cap) {
  if (c == nullptr || ops_cap < 0 || (d_trace == nullptr) != (ops_cap == 0) || (reinterpret_cast<uintptr_t>(d_trace) & 7) != 0) return PI0_EINVAL;
  c->loop_trace = d_trace;
  c->loop_trace_ops = ops_cap;
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  c->graphs.clear();
  return PI0_OK;
}

int pi0_set_graph_mode(pi0_ctx* c, int enabled) {
  if (c == nullptr) return PI0_EINVAL;
  c->graph_mode = enabled != 0;
  return PI0_OK;
}

int pi0_set_precision(pi0_ctx* c, int precision) {
  if (c == nullptr || (precision != PI0_PRECISION_BF16 && precision != PI0_PRECISION_MXFP8_PREFIX_MLP)) return PI0_EINVAL;
  if (precision == PI0_PRECISION_MXFP8_PREFIX_MLP && !c->wl.mx_ok) return PI0_EINVAL;   // widths not multiples of 256
  c->precision = precision;
  return PI0_OK;
}

int pi0_last_hip_error(const pi0_ctx* c) { return c ? c->last_hip : 0; }

int pi0_device_status(pi0_ctx* c, void* hip_stream) {
  if (c == nullptr) return PI0_EINVAL;
  if (!c->loaded) return PI0_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  unsigned flag = 0;
  hipError_t e = hipMemcpyAsync(&flag, at<unsigned>(c, c->wl.esync) + GB_ERR, sizeof(flag), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(c, e);
  return flag == 0u ? PI0_OK : PI0_ESTATE;
}

int pi0_kernel_count(const pi0_ctx* c, int n_views, int n_prompt) {
  if (c == nullptr || n_views < 1 || n_views > c->cfg.max_views || n_prompt < 0 || n_prompt > c->cfg.max_prompt) return 0;
  Run r{const_cast<pi0_ctx*>(c), nullptr, true};
  r.persistent_ok = true;
  run_prefill(r, n_views, n_prompt, nullptr);
  run_denoise(r, n_views * c->d.T + n_prompt, nullptr);
  return r.launches;
}

int pi0_load_weights(pi0_ctx* c, const void* d_blob, size_t blob_bytes, void* d_workspace, size_t ws_bytes, void* hip_stream) {
  if (c == nullptr || d_blob == nullptr || d_workspace == nullptr) return PI0_EINVAL;
  if ((reinterpret_cast<uintptr_t>(d_workspace) & 255) != 0 || (reinterpret_cast<uintptr_t>(d_blob) & 15) != 0) return PI0_EINVAL;
  if (blob_bytes != c->bl.total * 2) return PI0_EFORMAT;
  if (ws_bytes < c->wl.total) return PI0_ENOMEM;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  const Dims& d = c->d;
  const BlobLayout& b = c->bl;
  const WsLayout& w = c->wl;
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  c->graphs.clear();
  c->loaded = false;
  c->cur_views = 0;
  c->ws = reinterpret_cast<unsigned char*>(d_workspace);
  const bf16* B = reinterpret_cast<const bf16*>(d_blob);
  hipError_t e;
  if (!c->attrs_set) {
    e = gemm_init_attributes();
    if (e != hipSuccess) return fail_hip(c, e);
    e = attention_init_attributes();
    if (e != hipSuccess) return fail_hip(c, e);
    e = gemm_mx_init_attributes();
    if (e != hipSuccess) return fail_hip(c, e);
    e = expert_loop_init_attributes();
    if (e != hipSuccess) return fail_hip(c, e);
    {  // the persistent kernel's barrier needs all of its blocks resident: one per compute unit, 256 of them
      int dev = 0, cus = 0, per_cu = 0;
      e = hipGetDevice(&dev);
      if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      if (e == hipSuccess) e = expert_loop_max_blocks_per_cu(&per_cu);
      if (e != hipSuccess) return fail_hip(c, e);
      c->pk_ok = cus >= PK_BLOCKS && per_cu >= 1;
    }
    c->attrs_set = true;
  }
  e = static_scratch_ptr(&c->device, &c->static_scratch);
  if (e != hipSuccess) return fail_hip(c, e);
#define TRY(call) do { e = (call); if (e != hipSuccess) return fail_hip(c, e); } while (0)
  TRY(launch_fill_zero(s, c->ws + w.act_begin, w.total - w.act_begin));
  TRY(hipMemcpyAsync(c->ws + w.rope, c->h_rope.data(), c->h_rope.size() * 4, hipMemcpyHostToDevice, s));
  TRY(hipMemcpyAsync(c->ws + w.tau, c->h_tau.data(), c->h_tau.size() * 4, hipMemcpyHostToDevice, s));

  auto pack = [&](const PW& pw, PackSrc src, const bf16* ln_bias, const bf16* b0, const bf16* b1, const bf16* b2) -> hipError_t {
    hipError_t ee = launch_pack_weights(s, src, at<bf16>(c, pw.w), pw.n_pad, pw.k_pad);
    if (ee != hipSuccess) return ee;
    if (pw.colsum != 0 || pw.bias != 0) {
      const bf16* bs[3] = {b0, b1, b2};
      ee = launch_fold_vectors(s, src, ln_bias, bs, pw.colsum ? at<float>(c, pw.colsum) : nullptr,
                               pw.bias ? at<float>(c, pw.bias) : nullptr, pw.n_pad);
    }
    return ee;
  };
  auto src1 = [&](size_t off, int K, int N, int kscale, size_t gain_off) {
    PackSrc p;
    memset(&p, 0, sizeof(p));
    p.src[0] = B + off; p.cols[0] = N;
    p.K = K; p.n_true = N; p.rowmap = ROWMAP_CONCAT; p.kscale = kscale;
    p.gain = kscale != KSCALE_NONE ? B + gain_off : nullptr;
    return p;
  };
  // vision
  TRY(pack(w.patch, src1(b.patch_w, d.PD, d.Dv, KSCALE_NONE, 0), nullptr, B + b.patch_b, nullptr, nullptr));
  TRY(launch_bf16_to_f32(s, B + b.pos, at<float>(c, w.pos), (size_t)d.T * d.Dv));
  for (int l = 0; l < d.Lv; l++) {
    const BlobVis& v = b.vis[l];
    PackSrc q = src1(v.wq, d.Dv, d.Dv, KSCALE_GAIN, v.ln1g);
    q.src[1] = B + v.wk; q.cols[1] = d.Dv;
    q.src[2] = B + v.wv; q.cols[2] = d.Dv;
    q.n_true = 3 * d.Dv;
    TRY(pack(w.vis[l].qkv, q, B + v.ln1b, B + v.bq, B + v.bk, B + v.bv));
    TRY(pack(w.vis[l].o, src1(v.wo, d.Dv, d.Dv, KSCALE_NONE, 0), nullptr, B + v.bo, nullptr, nullptr));
    TRY(pack(w.vis[l].up, src1(v.w1, d.Dv, d.Fv, KSCALE_GAIN, v.ln2g), B + v.ln2b, B + v.b1, nullptr, nullptr));
    TRY(pack(w.vis[l].down, src1(v.w2, d.Fv, d.Dv, KSCALE_NONE, 0), nullptr, B + v.b2, nullptr, nullptr));
  }
  for (int l = 0; l < d.Lv; l++) {
    TRY(launch_gain_vector(s, B + b.vis[l].ln1g, at<float>(c, w.g_v1[l]), d.Dv, 0));
    TRY(launch_gain_vector(s, B + b.vis[l].ln2g, at<float>(c, w.g_v2[l]), d.Dv, 0));
  }
  TRY(launch_gain_vector(s, B + b.lnfg, at<float>(c, w.g_vf), d.Dv, 0));
  for (int l = 0; l < d.Ll; l++) {
    TRY(launch_gain_vector(s, B + b.llm[l].g_attn, at<float>(c, w.g_l1[l]), d.E, 1));
    TRY(launch_gain_vector(s, B + b.llm[l].g_mlp, at<float>(c, w.g_l2[l]), d.E, 1));
  }
  for (int l = 0; l < d.Le; l++) {
    TRY(launch_gain_vector(s, B + b.exp[l].g_attn, at<float>(c, w.g_e1[l]), d.X, 1));
    TRY(launch_gain_vector(s, B + b.exp[l].g_mlp, at<float>(c, w.g_e2[l]), d.X, 1));
  }
  TRY(launch_gain_vector(s, B + b.g_final, at<float>(c, w.g_ef), d.X, 1));
  TRY(pack(w.proj, src1(b.proj_w, d.Dv, d.E, KSCALE_GAIN, b.lnfg), B + b.lnfb, B + b.proj_b, nullptr, nullptr));
  if (c->cfg.vocab > 0) TRY(launch_copy_bf16(s, B + b.embed, at<bf16>(c, w.embed), (size_t)c->cfg.vocab * d.E));
  // prefix and expert transformers
  auto pack_tr = [&](const std::vector<BlobTr>& bt, const std::vector<WsTr>& wt, int L, int W, int M, bool skip_last) -> hipError_t {
    for (int l = 0; l < L; l++) {
      const BlobTr& t = bt[l];
      const bool last = skip_last && l == L - 1;
      PackSrc q;
      memset(&q, 0, sizeof(q));
      q.src[0] = B + t.wq; q.cols[0] = d.H * 256;
      q.src[1] = B + t.wk; q.cols[1] = 256;
      q.src[2] = B + t.wv; q.cols[2] = 256;
      q.K = W; q.rowmap = ROWMAP_ROPE_QKV; q.kscale = KSCALE_ONE_PLUS; q.gain = B + t.g_attn;
      q.q_heads = last ? 0 : d.H;
      q.n_true = (q.q_heads + 2) * 256;
      hipError_t ee = launch_pack_weights(s, q, at<bf16>(c, wt[l].qkv.w), wt[l].qkv.n_pad, wt[l].qkv.k_pad);
      if (ee != hipSuccess) return ee;
      if (last) continue;
      ee = launch_pack_weights(s, src1(t.wo, d.H * 256, W, KSCALE_NONE, 0), at<bf16>(c, wt[l].o.w), wt[l].o.n_pad, wt[l].o.k_pad);
      if (ee != hipSuccess) return ee;
      PackSrc g;
      memset(&g, 0, sizeof(g));
      g.src[0] = B + t.wg; g.cols[0] = M;
      g.src[1] = B + t.wu; g.cols[1] = M;
      g.K = W; g.n_true = 2 * M; g.rowmap = ROWMAP_PAIR; g.kscale = KSCALE_ONE_PLUS; g.gain = B + t.g_mlp;
      ee = launch_pack_weights(s, g, at<bf16>(c, wt[l].gu.w), wt[l].gu.n_pad, wt[l].gu.k_pad);
      if (ee != hipSuccess) return ee;
      ee = launch_pack_weights(s, src1(t.wd, M, W, KSCALE_NONE, 0), at<bf16>(c, wt[l].down.w), wt[l].down.n_pad, wt[l].down.k_pad);
      if (ee != hipSuccess) return ee;
      if (wt[l].gu8 != 0) {   // MXFP8 copies for the reduced-precision mode (same row maps)
        ee = launch_pack_weights_mx(s, g, c->ws + wt[l].gu8, c->ws + wt[l].gu8s, wt[l].gu.n_pad, wt[l].gu.k_pad);
        if (ee != hipSuccess) return ee;
        ee = launch_pack_weights_mx(s, src1(t.wd, M, W, KSCALE_NONE, 0), c->ws + wt[l].down8, c->ws + wt[l].down8s, wt[l].down.n_pad,
                                    wt[l].down.k_pad);
        if (ee != hipSuccess) return ee;
      }
    }
    return hipSuccess;
  };
  TRY(pack_tr(b.llm, w.llm, d.Ll, d.E, d.F, true));
  TRY(pack_tr(b.exp, w.exp, d.Le, d.X, d.Fx, false));
  // expert input / output heads
  TRY(launch_bf16_to_f32(s, B + b.state_w, at<float>(c, w.state_w), (size_t)d.SD * d.X));
  TRY(launch_bf16_to_f32(s, B + b.state_b, at<float>(c, w.state_b), (size_t)d.X));
  TRY(launch_time_fold(s, B + b.ain_w, B + b.ain_b, B + b.tin_w, B + b.tin_b, at<float>(c, w.tau), d.A, d.X, d.steps,
                       at<float>(c, w.wfold), at<float>(c, w.bias_tab)));
  TRY(pack(w.tout, src1(b.tout_w, d.X, d.X, KSCALE_NONE, 0), nullptr, B + b.tout_b, nullptr, nullptr));
  TRY(pack(w.outp, src1(b.out_w, d.X, d.A, KSCALE_ONE_PLUS, b.g_final), nullptr, B + b.out_b, nullptr, nullptr));
#undef TRY
  c->loaded = true;
  return PI0_OK;
}

int pi0_prefill(pi0_ctx* c, const float* d_images, int n_views, const int32_t* d_prompt_ids, int n_prompt, void* hip_stream) {
  if (c == nullptr) return PI0_EINVAL;
  if (!check_prefill_args(c, d_images, n_views, d_prompt_ids, n_prompt)) return PI0_EINVAL;
  if (!c->loaded) return PI0_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  c->cur_views = 0;
  hipError_t e = stage_inputs(c, s, d_images, n_views, d_prompt_ids, n_prompt, nullptr, nullptr);
  if (e != hipSuccess) return fail_hip(c, e);
  int rc = execute(c, KIND_PREFILL, n_views, n_prompt, s);
  if (rc != PI0_OK) return rc;
  if (c->ev_prefill[c->cur_slot] != nullptr) {
    e = hipEventRecord(c->ev_prefill[c->cur_slot], s);
    if (e != hipSuccess) return fail_hip(c, e);
  }
  c->cur_views = n_views;
  c->cur_prompt = n_prompt;
  return PI0_OK;
}

int pi0_denoise(pi0_ctx* c, const float* d_state, const float* d_noise, float* d_actions, void* hip_stream) {
  if (c == nullptr || d_state == nullptr || d_noise == nullptr || d_actions == nullptr) return PI0_EINVAL;
  if (!c->loaded || c->cur_views == 0) return PI0_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  hipError_t e = stage_inputs(c, s, nullptr, 0, nullptr, 0, d_state, d_noise);
  if (e != hipSuccess) return fail_hip(c, e);
  int rc = execute(c, KIND_DENOISE, c->cur_views, c->cur_prompt, s);
  if (rc != PI0_OK) return rc;
  e = launch_copy_f32(s, at<float>(c, c->wl.xa), d_actions, (size_t)c->cfg.chunk * c->d.A);
  return e == hipSuccess ? PI0_OK : fail_hip(c, e);
}

int pi0_denoise_static(pi0_ctx* c, const float* d_state, const float* d_noise, float* d_actions, void* hip_stream) {
  if (c == nullptr || d_state == nullptr || d_noise == nullptr || d_actions == nullptr) return PI0_EINVAL;
  if (c->wl.es_end - c->wl.es_begin > (size_t)PI0_STATIC_SCRATCH_BYTES) return PI0_ENOMEM;   // this geometry needs more than the static array holds
  if (!c->loaded || c->cur_views == 0) return PI0_ESTATE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != c->device || c->static_scratch == nullptr) return PI0_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  // the block's workspace offsets, rebased onto the static array (integer arithmetic: the sum is only ever
  // dereferenced at offsets inside [es_begin, es_end))
  unsigned char* ebase = reinterpret_cast<unsigned char*>(reinterpret_cast<uintptr_t>(c->static_scratch) - c->wl.es_begin);
  hipError_t e = stage_inputs(c, s, nullptr, 0, nullptr, 0, d_state, d_noise, ebase);
  if (e != hipSuccess) return fail_hip(c, e);
  Run r{c, s, false};
  r.slot_r = c->cur_slot;
  r.read_ahead = false;     // no second stream, no events: nothing is created here
  r.persistent_ok = false;  // per-operation launches, eagerly (a caller may be capturing the stream itself)
  r.ebase = ebase;
  run_denoise(r, c->cur_views * c->d.T + c->cur_prompt, nullptr);
  if (!r.ok()) return fail_hip(c, r.err);
  e = launch_copy_f32(s, ex<float>(r, c->wl.xa), d_actions, (size_t)c->cfg.chunk * c->d.A);
  return e == hipSuccess ? PI0_OK : fail_hip(c, e);
}

int pi0_infer(pi0_ctx* c, const float* d_images, int n_views, const int32_t* d_prompt_ids, int n_prompt, const float* d_state,
              const float* d_noise, float* d_actions, void* hip_stream) {
  if (c == nullptr || d_state == nullptr || d_noise == nullptr || d_actions == nullptr) return PI0_EINVAL;
  if (!check_prefill_args(c, d_images, n_views, d_prompt_ids, n_prompt)) return PI0_EINVAL;
  if (!c->loaded) return PI0_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  c->cur_views = 0;
  hipError_t e = stage_inputs(c, s, d_images, n_views, d_prompt_ids, n_prompt, d_state, d_noise);
  if (e != hipSuccess) return fail_hip(c, e);
  int rc = execute(c, KIND_INFER, n_views, n_prompt, s);
  if (rc != PI0_OK) return rc;
  if (c->ev_prefill[c->cur_slot] != nullptr) {
    e = hipEventRecord(c->ev_prefill[c->cur_slot], s);
    if (e != hipSuccess) return fail_hip(c, e);
  }
  c->cur_views = n_views;
  c->cur_prompt = n_prompt;
  e = launch_copy_f32(s, at<float>(c, c->wl.xa), d_actions, (size_t)c->cfg.chunk * c->d.A);
  return e == hipSuccess ? PI0_OK : fail_hip(c, e);
}

int pi0_stream_frame(pi0_ctx* c, const float* d_images, int n_views, const int32_t* d_prompt_ids, int n_prompt,
                     const float* d_state, const float* d_noise, float* d_actions, void* stream_prefill, void* stream_denoise) {
  if (c == nullptr || d_state == nullptr || d_noise == nullptr || d_actions == nullptr) return PI0_EINVAL;
  if (stream_prefill == nullptr || stream_denoise == nullptr || stream_prefill == stream_denoise) return PI0_EINVAL;
  if (!check_prefill_args(c, d_images, n_views, d_prompt_ids, n_prompt)) return PI0_EINVAL;
  if (!c->loaded || c->cur_views == 0) return PI0_ESTATE;
  hipStream_t sp = reinterpret_cast<hipStream_t>(stream_prefill), sd = reinterpret_cast<hipStream_t>(stream_denoise);
  hipError_t e = hipSuccess;
  const int cur = c->cur_slot, nxt = 1 - cur;
  const bool first_use = c->ev_prefill[0] == nullptr;
  for (int i = 0; i < 2 && e == hipSuccess; i++) {
    if (c->ev_prefill[i] == nullptr) e = hipEventCreateWithFlags(&c->ev_prefill[i], hipEventDisableTiming);
    if (e == hipSuccess && c->ev_denoise[i] == nullptr) e = hipEventCreateWithFlags(&c->ev_denoise[i], hipEventDisableTiming);
  }
  // first frame: the priming prefill was enqueued on stream_prefill before events existed
  if (e == hipSuccess && first_use) e = hipEventRecord(c->ev_prefill[cur], sp);
  if (e != hipSuccess) return fail_hip(c, e);
  // prefill of this frame into the other cache copy, once the last denoise that read that copy is done
  e = hipStreamWaitEvent(sp, c->ev_denoise[nxt], 0);
  if (e == hipSuccess) e = stage_inputs(c, sp, d_images, n_views, d_prompt_ids, n_prompt, nullptr, nullptr);
  if (e != hipSuccess) return fail_hip(c, e);
  int rc = execute(c, KIND_PREFILL, n_views, n_prompt, sp, nxt, nxt);
  if (rc != PI0_OK) return rc;
  e = hipEventRecord(c->ev_prefill[nxt], sp);
  // denoise against the copy the previous frame filled
  if (e == hipSuccess) e = hipStreamWaitEvent(sd, c->ev_prefill[cur], 0);
  if (e == hipSuccess) e = stage_inputs(c, sd, nullptr, 0, nullptr, 0, d_state, d_noise);
  if (e != hipSuccess) return fail_hip(c, e);
  // The denoise of a frame is the persistent loop on a part of the chip (frame_loop_blocks): a resident block of the
  // loop holds a whole compute unit, so its grid is what shares the chip between the two streams - the prefill's blocks
  // run on the compute units it leaves (measured at 1 view: 7.8 ms per frame with 160 blocks, 8.5 with 128, 9.1 as
  // per-operation launches).  With psb=0 it is per-operation launches without any reading ahead: the read-ahead kernel
  // keeps a wave on every SIMD for the whole loop, and the prefill's kernels have waves that take a SIMD's whole register
  // file (they would wait for the loop's end: +0.8 .. +1.2 ms); warm-up blocks inside the launches cost +0.2 .. +0.3 ms.
  rc = execute(c, KIND_DENOISE, c->cur_views, c->cur_prompt, sd, cur, cur, false);
  if (rc != PI0_OK) return rc;
  e = launch_copy_f32(sd, at<float>(c, c->wl.xa), d_actions, (size_t)c->cfg.chunk * c->d.A);
  if (e == hipSuccess) e = hipEventRecord(c->ev_denoise[cur], sd);
  if (e != hipSuccess) return fail_hip(c, e);
  c->cur_slot = nxt;
  c->cur_views = n_views;
  c->cur_prompt = n_prompt;
  return PI0_OK;
}

size_t pi0_debug_taps_elems(const pi0_config* cfg, int n_views, int n_prompt) {
  Dims d;
  if (cfg == nullptr || !derive_dims(*cfg, d)) return 0;
  if (n_views < 1 || n_views > cfg->max_views || n_prompt < 0 || n_prompt > cfg->max_prompt) return 0;
  const size_t I = (size_t)n_views * d.T, P = I + n_prompt;
  return (size_t)d.Lv * I * d.Dv + I * d.E + (size_t)(d.Ll - 1) * P * d.E + (size_t)2 * d.Ll * P * 256 +
         (size_t)2 * d.Le * 64 * d.X + (size_t)d.steps * cfg->chunk * d.A;
}

int pi0_debug_forward(pi0_ctx* c, const float* d_images, int n_views, const int32_t* d_prompt_ids, int n_prompt,
                      const float* d_state, const float* d_noise, float* d_actions, float* d_taps, size_t cap_elems,
                      void* hip_stream) {
  if (c == nullptr || d_state == nullptr || d_noise == nullptr || d_actions == nullptr || d_taps == nullptr) return PI0_EINVAL;
  if (!check_prefill_args(c, d_images, n_views, d_prompt_ids, n_prompt)) return PI0_EINVAL;
  if (!c->loaded) return PI0_ESTATE;
  if (cap_elems < pi0_debug_taps_elems(&c->cfg, n_views, n_prompt)) return PI0_ENOMEM;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  c->cur_views = 0;
  hipError_t e = stage_inputs(c, s, d_images, n_views, d_prompt_ids, n_prompt, d_state, d_noise);
  if (e != hipSuccess) return fail_hip(c, e);
  e = ensure_read_ahead(c);
  if (e != hipSuccess) return fail_hip(c, e);
  Run r{c, s, false};
  r.slot_w = r.slot_r = c->cur_slot;
  Taps taps;
  taps.base = d_taps;
  run_prefill(r, n_views, n_prompt, &taps);
  run_denoise(r, n_views * c->d.T + n_prompt, &taps);
  if (!r.ok()) return fail_hip(c, r.err);
  c->cur_views = n_views;
  c->cur_prompt = n_prompt;
  e = launch_copy_f32(s, at<float>(c, c->wl.xa), d_actions, (size_t)c->cfg.chunk * c->d.A);
  return e == hipSuccess ? PI0_OK : fail_hip(c, e);
}

int pi0_debug_profile(pi0_ctx* c, const float* d_images, int n_views, const int32_t* d_prompt_ids, int n_prompt,
                      const float* d_state, const float* d_noise, float* d_actions, int passes, double* h_class_us,
                      int* h_class_launches, void* hip_stream) {
  if (c == nullptr || d_state == nullptr || d_noise == nullptr || d_actions == nullptr || h_class_us == nullptr ||
      h_class_launches == nullptr || passes < 1 || passes > 64)
    return PI0_EINVAL;
  if (!check_prefill_args(c, d_images, n_views, d_prompt_ids, n_prompt)) return PI0_EINVAL;
  if (!c->loaded) return PI0_ESTATE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  for (int i = 0; i < PI0_OP_CLASSES; i++) {
    h_class_us[i] = 0.0;
    h_class_launches[i] = 0;
  }
  c->cur_views = 0;
  hipError_t e = stage_inputs(c, s, d_images, n_views, d_prompt_ids, n_prompt, d_state, d_noise);
  if (e != hipSuccess) return fail_hip(c, e);
  e = ensure_read_ahead(c);
  if (e != hipSuccess) return fail_hip(c, e);
  OpTimer timer;
  int rc = PI0_OK;
  for (int pass = 0; pass < passes && rc == PI0_OK; pass++) {
    Run r{c, s, false};
    r.slot_w = r.slot_r = c->cur_slot;
    r.timer = &timer;
    run_prefill(r, n_views, n_prompt, nullptr);
    run_denoise(r, n_views * c->d.T + n_prompt, nullptr);
    if (!r.ok()) rc = fail_hip(c, r.err);
  }
  e = hipStreamSynchronize(s);
  if (e != hipSuccess && rc == PI0_OK) rc = fail_hip(c, e);
  if (rc == PI0_OK) {
    for (size_t i = 0; i < timer.cls.size() && 2 * i + 1 < timer.ev.size(); i++) {
      float ms = 0.f;
      e = hipEventElapsedTime(&ms, timer.ev[2 * i], timer.ev[2 * i + 1]);
      if (e != hipSuccess) {
        rc = fail_hip(c, e);
        break;
      }
      h_class_us[timer.cls[i]] += (double)ms * 1000.0;
      h_class_launches[timer.cls[i]] += 1;
    }
  }
  for (hipEvent_t ev : timer.ev) (void)hipEventDestroy(ev);
  if (rc != PI0_OK) return rc;
  c->cur_views = n_views;
  c->cur_prompt = n_prompt;
  e = launch_copy_f32(s, at<float>(c, c->wl.xa), d_actions, (size_t)c->cfg.chunk * c->d.A);
  return e == hipSuccess ? PI0_OK : fail_hip(c, e);
}

}  // extern "C"
