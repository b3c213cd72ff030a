"""CPU oracle of one pi0 forward pass (test infrastructure, not a product path).

A plain, slow, unfused numpy implementation of what the paper's inference
program computes: SigLIP ViT over 1-3 views, the Gemma-style prefix transformer
whose keys and values are cached, and the action expert that integrates a flow
with 10 Euler steps against that cache (paper Section 2; every GEMM shape and its
scalar ops: Table 2; the algebraic rewrites this oracle deliberately does NOT
apply: Section 3.2 and Section 4).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this file; it shares no code with the
HIP library and imports nothing from it.

Precision: weights arrive as bfloat16 bit patterns and are widened exactly;
all arithmetic runs in `dtype` (float32 by default, float64 for cross-checks)
with no intermediate rounding.  numpy's matmul is the only library primitive.

Readings of points the paper leaves to its citations (all are conventions of
this build, "parity unpinned" against a trained pi0 because the paper prints no
activations): LayerNorm/RMSNorm eps 1e-6; RMSNorm gain (1 + g); tanh-GELU
everywhere; attention scale head_dim**-0.5; RoPE base 10000 with rotate-half
pairing (i, i + d/2); vision attention per view; learned additive position
embedding shared by all views; prompt embeddings scaled by sqrt(width) and placed
after the image tokens; time t runs 1.0 -> 0.1 with dt = -1/steps; time embedding
sin||cos with periods log-spaced 4e-3 .. 4; final RMSNorm before the action
out-projection, state row dropped.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import numpy as np

from . import mxfp8

EPS = 1e-6


# ----------------------------------------------------------------------------------------------
# scalar pieces
# ----------------------------------------------------------------------------------------------
def widen_bf16(bits: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Exact value of bfloat16 bit patterns (uint16) in `dtype`; float arrays pass through."""
    if bits.dtype == np.uint16:
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(dtype)
    return bits.astype(dtype)


def layer_norm(x, gain, bias):
    """(x - mean) / sqrt(biased var + eps) * gain + bias over the last axis (Table 2 "ln")."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + x.dtype.type(EPS)) * gain + bias


def rms_norm(x, g):
    """x / sqrt(mean(x^2) + eps) * (1 + g) over the last axis (Table 2 "rms")."""
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + x.dtype.type(EPS)) * (x.dtype.type(1.0) + g)


def gelu_tanh(x):
    c = x.dtype.type(math.sqrt(2.0 / math.pi))
    return x.dtype.type(0.5) * x * (x.dtype.type(1.0) + np.tanh(c * (x + x.dtype.type(0.044715) * x * x * x)))


def silu(x):
    return x / (x.dtype.type(1.0) + np.exp(-x))


def softmax_masked(logits, allowed):
    """Row softmax over the last axis; entries with allowed == False get weight exactly 0."""
    neg = np.where(allowed, logits, -np.inf)
    m = neg.max(axis=-1, keepdims=True)
    e = np.where(allowed, np.exp(neg - m), logits.dtype.type(0.0))
    return e / e.sum(axis=-1, keepdims=True)


def rope(u, positions, base=10000.0):
    """Rotary embedding on [..., T, d]: pairs (i, i + d/2), angle pos * base**(-2i/d)."""
    d = u.shape[-1]
    half = d // 2
    inv = np.asarray([base ** (-(2.0 * i) / d) for i in range(half)], dtype=np.float64)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv[None, :]
    c = np.cos(ang).astype(u.dtype)
    s = np.sin(ang).astype(u.dtype)
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def time_embedding(t, width, dtype, min_period=4e-3, max_period=4.0):
    """sin || cos of 2*pi*t / period_j with periods log-spaced from min to max (width/2 of them)."""
    half = width // 2
    frac = np.linspace(0.0, 1.0, half, dtype=np.float64)
    period = min_period * (max_period / min_period) ** frac
    ang = 2.0 * math.pi * float(t) / period
    return np.concatenate([np.sin(ang), np.cos(ang)]).astype(dtype)


def attention(q, k, v, allowed):
    """q [H, Tq, d], k/v [Hk, Tk, d] with Hk == H or Hk == 1 (shared kv head), allowed [Tq, Tk]."""
    H, Tq, d = q.shape
    out = np.empty((H, Tq, v.shape[-1]), dtype=q.dtype)
    scale = q.dtype.type(d ** -0.5)
    for h in range(H):
        kh = k[h if k.shape[0] > 1 else 0]
        vh = v[h if v.shape[0] > 1 else 0]
        p = softmax_masked((q[h] @ kh.T) * scale, allowed)
        out[h] = p @ vh
    return out


# ----------------------------------------------------------------------------------------------
# model
# ----------------------------------------------------------------------------------------------
class Weights:
    """Lazy widening view over name -> bf16-bits arrays."""

    def __init__(self, tensors: Dict[str, np.ndarray], dtype):
        self.t = tensors
        self.dtype = dtype

    def __getitem__(self, name):
        return widen_bf16(self.t[name], self.dtype)

    def mx(self, name):
        """Weight matrix [k, n] rounded through MXFP8 with blocks of 32 along k (its contraction axis)."""
        w = widen_bf16(self.t[name], np.float64)
        return np.ascontiguousarray(mxfp8.mx_round(w.T, np.float64).T).astype(self.dtype)


def patchify(cfg, images, dtype):
    """[V, H, W, 3] -> [V * T, patch*patch*3]; patch vector order (dy, dx, channel)."""
    V = images.shape[0]
    p, n = cfg.patch, cfg.img_size // cfg.patch
    x = images.astype(dtype).reshape(V, n, p, n, p, 3)       # v, py, dy, px, dx, c
    x = x.transpose(0, 1, 3, 2, 4, 5)                        # v, py, px, dy, dx, c
    return x.reshape(V * n * n, p * p * 3)


def vision_encoder(cfg, W: Weights, images, taps: Optional[dict] = None, joint_views: bool = False):
    """SigLIP tower + projector: images [V, H, W, 3] -> prefix image embeddings [V*T, llm_width]."""
    V = images.shape[0]
    T, D, Hn = cfg.tokens_per_view, cfg.vis_width, cfg.vis_heads
    dh = D // Hn
    h = patchify(cfg, images, W.dtype) @ W["vis.patch.w"] + W["vis.patch.b"]
    h = h + np.tile(W["vis.pos"], (V, 1))
    I = V * T
    if joint_views:
        allowed = np.ones((I, I), dtype=bool)
    else:
        view = np.arange(I) // T
        allowed = view[:, None] == view[None, :]
    for l in range(cfg.vis_layers):
        p = f"vis.{l}."
        a = layer_norm(h, W[p + "ln1.g"], W[p + "ln1.b"])
        q = (a @ W[p + "wq"] + W[p + "bq"]).reshape(I, Hn, dh).transpose(1, 0, 2)
        k = (a @ W[p + "wk"] + W[p + "bk"]).reshape(I, Hn, dh).transpose(1, 0, 2)
        v = (a @ W[p + "wv"] + W[p + "bv"]).reshape(I, Hn, dh).transpose(1, 0, 2)
        o = attention(q, k, v, allowed).transpose(1, 0, 2).reshape(I, D)
        h = h + o @ W[p + "wo"] + W[p + "bo"]
        m = layer_norm(h, W[p + "ln2.g"], W[p + "ln2.b"])
        h = h + gelu_tanh(m @ W[p + "w1"] + W[p + "b1"]) @ W[p + "w2"] + W[p + "b2"]
        if taps is not None:
            taps[f"vis.h.{l}"] = h.copy()
    e = layer_norm(h, W["vis.lnf.g"], W["vis.lnf.b"]) @ W["vis.proj.w"] + W["vis.proj.b"]
    if taps is not None:
        taps["vis.out"] = e.copy()
    return e


def _gemma_qkv(cfg, W, p, x, positions):
    Hn, dh = cfg.llm_q_heads, cfg.head_dim
    a = rms_norm(x, W[p + "g_attn"])
    T = x.shape[0]
    q = rope((a @ W[p + "wq"]).reshape(T, Hn, dh).transpose(1, 0, 2), positions)
    k = rope((a @ W[p + "wk"])[None], positions)
    v = (a @ W[p + "wv"])[None]
    return q, k, v


def _gemma_mlp(W, p, x):
    m = rms_norm(x, W[p + "g_mlp"])
    return (gelu_tanh(m @ W[p + "wg"]) * (m @ W[p + "wu"])) @ W[p + "wd"]


def _gemma_mlp_mxfp8(W, p, x):
    """The same feed-forward block with every GEMM operand rounded through MXFP8 (blocks of 32 along the
    contraction axis).  A convention of this build, not of the paper: the gain-scaled input x * (1 + g) is
    what gets quantised and the row's 1 / rms is applied to the products (power-of-two block scales do not
    commute with an arbitrary row factor, so the order is part of the definition); the gated product
    gelu(gate) * up is quantised before the down projection."""
    dt = x.dtype
    rstd = dt.type(1.0) / np.sqrt((x * x).mean(axis=-1, keepdims=True) + dt.type(EPS))
    xq = mxfp8.mx_round(x * (dt.type(1.0) + W[p + "g_mlp"]))
    gate = rstd * (xq @ W.mx(p + "wg"))
    up = rstd * (xq @ W.mx(p + "wu"))
    hq = mxfp8.mx_round(gelu_tanh(gate) * up)
    return hq @ W.mx(p + "wd")


def prefix_forward(cfg, W: Weights, images, prompt_ids=None, taps: Optional[dict] = None,
                   run_last_layer: bool = False, mlp_mxfp8: bool = False):
    """Vision tower, prompt embedding, and the prefix transformer.  Returns the per-layer
    key and value caches ([L, P, head_dim] each).  The last layer only produces its keys and
    values (Section 4.1: its attention and FFN feed nothing downstream) unless
    run_last_layer is set, which exists to test exactly that statement."""
    e = vision_encoder(cfg, W, images, taps)
    if prompt_ids is not None and len(prompt_ids) > 0:
        emb = W.t["llm.embed"][np.asarray(prompt_ids, dtype=np.int64)]
        emb = widen_bf16(emb, W.dtype) * W.dtype(math.sqrt(cfg.llm_width))
        x = np.concatenate([e, emb], axis=0)
    else:
        x = e
    P = x.shape[0]
    pos = np.arange(P)
    allowed = np.ones((P, P), dtype=bool)
    Ks = np.empty((cfg.llm_layers, P, cfg.head_dim), dtype=W.dtype)
    Vs = np.empty_like(Ks)
    for l in range(cfg.llm_layers):
        p = f"llm.{l}."
        q, k, v = _gemma_qkv(cfg, W, p, x, pos)
        Ks[l], Vs[l] = k[0], v[0]
        if l == cfg.llm_layers - 1 and not run_last_layer:
            break
        o = attention(q, k, v, allowed).transpose(1, 0, 2).reshape(P, -1)
        x = x + o @ W[p + "wo"]
        x = x + (_gemma_mlp_mxfp8(W, p, x) if mlp_mxfp8 else _gemma_mlp(W, p, x))
        if taps is not None:
            taps[f"llm.x.{l}"] = x.copy()
    return Ks, Vs


def suffix_allowed(P, S):
    """Attention permission of the S suffix rows (state, then actions) over P prefix + S suffix
    keys: everyone sees the prefix; the state row sees itself only; action rows see the state and
    every action row."""
    allowed = np.ones((S, P + S), dtype=bool)
    allowed[0, P + 1:] = False
    return allowed


def suffix_tokens(cfg, W: Weights, state, x, t):
    """[state token ; action-time tokens] at flow time t (Table 2 rows 1x32x1024, 63x32x1024,
    63x1024x1024, here unfolded: action up-projection, concat with the time encoding, two-layer
    MLP with SiLU)."""
    X = cfg.exp_width
    s = state.astype(W.dtype)[None] @ W["exp.state.w"] + W["exp.state.b"]
    ae = x @ W["exp.action_in.w"] + W["exp.action_in.b"]
    tau = time_embedding(t, X, W.dtype)
    cat = np.concatenate([ae, np.tile(tau[None], (x.shape[0], 1))], axis=1)
    z = silu(cat @ W["exp.time_in.w"] + W["exp.time_in.b"])
    tok = z @ W["exp.time_out.w"] + W["exp.time_out.b"]
    return np.concatenate([s, tok], axis=0)


def expert_velocity(cfg, W: Weights, Ks, Vs, state, x, t, taps: Optional[dict] = None, tag: str = ""):
    """One evaluation of the action expert: velocity field v(x, t) [chunk, action_dim]."""
    P = Ks.shape[1]
    S = cfg.suffix
    y = suffix_tokens(cfg, W, state, x, t)
    pos = np.arange(P, P + S)
    allowed = suffix_allowed(P, S)
    for l in range(cfg.exp_layers):
        p = f"exp.{l}."
        q, k, v = _gemma_qkv(cfg, W, p, y, pos)
        keys = np.concatenate([Ks[l], k[0]], axis=0)[None]
        vals = np.concatenate([Vs[l], v[0]], axis=0)[None]
        o = attention(q, keys, vals, allowed).transpose(1, 0, 2).reshape(S, -1)
        y = y + o @ W[p + "wo"]
        y = y + _gemma_mlp(W, p, y)
        if taps is not None:
            taps[f"exp.y.{tag}.{l}"] = y.copy()
    return rms_norm(y[1:], W["exp.g_final"]) @ W["exp.out.w"] + W["exp.out.b"]


def denoise(cfg, W: Weights, Ks, Vs, state, noise, taps: Optional[dict] = None, tap_steps=(0, 9)):
    """Euler integration of the flow from t = 1 (noise) to t = 0: x <- x + dt * v(x, t), dt = -1/steps."""
    x = noise.astype(W.dtype)
    dt = W.dtype(-1.0 / cfg.steps)
    for k in range(cfg.steps):
        t = 1.0 - k / cfg.steps
        tp = taps if (taps is not None and k in tap_steps) else None
        v = expert_velocity(cfg, W, Ks, Vs, state, x, t, tp, tag=str(k))
        x = x + dt * v
        if taps is not None:
            taps[f"exp.x.{k}"] = x.copy()
    return x


def pi0_forward(cfg, tensors: Dict[str, np.ndarray], images, state, noise, prompt_ids=None,
                dtype=np.float32, taps: Optional[dict] = None, prefix_mlp_mxfp8: bool = False):
    """images [V,H,W,3], state [state_dim], noise [chunk, action_dim] -> action chunk.
    prefix_mlp_mxfp8: the prefix transformer's feed-forward GEMMs take MXFP8-rounded operands."""
    W = Weights(tensors, dtype)
    Ks, Vs = prefix_forward(cfg, W, images, prompt_ids, taps, mlp_mxfp8=prefix_mlp_mxfp8)
    if taps is not None:
        taps["kcache"], taps["vcache"] = Ks.copy(), Vs.copy()
    return denoise(cfg, W, Ks, Vs, state, noise, taps, tap_steps=(0, cfg.steps - 1))


# ----------------------------------------------------------------------------------------------
# Independent second path: no cache, one joint sequence (used only to pin the cached path)
# ----------------------------------------------------------------------------------------------
def joint_velocity(cfg, tensors, images, state, x, t, prompt_ids=None, dtype=np.float64):
    """Velocity computed WITHOUT a KV cache: prefix tokens (routed through the prefix weights)
    and suffix tokens (routed through the expert weights) run side by side through every layer,
    sharing one attention over P + S keys with the three-block mask.  All layers run in full
    on both streams.  Must equal expert_velocity on cached keys/values (Section 4.1)."""
    W = Weights(tensors, dtype)
    e = vision_encoder(cfg, W, images)
    if prompt_ids is not None and len(prompt_ids) > 0:
        emb = widen_bf16(W.t["llm.embed"][np.asarray(prompt_ids, dtype=np.int64)], dtype)
        xp = np.concatenate([e, emb * dtype(math.sqrt(cfg.llm_width))], axis=0)
    else:
        xp = e
    P, S = xp.shape[0], cfg.suffix
    ys = suffix_tokens(cfg, W, state, x.astype(dtype), t)
    allowed = np.zeros((P + S, P + S), dtype=bool)
    allowed[:P, :P] = True
    allowed[P:, :] = suffix_allowed(P, S)
    pos = np.arange(P + S)
    Hn, dh = cfg.llm_q_heads, cfg.head_dim
    assert cfg.llm_layers == cfg.exp_layers
    for l in range(cfg.llm_layers):
        qs, ks, vs = [], [], []
        for pre, stream, ps in ((f"llm.{l}.", xp, pos[:P]), (f"exp.{l}.", ys, pos[P:])):
            q, k, v = _gemma_qkv(cfg, W, pre, stream, ps)
            qs.append(q); ks.append(k); vs.append(v)
        q = np.concatenate(qs, axis=1); k = np.concatenate(ks, axis=1); v = np.concatenate(vs, axis=1)
        o = attention(q, k, v, allowed).transpose(1, 0, 2).reshape(P + S, Hn * dh)
        xp = xp + o[:P] @ W[f"llm.{l}.wo"]
        xp = xp + _gemma_mlp(W, f"llm.{l}.", xp)
        ys = ys + o[P:] @ W[f"exp.{l}.wo"]
        ys = ys + _gemma_mlp(W, f"exp.{l}.", ys)
    return rms_norm(ys[1:], W["exp.g_final"]) @ W["exp.out.w"] + W["exp.out.b"]
