"""Seeded synthetic inputs for the pi0 forward pass: model dimensions, the
canonical (unfolded) weight-tensor table, and counter-based random generators.

This module holds no arithmetic of the method itself.  It only says which
tensors exist, how large they are, and fills them with reproducible random
numbers.  Both the CPU oracle's tests and the GPU path's tests draw their
inputs from here, so the two sides always see the same bytes.

Shapes follow Table 2 of the paper (rows x K x cols of every GEMM) and the
model description in its Section 2: a SigLIP ViT (width 1152, 16 heads of 72,
MLP 4304, patch 14 on 224x224 images), a Gemma-2B style prefix transformer
(width 2048, 8 query heads sharing 1 kv head of 256, gated MLP 16384) and an
action expert of the same shape at width 1024 / MLP 4096.

All weights are stored "x @ W" style: shape [in_features, out_features],
row-major, as bfloat16 bit patterns (uint16).
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Pi0Config:
    # vision tower
    vis_layers: int = 27
    vis_width: int = 1152
    vis_heads: int = 16
    vis_mlp: int = 4304
    img_size: int = 224
    patch: int = 14
    # prefix language model
    llm_layers: int = 18
    llm_width: int = 2048
    llm_q_heads: int = 8
    head_dim: int = 256
    llm_mlp: int = 16384
    # action expert
    exp_layers: int = 18
    exp_width: int = 1024
    exp_mlp: int = 4096
    # flow matching
    state_dim: int = 32
    action_dim: int = 32
    chunk: int = 63
    steps: int = 10
    # prompt embedding table rows (0 = no table in the blob, empty prompt only)
    vocab: int = 0
    max_views: int = 3
    max_prompt: int = 48

    @property
    def tokens_per_view(self) -> int:
        return (self.img_size // self.patch) ** 2

    @property
    def patch_dim(self) -> int:
        return self.patch * self.patch * 3

    @property
    def vis_head_dim(self) -> int:
        return self.vis_width // self.vis_heads

    @property
    def suffix(self) -> int:
        return self.chunk + 1


def full_config(vocab: int = 0) -> Pi0Config:
    """Full-depth model (27 / 18 / 18 layers)."""
    return Pi0Config(vocab=vocab)


def reduced_config(vocab: int = 0) -> Pi0Config:
    """Full widths, 2 / 2 / 2 layers: the small case the oracle finishes in seconds."""
    return Pi0Config(vis_layers=2, llm_layers=2, exp_layers=2, vocab=vocab)


def tiny_config() -> Pi0Config:
    """A toy geometry for brute-force checks of the oracle (pure Python loops)."""
    return Pi0Config(vis_layers=1, vis_width=8, vis_heads=2, vis_mlp=12, img_size=4, patch=2,
                     llm_layers=2, llm_width=12, llm_q_heads=2, head_dim=4, llm_mlp=16,
                     exp_layers=2, exp_width=8, exp_mlp=12, state_dim=3, action_dim=3,
                     chunk=3, steps=2, vocab=7, max_views=2, max_prompt=4)


# ----------------------------------------------------------------------------------------------
# canonical tensor table
# ----------------------------------------------------------------------------------------------
# kind: "w" = matrix / bias / embedding ~ N(0, 0.02^2)
#       "g" = RMSNorm gain under the (1 + g) convention ~ N(0, 0.02^2)
#       "ln" = LayerNorm gain stored directly, 1 + N(0, 0.02^2)
BLOB_ALIGN_ELEMS = 128  # every tensor starts at a multiple of 128 bf16 elements (256 bytes)


def tensor_table(cfg: Pi0Config) -> List[Tuple[str, Tuple[int, ...], str]]:
    """Names, shapes and kinds of all weight tensors, in blob order."""
    t: List[Tuple[str, Tuple[int, ...], str]] = []
    D, F, T = cfg.vis_width, cfg.vis_mlp, cfg.tokens_per_view
    t += [("vis.patch.w", (cfg.patch_dim, D), "w"), ("vis.patch.b", (D,), "w"), ("vis.pos", (T, D), "w")]
    for l in range(cfg.vis_layers):
        p = f"vis.{l}."
        t += [(p + "ln1.g", (D,), "ln"), (p + "ln1.b", (D,), "w"),
              (p + "wq", (D, D), "w"), (p + "bq", (D,), "w"),
              (p + "wk", (D, D), "w"), (p + "bk", (D,), "w"),
              (p + "wv", (D, D), "w"), (p + "bv", (D,), "w"),
              (p + "wo", (D, D), "w"), (p + "bo", (D,), "w"),
              (p + "ln2.g", (D,), "ln"), (p + "ln2.b", (D,), "w"),
              (p + "w1", (D, F), "w"), (p + "b1", (F,), "w"),
              (p + "w2", (F, D), "w"), (p + "b2", (D,), "w")]
    E = cfg.llm_width
    t += [("vis.lnf.g", (D,), "ln"), ("vis.lnf.b", (D,), "w"),
          ("vis.proj.w", (D, E), "w"), ("vis.proj.b", (E,), "w")]
    if cfg.vocab > 0:
        t += [("llm.embed", (cfg.vocab, E), "w")]
    H, Dh = cfg.llm_q_heads, cfg.head_dim
    for prefix, layers, W, M in (("llm", cfg.llm_layers, cfg.llm_width, cfg.llm_mlp),
                                ("exp", cfg.exp_layers, cfg.exp_width, cfg.exp_mlp)):
        for l in range(layers):
            p = f"{prefix}.{l}."
            t += [(p + "g_attn", (W,), "g"),
                  (p + "wq", (W, H * Dh), "w"), (p + "wk", (W, Dh), "w"), (p + "wv", (W, Dh), "w"),
                  (p + "wo", (H * Dh, W), "w"),
                  (p + "g_mlp", (W,), "g"),
                  (p + "wg", (W, M), "w"), (p + "wu", (W, M), "w"), (p + "wd", (M, W), "w")]
    X = cfg.exp_width
    t += [("exp.state.w", (cfg.state_dim, X), "w"), ("exp.state.b", (X,), "w"),
          ("exp.action_in.w", (cfg.action_dim, X), "w"), ("exp.action_in.b", (X,), "w"),
          ("exp.time_in.w", (2 * X, X), "w"), ("exp.time_in.b", (X,), "w"),
          ("exp.time_out.w", (X, X), "w"), ("exp.time_out.b", (X,), "w"),
          ("exp.g_final", (X,), "g"),
          ("exp.out.w", (X, cfg.action_dim), "w"), ("exp.out.b", (cfg.action_dim,), "w")]
    return t


def blob_layout(cfg: Pi0Config) -> Tuple[Dict[str, Tuple[int, Tuple[int, ...]]], int]:
    """name -> (element offset, shape) inside the flat bf16 blob, and total elements."""
    off = 0
    out: Dict[str, Tuple[int, Tuple[int, ...]]] = {}
    for name, shape, _ in tensor_table(cfg):
        out[name] = (off, shape)
        n = int(np.prod(shape))
        off += (n + BLOB_ALIGN_ELEMS - 1) // BLOB_ALIGN_ELEMS * BLOB_ALIGN_ELEMS
    return out, off


# ----------------------------------------------------------------------------------------------
# random numbers
# ----------------------------------------------------------------------------------------------
def _rng(seed: int, stream: int) -> np.random.Generator:
    """One independent Philox-4x64 stream per (seed, stream index)."""
    return np.random.Generator(np.random.Philox(key=(int(seed) << 32) | int(stream)))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (u >> np.uint32(16)).astype(np.uint16)


def _fill(args) -> None:
    dst, seed, idx, kind, std = args
    g = _rng(seed, idx)
    n = dst.size
    CH = 1 << 24
    for s in range(0, n, CH):
        m = min(CH, n - s)
        v = g.standard_normal(m, dtype=np.float32) * np.float32(std)
        if kind == "ln":
            v += np.float32(1.0)
        dst[s:s + m] = to_bf16_bits(v)


def make_weights(cfg: Pi0Config, seed: int = 0, std: float = 0.02, threads: int = 8,
                 overrides: Dict[str, float] | None = None) -> np.ndarray:
    """The flat weight blob (uint16 bf16 bits).  Tensor i of the table draws from stream i.

    `overrides` maps a tensor-name suffix (e.g. "wq") to a different std for tensors whose
    name ends with it: used by tests that need sharp attention logits.
    """
    layout, total = blob_layout(cfg)
    blob = np.zeros(total, dtype=np.uint16)
    jobs = []
    for idx, (name, shape, kind) in enumerate(tensor_table(cfg)):
        off, _ = layout[name]
        n = int(np.prod(shape))
        s = std
        if overrides:
            for suf, v in overrides.items():
                if name.endswith(suf):
                    s = v
        jobs.append((blob[off:off + n], seed, idx, kind, s))
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(_fill, jobs))
    else:
        for j in jobs:
            _fill(j)
    return blob


def blob_views(cfg: Pi0Config, blob: np.ndarray) -> Dict[str, np.ndarray]:
    """name -> uint16 view of the blob with the tensor's shape (no copies)."""
    layout, _ = blob_layout(cfg)
    return {name: blob[off:off + int(np.prod(shape))].reshape(shape) for name, (off, shape) in layout.items()}


def make_images(cfg: Pi0Config, n_views: int, seed: int = 1) -> np.ndarray:
    """[V, H, W, 3] float32, uniform in [-1, 1)."""
    g = _rng(seed, 0)
    return (g.random((n_views, cfg.img_size, cfg.img_size, 3), dtype=np.float32) * np.float32(2.0)
            - np.float32(1.0))


def make_state(cfg: Pi0Config, seed: int = 2) -> np.ndarray:
    return _rng(seed, 0).standard_normal(cfg.state_dim, dtype=np.float32)


def make_noise(cfg: Pi0Config, seed: int = 3) -> np.ndarray:
    return _rng(seed, 0).standard_normal((cfg.chunk, cfg.action_dim), dtype=np.float32)


def make_prompt(cfg: Pi0Config, n_prompt: int, seed: int = 4) -> np.ndarray:
    if n_prompt == 0:
        return np.zeros(0, dtype=np.int32)
    return _rng(seed, 0).integers(0, cfg.vocab, size=n_prompt, dtype=np.int32)
