"""How far bf16 GEMM inputs alone move the oracle (CPU only): the evidence behind the action bars of the GPU tests.

The HIP path feeds its matrix units bf16 operands (the paper runs everything in bf16, Section 8; accumulation and
statistics stay fp32).  Here the ORACLE is run with exactly that and nothing else changed: every matrix product
rounds both operands to bf16 first (weights are bf16 values already, so only activations, attention probabilities
and cached keys / values move).  The arithmetic is the oracle's own - the rounding is injected through an ndarray
subclass whose `@` rounds its operands, so no line of the oracle is touched.

  N(0, 0.02) weights (the benchmark's recipe)      -> a few 1e-3 of the action RMS: the 2e-2 bar of the task has a
                                                      factor of several in hand
  query / key projections 2.5 x wider (std 0.05)   -> 2e-2: the softmax is sharp (logit deviation about 5) and
                                                      amplifies input rounding; the GPU stress test that uses this
                                                      configuration (test_sharp_attention_masks) takes 5e-2, the
                                                      same factor 2.5 above the rounding-only figure that the 2e-2
                                                      bar has on the benchmark's weights
  4 x wider (std 0.08)                             -> far beyond any such bar: sharper settings test the conditioning
                                                      of the problem, not an implementation
"""
import os

import numpy as np
import pytest

from oracle import pi0_oracle as O
from paper_2510_26742_amd import synth


def bf16_round(x):
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


class Bf16Operands(np.ndarray):
    """float32 array whose matrix products round both operands to bf16 (round to nearest even) first."""

    def __matmul__(self, other):
        return np.matmul(bf16_round(np.asarray(self)), bf16_round(np.asarray(other))).view(Bf16Operands)

    def __rmatmul__(self, other):
        return np.matmul(bf16_round(np.asarray(other)), bf16_round(np.asarray(self))).view(Bf16Operands)


def cache_delta(plain_taps, rounded_taps, name, layer):
    """max |delta| of one layer of the key / value cache over the layer's RMS, the rounded run's cache stored as bf16
    (as the HIP path stores it)."""
    r = np.asarray(plain_taps[name][layer])
    g = bf16_round(np.asarray(rounded_taps[name][layer]))
    return float(np.abs(g - r).max()) / float(np.sqrt((r.astype(np.float64) ** 2).mean()))


def forward(cfg, tensors, img, st, nz, ids, rounded, monkeypatch, taps=None):
    if not rounded:
        return O.pi0_forward(cfg, tensors, img, st, nz, ids, taps=taps)
    # attention() and softmax_masked() build their results in fresh plain arrays: hand them on as the subclass,
    # so that the products they feed (P @ V, the O projection) round their inputs too
    att, sm = O.attention, O.softmax_masked
    monkeypatch.setattr(O, "attention", lambda *a: att(*a).view(Bf16Operands))
    monkeypatch.setattr(O, "softmax_masked", lambda *a: sm(*a).view(Bf16Operands))
    out = O.pi0_forward(cfg, tensors, img.view(Bf16Operands), st.view(Bf16Operands), nz.view(Bf16Operands), ids, taps=taps)
    monkeypatch.undo()
    return np.asarray(out)


def test_rounding_helper_is_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -3.1415927, 0.0], dtype=np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -3.140625, 0.0], dtype=np.float32)
    np.testing.assert_array_equal(bf16_round(x), want)
    a = np.arange(12, dtype=np.float32).reshape(3, 4).view(Bf16Operands) * np.float32(1.001)
    assert isinstance(a @ np.ones((4, 2), np.float32), Bf16Operands)
    np.testing.assert_array_equal(np.asarray(a @ np.eye(4, dtype=np.float32)), bf16_round(np.asarray(a)))


@pytest.mark.parametrize("std, lo, hi, cache_hi", [(None, 5e-4, 8e-3, 0.135 / 2.5), (0.05, 8e-3, 5e-2 / 1.5, 0.30 / 2.5),
                                                  (0.08, 5e-2, 10.0, None)])
def test_oracle_moves_this_much_under_bf16_operands(std, lo, hi, cache_hi, monkeypatch):
    cfg = synth.reduced_config(vocab=1024)
    overrides = {"wq": std, "wk": std} if std else None
    blob = synth.make_weights(cfg, seed=5, overrides=overrides)       # the GPU stress test's seed and inputs
    tensors = synth.blob_views(cfg, blob)
    img, st, nz = synth.make_images(cfg, 2, seed=1), synth.make_state(cfg, seed=2), synth.make_noise(cfg, seed=3)
    ids = synth.make_prompt(cfg, 7, seed=4)
    tp, tr = {}, {}
    plain = forward(cfg, tensors, img, st, nz, ids, False, monkeypatch, tp)
    rounded = forward(cfg, tensors, img, st, nz, ids, True, monkeypatch, tr)
    rms = float(np.sqrt((plain.astype(np.float64) ** 2).mean()))
    delta = float(np.abs(rounded - plain).max()) / rms
    cache = max(cache_delta(tp, tr, n, l) for n in ("kcache", "vcache") for l in range(cfg.llm_layers))
    print(f"wq/wk std {std}: bf16 operands move the oracle's actions by {delta:.3e} of their RMS, a cache element by "
          f"up to {cache:.3e} of its layer's RMS")
    assert lo <= delta <= hi, delta
    # the GPU tests' cache bar (max |delta| / RMS per layer: 0.135, and 0.30 in the sharp configuration) is 2.5 x
    # what rounding alone does here
    if cache_hi is not None:
        assert cache <= cache_hi, cache


def test_full_depth_under_bf16_operands(monkeypatch):
    """The benchmark's own model (27/18/18 layers, 1 view): bf16 operands alone move the actions by about 4e-3 of
    their RMS - where the HIP path is measured too (4e-3 .. 6e-3), i.e. it sits at the floor its operand precision
    sets - and a cache element by up to 5.4e-2 of its layer's RMS at the deepest layers (2e-2 at the first), which is
    what the GPU tests' cache bar of 0.135 = 2.5 x 5.4e-2 rests on."""
    cfg = synth.full_config()
    tensors = synth.blob_views(cfg, synth.make_weights(cfg, seed=0, threads=8))
    img, st, nz = synth.make_images(cfg, 1, seed=1), synth.make_state(cfg, seed=2), synth.make_noise(cfg, seed=3)
    tp, tr = {}, {}
    plain = forward(cfg, tensors, img, st, nz, None, False, monkeypatch, tp)
    rounded = forward(cfg, tensors, img, st, nz, None, True, monkeypatch, tr)
    rms = float(np.sqrt((plain.astype(np.float64) ** 2).mean()))
    delta = float(np.abs(rounded - plain).max()) / rms
    per_layer = [max(cache_delta(tp, tr, n, l) for n in ("kcache", "vcache")) for l in range(cfg.llm_layers)]
    print(f"full model: actions {delta:.3e}; cache per layer " + " ".join(f"{d:.3f}" for d in per_layer))
    assert 1e-3 <= delta <= 8e-3
    assert max(per_layer) <= 0.135 / 2.5 * 1.05 and per_layer[0] <= 0.03


@pytest.mark.skipif(not os.environ.get("PI0_SLOW_TESTS"), reason="about 8 minutes of numpy (two MXFP8-oracle passes of the full "
                    "model); set PI0_SLOW_TESTS=1.  Figures of the last run are in the docstring")
def test_full_depth_mxfp8_oracle_under_bf16_operands(monkeypatch):
    """The reduced-precision mode's oracle (prefix feed-forward operands through MXFP8) at full depth, plain against
    bf16 GEMM operands: quantisation is discontinuous, so the two runs part ways layer by layer.  Last run: prefix
    hidden-state cosines 0.99957 0.99886 0.99811 0.99736 0.99664 0.99598 0.99541 0.99469 0.99413 0.99358 0.99297 0.99242
    0.99194 0.99150 0.99107 0.99068 0.99024 (layers 0 .. 16); key cache down to 0.98953; worst single token row 0.98712;
    expert hidden states >= 0.99993; actions 1.69e-2 of their RMS.  The GPU test of the mode at full depth takes its
    bars from these (cosine 0.985 / 0.97 per row, actions 2.5 x 1.7e-2)."""
    def cosine(a, b):
        a, b = np.asarray(a, dtype=np.float64).ravel(), np.asarray(b, dtype=np.float64).ravel()
        return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))
    cfg = synth.full_config()
    tensors = synth.blob_views(cfg, synth.make_weights(cfg, seed=0, threads=8))
    img, st, nz = synth.make_images(cfg, 1, seed=1), synth.make_state(cfg, seed=2), synth.make_noise(cfg, seed=3)
    tp, tr = {}, {}
    plain = O.pi0_forward(cfg, tensors, img, st, nz, None, taps=tp, prefix_mlp_mxfp8=True)
    att, sm = O.attention, O.softmax_masked
    monkeypatch.setattr(O, "attention", lambda *a: att(*a).view(Bf16Operands))
    monkeypatch.setattr(O, "softmax_masked", lambda *a: sm(*a).view(Bf16Operands))
    rounded = np.asarray(O.pi0_forward(cfg, tensors, img.view(Bf16Operands), st.view(Bf16Operands), nz.view(Bf16Operands), None,
                                       taps=tr, prefix_mlp_mxfp8=True))
    monkeypatch.undo()
    rms = float(np.sqrt((plain.astype(np.float64) ** 2).mean()))
    delta = float(np.abs(rounded - plain).max()) / rms
    cos = [cosine(tp[f"llm.x.{l}"], tr[f"llm.x.{l}"]) for l in range(cfg.llm_layers - 1)]
    print(f"actions {delta:.3e}; llm.x cosines " + " ".join(f"{c:.5f}" for c in cos))
    assert 5e-3 <= delta <= 4.2e-2 / 1.5
    assert 0.985 + 0.003 <= min(cos) and cos[3] < 0.999
