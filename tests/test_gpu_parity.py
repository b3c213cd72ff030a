"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Bars (from the benchmark spec): actions max|delta| <= 2e-2 * RMS(oracle actions); every per-layer
hidden state (vision, prefix, expert at the first and last Euler step) and every layer of the
key/value cache has cosine similarity >= 0.999 with the oracle.  Integer-free path, so nothing
here is bit-exact against the oracle; bit-exactness is required between the library's own
eager, graph and replayed runs.
"""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import pi0_oracle as O
from paper_2510_26742_amd import binding, synth

pytestmark = pytest.mark.gpu

ACTION_TOL = 2e-2
COS_MIN = 0.999
# MXFP8 mode against the MXFP8 oracle.  Both sides quantise by the same rule, but their inputs differ by the bf16
# path's own error (~2^-9 relative), so a few percent of the elements land on neighbouring FP8 codes (one code =
# 2^-4 .. 2^-3 relative): the per-layer agreement is looser than in bf16 (measured worst cosine 0.9995), the
# actions stay within the bf16 bar (measured 6e-3 of their RMS).
SHARP_ACTION_TOL = 5e-2     # see test_sharp_attention_masks and tests/test_bf16_sensitivity.py
MX_ACTION_TOL = 2e-2
MX_COS_MIN = 0.998
MX_ROW_COS_MIN = 0.99
# ... and at full depth (17 quantised layers).  Quantisation is discontinuous: two runs whose inputs differ by the
# bf16 path's rounding land on neighbouring codes here and there, and every layer widens the gap.  What that does to
# the MXFP8 ORACLE ITSELF was measured on the CPU (tests/test_bf16_sensitivity.py, the slow test): with bf16 GEMM
# operands and nothing else changed its prefix hidden states fall from cosine 0.9996 (layer 0) through 0.9974 (layer 3)
# to 0.990 (layer 16) against its own plain run, the cache to 0.9895, single token rows to 0.987, and the actions move
# by 1.7e-2 of their RMS.  The HIP path measures the same figures (0.99735 at layer 3).  Bars: a margin below those
# cosines, 2.5 x the action figure.
MX_FULL_COS_MIN = 0.985
MX_FULL_ROW_COS_MIN = 0.97
MX_FULL_ACTION_TOL = 4.2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def cosine(a, b):
    a = a.astype(np.float64).ravel()
    b = b.astype(np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b) + 1e-300))


class Case:
    """One (config, weights) pair loaded on the GPU plus the oracle-side view of the same bytes."""

    def __init__(self, cfg, seed=0, overrides=None, tune=None):
        self.cfg = cfg
        self.dev = torch.device("cuda:0")
        say(f"[case] generating weights layers={cfg.vis_layers}/{cfg.llm_layers}/{cfg.exp_layers} vocab={cfg.vocab}")
        self.blob = synth.make_weights(cfg, seed=seed, overrides=overrides)
        self.tensors = synth.blob_views(cfg, self.blob)
        self.stream = torch.cuda.Stream(device=self.dev)
        self.m = binding.Pi0(cfg, tune=tune)
        d_blob = torch.from_numpy(self.blob.view(np.int16)).to(self.dev)
        say("[case] pi0_load_weights")
        self.m.pi0_load_weights(d_blob, self.stream)
        self.stream.synchronize()
        del d_blob
        say("[case] loaded")

    def inputs(self, n_views, n_prompt, seed_shift=0):
        cfg = self.cfg
        img = synth.make_images(cfg, n_views, seed=1 + seed_shift)
        st = synth.make_state(cfg, seed=2 + seed_shift)
        nz = synth.make_noise(cfg, seed=3 + seed_shift)
        ids = synth.make_prompt(cfg, n_prompt, seed=4 + seed_shift)
        return img, st, nz, ids

    def to_dev(self, img, st, nz, ids):
        d = self.dev
        d_ids = torch.from_numpy(ids).to(d) if len(ids) else None
        return torch.from_numpy(img).to(d), torch.from_numpy(st).to(d), torch.from_numpy(nz).to(d), d_ids

    def debug_forward(self, img, st, nz, ids):
        cfg = self.cfg
        n_views, n_prompt = img.shape[0], len(ids)
        d_img, d_st, d_nz, d_ids = self.to_dev(img, st, nz, ids)
        n_taps = binding.pi0_debug_taps_elems(cfg, n_views, n_prompt)
        d_taps = torch.zeros(n_taps, dtype=torch.float32, device=self.dev)
        d_act = torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=self.dev)
        say(f"[gpu] pi0_debug_forward views={n_views} prompt={n_prompt}")
        self.m.pi0_debug_forward(d_img, n_views, d_ids, n_prompt, d_st, d_nz, d_act, d_taps, self.stream)
        self.stream.synchronize()
        say("[gpu] done")
        return d_act.cpu().numpy(), d_taps.cpu().numpy()

    def infer(self, img, st, nz, ids):
        cfg = self.cfg
        d_img, d_st, d_nz, d_ids = self.to_dev(img, st, nz, ids)
        d_act = torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=self.dev)
        self.m.pi0_infer(d_img, img.shape[0], d_ids, len(ids), d_st, d_nz, d_act, self.stream)
        self.stream.synchronize()
        return d_act.cpu().numpy()

    def denoise_only(self, st, nz):
        """pi0_denoise on the cache of the last prefill."""
        cfg = self.cfg
        d_st, d_nz = torch.from_numpy(st).to(self.dev), torch.from_numpy(nz).to(self.dev)
        d_act = torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=self.dev)
        self.m.pi0_denoise(d_st, d_nz, d_act, self.stream)
        self.stream.synchronize()
        return d_act.cpu().numpy()

    def close(self):
        self.m.close()
        self.m.workspace = None
        torch.cuda.empty_cache()


class TalkingTaps(dict):
    """Tap dictionary that reports every tensor the oracle stores: progress lines of a long oracle run (the MXFP8
    oracle of the full model quantises 1.7 G weights in numpy) that come from the run itself."""

    def __setitem__(self, key, value):
        if key.startswith(("llm.x", "vis.out", "kcache")):
            say(f"[oracle] ... {key}")
        super().__setitem__(key, value)


def split_taps(cfg, taps, n_views, n_prompt):
    I = n_views * cfg.tokens_per_view
    P = I + n_prompt
    out, off = {}, 0

    def take(name, shape):
        nonlocal off
        n = int(np.prod(shape))
        out[name] = taps[off:off + n].reshape(shape)
        off += n

    for l in range(cfg.vis_layers):
        take(f"vis.h.{l}", (I, cfg.vis_width))
    take("vis.out", (I, cfg.llm_width))
    for l in range(cfg.llm_layers - 1):
        take(f"llm.x.{l}", (P, cfg.llm_width))
    take("kcache", (cfg.llm_layers, P, cfg.head_dim))
    take("vcache", (cfg.llm_layers, P, cfg.head_dim))
    for k in (0, cfg.steps - 1):
        for l in range(cfg.exp_layers):
            take(f"exp.y.{k}.{l}", (cfg.suffix, cfg.exp_width))
    for k in range(cfg.steps):
        take(f"exp.x.{k}", (cfg.chunk, cfg.action_dim))
    assert off == taps.size
    return out


# Key / value cache, element by element (the one tensor that crosses the prefill / denoise boundary): max |delta| over
# a layer relative to that layer's RMS.  The bar is 2.5 x what bf16 GEMM operands alone do to the ORACLE's cache
# (tests/test_bf16_sensitivity.py, CPU: up to 5.4e-2 at the deepest layers of the full model, 1.2e-1 in the
# sharp-attention configuration): the same factor that the task's 2e-2 action bar has over the rounding-only 4e-3 to
# 8e-3 of the actions.
CACHE_TOL = 0.135
SHARP_CACHE_TOL = 0.30


def check_against_oracle(case, n_views, n_prompt, seed_shift=0, label="", action_tol=ACTION_TOL, mxfp8=False, cos_min=COS_MIN,
                         row_cos_min=0.995, cache_tol=CACHE_TOL):
    cfg = case.cfg
    img, st, nz, ids = case.inputs(n_views, n_prompt, seed_shift)
    say(f"[oracle] forward {label}")
    ref_taps = TalkingTaps() if (mxfp8 and cfg.llm_layers > 4) else {}
    ref = O.pi0_forward(cfg, case.tensors, img, st, nz, ids, dtype=np.float32, taps=ref_taps, prefix_mlp_mxfp8=mxfp8)
    act, taps = case.debug_forward(img, st, nz, ids)
    got = split_taps(cfg, taps, n_views, n_prompt)
    assert np.isfinite(act).all() and np.isfinite(taps).all()
    worst = (1.0, None)
    worst_cache = (0.0, None)
    for name, g in got.items():
        r = ref_taps[name]
        if name in ("kcache", "vcache"):
            for l in range(cfg.llm_layers):
                c = cosine(g[l], r[l])
                worst = min(worst, (c, f"{name}[{l}]"))
                assert c >= cos_min, (label, name, l, c)
                d = float(np.abs(g[l] - r[l]).max()) / math.sqrt(float((r[l].astype(np.float64) ** 2).mean()))
                worst_cache = max(worst_cache, (d, f"{name}[{l}]"))
                assert cache_tol is None or d <= cache_tol, (label, name, l, d)
        else:
            c = cosine(g, r)
            worst = min(worst, (c, name))
            assert c >= cos_min, (label, name, c)
            if name.startswith(("vis.h", "llm.x", "exp.y")):      # per-token cosine, catches single bad rows
                rows = [cosine(g[i], r[i]) for i in range(g.shape[0])]
                assert min(rows) >= row_cos_min, (label, name, int(np.argmin(rows)), min(rows))
                if name.startswith("exp.y"):
                    # the mask's edges by name: the state row (prefix + itself only), the first and the last action row
                    for i in (0, 1, cfg.suffix - 1):
                        assert rows[i] >= row_cos_min, (label, name, "suffix row", i, rows[i])
    rms = math.sqrt(float((ref.astype(np.float64) ** 2).mean()))
    err = float(np.abs(act - ref).max()) / rms
    say(f"[parity] {label}: actions max|d|/rms = {err:.3e}, worst cosine {worst[0]:.6f} at {worst[1]}, "
        f"cache max|d|/rms {worst_cache[0]:.3e} at {worst_cache[1]}")
    assert err <= action_tol, (label, err)
    np.testing.assert_array_equal(act, got[f"exp.x.{cfg.steps - 1}"])
    return act, ref


@pytest.fixture(scope="module")
def reduced():
    c = Case(synth.reduced_config(vocab=1024))
    yield c
    c.close()


def test_reduced_one_view(reduced):
    check_against_oracle(reduced, 1, 0, label="reduced 1 view")


def test_reduced_two_and_three_views(reduced):
    check_against_oracle(reduced, 2, 0, label="reduced 2 views")
    check_against_oracle(reduced, 3, 0, label="reduced 3 views")


def test_reduced_prompt_ragged_prefix(reduced):
    # 3 views + 48 prompt tokens: P = 816 is not a multiple of 32 (ragged key chunk, ragged row tile)
    check_against_oracle(reduced, 3, 48, label="reduced 3 views + 48 prompt")
    # 1 view + 1 prompt token: smallest ragged tail
    check_against_oracle(reduced, 1, 1, seed_shift=10, label="reduced 1 view + 1 prompt")


def test_graph_replay_is_bitwise_equal_to_eager(reduced):
    img, st, nz, ids = reduced.inputs(2, 0)
    eager, _ = reduced.debug_forward(img, st, nz, ids)
    reduced.m.pi0_set_graph_mode(True)
    runs = []
    for i in range(4):                       # first call captures, the rest replay
        runs.append(reduced.infer(img, st, nz, ids))
        # unrelated eager work between replays
        other = reduced.inputs(1, 0, seed_shift=20 + i)
        reduced.infer(*other)
    for r in runs:
        np.testing.assert_array_equal(r, eager)
    reduced.m.pi0_set_graph_mode(False)
    np.testing.assert_array_equal(reduced.infer(img, st, nz, ids), eager)
    reduced.m.pi0_set_graph_mode(True)


def test_prefill_then_denoise_and_streaming(reduced):
    cfg = reduced.cfg
    img, st, nz, ids = reduced.inputs(2, 0)
    full = reduced.infer(img, st, nz, ids)
    d_img, d_st, d_nz, _ = reduced.to_dev(img, st, nz, ids)
    d_act = torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=reduced.dev)
    reduced.m.pi0_prefill(d_img, 2, None, 0, reduced.stream)
    reduced.m.pi0_denoise(d_st, d_nz, d_act, reduced.stream)
    reduced.stream.synchronize()
    np.testing.assert_array_equal(d_act.cpu().numpy(), full)
    # streaming use: fresh state/noise on the same cache, output aliasing the noise buffer
    W = O.Weights(reduced.tensors, np.float32)
    Ks, Vs = O.prefix_forward(cfg, W, img, None)
    for j in range(2):
        st2 = synth.make_state(cfg, seed=50 + j)
        nz2 = synth.make_noise(cfg, seed=100 + j)
        ref = O.denoise(cfg, W, Ks, Vs, st2, nz2)
        d_buf = torch.from_numpy(nz2).to(reduced.dev)
        reduced.m.pi0_denoise(torch.from_numpy(st2).to(reduced.dev), d_buf, d_buf, reduced.stream)
        reduced.stream.synchronize()
        rms = math.sqrt(float((ref.astype(np.float64) ** 2).mean()))
        err = float(np.abs(d_buf.cpu().numpy() - ref).max()) / rms
        say(f"[parity] streaming chunk {j}: {err:.3e}")
        assert err <= ACTION_TOL


def test_denoise_without_prefill_is_an_error():
    cfg = synth.reduced_config()
    m = binding.Pi0(cfg)
    x = torch.zeros(4096, dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.Pi0Error) as e:
        m.pi0_denoise(x, x, x, None)
    assert e.value.code == binding.PI0_ESTATE
    m.close()


def test_sharp_attention_masks():
    """N(0, 0.02) weights give nearly uniform attention, which hides mask / RoPE / scale bugs.
    Query/key projections drawn 2.5x wider give logits with a standard deviation of about 5 in the
    prefix and expert (3 in the vision tower): attention is concentrated on a few keys, so a wrong
    mask block, position offset or softmax scale moves the hidden states far beyond the cosine bar.
    Much sharper settings are not a fair test of any bf16 implementation: the logit error is the
    relative error of q and k times the logit magnitude, and at a logit deviation of 30 the oracle
    itself turns a 4.5 % input perturbation into a cosine of 0.96 after one layer.  For the same
    reason the action bar of this stress configuration is 5e-2 (the 2e-2 bar belongs to the
    N(0, 0.02) workloads); the per-layer cosine bar is unchanged.  Where 5e-2 comes from is a CPU test
    (tests/test_bf16_sensitivity.py): the oracle itself, with nothing changed but its GEMM inputs rounded to
    bf16, moves by 2.0e-2 of the action RMS on exactly this case (3e-3 on the N(0, 0.02) weights, where the
    bar is 2e-2: the same factor 2.5 above the rounding-only figure), and by 0.18 at a deviation of 0.08."""
    case = Case(synth.reduced_config(vocab=1024), seed=5, overrides={"wq": 0.05, "wk": 0.05})
    try:
        check_against_oracle(case, 2, 7, label="sharp attention 2 views + 7 prompt", action_tol=SHARP_ACTION_TOL,
                             cache_tol=SHARP_CACHE_TOL)
    finally:
        case.close()


def test_full_model_all_view_counts():
    """The benchmark's workloads (full depth; one, two and three views; empty prompt, Table 1) end to
    end against the oracle, in the launch configuration the benchmark times (graph replay)."""
    case = Case(synth.full_config())
    try:
        for n_views in (1, 2, 3):
            act, ref = check_against_oracle(case, n_views, 0, label=f"full {n_views} view")
            # the graph path the benchmark times gives the same bits
            img, st, nz, ids = case.inputs(n_views, 0)
            np.testing.assert_array_equal(case.infer(img, st, nz, ids), act)
            np.testing.assert_array_equal(case.infer(img, st, nz, ids), act)
        # the reduced-precision mode at full depth against the oracle in the same mode (17 quantised layers)
        case.m.pi0_set_precision("mxfp8_prefix_mlp")
        act, _ = check_against_oracle(case, 1, 0, label="full 1 view, mxfp8 prefix feed-forward", mxfp8=True,
                                      action_tol=MX_FULL_ACTION_TOL, cos_min=MX_FULL_COS_MIN,
                                      row_cos_min=MX_FULL_ROW_COS_MIN, cache_tol=None)
        img, st, nz, ids = case.inputs(1, 0)
        np.testing.assert_array_equal(case.infer(img, st, nz, ids), act)
        case.m.pi0_set_precision("bf16")
    finally:
        case.close()


def test_full_model_three_views_and_prompt_with_the_full_embedding_table():
    """The largest configuration: full depth, 3 views + a 48-token prompt drawn from the 257152-row embedding table
    (816 prefix tokens: ragged last key chunk, four key shares in the expert's attention, the 256-token gate||up
    tile), end to end against the oracle; the graph path gives the same bits; and the streaming use - pi0_denoise
    alone on that cache with fresh state / noise - against the oracle's denoise on its own cache."""
    cfg = synth.full_config(vocab=257152)
    case = Case(cfg)
    try:
        n_views, n_prompt = 3, 48
        act, ref = check_against_oracle(case, n_views, n_prompt, label="full 3 views + 48 prompt, 257152-row table")
        img, st, nz, ids = case.inputs(n_views, n_prompt)
        assert int(ids.max()) > 65536          # the gather reaches rows far into the table
        np.testing.assert_array_equal(case.infer(img, st, nz, ids), act)
        np.testing.assert_array_equal(case.infer(img, st, nz, ids), act)
        W = O.Weights(case.tensors, np.float32)
        say("[oracle] prefix for the streaming chunks")
        Ks, Vs = O.prefix_forward(cfg, W, img, ids)
        for j in range(2):
            st2, nz2 = synth.make_state(cfg, seed=50 + j), synth.make_noise(cfg, seed=100 + j)
            want = O.denoise(cfg, W, Ks, Vs, st2, nz2)
            got = case.denoise_only(st2, nz2)
            rms = math.sqrt(float((want.astype(np.float64) ** 2).mean()))
            err = float(np.abs(got - want).max()) / rms
            say(f"[parity] full model, 816 prefix tokens, streaming chunk {j}: {err:.3e}")
            assert err <= ACTION_TOL
        case.m.pi0_device_status(case.stream)
    finally:
        case.close()


def test_sync_overhead_microbenchmark():
    """Table 3's experiment (Section 5.2): every ordering mode applies exactly n_ops updates; the software
    barriers terminate; one unsynchronised kernel is the cheapest variant."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(device=dev)
    g = torch.Generator().manual_seed(7)
    x0 = torch.randint(-8, 8, (256, 1024), generator=g).float()
    b = torch.randint(0, 3, (256, 1024), generator=g).float()
    n_ops, reps = 1378, 2
    times = {}
    for mode in ("eager", "graph", "barrier", "barrier_fence", "fused"):
        say(f"[gpu] pi0_sync_bench {mode}")
        d_x, d_b = x0.to(dev), b.to(dev)
        d_state = torch.zeros(2, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        times[mode] = binding.pi0_sync_bench(mode, n_ops, reps, d_x, d_b, d_state, stream)
        torch.testing.assert_close(d_x.cpu(), x0 + reps * n_ops * b, rtol=0, atol=0)
        assert int(d_state[1].item()) == 0
    say("[sync] ms per 1378 updates: " + ", ".join(f"{k} {v:.3f}" for k, v in times.items()))
    assert times["fused"] < times["graph"] < times["eager"] * 1.5
    assert times["fused"] < times["barrier"]


def test_attainable_peak_microbenchmarks():
    """The two device micro-benchmarks behind the roofline fractions (Section 5.1): a streaming read and a
    register-resident bf16 MFMA loop finish, leave their input alone and land between a floor that any
    working MI355X exceeds and the published peak."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(device=dev)
    g = torch.Generator().manual_seed(11)
    n = (512 << 20) // 4 + 12                                  # 512 MiB and a ragged tail of 3 sixteen-byte words
    host = torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), dtype=torch.int32, generator=g)
    buf = host.to(dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    say("[gpu] pi0_peak_bench hbm_read")
    gbps = binding.pi0_peak_bench("hbm_read", buf, n * 4, 0, 10, sink, stream)
    say("[gpu] pi0_peak_bench mfma_bf16")
    tflops = binding.pi0_peak_bench("mfma_bf16", None, 0, 2048, 10, sink, stream)
    say(f"[peak] HBM read {gbps:.0f} GB/s, bf16 MFMA {tflops:.0f} TFLOP/s")
    assert 1500.0 < gbps < 8000.0
    assert 500.0 < tflops < 2600.0
    say("[gpu] pi0_peak_bench cache_read")
    l2 = binding.pi0_peak_bench("cache_read", buf, 8 << 20, 32, 5, sink, stream)    # 1 MiB per die, shared by its 32 blocks
    say(f"[peak] L2 hits into the compute units {l2:.0f} GB/s")
    assert 4000.0 < l2 < 256 * 64 * 3.0        # above HBM's rate, below 64 B/clk per compute unit at 3 GHz
    with pytest.raises(binding.Pi0Error):
        binding.pi0_peak_bench("cache_read", buf, 8 << 20, 0, 1, sink, stream)
    with pytest.raises(binding.Pi0Error):
        binding.pi0_peak_bench("cache_read", buf, 1000, 4, 1, sink, stream)
    assert torch.equal(buf.cpu(), host)
    with pytest.raises(binding.Pi0Error):
        binding.pi0_peak_bench("hbm_read", buf, n * 4 + 4, 0, 1, sink, stream)
    # clock samples around ~0.2 s of streaming reads: a plausible shader clock
    c0 = torch.zeros(2, dtype=torch.int64, device=dev)
    c1 = torch.zeros(2, dtype=torch.int64, device=dev)
    binding.pi0_clock_sample(c0, stream)
    binding.pi0_peak_bench("hbm_read", buf, n * 4, 0, 1000, sink, stream)
    binding.pi0_peak_bench("hbm_read", buf, n * 4, 0, 1000, sink, stream)
    binding.pi0_clock_sample(c1, stream)
    stream.synchronize()
    ghz = binding.shader_clock_ghz(c0.cpu().tolist(), c1.cpu().tolist())
    say(f"[peak] shader clock {ghz:.3f} GHz")
    assert 0.5 < ghz < 3.0


def test_read_ahead_kernel_follows_its_counter_and_gives_up_when_it_stalls():
    """The expert's read-ahead kernel (Section 5.2's prefetch across synchronisation points) alone on a stream:
    with the counter ahead of it, it walks the whole buffer; with a counter that never moves, every block gives
    up after one bound instead of waiting for a partner stream that is not there; it writes nothing."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(device=dev)
    g = torch.Generator().manual_seed(5)
    host = torch.randint(-2 ** 31, 2 ** 31 - 1, ((256 << 20) // 4,), dtype=torch.int32, generator=g)
    buf = host.to(dev)
    sink = torch.zeros(1024, dtype=torch.int32, device=dev)
    prog = torch.zeros(1, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    say("[gpu] pi0_read_ahead_probe, unpaced")
    binding.pi0_read_ahead_probe(buf, 8, 4, 32, prog, 100000, 256, sink, stream)              # first launch: code upload
    ms_free = binding.pi0_read_ahead_probe(buf, 8, 4, 32, prog, 100000, 256, sink, stream)    # lead 32 of 32: 4 x 256 MiB, no waits
    say(f"[read-ahead] 1 GiB unpaced: {ms_free:.3f} ms ({1.074 / ms_free:.2f} TB/s)")
    assert 0.03 < ms_free < 20.0
    # a compute stream that is far ahead: every slice is skipped
    prog.fill_(1 << 20)
    torch.cuda.synchronize()
    say("[gpu] pi0_read_ahead_probe, counter far ahead")
    ms_skip = binding.pi0_read_ahead_probe(buf, 8, 4, 1, prog, 100000, 256, sink, stream)
    say(f"[read-ahead] all 32 slices skipped: {ms_skip:.3f} ms")
    assert ms_skip < 0.5 * ms_free
    prog.zero_()
    torch.cuda.synchronize()
    say("[gpu] pi0_read_ahead_probe, counter never moves, bound 1 ms")
    ms_1 = binding.pi0_read_ahead_probe(buf, 8, 4, 1, prog, 100000, 256, sink, stream)        # slice 0, then one wait of 1 ms
    say("[gpu] pi0_read_ahead_probe, counter never moves, bound 20 us")
    ms_2 = binding.pi0_read_ahead_probe(buf, 8, 4, 1, prog, 2000, 256, sink, stream)
    say(f"[read-ahead] stalled: {ms_1:.3f} ms with a 1 ms bound, {ms_2:.3f} ms with a 20 us bound")
    assert 0.9 < ms_1 < 3.0
    assert ms_2 < 0.5
    # the counter lets it through slices 1 and 2 of 8 (lead 1: slice i needs counter >= i; slice 0 is skipped as stale),
    # then it stalls for one bound
    prog.fill_(2)
    torch.cuda.synchronize()
    say("[gpu] pi0_read_ahead_probe, counter at 2, bound 1 ms")
    ms_3 = binding.pi0_read_ahead_probe(buf, 8, 1, 1, prog, 100000, 256, sink, stream)
    assert 0.9 < ms_3 < 3.0
    # two slices ahead of the counter instead of one: slice i needs counter >= i - 1, so a counter of 6 lets it reach the end
    prog.fill_(6)
    torch.cuda.synchronize()
    say("[gpu] pi0_read_ahead_probe, counter at 6, two ahead")
    ms_4 = binding.pi0_read_ahead_probe(buf, 8, 1, 2, prog, 100000, 256, sink, stream)
    assert ms_4 < 0.9
    assert torch.equal(buf.cpu(), host) and int(sink.abs().sum()) == 0 and int(prog.item()) == 6
    with pytest.raises(binding.Pi0Error):
        binding.pi0_read_ahead_probe(buf, 7, 1, 1, prog, 1000, 256, sink, stream)               # 256 MiB is not 7 * 16 * n


def test_mxfp8_prefix_mlp_against_mxfp8_oracle(reduced):
    """Reduced-precision mode (prefix gate||up / down on MXFP8 operands) against the oracle that rounds the same
    operands through MXFP8 by the format's definition; the mode really changes the numbers; switching back
    restores the bf16 results bit for bit."""
    img, st, nz, ids = reduced.inputs(1, 0)
    before = reduced.infer(img, st, nz, ids)
    reduced.m.pi0_set_precision("mxfp8_prefix_mlp")
    try:
        act1, ref1 = check_against_oracle(reduced, 1, 0, label="mxfp8 1 view", mxfp8=True, action_tol=MX_ACTION_TOL,
                                          cos_min=MX_COS_MIN, row_cos_min=MX_ROW_COS_MIN, cache_tol=2 * CACHE_TOL)
        check_against_oracle(reduced, 3, 48, label="mxfp8 3 views + 48 prompt", mxfp8=True, action_tol=MX_ACTION_TOL,
                             cos_min=MX_COS_MIN, row_cos_min=MX_ROW_COS_MIN, cache_tol=2 * CACHE_TOL)
        # graph replays of the mode equal its eager debug pass
        np.testing.assert_array_equal(reduced.infer(img, st, nz, ids), act1)
        np.testing.assert_array_equal(reduced.infer(img, st, nz, ids), act1)
        # not the bf16 path under another name: the prefix hidden state is much closer to the MXFP8 oracle than to
        # the plain one
        taps_plain, taps_mx = {}, {}
        O.pi0_forward(reduced.cfg, reduced.tensors, img, st, nz, ids, taps=taps_plain)
        O.pi0_forward(reduced.cfg, reduced.tensors, img, st, nz, ids, taps=taps_mx, prefix_mlp_mxfp8=True)
        _, taps = reduced.debug_forward(img, st, nz, ids)
        x0 = split_taps(reduced.cfg, taps, 1, 0)["llm.x.0"]
        d_mx, d_plain = 1 - cosine(x0, taps_mx["llm.x.0"]), 1 - cosine(x0, taps_plain["llm.x.0"])
        say(f"[mxfp8] 1 - cos of llm.x.0: {d_mx:.2e} to the MXFP8 oracle, {d_plain:.2e} to the plain oracle")
        assert d_mx < 0.5 * d_plain
        assert np.abs(act1 - before).max() > 0
    finally:
        reduced.m.pi0_set_precision("bf16")
    np.testing.assert_array_equal(reduced.infer(img, st, nz, ids), before)
    with pytest.raises(binding.Pi0Error):
        reduced.m._check(binding.lib().pi0_set_precision(reduced.m._ctx, 2))


def test_two_stream_frames_match_sequential(reduced):
    """Section 6's concurrent mode: frame k's prefill runs beside the denoise against frame k-1's cache
    (double-buffered).  Same kernels, so every chunk must equal, bit for bit, what pi0_prefill +
    pi0_denoise give sequentially; view counts change between frames; no host synchronisation
    between frames."""
    cfg, m, dev = reduced.cfg, reduced.m, reduced.dev
    sp, sd = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
    views = [1, 2, 1, 3, 2]
    frames = [reduced.inputs(v, 0, seed_shift=40 + k) for k, v in enumerate(views)]
    dev_frames = [reduced.to_dev(*f) for f in frames]
    torch.cuda.synchronize()
    # sequential reference: actions of frame k use the cache of frame k-1
    ref = []
    for k in range(1, len(views)):
        d_img, _, _, _ = dev_frames[k - 1]
        _, d_st, d_nz, _ = dev_frames[k]
        out = torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=dev)
        m.pi0_prefill(d_img, views[k - 1], None, 0, reduced.stream)
        m.pi0_denoise(d_st, d_nz, out, reduced.stream)
        reduced.stream.synchronize()
        ref.append(out.cpu().numpy())
    # the denoise of a frame: the persistent loop on a part of the chip (default grid, and an odd one), or per-operation
    # launches (psb=0); the second round of each replays the captured graphs
    for tune in ("psb=-1", "psb=-1", "psb=0", "psb=0", "psb=72", "psb=-1"):
        m.pi0_tune(tune)
        outs = [torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=dev) for _ in views[1:]]
        say(f"[gpu] pi0_stream_frame {tune}")
        m.pi0_prefill(dev_frames[0][0], views[0], None, 0, sp)
        for k in range(1, len(views)):
            d_img, d_st, d_nz, _ = dev_frames[k]
            m.pi0_stream_frame(d_img, views[k], None, 0, d_st, d_nz, outs[k - 1], sp, sd)
        sp.synchronize()
        sd.synchronize()
        m.pi0_device_status(sd)      # no bounded wait of the loop ran out
        for k, (o, r) in enumerate(zip(outs, ref)):
            np.testing.assert_array_equal(o.cpu().numpy(), r, err_msg=f"{tune} frame {k + 1}")
    # one streamed frame against the oracle itself: the chunk of frame 3 belongs to frame 2's images
    k = 3
    say("[oracle] streamed frame")
    want = O.pi0_forward(cfg, reduced.tensors, frames[k - 1][0], frames[k][1], frames[k][2], None)
    rms = math.sqrt(float((want.astype(np.float64) ** 2).mean()))
    err = float(np.abs(outs[k - 1].cpu().numpy() - want).max()) / rms
    say(f"[parity] streamed frame {k}: {err:.3e}")
    assert err <= ACTION_TOL
    # the plain entry points keep working on whichever cache copy is current after streaming
    k = 2
    d_img, _, _, _ = dev_frames[k - 1]
    _, d_st, d_nz, _ = dev_frames[k]
    out = torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=dev)
    m.pi0_infer(d_img, views[k - 1], None, 0, d_st, d_nz, out, reduced.stream)
    reduced.stream.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), ref[k - 1])
    m.pi0_denoise(d_st, d_nz, out, reduced.stream)
    reduced.stream.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), ref[k - 1])


def test_persistent_denoise_loop_equals_per_operation_launches():
    """The denoise loop as one persistent kernel with software grid barriers (Section 5.2) runs the same bodies on
    the same work items as the per-operation launches: same bits, for one prefix share (1 view), two (2 views), three
    (3 views) and four ragged ones (3 views + 48 prompt tokens), as a graph replay and eagerly, also through
    pi0_denoise alone on the cached prefix with fresh noise; no barrier wait runs out."""
    cfg = synth.reduced_config(vocab=1024)
    shapes = [(1, 0), (2, 0), (3, 0), (3, 48), (1, 7)]
    outs = {}
    for tune in ("pdn=0", "pdn=1"):
        case = Case(cfg, tune=tune)
        try:
            for n_views, n_prompt in shapes:
                say(f"[gpu] {tune} views={n_views} prompt={n_prompt}")
                img, st, nz, ids = case.inputs(n_views, n_prompt)
                a = case.infer(img, st, nz, ids)
                b = case.infer(img, st, nz, ids)          # replay
                case.m.pi0_set_graph_mode(False)
                c = case.infer(img, st, nz, ids)          # eager
                case.m.pi0_set_graph_mode(True)
                np.testing.assert_array_equal(a, b)
                np.testing.assert_array_equal(a, c)
                # streaming use: denoise alone on the cache of the prefill above, other state / noise
                _, st2, nz2, _ = case.inputs(n_views, n_prompt, seed_shift=50)
                d = case.denoise_only(st2, nz2)
                assert np.isfinite(d).all() and not np.array_equal(d, a)
                outs[(tune, n_views, n_prompt)] = (a, d)
            case.m.pi0_device_status(case.stream)
            n_launch = case.m.pi0_kernel_count(1, 0)
            say(f"[gpu] {tune}: {n_launch} launches per pi0_infer at 1 view")
            outs[(tune, "launches")] = n_launch
        finally:
            case.close()
    for n_views, n_prompt in shapes:
        for i, what in enumerate(("infer", "denoise")):
            np.testing.assert_array_equal(outs[("pdn=1", n_views, n_prompt)][i], outs[("pdn=0", n_views, n_prompt)][i],
                                          err_msg=f"{what} views={n_views} prompt={n_prompt}")
    # 5 launches per layer-step and 3 per Euler step become 3 launches in all
    assert outs[("pdn=0", "launches")] - outs[("pdn=1", "launches")] >= 10 * (5 * cfg.exp_layers + 3) - 3


def test_reading_ahead_changes_no_bit():
    """The expert's read-ahead kernel and the warm-up blocks only load: the actions of a pass with either of them,
    with neither, and with another shape of the read-ahead kernel are the same bits (graph replay and eager), and the
    persistent loop gives the bits of the per-operation launches, whatever its idle blocks read ahead (pra).  The number of blocks that share the value slices of the
    expert attention fixes how the second product is shared out over a block's waves, i.e. the order of an fp32 sum:
    for each such number the persistent loop and the launches agree bit for bit, and between the numbers the actions
    differ by rounding only."""
    import os
    outs = {}
    for tune in ("", "pdn=0", "pdn=0,ras=0", "pdn=0,ras=0,pfq=0,pfa=0,pfo=0,pfd=0", "pdn=0,ras=128,rat=128,rad=3,ral=2", "pdn=0,avs=1",
                 "pdn=0,avs=8", "avs=1", "avs=8", "pdn=0,avs=2", "avs=2", "pra=0", "pra=63"):
        if tune:
            os.environ["PI0_TUNE"] = tune
        try:
            case = Case(synth.reduced_config(vocab=1024))
        finally:
            os.environ.pop("PI0_TUNE", None)
        try:
            img, st, nz, ids = case.inputs(2, 16)
            say(f"[gpu] pi0_infer tune={tune!r}")
            a = case.infer(img, st, nz, ids)
            b = case.infer(img, st, nz, ids)          # replay
            case.m.pi0_set_graph_mode(False)
            c = case.infer(img, st, nz, ids)          # eager
            np.testing.assert_array_equal(a, b)
            np.testing.assert_array_equal(a, c)
            outs[tune] = a
        finally:
            case.close()
    for tune, a in outs.items():
        if "avs" not in tune:
            np.testing.assert_array_equal(a, outs[""], err_msg=f"PI0_TUNE={tune}")
    for n in (1, 2, 8):   # avs=1 has no persistent form: both runs are the launches
        np.testing.assert_array_equal(outs[f"avs={n}"], outs[f"pdn=0,avs={n}"], err_msg=f"avs={n}")
        rms = float(np.sqrt(np.mean(outs[""].astype(np.float64) ** 2)))
        d = float(np.abs(outs[f"avs={n}"].astype(np.float64) - outs[""]).max())
        say(f"[parity] avs={n} vs default: max|delta| {d / rms:.2e} of RMS")
        # another order of an fp32 sum flips a bf16 rounding of the attention output here and there, and a flipped rounding
        # travels like any other: the bar is that of rounding alone (3e-3 of RMS moves the ORACLE under bf16 operands,
        # tests/test_bf16_sensitivity.py), measured 2.3e-3
        assert d <= 5e-3 * rms


@pytest.mark.parametrize("tune", [
    "ae16=0,qms=0,ksplit=0,pfq=0,pfa=0,pfo=0,pfd=0,lgu=0,ld=0",                        # 32x32 expert tiles, no warm-up, no key shares, 256x128 gate||up and down
    "vis=0,vqkv=0,vup=0,lqkv=0,lgu=1,vo=0,vd=0,lo=0,ld=1,zvo=6,zvd=17,zlo=8,zld=4",    # the other tile of every prefill GEMM
    "vis=5,vqkv=5,vup=5,lqkv=5,vo=5,vd=5,lo=5,zvo=1,zvd=2,zlo=1,kcps=4",               # 64x64 tiles, few splits, small key shares
    "lgu=6,ld=7,zld=4",                                                                # two feature tiles per wave: 256x256 gate||up, 128x256 down
    "lgu=7,ld=6,zld=8",                                                                # ... and the other way round
    "lgu=10,ld=10,zld=8",                                                              # 192-token tiles (768 tokens in four)
    "vis=9,vqkv=9,vup=9,lqkv=9,vo=9,vd=9,lo=9,zvo=2,zvd=3,zlo=2,fko=0,fkl=0",          # 128x128 tiles everywhere they exist
    "vqkv=11,vup=11,lqkv=11,vo=11,vd=11,lo=11,fko=0,fkl=0",                            # 64x128 tiles cut for two resident blocks per compute unit
    "fko=1,fkl=1",                                                                     # O projections over the whole k range, residual epilogue in the GEMM
    "fko=0,fkl=0",                                                                     # ... and as split-K partial GEMMs + reduction
    "ras=64,ral=2,rat=128,rad=8",                                                      # expert read-ahead kernel: other shape, two layers ahead
    "ras=0",                                                                           # ... and none: warm-up blocks inside the expert's launches
    "avs=1",                                                                           # expert attention: one block per (query tile, head)
    "avs=8,ras=0",                                                                     # ... its value slices over 8 blocks, warm-up blocks in the launch
])
def test_alternative_kernel_choices(tune):
    """Every tile / split / warm-up choice the tuning variable can select computes the same function."""
    import os
    os.environ["PI0_TUNE"] = tune
    try:
        case = Case(synth.reduced_config(vocab=1024))
    finally:
        del os.environ["PI0_TUNE"]
    try:
        check_against_oracle(case, 3, 48, label=f"tune {tune}")
        check_against_oracle(case, 1, 0, label=f"tune {tune} (1 view)")
    finally:
        case.close()
