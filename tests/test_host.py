"""Host-side checks that need no GPU: the library loads, exports what the header declares,
rejects bad arguments before touching the GPU, and agrees with the generators on blob size.
Also pins the roofline calculator to the numbers the paper prints in Table 2 / Section 5.1."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2510_26742_amd import binding, roofline, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding.lib()


def test_header_symbols_are_exported(L):
    declared = []
    for name in ("pi0.h", "pi0_bench.h"):
        hdr = open(os.path.join(ROOT, "include", name)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
        found = set(re.findall(r"\b(pi0_[a-z_0-9]+)\s*\(", hdr))
        assert found, f"no declarations found in {name}"
        declared += sorted(found)
    declared = sorted(set(declared))
    assert sorted(binding.EXPORTS) == declared
    for name in declared:
        assert hasattr(L, name), name


def test_strerror(L):
    for code in (0, -1, -2, -3, -4, -5, -99):
        s = L.pi0_strerror(code)
        assert s and len(s) > 1


@pytest.mark.parametrize("cfg", [synth.reduced_config(), synth.full_config(), synth.full_config(vocab=257152)])
def test_blob_size_matches_generator_layout(L, cfg):
    _, total = synth.blob_layout(cfg)
    assert binding.pi0_weights_bytes(cfg) == total * 2
    assert binding.pi0_workspace_bytes(cfg) > total * 2 * 0.9


def test_full_model_sizes_are_plausible(L):
    cfg = synth.full_config()
    gb = binding.pi0_weights_bytes(cfg) / 1e9
    assert 5.0 < gb < 6.5          # ~2.7-3.2 B parameters in bf16 (SigLIP 0.4 B, Gemma 2 B+, expert 0.3 B)
    assert binding.pi0_workspace_bytes(cfg) < 8e9


def test_create_rejects_bad_geometry(L):
    good = synth.reduced_config()
    bad = [dict(head_dim=128), dict(chunk=31), dict(vis_width=1150), dict(exp_layers=3), dict(steps=0),
           dict(max_views=0), dict(patch=15), dict(state_dim=33), dict(vis_heads=7), dict(llm_layers=1),
           dict(max_views=4, max_prompt=1),      # 1025 prefix tokens: beyond the attention kernels' 32 key chunks
           dict(img_size=448),                   # 1024 tokens per view: beyond one round of the vision attention
           dict(vis_heads=18)]                   # vision head dim 64: no such attention variant
    for kw in bad:
        c = binding.to_c_config(synth.dataclasses.replace(good, **kw))
        ctx = ctypes.c_void_p()
        assert L.pi0_create(ctypes.byref(c), ctypes.byref(ctx)) == binding.PI0_EINVAL, kw
        assert not ctx
        assert L.pi0_weights_bytes(ctypes.byref(c)) == 0
        assert L.pi0_workspace_bytes(ctypes.byref(c)) == 0
    ctx = ctypes.c_void_p()
    assert L.pi0_create(None, ctypes.byref(ctx)) == binding.PI0_EINVAL
    c = binding.to_c_config(good)
    assert L.pi0_create(ctypes.byref(c), None) == binding.PI0_EINVAL


def test_error_paths_before_any_gpu_call(L):
    cfg = synth.reduced_config()
    c = binding.to_c_config(cfg)
    ctx = ctypes.c_void_p()
    assert L.pi0_create(ctypes.byref(c), ctypes.byref(ctx)) == 0
    fake = 0x10000                       # never dereferenced: every call below fails its checks first
    nbytes = binding.pi0_weights_bytes(cfg)
    ws = binding.pi0_workspace_bytes(cfg)
    assert L.pi0_load_weights(ctx, None, nbytes, fake, ws, None) == binding.PI0_EINVAL
    assert L.pi0_load_weights(ctx, fake, nbytes, None, ws, None) == binding.PI0_EINVAL
    assert L.pi0_load_weights(ctx, fake, nbytes, fake + 8, ws, None) == binding.PI0_EINVAL      # misaligned
    assert L.pi0_load_weights(ctx, fake, nbytes - 2, fake, ws, None) == binding.PI0_EFORMAT
    assert L.pi0_load_weights(ctx, fake, nbytes, fake, ws - 1, None) == binding.PI0_ENOMEM
    assert L.pi0_load_weights(None, fake, nbytes, fake, ws, None) == binding.PI0_EINVAL
    # not loaded yet
    assert L.pi0_prefill(ctx, fake, 1, None, 0, None) == binding.PI0_ESTATE
    assert L.pi0_denoise(ctx, fake, fake, fake, None) == binding.PI0_ESTATE
    assert L.pi0_infer(ctx, fake, 1, None, 0, fake, fake, fake, None) == binding.PI0_ESTATE
    # argument checks win over state checks
    assert L.pi0_prefill(ctx, None, 1, None, 0, None) == binding.PI0_EINVAL
    assert L.pi0_prefill(ctx, fake, 0, None, 0, None) == binding.PI0_EINVAL
    assert L.pi0_prefill(ctx, fake, 4, None, 0, None) == binding.PI0_EINVAL
    assert L.pi0_prefill(ctx, fake, 1, None, 3, None) == binding.PI0_EINVAL         # ids missing
    assert L.pi0_prefill(ctx, fake, 1, fake, 3, None) == binding.PI0_EINVAL         # no embedding table (vocab 0)
    assert L.pi0_prefill(ctx, fake, 1, fake, 49, None) == binding.PI0_EINVAL
    assert L.pi0_denoise(ctx, None, fake, fake, None) == binding.PI0_EINVAL
    assert L.pi0_infer(ctx, fake, 1, None, 0, fake, fake, None, None) == binding.PI0_EINVAL
    assert L.pi0_debug_forward(ctx, fake, 1, None, 0, fake, fake, fake, None, 0, None) == binding.PI0_EINVAL
    # two-stream frame: streams must be two different non-null streams, and a prefill must exist
    assert L.pi0_stream_frame(ctx, fake, 1, None, 0, fake, fake, fake, None, fake) == binding.PI0_EINVAL
    assert L.pi0_stream_frame(ctx, fake, 1, None, 0, fake, fake, fake, fake, fake) == binding.PI0_EINVAL
    assert L.pi0_stream_frame(ctx, fake, 1, None, 0, fake, None, fake, fake, fake + 64) == binding.PI0_EINVAL
    assert L.pi0_stream_frame(ctx, fake, 1, None, 0, fake, fake, fake, fake, fake + 64) == binding.PI0_ESTATE
    # per-class timing run
    us = (ctypes.c_double * len(binding.OP_CLASSES))()
    n = (ctypes.c_int * len(binding.OP_CLASSES))()
    assert L.pi0_debug_profile(ctx, fake, 1, None, 0, fake, fake, fake, 0, us, n, None) == binding.PI0_EINVAL
    assert L.pi0_debug_profile(ctx, fake, 1, None, 0, fake, fake, fake, 1, None, n, None) == binding.PI0_EINVAL
    assert L.pi0_debug_profile(ctx, fake, 1, None, 0, fake, fake, fake, 1, us, n, None) == binding.PI0_ESTATE
    assert L.pi0_last_hip_error(ctx) == 0
    L.pi0_destroy(ctx)
    L.pi0_destroy(None)


def test_sync_bench_rejects_bad_arguments(L):
    fake = 0x10000
    ms = ctypes.c_double(0.0)
    ok = (1, 10, 1, fake, fake, fake)
    assert L.pi0_sync_bench(5, 10, 1, fake, fake, fake, ctypes.byref(ms), None) == binding.PI0_EINVAL      # unknown mode
    assert L.pi0_sync_bench(-1, 10, 1, fake, fake, fake, ctypes.byref(ms), None) == binding.PI0_EINVAL
    assert L.pi0_sync_bench(0, 0, 1, fake, fake, fake, ctypes.byref(ms), None) == binding.PI0_EINVAL       # no updates
    assert L.pi0_sync_bench(0, 10, 0, fake, fake, fake, ctypes.byref(ms), None) == binding.PI0_EINVAL      # no repetitions
    assert L.pi0_sync_bench(0, 10, 1, None, fake, fake, ctypes.byref(ms), None) == binding.PI0_EINVAL
    assert L.pi0_sync_bench(0, 10, 1, fake + 4, fake, fake, ctypes.byref(ms), None) == binding.PI0_EINVAL  # misaligned
    assert L.pi0_sync_bench(0, 10, 1, fake, fake, None, ctypes.byref(ms), None) == binding.PI0_EINVAL
    assert L.pi0_sync_bench(0, 10, 1, fake, fake, fake, None, None) == binding.PI0_EINVAL
    assert len(binding.OP_CLASSES) == 21 and binding.SYNC_MODES["fused"] == 4


def test_set_precision_arguments(L):
    cfg = synth.reduced_config(vocab=16)
    c = binding.to_c_config(cfg)
    ctx = ctypes.c_void_p()
    assert L.pi0_create(ctypes.byref(c), ctypes.byref(ctx)) == 0
    n_bf16 = L.pi0_kernel_count(ctx, 1, 0)
    assert L.pi0_set_precision(None, 0) == binding.PI0_EINVAL
    assert L.pi0_set_precision(ctx, 2) == binding.PI0_EINVAL and L.pi0_set_precision(ctx, -1) == binding.PI0_EINVAL
    assert L.pi0_set_precision(ctx, 1) == binding.PI0_OK
    # per prefix layer with a feed-forward block: the O projection keeps its reduction launch (it quantises gate||up's input)
    assert L.pi0_kernel_count(ctx, 1, 0) == n_bf16 + (cfg.llm_layers - 1)
    assert L.pi0_set_precision(ctx, 0) == binding.PI0_OK and L.pi0_kernel_count(ctx, 1, 0) == n_bf16
    L.pi0_destroy(ctx)
    # widths that are not multiples of 256 cannot use the MXFP8 kernels
    import dataclasses
    odd = binding.to_c_config(dataclasses.replace(cfg, llm_width=2048 + 64))
    ctx2 = ctypes.c_void_p()
    if L.pi0_create(ctypes.byref(odd), ctypes.byref(ctx2)) == 0:
        assert L.pi0_set_precision(ctx2, 1) == binding.PI0_EINVAL
        L.pi0_destroy(ctx2)


def test_peak_bench_rejects_bad_arguments(L):
    fake = 0x10000
    out = ctypes.c_double(0.0)
    r = ctypes.byref(out)
    assert L.pi0_peak_bench(3, fake, 1 << 20, 16, 1, fake, r, None) == binding.PI0_EINVAL          # unknown kind
    assert L.pi0_peak_bench(2, None, 1 << 20, 16, 1, fake, r, None) == binding.PI0_EINVAL          # cache read: no buffer
    assert L.pi0_peak_bench(2, fake, 1 << 15, 16, 1, fake, r, None) == binding.PI0_EINVAL          # slices too small
    assert L.pi0_peak_bench(2, fake, (1 << 20) + 64, 16, 1, fake, r, None) == binding.PI0_EINVAL   # not 8 equal slices of 16-byte words
    assert L.pi0_peak_bench(2, fake, 1 << 20, 0, 1, fake, r, None) == binding.PI0_EINVAL           # no passes
    assert L.pi0_peak_bench(0, None, 1 << 20, 0, 1, fake, r, None) == binding.PI0_EINVAL            # no buffer
    assert L.pi0_peak_bench(0, fake, 0, 0, 1, fake, r, None) == binding.PI0_EINVAL                  # nothing to read
    assert L.pi0_peak_bench(0, fake, (1 << 20) + 8, 0, 1, fake, r, None) == binding.PI0_EINVAL      # not whole 16-byte words
    assert L.pi0_peak_bench(0, fake + 8, 1 << 20, 0, 1, fake, r, None) == binding.PI0_EINVAL        # misaligned
    assert L.pi0_peak_bench(1, None, 0, 0, 1, fake, r, None) == binding.PI0_EINVAL                  # no rounds
    assert L.pi0_peak_bench(1, None, 0, (1 << 22) + 1, 1, fake, r, None) == binding.PI0_EINVAL      # too many rounds
    assert L.pi0_peak_bench(1, None, 0, 16, 0, fake, r, None) == binding.PI0_EINVAL                 # no repetitions
    assert L.pi0_peak_bench(1, None, 0, 16, 1, None, r, None) == binding.PI0_EINVAL                 # no sink
    assert L.pi0_peak_bench(1, None, 0, 16, 1, fake, None, None) == binding.PI0_EINVAL              # no result
    assert binding.PEAK_KINDS == {"hbm_read": 0, "mfma_bf16": 1, "cache_read": 2}


def test_clock_sample_rejects_bad_arguments(L):
    assert L.pi0_clock_sample(None, None) == binding.PI0_EINVAL
    assert L.pi0_clock_sample(0x10004, None) == binding.PI0_EINVAL        # not 8-byte aligned
    assert binding.shader_clock_ghz([100, 10], [2500, 110]) == 2.4        # 2400 cycles in 100 ticks of 10 ns


def test_read_ahead_probe_rejects_bad_arguments(L):
    fake = 0x10000
    out = ctypes.c_double(0.0)
    r = ctypes.byref(out)
    ok = dict(buf=fake, nbytes=1 << 20, layers=4, steps=2, lead=1, prog=fake, ticks=1000, blocks=64, sink=fake)

    def call(**kw):
        a = dict(ok, **kw)
        return L.pi0_read_ahead_probe(a["buf"], a["nbytes"], a["layers"], a["steps"], a["lead"], a["prog"], a["ticks"], a["blocks"],
                                      a["sink"], kw.get("res", r), None)
    for bad in (dict(buf=None), dict(prog=None), dict(sink=None), dict(res=None), dict(buf=fake + 8),     # null / misaligned
                dict(layers=0), dict(steps=0), dict(lead=0), dict(ticks=0), dict(blocks=0), dict(blocks=1025),
                dict(nbytes=0), dict(nbytes=(1 << 20) + 16),                                               # not layers * 16
                dict(nbytes=1 << 33, layers=2)):                                                           # slice of 4 GiB
        assert call(**bad) == binding.PI0_EINVAL, bad


def test_kernel_count_and_taps(L):
    cfg = synth.full_config()
    c = binding.to_c_config(cfg)
    ctx = ctypes.c_void_p()
    assert L.pi0_create(ctypes.byref(c), ctypes.byref(ctx)) == 0
    n1 = L.pi0_kernel_count(ctx, 1, 0)
    n2 = L.pi0_kernel_count(ctx, 2, 0)
    # up to 256 tokens the O projections carry their residual epilogue themselves; beyond, each is followed
    # by a split-K reduction launch: 27 vision layers, 17 prefix layers with an O projection
    assert 900 < n1 < 2000 and n2 == n1 + cfg.vis_layers + (cfg.llm_layers - 1)
    assert L.pi0_kernel_count(ctx, 3, 0) == n2
    assert L.pi0_kernel_count(ctx, 0, 0) == 0
    # 261 prefix tokens: the prompt embedding gather, and the prefix reductions are back
    assert L.pi0_kernel_count(ctx, 1, 5) == n1 + 1 + (cfg.llm_layers - 1)
    assert L.pi0_kernel_count(ctx, 1, 49) == 0
    L.pi0_destroy(ctx)
    I, P = 256, 256
    exp = (27 * I * 1152 + I * 2048 + 17 * P * 2048 + 2 * 18 * P * 256 + 2 * 18 * 64 * 1024 + 10 * 63 * 32)
    assert binding.pi0_debug_taps_elems(cfg, 1, 0) == exp


def test_tuning_variable_is_parsed_by_key_and_range(L):
    """pi0_tune parses whole keys only (`vo` is not found inside `zvo`), values outside a key's range
    are ignored, unknown keys do nothing.  Seen through the launch count: a one-launch O projection drops a reduction
    launch per layer, the plain expert QKV / 32 x 32 expert tiles change nothing in the count."""
    import os
    cfg = synth.full_config()
    c = binding.to_c_config(cfg)

    def count(tune, views=1):
        ctx = ctypes.c_void_p()
        assert L.pi0_create(ctypes.byref(c), ctypes.byref(ctx)) == 0
        if tune is not None:
            assert L.pi0_tune(ctx, tune.encode()) == 0
        n = L.pi0_kernel_count(ctx, views, 0)
        L.pi0_destroy(ctx)
        return n
    base = count(None)
    vis, llm = cfg.vis_layers, cfg.llm_layers - 1
    assert count("") == base and count("nonsense=3,,=,x") == base
    assert count("fko=0") == base + vis and count("fkl=0") == base + llm and count("fko=0,fkl=0") == base + vis + llm
    assert count("fko=7") == base and count("fko=-1") == base            # out of range: ignored
    assert count("xfko=0") == base and count("fko0=0") == base           # not the key
    assert count("zvo=1,fko=0") == base + vis                            # a key after another one
    assert count("fko=1,fkl=1", views=2) == count(None, views=2) - vis - llm
    assert count("ras=0") == base and count("ras=4096,rad=8,ral=8,avs=8,qms=0,ae16=0") == base


# ---------------------------------------------------------------------------- roofline pins
def test_roofline_reproduces_table2_and_section5():
    cfg = synth.full_config()
    ops = roofline.table2_ops(cfg, 2, 0)
    b = roofline.stage_bounds_ms(ops, roofline.RTX4090_BW, roofline.RTX4090_MACS)
    # bold totals of Table 2 (two views)
    assert abs(b["vision"] - 2.485) < 2e-3
    assert abs(b["llm"] - 10.727) < 2e-3
    assert abs(b["expert"] - 6.486) < 2e-3
    assert abs(b["total"] - 19.698) < 3e-3
    # individual rows printed in the table's roofline column
    rows = {(o.stage, o.name): o.bound_s(roofline.RTX4090_BW, roofline.RTX4090_MACS) * 1e3 for o in ops}
    assert abs(rows[("vision", "qkv")] - 0.602) < 1e-3
    assert abs(rows[("vision", "attention")] - 0.178) < 1e-3
    assert abs(rows[("llm", "gate+up")] - 6.391) < 1e-3
    assert abs(rows[("llm", "down")] - 3.195) < 1e-3
    assert abs(rows[("expert", "gate+up")] - 2.990) < 1e-3
    assert abs(rows[("expert", "scores")] - 0.149) < 1e-3
    # 1378 matmuls (Section 5.2)
    assert roofline.matmul_count(ops) == 1378
    # sums for one and three views (Section 5.1 prints 12.8 and 26.7)
    b1 = roofline.stage_bounds_ms(roofline.table2_ops(cfg, 1, 0), roofline.RTX4090_BW, roofline.RTX4090_MACS)
    b3 = roofline.stage_bounds_ms(roofline.table2_ops(cfg, 3, 0), roofline.RTX4090_BW, roofline.RTX4090_MACS)
    assert abs(b1["total"] - 12.8) < 0.1 and abs(b3["total"] - 26.7) < 0.1


def test_static_scratch_entry_point_rejects_what_does_not_fit(L):
    """pi0_denoise_static keeps the expert's scratch in a device array of PI0_STATIC_SCRATCH_BYTES inside the library:
    a geometry that needs more is refused with ENOMEM before anything else is looked at (no GPU call), one that fits
    gets as far as the state check (no weights loaded here)."""
    dummy = ctypes.c_void_p(256)     # never dereferenced: every check below fails before a GPU call
    for kw, want in ((dict(exp_mlp=16384), binding.PI0_ENOMEM), (dict(), binding.PI0_ESTATE)):
        c = binding.to_c_config(synth.dataclasses.replace(synth.full_config(), **kw))
        ctx = ctypes.c_void_p()
        assert L.pi0_create(ctypes.byref(c), ctypes.byref(ctx)) == 0
        assert L.pi0_denoise_static(ctx, dummy, dummy, dummy, None) == want
        assert L.pi0_denoise_static(ctx, None, dummy, dummy, None) == binding.PI0_EINVAL
        L.pi0_destroy(ctx)


def test_traffic_profile_is_what_bench_reads():
    """bench.py takes `traffic` from profiles/traffic_full_pi0.json: per view count the dominant kernel's HBM-side bytes per
    launch and a table by kernel family, with the commit and the calibration it was taken at."""
    import json
    t = json.load(open(os.path.join(ROOT, "profiles", "traffic_full_pi0.json")))
    assert re.fullmatch(r"[0-9a-f]{7,40}", t["commit"])
    assert 1.5 < t["calibration"]["fetch_factor"] < 2.5 and 0.8 < t["calibration"]["write_factor"] < 1.2
    algorithmic = 6.9e9            # the expert's weights, 10 times (roofline.class_work gives the exact figure)
    for v in ("1", "2", "3"):
        row = t["by_views"][v]
        assert algorithmic < row["expert_loop_kernel"] < 4 * algorithmic
        assert row["families"]["expert_loop_kernel"]["launches"] == 1
        for fam in ("gemm_kernel", "attention_kernel", "splitk_reduce_kernel"):
            assert row["families"][fam]["bytes_per_launch"] > 0
