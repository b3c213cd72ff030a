"""GPU: pi0_denoise_static (the entry point for callers that cannot allocate: the expert's scratch lives in a device
array inside the library) against pi0_denoise on the same cached prefix, bit for bit, on two calls in a row - the
second on a smaller prefix, so that whatever the first call left in the shared array must not matter."""
import sys

import numpy as np
import pytest
import torch

from paper_2510_26742_amd import binding, synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def test_static_scratch_denoise_matches_workspace_denoise():
    cfg = synth.reduced_config(vocab=1024)
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(device=dev)
    say("[gpu] no-alloc: weights")
    blob = synth.make_weights(cfg, seed=0)
    m = binding.Pi0(cfg)
    d_blob = torch.from_numpy(blob.view(np.int16)).to(dev)
    m.pi0_load_weights(d_blob, stream)
    stream.synchronize()
    del d_blob
    try:
        for call, (n_views, n_prompt) in enumerate([(3, 48), (1, 0)]):     # 816 prefix tokens (4 key shares), then 256
            say(f"[gpu] no-alloc: call {call}: views={n_views} prompt={n_prompt}")
            img = torch.from_numpy(synth.make_images(cfg, n_views, seed=11 + call)).to(dev)
            ids = torch.from_numpy(synth.make_prompt(cfg, n_prompt, seed=14 + call)).to(dev) if n_prompt else None
            st = torch.from_numpy(synth.make_state(cfg, seed=12 + call)).to(dev)
            nz = torch.from_numpy(synth.make_noise(cfg, seed=13 + call)).to(dev)
            want = torch.empty((cfg.chunk, cfg.action_dim), dtype=torch.float32, device=dev)
            got = torch.full((cfg.chunk, cfg.action_dim), float("nan"), dtype=torch.float32, device=dev)
            m.pi0_prefill(img, n_views, ids, n_prompt, stream)
            m.pi0_denoise(st, nz, want, stream)
            stream.synchronize()
            m.pi0_denoise_static(st, nz, got, stream)
            stream.synchronize()
            w, g = want.cpu().numpy(), got.cpu().numpy()
            assert np.isfinite(w).all() and np.abs(w).max() > 0
            np.testing.assert_array_equal(g, w, err_msg=f"call {call}")
        m.pi0_device_status(stream)
        with pytest.raises(binding.Pi0Error):     # null output
            m.pi0_denoise_static(st, nz, None, stream)
    finally:
        m.close()
        m.workspace = None
        torch.cuda.empty_cache()
