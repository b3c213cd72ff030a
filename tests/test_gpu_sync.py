"""GPU: grid synchronisation with a data dependency between blocks (Section 5.2 of the paper: software barriers
inside one persistent kernel).  Every (barrier, data path) pair must reproduce, bit for bit, a host simulation
of the dependent updates: a data path that leaves a stale copy in some cache fails here."""
import sys

import numpy as np
import pytest
import torch

from paper_2510_26742_amd import binding

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def simulate(x0, b, fan, n_ops):
    """x_{k+1}[r] = max_{j = 1 .. fan} x_k[(r + j) mod 256] + b[r], n_ops times (exact in fp32 for small integers)."""
    x = x0.copy()
    for _ in range(n_ops):
        m = np.roll(x, -1, axis=0)
        for j in range(2, fan + 1):
            np.maximum(m, np.roll(x, -j, axis=0), out=m)
        x = m + b
    return x


@pytest.mark.parametrize("barrier", ["counter", "xcd", "flags", "flags8", "groupadd", "xcc"])
@pytest.mark.parametrize("data", ["bypass", "inv", "fence", "fresh", "wback"])
def test_dependent_updates_are_exact(barrier, data):
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(device=dev)
    rng = np.random.default_rng(5)
    x0 = rng.integers(-8, 8, (256, 1024)).astype(np.float32)
    b = rng.integers(-2, 3, (256, 1024)).astype(np.float32)
    n_ops, fan = 150, 5
    planes = n_ops + 1 if data == "fresh" else 2
    say(f"[gpu] pi0_sync_dep_bench {barrier} {data} fan={fan} n_ops={n_ops} planes={planes}")
    d_x = torch.zeros((planes, 256, 1024), dtype=torch.float32, device=dev)
    d_x[0] = torch.from_numpy(x0).to(dev)
    d_b = torch.from_numpy(b).to(dev)
    d_state = torch.zeros(9216, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    ms = binding.pi0_sync_dep_bench(barrier, data, fan, n_ops, 1, d_x, d_b, d_state, stream)
    want = simulate(x0, b, fan, n_ops)
    got = d_x[n_ops % planes].cpu().numpy()
    say(f"[sync-dep] {barrier}/{data}: {ms * 1e3 / n_ops:.2f} us per update")
    np.testing.assert_array_equal(got, want)


def test_independent_updates_and_argument_checks():
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream(device=dev)
    x0 = torch.arange(256 * 1024, dtype=torch.float32).reshape(256, 1024) % 17
    b = torch.ones(256, 1024)
    d_b = b.to(dev)
    d_state = torch.zeros(9216, dtype=torch.int32, device=dev)
    for barrier in ("counter", "xcd", "flags", "flags8", "groupadd", "xcc"):
        say(f"[gpu] pi0_sync_dep_bench {barrier} none")
        d_x = x0.clone().reshape(1, 256, 1024).to(dev)
        torch.cuda.synchronize()
        binding.pi0_sync_dep_bench(barrier, "none", 1, 300, 2, d_x, d_b, d_state, stream)
        torch.testing.assert_close(d_x[0].cpu(), x0 + 600 * b, rtol=0, atol=0)
    d_x = torch.zeros((2, 256, 1024), dtype=torch.float32, device=dev)
    with pytest.raises(binding.Pi0Error):   # a fresh plane per update needs n_ops + 1 planes
        binding.pi0_sync_dep_bench("flags", "fresh", 1, 10, 1, d_x, d_b, d_state, stream)
    with pytest.raises(binding.Pi0Error):   # fan beyond 32 rows
        binding.pi0_sync_dep_bench("flags", "bypass", 33, 10, 1, d_x, d_b, d_state, stream)
    with pytest.raises(binding.Pi0Error):   # dependent data needs two planes
        binding.pi0_sync_dep_bench("flags", "bypass", 1, 10, 1, d_x[:1], d_b, d_state, stream)
