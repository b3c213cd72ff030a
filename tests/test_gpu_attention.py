"""GPU: the three attention kernels of the pass (Table 2: SigLIP attention per view; prefix attention with a shared
key/value head; the action expert's attention over [prefix cache ; its own 64 keys] with the state/action block
mask), each on its own against the oracle's attention in float64, with logits of order one so that the softmax is far
from uniform and the masks matter.

Operands are bf16-representable, so both sides see the same numbers.  What the kernels round: the probabilities
(to bf16, relative 2^-9, before the second product) and the output (to bf16); both products accumulate in fp32.
|delta| <= 2^-9 |out| + 2^-9 sum_j p_j |v_j| <= 2^-8 max|v|, which is the bar below; a wrong mask, a wrong key
offset or a wrong merge of key shares moves rows by O(1).
Rows are built so that the mask edges carry the mass: chosen query rows point at the last prefix key, the first and
last suffix key, and the state row points at a key it must NOT see."""
import sys

import numpy as np
import pytest
import torch

from oracle import pi0_oracle as orc
from paper_2510_26742_amd import binding

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def bf16_round(x):
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def draw(rng, *shape):
    return bf16_round(rng.standard_normal(shape))


def merge_shares(out, ml, Tq):
    """Merge of key shares as the consumer defines it: sum_z c_z out_z, c_z = l_z exp(m_z - max m) / sum."""
    Z, _, HD = out.shape
    H = ml.shape[1]
    d = HD // H
    m = ml[:, :, :Tq, 0].astype(np.float64)
    l = ml[:, :, :Tq, 1].astype(np.float64)
    c = l * np.exp(m - m.max(axis=0, keepdims=True))
    c /= c.sum(axis=0, keepdims=True)                       # [Z, H, Tq]
    o = out.astype(np.float64).reshape(Z, Tq, H, d)
    return np.einsum("zht,zthd->thd", c, o).reshape(Tq, HD)


def run(q, k0, v0, k1=None, v1=None, **kw):
    dev = torch.device("cuda:0")
    t = [None if a is None else torch.from_numpy(a).to(dev) for a in (q, k0, v0, k1, v1)]
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    out, ml = binding.pi0_attention_probe(*t, stream=stream, **kw)
    out = out.cpu().numpy()
    if ml is None:
        return out[0]
    return merge_shares(out, ml.cpu().numpy(), q.shape[1])


def check(name, got, want, vmax):
    H, Tq, d = want.shape
    want2 = want.transpose(1, 0, 2).reshape(Tq, H * d)
    delta = np.abs(got - want2)
    bar = 2.0 ** -8 * vmax
    rms = float(np.sqrt(np.mean(delta ** 2)))
    say(f"[attention] {name}: max|delta| {delta.max():.3e} (bar {bar:.3e}) at row {int(np.argmax(delta.max(axis=1)))}, rms {rms:.3e}")
    assert np.isfinite(got).all()
    assert delta.max() <= bar
    assert rms <= 2.0 ** -12 * vmax   # measured 1.2e-4 .. 3.3e-4


def test_vision_attention_per_view():
    # 16 heads of 72, 3 views of 256 tokens each; a row only sees its own view
    rng = np.random.default_rng(11)
    H, d, T, views = 16, 72, 256, 3
    q, k, v = draw(rng, H, views * T, d), draw(rng, H, views * T, d), draw(rng, H, views * T, d)
    # a row of view 1 that would, without the view mask, put all its weight on a key of view 0
    q[:, T + 3] = 3.0 * k[:, 5]
    q[:, 2 * T + 255] = 3.0 * k[:, 2 * T]       # last row of the last view -> first key of its view
    q = bf16_round(q)
    allowed = np.zeros((views * T, views * T), dtype=bool)
    for i in range(views):
        allowed[i * T:(i + 1) * T, i * T:(i + 1) * T] = True
    say(f"[gpu] pi0_attention_probe vision heads={H} d={d} views={views}")
    got = run(q, k, v, view_tokens=T)
    want = orc.attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), allowed)
    check("vision 3 views", got, want, np.abs(v).max())


@pytest.mark.parametrize("P", [256, 263, 519, 816])
def test_prefix_attention_shared_head(P):
    # 8 query heads of 256 over one key/value head, whole prefix visible; P = 816 is ragged (25.5 chunks of 32)
    rng = np.random.default_rng(100 + P)
    H, d = 8, 256
    q, k, v = draw(rng, H, P, d), draw(rng, 1, P, d), draw(rng, 1, P, d)
    q[:, 0] = 2.0 * k[0, P - 1]        # first row -> last key
    q[:, P - 1] = 2.0 * k[0, 0]        # last row -> first key
    allowed = np.ones((P, P), dtype=bool)
    say(f"[gpu] pi0_attention_probe prefix P={P}")
    got = run(q, k, v)
    want = orc.attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), allowed)
    check(f"prefix P={P}", got, want, np.abs(v).max())


@pytest.mark.parametrize("P,cps,v_split", [(256, 0, 4), (263, 8, 2), (519, 8, 2), (816, 8, 2), (816, 7, 2), (40, 0, 4)])
def test_expert_attention_block_mask_and_key_shares(P, cps, v_split):
    """64 suffix rows over P cached keys and their own 64 keys.  Row 0 (state) sees the prefix and itself only; rows
    1 .. 63 see everything.  cps = chunks of 32 keys per share: 263 keys -> 2 shares (8 chunks + 1), 519 -> 3 shares, 816 -> 4 shares with a ragged
    last one (2 chunks, 16 keys in the last) or, at 7, a full fourth share of 5 chunks."""
    rng = np.random.default_rng(200 + P + cps)
    H, d, S = 8, 256, 64
    q, k0, v0 = draw(rng, H, S, d), draw(rng, 1, P, d), draw(rng, 1, P, d)
    k1, v1 = draw(rng, 1, S, d), draw(rng, 1, S, d)
    q[:, 0] = 2.0 * k1[0, 1]           # the state row points at action key 1, which it must not see
    q[:, 1] = 2.0 * k1[0, 0]           # first action row -> state key (first suffix key)
    q[:, 5] = 2.0 * k0[0, P - 1]       # -> last prefix key
    q[:, 6] = 2.0 * k1[0, S - 1]       # -> last suffix key
    q[:, S - 1] = 2.0 * k0[0, 0]       # last row -> first prefix key
    k = np.concatenate([k0, k1], axis=1).astype(np.float64)
    v = np.concatenate([v0, v1], axis=1).astype(np.float64)
    allowed = orc.suffix_allowed(P, S)
    say(f"[gpu] pi0_attention_probe expert P={P} chunks_per_share={cps} v_split={v_split}")
    got = run(q, k0, v0, k1, v1, suffix_mask=True, chunks_per_share=cps, v_split=v_split)
    want = orc.attention(q.astype(np.float64), k, v, allowed)
    vmax = np.abs(v).max()
    check(f"expert P={P} cps={cps}", got, want, vmax)
    # the named rows on their own: state row, first and last action row, and the rows sitting on the mask edges
    want2 = want.transpose(1, 0, 2).reshape(S, H * d)
    for r in (0, 1, 5, 6, S - 1):
        assert np.abs(got[r] - want2[r]).max() <= 2.0 ** -8 * vmax, r
    # the state row must not depend on the action keys at all: other action keys / values, same bits in row 0
    k1b, v1b = k1.copy(), v1.copy()
    k1b[0, 1:] = draw(rng, S - 1, d)
    v1b[0, 1:] = draw(rng, S - 1, d)
    got_b = run(q, k0, v0, k1b, v1b, suffix_mask=True, chunks_per_share=cps, v_split=v_split)
    np.testing.assert_array_equal(got_b[0], got[0])
    assert np.abs(got_b[1:] - got[1:]).max() > 0.1


def test_probe_rejects_what_the_kernels_do_not_support():
    dev = torch.device("cuda:0")
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device=dev)
    with pytest.raises(binding.Pi0Error):
        binding.pi0_attention_probe(z(8, 64, 128), z(1, 64, 128), z(1, 64, 128))             # head dim
    with pytest.raises(binding.Pi0Error):
        binding.pi0_attention_probe(z(8, 64, 256), z(2, 64, 256), z(2, 64, 256))             # key heads
    with pytest.raises(binding.Pi0Error):
        binding.pi0_attention_probe(z(8, 64, 256), z(1, 1056, 256), z(1, 1056, 256))         # too many keys
    with pytest.raises(binding.Pi0Error):
        binding.pi0_attention_probe(z(16, 512, 72), z(16, 512, 72), z(16, 512, 72), view_tokens=200)
