"""Pins for the oracle's MXFP8 rounding (OCP FP8 E4M3 elements, E8M0 scale per 32 elements): the format's
closed forms, a brute-force nearest-value search, torch's float8_e4m3fn cast as an independent library
routine, and invariants of the block scaling.  Nothing here touches the HIP library."""
import math

import numpy as np
import torch

from oracle import mxfp8 as M
from oracle import pi0_oracle as O

R = np.random.default_rng(11)
FINITE = np.array([c for c in range(256) if (c & 0x7f) != 0x7f], dtype=np.uint8)


def test_e4m3_decode_closed_forms():
    d = M.e4m3_decode(np.arange(256, dtype=np.uint8)).astype(np.float64)
    assert d[0x00] == 0.0 and d[0x38] == 1.0 and d[0xb8] == -1.0
    assert d[0x01] == 2.0 ** -9 and d[0x07] == 7 * 2.0 ** -9 and d[0x08] == 2.0 ** -6     # subnormals, smallest normal
    assert d[0x7e] == 448.0 and d[0x40] == 2.0 and d[0x3c] == 1.5
    assert math.isnan(d[0x7f]) and math.isnan(d[0xff])
    pos = d[:0x7f]
    assert np.all(np.diff(pos) > 0)                       # codes order the positive values
    np.testing.assert_array_equal(d[0x80:0xff], -pos)     # sign bit only flips the sign
    # spacing doubles with every exponent step: 8 mantissa steps per binade
    for e in range(1, 15):
        base = d[e << 3]
        np.testing.assert_array_equal(d[(e << 3):(e << 3) + 8][: (7 if e == 15 else 8)],
                                      base * (1 + np.arange(8) / 8.0)[: (7 if e == 15 else 8)])


def test_e4m3_encode_inverts_decode_and_saturates():
    np.testing.assert_array_equal(M.e4m3_encode(M.e4m3_decode(FINITE)) & 0x7f, FINITE & 0x7f)
    assert M.e4m3_encode(np.array([-0.0]))[0] == 0x80
    np.testing.assert_array_equal(M.e4m3_encode(np.array([449.0, 1e9, -500.0, -1e30])), [0x7e, 0x7e, 0xfe, 0xfe])


def brute_nearest(x):
    """Nearest finite E4M3 code by exhaustive search, ties to the code with an even mantissa."""
    vals = M.e4m3_decode(np.arange(0x7f, dtype=np.uint8)).astype(np.float64)      # positive codes 0 .. 0x7e
    a = min(abs(x), 448.0)
    err = np.abs(vals - a)
    best = np.flatnonzero(err == err.min())
    c = int(best[0]) if len(best) == 1 else int([b for b in best if b % 2 == 0][0])
    return c | (0x80 if math.copysign(1.0, x) < 0 else 0)


def test_e4m3_encode_matches_brute_force_including_ties():
    vals = M.e4m3_decode(np.arange(0x7f, dtype=np.uint8)).astype(np.float64)
    mids = (vals[:-1] + vals[1:]) / 2                      # exact ties between neighbours
    probes = np.concatenate([mids, mids * (1 + 1e-9), mids * (1 - 1e-9), vals, R.uniform(-460, 460, 3000),
                             R.normal(0, 1, 3000), R.normal(0, 0.01, 3000), -mids])
    got = M.e4m3_encode(probes)
    want = np.array([brute_nearest(float(p)) for p in probes], dtype=np.uint8)
    np.testing.assert_array_equal(got, want)
    # the ties the format's definition fixes: 17 -> 16, 19 -> 20, 1.0625 -> 1, 1.1875 -> 1.25, 2^-10 -> 0
    np.testing.assert_array_equal(M.e4m3_decode(M.e4m3_encode(np.array([17.0, 19.0, 1.0625, 1.1875, 2.0 ** -10]))),
                                  [16.0, 20.0, 1.0, 1.25, 0.0])


def test_e4m3_encode_matches_torch_cast():
    x = np.concatenate([R.uniform(-448, 448, 20000), R.normal(0, 1, 20000), R.normal(0, 1e-2, 20000)]).astype(np.float32)
    t = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(M.e4m3_encode(x), t)


def test_mx_scale_closed_forms_and_invariants():
    blk = np.zeros((1, 32))
    blk[0, 3] = 1.0
    codes, sc = M.mx_quantize(blk)
    assert sc[0, 0] == 127 - 8 and codes[0, 3] == 0x78 and M.mx_dequantize(codes, sc, np.float64)[0, 3] == 1.0   # 1 = 256 * 2^-8
    blk[0, 3] = 448.0
    assert M.mx_quantize(blk)[1][0, 0] == 127 and M.mx_quantize(blk)[0][0, 3] == 0x7e
    blk[0, 3] = 511.0                                     # floor(log2) still 8: the element saturates
    assert M.mx_quantize(blk)[1][0, 0] == 127 and M.mx_quantize(blk)[0][0, 3] == 0x7e
    blk[0, 3] = 512.0
    assert M.mx_quantize(blk)[1][0, 0] == 128 and M.mx_quantize(blk)[0][0, 3] == 0x78
    z = M.mx_quantize(np.zeros((2, 64)))
    assert np.all(z[0] == 0) and np.all(z[1] == 0)
    x = R.normal(0, 1, (5, 96))
    c1, s1 = M.mx_quantize(x)
    c2, s2 = M.mx_quantize(x * 8.0)                       # a power-of-two factor moves only the scales
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(s1.astype(int) + 3, s2.astype(int))
    y = x.copy()
    y[:, 32:64] *= 1000.0                                 # blocks are independent
    c3, s3 = M.mx_quantize(y)
    np.testing.assert_array_equal(c1[:, :32], c3[:, :32])
    np.testing.assert_array_equal(c1[:, 64:], c3[:, 64:])
    np.testing.assert_array_equal(s1[:, [0, 2]], s3[:, [0, 2]])
    # error bound: the block maximum lands in [256, 512) * scale, so every element is within half an E4M3
    # step of that binade (32 * scale / 2) - or, saturated, within 64 * scale
    d = M.mx_dequantize(c1, s1, np.float64)
    scale = np.ldexp(1.0, s1.astype(int) - 127)
    assert np.all(np.abs(d - x).reshape(5, 3, 32) <= 64.0 * scale[..., None])
    unsat = np.abs(x).reshape(5, 3, 32) <= 448.0 * scale[..., None]
    assert np.all(np.abs(d - x).reshape(5, 3, 32)[unsat] <= (16.0 * np.broadcast_to(scale[..., None], (5, 3, 32)))[unsat])
    # values that are representable next to their block maximum are kept exactly: mantissa below 1.875 (a
    # maximum of 1.875 * 2^k lands on 480 * scale and saturates, by the format's rule) and at most 6 binades apart
    narrow = np.array([c for c in FINITE if 8 <= ((c >> 3) & 15) <= 14 and (c & 7) <= 6], dtype=np.uint8)
    rep = M.e4m3_decode(R.choice(narrow, size=(4, 64))).astype(np.float64)
    np.testing.assert_array_equal(M.mx_round(rep * 2.0 ** -5), rep * 2.0 ** -5)
    top = np.zeros((1, 32))
    top[0, 0] = 1.875 * 2.0 ** -3
    assert M.mx_round(top)[0, 0] == 1.75 * 2.0 ** -3


def test_mxfp8_mlp_matches_loops():
    """The oracle's MXFP8 feed-forward block against per-element Python loops written from the same definition."""
    E, F_ = 64, 96
    def bits(a):
        return (np.asarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    t = {"l.g_mlp": bits(R.normal(0, 0.1, E)), "l.wg": bits(R.normal(0, 0.2, (E, F_))),
         "l.wu": bits(R.normal(0, 0.2, (E, F_))), "l.wd": bits(R.normal(0, 0.2, (F_, E)))}
    W = O.Weights(t, np.float64)
    x = R.normal(0, 1.5, (3, E))
    got = O._gemma_mlp_mxfp8(W, "l.", x)

    def q32(v):   # one block of 32 values -> dequantised values
        amax = max(abs(float(u)) for u in v)
        se = (math.frexp(amax)[1] - 1 - 8) if amax > 0 else -127
        return [float(M.e4m3_decode(np.array([brute_nearest(float(u) / 2.0 ** se)], dtype=np.uint8))[0]) * 2.0 ** se for u in v]

    def qrow(v):
        out = []
        for b in range(0, len(v), 32):
            out += q32(v[b:b + 32])
        return np.array(out)

    g, wg, wu, wd = (W["l.g_mlp"], W["l.wg"], W["l.wu"], W["l.wd"])
    wgq = np.stack([qrow(wg[:, n]) for n in range(F_)], axis=1)
    wuq = np.stack([qrow(wu[:, n]) for n in range(F_)], axis=1)
    wdq = np.stack([qrow(wd[:, n]) for n in range(E)], axis=1)
    want = np.zeros((3, E))
    for m in range(3):
        rstd = 1.0 / math.sqrt(float(np.mean(x[m] ** 2)) + 1e-6)
        xq = qrow(x[m] * (1.0 + g))
        h = np.zeros(F_)
        for n in range(F_):
            gate = rstd * float(np.dot(xq, wgq[:, n]))
            up = rstd * float(np.dot(xq, wuq[:, n]))
            gl = 0.5 * gate * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (gate + 0.044715 * gate ** 3)))
            h[n] = gl * up
        want[m] = qrow(h) @ wdq
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # and the rounding really changes the result at the expected scale (a dropped quantisation would pass nothing above)
    plain = O._gemma_mlp(W, "l.", x)
    rel = np.abs(got - plain).max() / np.abs(plain).max()
    assert 1e-3 < rel < 0.2
