"""Scalar, index-by-index pi0 forward for toy geometries (pure Python floats, no numpy math).

Written separately from the oracle, in a different style (explicit loops over token, head and
feature indices, dictionaries of nested lists), so that a transposed operand, a wrong index or a
mis-ordered concatenation in the vectorised oracle shows up as a mismatch on tiny inputs.
Follows the paper's Section 2 description and the op list of its Table 2, unfused.
"""
import math


def bf16_val(bits):
    import struct
    return struct.unpack("<f", struct.pack("<I", int(bits) << 16))[0]


def load(tensors):
    out = {}
    for k, a in tensors.items():
        if a.ndim == 1:
            out[k] = [bf16_val(v) for v in a]
        else:
            out[k] = [[bf16_val(v) for v in row] for row in a]
    return out


def matvec(x, W, b=None):
    n_out = len(W[0])
    y = [0.0] * n_out
    for j in range(n_out):
        s = 0.0
        for i in range(len(x)):
            s += x[i] * W[i][j]
        y[j] = s + (b[j] if b is not None else 0.0)
    return y


def ln(x, g, b):
    n = len(x)
    mu = sum(x) / n
    var = sum((v - mu) ** 2 for v in x) / n
    return [(x[i] - mu) / math.sqrt(var + 1e-6) * g[i] + b[i] for i in range(n)]


def rms(x, g):
    n = len(x)
    ms = sum(v * v for v in x) / n
    return [x[i] / math.sqrt(ms + 1e-6) * (1.0 + g[i]) for i in range(n)]


def gelu(v):
    return 0.5 * v * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))


def rope_vec(u, pos):
    d = len(u)
    h = d // 2
    out = [0.0] * d
    for i in range(h):
        ang = pos * (10000.0 ** (-2.0 * i / d))
        c, s = math.cos(ang), math.sin(ang)
        out[i] = u[i] * c - u[i + h] * s
        out[i + h] = u[i + h] * c + u[i] * s
    return out


def attend(qrow, keys, vals, allowed_idx):
    d = len(qrow)
    logits = {j: sum(qrow[c] * keys[j][c] for c in range(d)) / math.sqrt(d) for j in allowed_idx}
    m = max(logits.values())
    e = {j: math.exp(v - m) for j, v in logits.items()}
    z = sum(e.values())
    out = [0.0] * len(vals[allowed_idx[0]])
    for j, w in e.items():
        for c in range(len(out)):
            out[c] += w / z * vals[j][c]
    return out


def vision(cfg, W, images):
    V = len(images)
    n = cfg.img_size // cfg.patch
    toks = []
    for v in range(V):
        for py in range(n):
            for px in range(n):
                u = []
                for dy in range(cfg.patch):
                    for dx in range(cfg.patch):
                        for c in range(3):
                            u.append(float(images[v][py * cfg.patch + dy][px * cfg.patch + dx][c]))
                h = matvec(u, W["vis.patch.w"], W["vis.patch.b"])
                pos = W["vis.pos"][py * n + px]
                toks.append([h[i] + pos[i] for i in range(len(h))])
    T = n * n
    D, Hn = cfg.vis_width, cfg.vis_heads
    dh = D // Hn
    for l in range(cfg.vis_layers):
        p = f"vis.{l}."
        a = [ln(t, W[p + "ln1.g"], W[p + "ln1.b"]) for t in toks]
        q = [matvec(t, W[p + "wq"], W[p + "bq"]) for t in a]
        k = [matvec(t, W[p + "wk"], W[p + "bk"]) for t in a]
        vv = [matvec(t, W[p + "wv"], W[p + "bv"]) for t in a]
        new = []
        for i in range(len(toks)):
            view = i // T
            idx = list(range(view * T, view * T + T))
            o = []
            for h in range(Hn):
                sl = slice(h * dh, (h + 1) * dh)
                o += attend(q[i][sl], {j: k[j][sl] for j in idx}, {j: vv[j][sl] for j in idx}, idx)
            r = matvec(o, W[p + "wo"], W[p + "bo"])
            new.append([toks[i][c] + r[c] for c in range(D)])
        toks = new
        for i in range(len(toks)):
            m = ln(toks[i], W[p + "ln2.g"], W[p + "ln2.b"])
            hid = [gelu(v) for v in matvec(m, W[p + "w1"], W[p + "b1"])]
            r = matvec(hid, W[p + "w2"], W[p + "b2"])
            toks[i] = [toks[i][c] + r[c] for c in range(D)]
    return [matvec(ln(t, W["vis.lnf.g"], W["vis.lnf.b"]), W["vis.proj.w"], W["vis.proj.b"]) for t in toks]


def gemma_layer_qkv(cfg, W, p, xs, pos0):
    Hn, dh = cfg.llm_q_heads, cfg.head_dim
    qs, ks, vs = [], [], []
    for i, x in enumerate(xs):
        a = rms(x, W[p + "g_attn"])
        q = matvec(a, W[p + "wq"])
        qs.append([rope_vec(q[h * dh:(h + 1) * dh], pos0 + i) for h in range(Hn)])
        ks.append(rope_vec(matvec(a, W[p + "wk"]), pos0 + i))
        vs.append(matvec(a, W[p + "wv"]))
    return qs, ks, vs


def gemma_mlp(W, p, x):
    m = rms(x, W[p + "g_mlp"])
    g = matvec(m, W[p + "wg"])
    u = matvec(m, W[p + "wu"])
    r = matvec([gelu(g[i]) * u[i] for i in range(len(g))], W[p + "wd"])
    return [x[i] + r[i] for i in range(len(x))]


def forward(cfg, tensors, images, state, noise, prompt_ids):
    W = load(tensors)
    xs = vision(cfg, W, images)
    for t in prompt_ids:
        xs.append([v * math.sqrt(cfg.llm_width) for v in W["llm.embed"][int(t)]])
    P = len(xs)
    Hn = cfg.llm_q_heads
    cacheK, cacheV = [], []
    for l in range(cfg.llm_layers):
        p = f"llm.{l}."
        qs, ks, vs = gemma_layer_qkv(cfg, W, p, xs, 0)
        cacheK.append(ks)
        cacheV.append(vs)
        if l == cfg.llm_layers - 1:
            break
        for i in range(P):
            o = []
            for h in range(Hn):
                o += attend(qs[i][h], ks, vs, list(range(P)))
            r = matvec(o, W[p + "wo"])
            xs[i] = [xs[i][c] + r[c] for c in range(len(r))]
        xs = [gemma_mlp(W, p, x) for x in xs]
    X = cfg.exp_width
    x = [[float(v) for v in row] for row in noise]
    st = matvec([float(v) for v in state], W["exp.state.w"], W["exp.state.b"])
    S = cfg.chunk + 1
    for k in range(cfg.steps):
        t = 1.0 - k / cfg.steps
        half = X // 2
        per = [4e-3 * (4.0 / 4e-3) ** (j / (half - 1)) for j in range(half)]
        tau = [math.sin(2 * math.pi * t / pj) for pj in per] + [math.cos(2 * math.pi * t / pj) for pj in per]
        ys = [list(st)]
        for row in x:
            ae = matvec(row, W["exp.action_in.w"], W["exp.action_in.b"])
            z = matvec(ae + tau, W["exp.time_in.w"], W["exp.time_in.b"])
            z = [v / (1.0 + math.exp(-v)) for v in z]
            ys.append(matvec(z, W["exp.time_out.w"], W["exp.time_out.b"]))
        for l in range(cfg.exp_layers):
            p = f"exp.{l}."
            qs, ks, vs = gemma_layer_qkv(cfg, W, p, ys, P)
            keys = cacheK[l] + ks
            vals = cacheV[l] + vs
            new = []
            for i in range(S):
                idx = list(range(P)) + ([P] if i == 0 else list(range(P, P + S)))
                o = []
                for h in range(Hn):
                    o += attend(qs[i][h], keys, vals, idx)
                r = matvec(o, W[p + "wo"])
                new.append([ys[i][c] + r[c] for c in range(X)])
            ys = [gemma_mlp(W, p, y) for y in new]
        for i in range(cfg.chunk):
            v = matvec(rms(ys[i + 1], W["exp.g_final"]), W["exp.out.w"], W["exp.out.b"])
            x[i] = [x[i][c] - v[c] / cfg.steps for c in range(len(v))]
    return x, cacheK, cacheV
