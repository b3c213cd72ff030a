"""The paper's roofline model (Section 5.1) and the op list of its Table 2, parameterised by the
number of views / prompt tokens, for use by the benchmark.

For one bf16 GEMM of N x K x M (rows x reduction x columns) the bound is
    t = max(2*K*M / bandwidth, N*K*M / mac_rate)
i.e. only the weight matrix is charged to memory (activations are assumed cache resident), and
per-op bounds are summed.  Attention rows are charged their MACs only.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

RTX4090_BW = 1.01e12          # bytes/s, the paper's constant
RTX4090_MACS = 91.4e12        # bf16 MAC/s at the boost clock the paper observed
MI355X_BW = 8.0e12            # bytes/s, HBM3E spec sheet
MI355X_MACS = 2.5e15 / 2      # dense bf16 MFMA: 2.5 PFLOP/s = 1.25 PMAC/s


@dataclass
class Op:
    stage: str      # "vision" | "llm" | "expert"
    name: str
    rows: int       # N
    k: int          # K
    cols: int       # M
    count: int
    attn: bool = False   # attention row: MACs only (rows * k * cols already the MAC count of one call)
    matmuls: int = 1     # how many matmuls the paper counts for one call

    @property
    def macs(self) -> float:
        return float(self.rows) * self.k * self.cols * self.count

    @property
    def weight_bytes(self) -> float:
        return 0.0 if self.attn else 2.0 * self.k * self.cols * self.count

    def bound_s(self, bw: float, macs: float) -> float:
        per_call_mem = 0.0 if self.attn else 2.0 * self.k * self.cols / bw
        per_call_cmp = float(self.rows) * self.k * self.cols / macs
        return max(per_call_mem, per_call_cmp) * self.count


def table2_ops(cfg, n_views: int, n_prompt: int = 0, joint_vision_attention: bool = True) -> List[Op]:
    """Rows of Table 2 for the given input shape.  With n_views=2, n_prompt=0 these are exactly
    the printed rows.  joint_vision_attention=True reproduces the table's accounting of vision
    attention as one T x T problem over all views; False charges it per view (what is computed)."""
    T = cfg.tokens_per_view
    I = n_views * T
    P = I + n_prompt
    S = cfg.suffix
    Dv, Fv, Hv = cfg.vis_width, cfg.vis_mlp, cfg.vis_heads
    E, H, Dh, F = cfg.llm_width, cfg.llm_q_heads, cfg.head_dim, cfg.llm_mlp
    X, Fx = cfg.exp_width, cfg.exp_mlp
    Lv, Ll, Le, steps = cfg.vis_layers, cfg.llm_layers, cfg.exp_layers, cfg.steps
    ops = [Op("vision", "patch embed", I, cfg.patch_dim, Dv, 1),
           Op("vision", "qkv", I, Dv, 3 * Dv, Lv)]
    if joint_vision_attention:
        ops.append(Op("vision", "attention", Hv * I, 2 * I, Dv // Hv, Lv, attn=True, matmuls=2))
    else:
        ops.append(Op("vision", "attention", Hv * I, 2 * T, Dv // Hv, Lv, attn=True, matmuls=2))
    ops += [Op("vision", "o", I, Dv, Dv, Lv),
            Op("vision", "up", I, Dv, Fv, Lv),
            Op("vision", "down", I, Fv, Dv, Lv),
            Op("llm", "projector", I, Dv, E, 1),
            Op("llm", "qkv", P, E, (H + 2) * Dh, Ll),
            Op("llm", "attention", H * P, 2 * P, Dh, Ll - 1, attn=True, matmuls=2),
            Op("llm", "o", P, H * Dh, E, Ll - 1),
            Op("llm", "gate+up", P, E, 2 * F, Ll - 1),
            Op("llm", "down", P, F, E, Ll - 1),
            Op("expert", "state", 1, cfg.state_dim, X, 1),
            Op("expert", "action-time 1", cfg.chunk, cfg.action_dim, X, steps),
            Op("expert", "action-time 2", cfg.chunk, X, X, steps),
            Op("expert", "qkv", S, X, (H + 2) * Dh, Le * steps),
            Op("expert", "scores", H * S, Dh, P + S, Le * steps),
            Op("expert", "pv", H * S, P + S, Dh, Le * steps),
            Op("expert", "o", S, H * Dh, X, Le * steps),
            Op("expert", "gate+up", S, X, 2 * Fx, Le * steps),
            Op("expert", "down", S, Fx, X, Le * steps),
            Op("expert", "out + euler", cfg.chunk, X, cfg.action_dim, steps)]
    return ops


def stage_bounds_ms(ops: List[Op], bw: float, macs: float) -> dict:
    out = {"vision": 0.0, "llm": 0.0, "expert": 0.0}
    for o in ops:
        out[o.stage] += o.bound_s(bw, macs) * 1e3
    out["total"] = out["vision"] + out["llm"] + out["expert"]
    return out


def matmul_count(ops: List[Op]) -> int:
    return sum(o.count * o.matmuls for o in ops)


def weight_bytes(ops: List[Op], stage: str | None = None) -> float:
    return sum(o.weight_bytes for o in ops if stage is None or o.stage == stage)


def total_macs(ops: List[Op], stage: str | None = None) -> float:
    return sum(o.macs for o in ops if stage is None or o.stage == stage)
