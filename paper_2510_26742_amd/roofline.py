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


MI355X_FLOPS = 2.5e15         # dense bf16 MFMA FLOP/s


def class_work(cfg, n_views: int, n_prompt: int = 0) -> dict:
    """Algorithmic work of ONE launch of every operation class the library times
    (binding.OP_CLASSES): name -> (bytes, flops).

    Bytes are what the operation must move if every operand crossed HBM exactly once: the bf16
    weight matrix, the bf16 input activations, and the final outputs (fp32 residual read and
    write plus its bf16 copy for residual projections, bf16 otherwise; keys and values for the
    attention rows).  Split-K partial sums are an implementation artefact and are not counted;
    the reduction launches and the small non-GEMM launches ("reduce", "misc") have no entry.
    """
    T = cfg.tokens_per_view
    I = n_views * T
    P = I + n_prompt
    S = cfg.suffix
    Dv, Fv = cfg.vis_width, cfg.vis_mlp
    E, H, Dh, F = cfg.llm_width, cfg.llm_q_heads, cfg.head_dim, cfg.llm_mlp
    X, Fx = cfg.exp_width, cfg.exp_mlp

    def gemm(m, k, n, out_bytes):
        return (2.0 * k * n + 2.0 * m * k + out_bytes, 2.0 * m * k * n)

    def resid(m, n):            # fp32 residual in and out, bf16 copy
        return m * n * (4 + 4 + 2)

    qkv_n = (H + 2) * Dh
    return {
        "vis_patch": gemm(I, cfg.patch_dim, Dv, resid(I, Dv)),
        "vis_qkv": gemm(I, Dv, 3 * Dv, 2.0 * I * 3 * Dv),
        "vis_attn": (2.0 * I * Dv * 4, 2.0 * 2 * I * T * Dv),
        "vis_o": gemm(I, Dv, Dv, resid(I, Dv)),
        "vis_up": gemm(I, Dv, Fv, 2.0 * I * Fv),
        "vis_down": gemm(I, Fv, Dv, resid(I, Dv)),
        "vis_proj": gemm(I, Dv, E, I * E * 6.0),
        "llm_qkv": gemm(P, E, qkv_n, 2.0 * P * qkv_n),
        "llm_attn": (2.0 * P * H * Dh * 2 + 2.0 * P * Dh * 2, 2.0 * 2 * H * P * P * Dh),
        "llm_o": gemm(P, H * Dh, E, resid(P, E)),
        "llm_gateup": gemm(P, E, 2 * F, 2.0 * P * F),
        "llm_down": gemm(P, F, E, resid(P, E)),
        "exp_qkv": gemm(S, X, qkv_n, 2.0 * S * qkv_n),
        "exp_attn": (2.0 * S * H * Dh * 2 + 2.0 * (P + S) * Dh * 2, 2.0 * 2 * H * S * (P + S) * Dh),
        "exp_o": gemm(S, H * Dh, X, resid(S, X)),
        "exp_gateup": gemm(S, X, 2 * Fx, 2.0 * S * Fx),
        "exp_down": gemm(S, Fx, X, resid(S, X)),
        "exp_out": gemm(S, X, cfg.action_dim, 8.0 * cfg.chunk * cfg.action_dim),
    }


def class_rooflines(work: dict, timing: dict) -> list:
    """work: class_work(); timing: {class: (total_us, launches)} -> rows sorted by total time, each with
    the class's bound ("hbm" or "mfma"), its achieved rate against the MI355X peak, and the fraction."""
    rows = []
    for name, (total_us, launches) in timing.items():
        if launches == 0:
            continue
        avg_us = total_us / launches
        row = {"class": name, "launches": launches, "avg_us": round(avg_us, 3), "total_us": round(total_us, 1)}
        if name in work:
            b, f = work[name]
            t_mem, t_cmp = b / MI355X_BW, f / MI355X_FLOPS
            if t_mem >= t_cmp:
                ach = b / (avg_us * 1e-6) / 1e9
                row.update(bound="hbm", achieved=round(ach, 1), peak=MI355X_BW / 1e9, unit="GB/s",
                           frac=round(ach / (MI355X_BW / 1e9), 4), algorithmic_bytes=int(b))
            else:
                ach = f / (avg_us * 1e-6) / 1e12
                row.update(bound="mfma", achieved=round(ach, 1), peak=MI355X_FLOPS / 1e12, unit="TFLOP/s",
                           frac=round(ach / (MI355X_FLOPS / 1e12), 4), algorithmic_flops=int(f))
        rows.append(row)
    rows.sort(key=lambda r: -r["total_us"])
    return rows


# which kernel (template family, as rocprofv3 names it) runs each operation class
KERNEL_OF_CLASS = {
    "vis_patch": "gemm_kernel", "vis_qkv": "gemm_kernel", "vis_o": "gemm_kernel", "vis_up": "gemm_kernel",
    "vis_down": "gemm_kernel", "vis_proj": "gemm_kernel", "llm_qkv": "gemm_kernel", "llm_o": "gemm_kernel",
    "llm_gateup": "gemm_kernel", "llm_down": "gemm_kernel",
    "vis_attn": "attention_kernel", "llm_attn": "attention_kernel", "exp_attn": "attention_kernel",
    "exp_qkv": "gemm_skinny_kernel", "exp_gateup": "gemm_skinny_kernel", "exp_out": "gemm_skinny_kernel",
    "exp_o": "gemm_skinny16_kernel", "exp_down": "gemm_skinny16_kernel",
    "reduce": "splitk_reduce_kernel",
}


def kernel_of_class(name: str, prefix_tokens: int | None = None):
    """Kernel template family that runs an operation class.  Up to 256 tokens the library's default schedule runs
    the vision QKV projection and the vision and prefix O projections on gemm_entry_kernel (every load issued at
    entry; the O projections over the whole k range with the residual epilogue in the GEMM)."""
    if prefix_tokens is not None and prefix_tokens <= 256 and name in ("vis_qkv", "vis_o", "llm_o"):
        return "gemm_entry_kernel"
    return KERNEL_OF_CLASS.get(name)


def kernel_rooflines(work: dict, timing: dict, traffic: dict | None = None, prefix_tokens: int | None = None) -> list:
    """Per kernel (all launches of one template family): total time, launches, algorithmic bytes and flops summed
    over its launches, the bound that dominates, the achieved rate over the kernel's total time and the
    fraction of the MI355X peak; `traffic` (measured HBM-side bytes per launch by class) is averaged over the
    launches it covers, None if a class of the family has no counter figure."""
    fam = {}
    for name, (total_us, launches) in timing.items():
        k = kernel_of_class(name, prefix_tokens)
        if k is None or launches == 0 or name not in work:
            continue
        f = fam.setdefault(k, {"kernel": k, "classes": [], "launches": 0, "total_us": 0.0, "bytes": 0.0, "flops": 0.0,
                               "traffic": 0.0, "traffic_ok": True})
        b, fl = work[name]
        f["classes"].append(name)
        f["launches"] += launches
        f["total_us"] += total_us
        f["bytes"] += b * launches
        f["flops"] += fl * launches
        if traffic and name in traffic:
            f["traffic"] += traffic[name] * launches
        else:
            f["traffic_ok"] = False
    rows = []
    for f in fam.values():
        t = f["total_us"] * 1e-6
        t_mem, t_cmp = f["bytes"] / MI355X_BW, f["flops"] / MI355X_FLOPS
        row = {"kernel": f["kernel"], "classes": f["classes"], "launches": f["launches"],
               "avg_us": round(f["total_us"] / f["launches"], 3), "total_us": round(f["total_us"], 1),
               "algorithmic_bytes_per_launch": int(f["bytes"] / f["launches"]),
               "algorithmic_flops_per_launch": int(f["flops"] / f["launches"]),
               "traffic": int(f["traffic"] / f["launches"]) if f["traffic_ok"] else None}
        if t_mem >= t_cmp:
            ach = f["bytes"] / t / 1e9
            row.update(bound="hbm", achieved=round(ach, 1), peak=MI355X_BW / 1e9, unit="GB/s", frac=round(ach / (MI355X_BW / 1e9), 4))
        else:
            ach = f["flops"] / t / 1e12
            row.update(bound="mfma", achieved=round(ach, 1), peak=MI355X_FLOPS / 1e12, unit="TFLOP/s",
                       frac=round(ach / (MI355X_FLOPS / 1e12), 4))
        rows.append(row)
    rows.sort(key=lambda r: -r["total_us"])
    return rows
