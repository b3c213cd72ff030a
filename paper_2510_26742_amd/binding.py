"""ctypes binding of libpi0_hip.so: the same names as include/pi0.h, argument marshalling only.

PyTorch is used for what it is good at here: owning device memory and streams.  Every step of
the forward pass runs in the library's HIP kernels; there is no fallback path, and loading
fails loudly if the shared library has not been built.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpi0_hip.so")

EXPORTS = ["pi0_create", "pi0_destroy", "pi0_weights_bytes", "pi0_workspace_bytes", "pi0_load_weights",
           "pi0_prefill", "pi0_denoise", "pi0_denoise_static", "pi0_infer", "pi0_debug_taps_elems", "pi0_debug_forward", "pi0_debug_profile", "pi0_sync_bench", "pi0_peak_bench", "pi0_clock_sample", "pi0_read_ahead_probe", "pi0_stream_frame",
           "pi0_set_graph_mode", "pi0_set_precision", "pi0_kernel_count", "pi0_strerror", "pi0_last_hip_error",
           "pi0_sync_dep_bench", "pi0_tune", "pi0_device_status", "pi0_loop_trace_ops", "pi0_set_loop_trace", "pi0_attention_probe"]

# enum pi0_op_class, in order
OP_CLASSES = ["misc", "vis_patch", "vis_qkv", "vis_attn", "vis_o", "vis_up", "vis_down", "vis_proj", "reduce",
              "llm_qkv", "llm_attn", "llm_o", "llm_gateup", "llm_down", "exp_embed", "exp_qkv", "exp_attn", "exp_o",
              "exp_gateup", "exp_down", "exp_out"]

PI0_OK, PI0_EINVAL, PI0_ESTATE, PI0_ENOMEM, PI0_EFORMAT, PI0_EHIP = 0, -1, -2, -3, -4, -5

_FIELDS = ["vis_layers", "vis_width", "vis_heads", "vis_mlp", "img_size", "patch", "llm_layers", "llm_width",
           "llm_q_heads", "head_dim", "llm_mlp", "exp_layers", "exp_width", "exp_mlp", "state_dim", "action_dim",
           "chunk", "steps", "vocab", "max_views", "max_prompt"]


class Pi0ConfigC(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in _FIELDS]


def to_c_config(cfg) -> Pi0ConfigC:
    """Any object with the pi0_config field names (e.g. synth.Pi0Config) -> C struct."""
    return Pi0ConfigC(**{f: int(getattr(cfg, f)) for f in _FIELDS})


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        cfgp = ctypes.POINTER(Pi0ConfigC)
        L.pi0_create.argtypes = [cfgp, ctypes.POINTER(vp)]
        L.pi0_create.restype = i32
        L.pi0_destroy.argtypes = [vp]
        L.pi0_destroy.restype = None
        L.pi0_weights_bytes.argtypes = [cfgp]
        L.pi0_weights_bytes.restype = sz
        L.pi0_workspace_bytes.argtypes = [cfgp]
        L.pi0_workspace_bytes.restype = sz
        L.pi0_load_weights.argtypes = [vp, vp, sz, vp, sz, vp]
        L.pi0_load_weights.restype = i32
        L.pi0_prefill.argtypes = [vp, vp, i32, vp, i32, vp]
        L.pi0_prefill.restype = i32
        L.pi0_denoise.argtypes = [vp, vp, vp, vp, vp]
        L.pi0_denoise.restype = i32
        L.pi0_denoise_static.argtypes = [vp, vp, vp, vp, vp]
        L.pi0_denoise_static.restype = i32
        L.pi0_infer.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, vp]
        L.pi0_infer.restype = i32
        L.pi0_debug_taps_elems.argtypes = [cfgp, i32, i32]
        L.pi0_debug_taps_elems.restype = sz
        L.pi0_debug_forward.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        L.pi0_debug_forward.restype = i32
        L.pi0_debug_profile.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, i32, ctypes.POINTER(ctypes.c_double),
                                        ctypes.POINTER(ctypes.c_int), vp]
        L.pi0_debug_profile.restype = i32
        L.pi0_stream_frame.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, vp, vp]
        L.pi0_stream_frame.restype = i32
        L.pi0_sync_bench.argtypes = [i32, i32, i32, vp, vp, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.pi0_sync_bench.restype = i32
        L.pi0_sync_dep_bench.argtypes = [i32, i32, i32, i32, i32, vp, i32, vp, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.pi0_sync_dep_bench.restype = i32
        L.pi0_attention_probe.argtypes = [i32] * 10 + [ctypes.c_float] + [vp] * 8
        L.pi0_attention_probe.restype = i32
        L.pi0_device_status.argtypes = [vp, vp]
        L.pi0_device_status.restype = i32
        L.pi0_loop_trace_ops.argtypes = [vp]
        L.pi0_loop_trace_ops.restype = i32
        L.pi0_set_loop_trace.argtypes = [vp, vp, i32]
        L.pi0_set_loop_trace.restype = i32
        L.pi0_tune.argtypes = [vp, ctypes.c_char_p]
        L.pi0_tune.restype = i32
        L.pi0_peak_bench.argtypes = [i32, vp, sz, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.pi0_peak_bench.restype = i32
        L.pi0_clock_sample.argtypes = [vp, vp]
        L.pi0_clock_sample.restype = i32
        L.pi0_read_ahead_probe.argtypes = [vp, sz, i32, i32, i32, vp, ctypes.c_longlong, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.pi0_read_ahead_probe.restype = i32
        L.pi0_set_graph_mode.argtypes = [vp, i32]
        L.pi0_set_graph_mode.restype = i32
        L.pi0_set_precision.argtypes = [vp, i32]
        L.pi0_set_precision.restype = i32
        L.pi0_kernel_count.argtypes = [vp, i32, i32]
        L.pi0_kernel_count.restype = i32
        L.pi0_strerror.argtypes = [i32]
        L.pi0_strerror.restype = ctypes.c_char_p
        L.pi0_last_hip_error.argtypes = [vp]
        L.pi0_last_hip_error.restype = i32
        _lib = L
    return _lib


class Pi0Error(RuntimeError):
    def __init__(self, code: int, hip: int = 0):
        self.code = code
        self.hip = hip
        msg = lib().pi0_strerror(code).decode()
        super().__init__(f"pi0 error {code}: {msg}" + (f" (hipError_t {hip})" if hip else ""))


def pi0_weights_bytes(cfg) -> int:
    c = to_c_config(cfg)
    return int(lib().pi0_weights_bytes(ctypes.byref(c)))


def pi0_workspace_bytes(cfg) -> int:
    c = to_c_config(cfg)
    return int(lib().pi0_workspace_bytes(ctypes.byref(c)))


def pi0_debug_taps_elems(cfg, n_views: int, n_prompt: int) -> int:
    c = to_c_config(cfg)
    return int(lib().pi0_debug_taps_elems(ctypes.byref(c), n_views, n_prompt))


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


SYNC_MODES = {"eager": 0, "graph": 1, "barrier": 2, "barrier_fence": 3, "fused": 4}


def pi0_sync_bench(mode: str, n_ops: int, reps: int, d_x, d_b, d_state, stream=None) -> float:
    """Milliseconds of one repetition of n_ops dependent x += b updates under the given ordering mode."""
    ms = ctypes.c_double(0.0)
    s = None if stream is None else int(stream.cuda_stream)
    rc = lib().pi0_sync_bench(SYNC_MODES[mode], int(n_ops), int(reps), _ptr(d_x), _ptr(d_b), _ptr(d_state),
                              ctypes.byref(ms), s)
    if rc != PI0_OK:
        raise Pi0Error(rc)
    return float(ms.value)


BARRIERS = {"counter": 0, "xcd": 1, "flags": 2, "flags8": 3, "groupadd": 4, "xcc": 5}
SYNC_DATA = {"none": 0, "bypass": 1, "inv": 2, "fence": 3, "fresh": 4, "wback": 5}


def pi0_sync_dep_bench(barrier: str, data: str, fan: int, n_ops: int, reps: int, d_x, d_b, d_state, stream=None) -> float:
    """Milliseconds of one repetition of n_ops updates x_{k+1}[r] = max_j x_k[r + j] + b[r] (d_x: [planes, 256, 1024])."""
    ms = ctypes.c_double(0.0)
    s = None if stream is None else int(stream.cuda_stream)
    rc = lib().pi0_sync_dep_bench(BARRIERS[barrier], SYNC_DATA[data], int(fan), int(n_ops), int(reps), _ptr(d_x),
                                  int(d_x.shape[0]), _ptr(d_b), _ptr(d_state), ctypes.byref(ms), s)
    if rc != PI0_OK:
        raise Pi0Error(rc)
    return float(ms.value)


def pi0_attention_probe(q, k0, v0, k1=None, v1=None, *, view_tokens=0, suffix_mask=False, chunks_per_share=0, v_split=0,
                        scale=None, stream=None):
    """Attention kernels of the pass on fp32 device tensors in natural order: q [H, Tq, d], k0 / v0 [Hk, n0, d],
    k1 / v1 [1, 64, d] or None.  Returns (out [shares, Tq, H * d], ml [shares, H, ceil32(Tq), 2] or None)."""
    import torch
    H, Tq, d = q.shape
    Hk, n0, _ = k0.shape
    n1 = 0 if k1 is None else int(k1.shape[1])
    c0 = (n0 + 31) // 32
    shares = -(-c0 // chunks_per_share) if chunks_per_share > 0 and c0 > chunks_per_share else 1
    out = torch.empty((shares, Tq, H * d), dtype=torch.float32, device=q.device)
    ml = torch.empty((shares, H, (Tq + 31) // 32 * 32, 2), dtype=torch.float32, device=q.device) if shares > 1 else None
    ts = [t.contiguous() if t is not None else None for t in (q, k0, v0, k1, v1)]
    s = None if stream is None else int(stream.cuda_stream)
    rc = lib().pi0_attention_probe(H, Hk, d, Tq, n0, n1, int(view_tokens), int(bool(suffix_mask)), int(chunks_per_share),
                                   int(v_split), float(d ** -0.5 if scale is None else scale),
                                   *[None if t is None else _ptr(t) for t in ts], _ptr(out), None if ml is None else _ptr(ml), s)
    if rc != PI0_OK:
        raise Pi0Error(rc)
    return out, ml


def pi0_clock_sample(d_out, stream=None):
    """Enqueue a sample of (shader cycle counter, 100 MHz counter) into the int64[2] device tensor d_out."""
    s = None if stream is None else int(stream.cuda_stream)
    rc = lib().pi0_clock_sample(_ptr(d_out), s)
    if rc != PI0_OK:
        raise Pi0Error(rc)


def pi0_read_ahead_probe(d_buf, layers: int, steps: int, lead: int, d_progress, wait_ticks: int, blocks: int, d_sink,
                         stream=None) -> float:
    """Milliseconds one read-ahead kernel takes over d_buf (cut into `layers` slices) at the pace *d_progress allows."""
    ms = ctypes.c_double(0.0)
    s = None if stream is None else int(stream.cuda_stream)
    nbytes = 0 if d_buf is None else int(d_buf.numel() * d_buf.element_size())
    rc = lib().pi0_read_ahead_probe(_ptr(d_buf), nbytes, int(layers), int(steps), int(lead), _ptr(d_progress),
                                    int(wait_ticks), int(blocks), _ptr(d_sink), ctypes.byref(ms), s)
    if rc != PI0_OK:
        raise Pi0Error(rc)
    return float(ms.value)


def shader_clock_ghz(sample0, sample1) -> float:
    """Average shader clock between two pi0_clock_sample results (host tensors / sequences of 2 ints)."""
    cyc, ticks = int(sample1[0]) - int(sample0[0]), int(sample1[1]) - int(sample0[1])
    return cyc / (ticks * 10.0) if ticks > 0 else float("nan")


PEAK_KINDS = {"hbm_read": 0, "mfma_bf16": 1, "cache_read": 2}
PRECISIONS = {"bf16": 0, "mxfp8_prefix_mlp": 1}


def pi0_peak_bench(kind: str, d_buf, nbytes: int, iters: int, reps: int, d_sink, stream=None) -> float:
    """GB/s of a streaming read of nbytes at d_buf ("hbm_read") or TFLOP/s of a register-resident bf16 MFMA loop."""
    out = ctypes.c_double(0.0)
    s = None if stream is None else int(stream.cuda_stream)
    rc = lib().pi0_peak_bench(PEAK_KINDS[kind], _ptr(d_buf), int(nbytes), int(iters), int(reps), _ptr(d_sink),
                              ctypes.byref(out), s)
    if rc != PI0_OK:
        raise Pi0Error(rc)
    return float(out.value)


class Pi0:
    """Thin handle over pi0_ctx.  All tensor arguments are torch CUDA tensors (device memory)."""

    def __init__(self, cfg, tune: Optional[str] = None):
        """tune: kernel choices for tuning runs (pi0_tune); None takes the PI0_TUNE environment variable if set."""
        self.cfg = cfg
        self._c = to_c_config(cfg)
        self._ctx = ctypes.c_void_p()
        rc = lib().pi0_create(ctypes.byref(self._c), ctypes.byref(self._ctx))
        if rc != PI0_OK:
            raise Pi0Error(rc)
        self.workspace = None
        if tune is None:
            tune = os.environ.get("PI0_TUNE")
        if tune:
            self.pi0_tune(tune)

    def pi0_tune(self, spec: str):
        self._check(lib().pi0_tune(self._ctx, spec.encode()))

    def close(self):
        if self._ctx:
            lib().pi0_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != PI0_OK:
            raise Pi0Error(rc, lib().pi0_last_hip_error(self._ctx) if rc == PI0_EHIP else 0)

    @staticmethod
    def _stream(stream) -> Optional[int]:
        if stream is None:
            return None
        return int(stream.cuda_stream) or None

    def pi0_load_weights(self, d_blob, stream=None):
        """d_blob: uint16/bfloat16 CUDA tensor holding the canonical blob.  Allocates the workspace
        through torch (the caller-owned memory of the C ABI) and keeps it alive on this object."""
        import torch
        need = pi0_workspace_bytes(self.cfg)
        self.workspace = torch.empty(need + 256, dtype=torch.uint8, device=d_blob.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        nbytes = d_blob.numel() * d_blob.element_size()
        self._check(lib().pi0_load_weights(self._ctx, _ptr(d_blob), nbytes, self._ws_ptr, need, self._stream(stream)))

    def pi0_prefill(self, d_images, n_views, d_prompt_ids=None, n_prompt=0, stream=None):
        self._check(lib().pi0_prefill(self._ctx, _ptr(d_images), n_views, _ptr(d_prompt_ids), n_prompt, self._stream(stream)))

    def pi0_denoise(self, d_state, d_noise, d_actions, stream=None):
        self._check(lib().pi0_denoise(self._ctx, _ptr(d_state), _ptr(d_noise), _ptr(d_actions), self._stream(stream)))

    def pi0_denoise_static(self, d_state, d_noise, d_actions, stream=None):
        self._check(lib().pi0_denoise_static(self._ctx, _ptr(d_state), _ptr(d_noise), _ptr(d_actions), self._stream(stream)))

    def pi0_infer(self, d_images, n_views, d_prompt_ids, n_prompt, d_state, d_noise, d_actions, stream=None):
        self._check(lib().pi0_infer(self._ctx, _ptr(d_images), n_views, _ptr(d_prompt_ids), n_prompt, _ptr(d_state),
                                    _ptr(d_noise), _ptr(d_actions), self._stream(stream)))

    def pi0_stream_frame(self, d_images, n_views, d_prompt_ids, n_prompt, d_state, d_noise, d_actions, stream_prefill,
                         stream_denoise):
        self._check(lib().pi0_stream_frame(self._ctx, _ptr(d_images), n_views, _ptr(d_prompt_ids), n_prompt, _ptr(d_state),
                                           _ptr(d_noise), _ptr(d_actions), int(stream_prefill.cuda_stream),
                                           int(stream_denoise.cuda_stream)))

    def pi0_debug_forward(self, d_images, n_views, d_prompt_ids, n_prompt, d_state, d_noise, d_actions, d_taps, stream=None):
        self._check(lib().pi0_debug_forward(self._ctx, _ptr(d_images), n_views, _ptr(d_prompt_ids), n_prompt, _ptr(d_state),
                                            _ptr(d_noise), _ptr(d_actions), _ptr(d_taps), d_taps.numel(),
                                            self._stream(stream)))

    def pi0_debug_profile(self, d_images, n_views, d_prompt_ids, n_prompt, d_state, d_noise, d_actions, passes=1, stream=None):
        """-> {class name: (total microseconds, launches)} over `passes` eager, event-bracketed passes."""
        us = (ctypes.c_double * len(OP_CLASSES))()
        n = (ctypes.c_int * len(OP_CLASSES))()
        self._check(lib().pi0_debug_profile(self._ctx, _ptr(d_images), n_views, _ptr(d_prompt_ids), n_prompt, _ptr(d_state),
                                            _ptr(d_noise), _ptr(d_actions), int(passes), us, n, self._stream(stream)))
        return {name: (float(us[i]), int(n[i])) for i, name in enumerate(OP_CLASSES)}

    def pi0_device_status(self, stream=None):
        """Synchronises the stream; raises if a bounded wait inside a kernel ran out."""
        self._check(lib().pi0_device_status(self._ctx, self._stream(stream)))

    def pi0_loop_trace_ops(self) -> int:
        return int(lib().pi0_loop_trace_ops(self._ctx))

    def pi0_set_loop_trace(self, d_trace):
        """d_trace: int64 CUDA tensor [ops, 256, 8] or None (off)."""
        self._check(lib().pi0_set_loop_trace(self._ctx, _ptr(d_trace), 0 if d_trace is None else int(d_trace.shape[0])))

    def pi0_set_graph_mode(self, enabled: bool):
        self._check(lib().pi0_set_graph_mode(self._ctx, 1 if enabled else 0))

    def pi0_set_precision(self, precision: str):
        self._check(lib().pi0_set_precision(self._ctx, PRECISIONS[precision]))

    def pi0_kernel_count(self, n_views: int, n_prompt: int) -> int:
        return int(lib().pi0_kernel_count(self._ctx, n_views, n_prompt))
