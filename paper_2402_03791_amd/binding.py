"""ctypes binding of libzpp.so.  Names mirror include/zpp.h; every step of the path runs in the
library's kernels.  There is no CPU fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzpp.so")
_lib = None

EXPORTS = [
    "zpp_stage_create", "zpp_stage_destroy", "zpp_stage_param_count", "zpp_stage_workspace_bytes",
    "zpp_stage_layout_size", "zpp_stage_param_layout", "zpp_stage_bind", "stage_materialize_params",
    "zpp_stage_params_changed",
    "stage_forward", "stage_backward", "stage_backward_accumulate", "stage_backward_input", "stage_backward_weight", "stage_backward_weight_group",
    "stage_forward_group", "stage_backward_input_group", "stage_backward_accumulate_group",
    "stage_accumulate_grads", "shard_adam_step", "shard_adam_step_ranges", "zpp_stage_decay_ranges",
    "zpp_stage_end_unit",
    "zpp_stage_counters", "zpp_stage_region", "zpp_last_error", "zpp_version",
    "zpp_profile_enable", "zpp_profile_reset", "zpp_profile_read",
    "zpp_op_gemm_bf16_nt", "zpp_op_gemm_bf16_tt", "zpp_op_gemm_bf16_tt_group", "zpp_op_gemm_bf16_nn", "zpp_op_attention_fwd", "zpp_op_attention_bwd", "zpp_op_flat_adam",
    "zpp_op_flat_accumulate", "zpp_op_flat_materialize", "zpp_op_attention_bwd_noalloc",
    "zpp_op_attention_bwd_noalloc_max_rows",
    "zpp_device_create", "zpp_device_create_per_stage", "zpp_device_destroy", "zpp_device_stage_count", "zpp_device_param_count",
    "zpp_device_workspace_bytes", "zpp_device_memory_terms", "zpp_device_stage", "zpp_device_bind",
    "device_forward_unit", "device_backward_unit", "device_adam_step", "zpp_device_end_unit",
    "zpp_plan_tp_comm", "zpp_plan_zeropp_comm", "zpp_plan_zeropp_wins", "zpp_plan_bubbles", "zpp_plan_max_memory",
    "zpp_plan_pp_method", "zpp_plan_choose",
]


class ZppError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"zpp status {status}: {message}")
        self.status = status


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("arch", "n_blocks", "hidden", "n_heads", "ffn", "seq", "micro_batch",
                                              "unit_mbs", "compute_dtype", "gelu_mode")] + \
               [("norm_eps", ctypes.c_float), ("rope_base", ctypes.c_float), ("split_backward", ctypes.c_int32),
                ("recompute", ctypes.c_int32), ("group_mbs", ctypes.c_int32)]


class _AdamRange(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_uint64), ("count", ctypes.c_uint64), ("lr", ctypes.c_float),
                ("weight_decay", ctypes.c_float)]


class PlanModel(ctypes.Structure):
    """zpp_plan_model of include/zpp_plan.h (the paper's symbols)."""
    _fields_ = [(n, ctypes.c_int64) for n in ("L", "h", "s", "b", "B", "P", "D")] + \
               [("Mw", ctypes.c_double), ("Ma", ctypes.c_double)]


class _PlanChoice(ctypes.Structure):
    _fields_ = [("U", ctypes.c_int64), ("V", ctypes.c_int64), ("memory", ctypes.c_double),
                ("comm", ctypes.c_double), ("bubbles", ctypes.c_double)]


class _Adam(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("lr", "beta1", "beta2", "eps", "weight_decay", "grad_scale")] + \
               [(n, ctypes.c_int32) for n in ("step", "decoupled_wd", "zero_grad", "write_back")]


def load_library(path: str | None = None):
    """Loads libzpp.so (built by paper_2402_03791_amd/build.py).  Raises if it is not there."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or _LIB_PATH
    # PyTorch owns the device memory and streams this library works on, and its wheel bundles a HIP
    # runtime with the same soname as the system one.  Import torch first so that one runtime serves
    # both; the other order leaves the process with two runtimes and no usable device.
    import torch  # noqa: F401
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2402_03791_amd.build` "
                                "(there is no fallback path)")
    L = ctypes.CDLL(path)
    vp, i32, i64, u64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_float
    L.zpp_stage_create.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(vp)]
    L.zpp_stage_destroy.argtypes = [vp]
    L.zpp_stage_destroy.restype = None
    L.zpp_stage_param_count.argtypes = [vp]
    L.zpp_stage_param_count.restype = u64
    L.zpp_stage_workspace_bytes.argtypes = [vp]
    L.zpp_stage_workspace_bytes.restype = u64
    L.zpp_stage_layout_size.argtypes = [vp]
    L.zpp_stage_param_layout.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(u64),
                                         ctypes.POINTER(u64), ctypes.POINTER(u64)]
    L.zpp_stage_bind.argtypes = [vp, vp, vp, vp, vp, vp, u64]
    L.stage_materialize_params.argtypes = [vp, vp]
    L.zpp_stage_params_changed.argtypes = [vp]
    L.stage_forward.argtypes = [vp, i32, vp, vp, vp]
    L.stage_backward.argtypes = [vp, i32, vp, vp, vp]
    L.stage_backward_accumulate.argtypes = [vp, i32, vp, vp, f32, vp]
    L.stage_backward_input.argtypes = [vp, i32, vp, vp, vp]
    L.stage_backward_weight.argtypes = [vp, i32, i32, f32, vp]
    L.stage_backward_weight_group.argtypes = [vp, i32, i32, f32, vp]
    L.stage_forward_group.argtypes = [vp, i32, i32, vp, vp, vp]
    L.stage_backward_input_group.argtypes = [vp, i32, i32, vp, vp, vp]
    L.stage_backward_accumulate_group.argtypes = [vp, i32, i32, vp, vp, f32, vp]
    L.stage_accumulate_grads.argtypes = [vp, i32, f32, vp]
    L.shard_adam_step.argtypes = [vp, u64, u64, ctypes.POINTER(_Adam), vp]
    L.shard_adam_step_ranges.argtypes = [vp, ctypes.POINTER(_AdamRange), i32, ctypes.POINTER(_Adam), vp]
    L.zpp_stage_decay_ranges.argtypes = [vp, f32, f32, ctypes.POINTER(_AdamRange), i32]
    L.zpp_stage_end_unit.argtypes = [vp]
    L.zpp_stage_counters.argtypes = [vp, ctypes.POINTER(u64), ctypes.POINTER(u64)]
    L.zpp_stage_counters.restype = None
    L.zpp_stage_region.argtypes = [vp, ctypes.c_char_p, i32, i32, ctypes.POINTER(vp), ctypes.POINTER(u64),
                                   ctypes.POINTER(i32)]
    L.zpp_device_create.argtypes = [ctypes.POINTER(_Config), i32, i32, ctypes.POINTER(vp)]
    L.zpp_device_create_per_stage.argtypes = [ctypes.POINTER(_Config), i32, i32, ctypes.POINTER(i32), ctypes.POINTER(vp)]
    L.zpp_device_destroy.argtypes = [vp]
    L.zpp_device_destroy.restype = None
    L.zpp_device_stage_count.argtypes = [vp]
    L.zpp_device_param_count.argtypes = [vp]
    L.zpp_device_param_count.restype = u64
    L.zpp_device_workspace_bytes.argtypes = [vp]
    L.zpp_device_workspace_bytes.restype = u64
    L.zpp_device_memory_terms.argtypes = [vp, ctypes.POINTER(u64), ctypes.POINTER(u64), ctypes.POINTER(u64)]
    L.zpp_device_stage.argtypes = [vp, i32]
    L.zpp_device_stage.restype = vp
    L.zpp_device_bind.argtypes = [vp, vp, vp, vp, vp, vp, u64]
    L.device_forward_unit.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp]
    L.device_backward_unit.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), f32, vp, vp]
    L.device_adam_step.argtypes = [vp, ctypes.POINTER(_Adam), vp]
    L.zpp_device_end_unit.argtypes = [vp]
    pm, dbl = ctypes.POINTER(PlanModel), ctypes.c_double
    L.zpp_plan_tp_comm.argtypes = [pm]
    L.zpp_plan_tp_comm.restype = dbl
    L.zpp_plan_zeropp_comm.argtypes = [pm, i64]
    L.zpp_plan_zeropp_comm.restype = dbl
    L.zpp_plan_zeropp_wins.argtypes = [pm, i64]
    L.zpp_plan_bubbles.argtypes = [pm, i64]
    L.zpp_plan_bubbles.restype = dbl
    L.zpp_plan_max_memory.argtypes = [pm, i64, i64] + [ctypes.POINTER(dbl)] * 3
    L.zpp_plan_max_memory.restype = dbl
    L.zpp_plan_pp_method.argtypes = [pm, i32, i64] + [ctypes.POINTER(dbl)] * 3
    L.zpp_plan_choose.argtypes = [pm, dbl, ctypes.POINTER(_PlanChoice)]
    L.zpp_profile_enable.argtypes = [i32]
    L.zpp_profile_reset.restype = None
    L.zpp_profile_read.argtypes = [i32, ctypes.POINTER(u64), ctypes.POINTER(ctypes.c_double),
                                   ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    L.zpp_last_error.restype = ctypes.c_char_p
    L.zpp_version.restype = ctypes.c_char_p
    L.zpp_op_gemm_bf16_nt.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, vp, i32, i32, vp]
    L.zpp_op_gemm_bf16_tt.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp]
    L.zpp_op_gemm_bf16_nn.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp]
    L.zpp_op_gemm_bf16_tt_group.argtypes = [i32, vp, vp, i64, vp, vp, vp, vp, vp, vp, i32, vp]
    L.zpp_op_attention_fwd.argtypes = [i32, i32, vp, vp, vp, i64, i64, i64, i64, vp]
    L.zpp_op_attention_bwd.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, vp]
    L.zpp_op_attention_bwd_noalloc.argtypes = [i32, i32, vp, vp, vp, vp, vp, i64, i64, i64, i64, vp]
    L.zpp_op_attention_bwd_noalloc_max_rows.restype = u64
    L.zpp_op_flat_adam.argtypes = [vp, vp, vp, vp, u64, ctypes.POINTER(_Adam), vp]
    L.zpp_op_flat_accumulate.argtypes = [vp, vp, u64, f32, vp]
    L.zpp_op_flat_materialize.argtypes = [vp, vp, u64, i32, vp]
    if path == _LIB_PATH:
        _lib = L
    return L


def lib():
    return load_library()


def _check(status: int):
    if status != 0:
        raise ZppError(status, lib().zpp_last_error().decode())


@dataclass
class StageConfig:
    arch: int
    n_blocks: int
    hidden: int
    n_heads: int
    ffn: int
    seq: int
    micro_batch: int
    unit_mbs: int
    compute_dtype: int
    gelu_mode: int = 0
    norm_eps: float = 1e-5
    rope_base: float = 10000.0
    split_backward: int = 0
    recompute: int = 0     # 0 none, 1 full, 2 selective
    group_mbs: int = 0

    @classmethod
    def from_shape(cls, shape, split_backward: int = 0, recompute: int = 0, group_mbs: int = 0) -> "StageConfig":
        g = (lambda k: shape[k]) if isinstance(shape, dict) else (lambda k: getattr(shape, k))
        return cls(*(g(k) for k in ("arch", "n_blocks", "hidden", "n_heads", "ffn", "seq", "micro_batch", "unit_mbs",
                                    "compute_dtype", "gelu_mode", "norm_eps", "rope_base")), split_backward, recompute,
                   group_mbs)

    def _c(self) -> _Config:
        return _Config(self.arch, self.n_blocks, self.hidden, self.n_heads, self.ffn, self.seq, self.micro_batch,
                       self.unit_mbs, self.compute_dtype, self.gelu_mode, self.norm_eps, self.rope_base,
                       self.split_backward, self.recompute, self.group_mbs)


def _adam_struct(lr, beta1, beta2, eps, weight_decay, grad_scale=1.0, step=1, decoupled_wd=1, zero_grad=0,
                 write_back=0) -> _Adam:
    return _Adam(lr, beta1, beta2, eps, weight_decay, grad_scale, step, decoupled_wd, zero_grad, write_back)


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class Stage:
    """A stage handle.  With ``allocate=True`` it also owns torch tensors for P, G, M, V and the
    workspace and binds them; otherwise call :meth:`bind` with your own tensors."""

    def __init__(self, cfg, device: str | None = "cuda:0", allocate: bool = True, split_backward: int = 0,
                 recompute: int = 0, group_mbs: int = 0):
        self.cfg = cfg if isinstance(cfg, StageConfig) else StageConfig.from_shape(cfg, int(split_backward),
                                                                                   int(recompute), int(group_mbs))
        self._h = ctypes.c_void_p()
        c = self.cfg._c()
        _check(lib().zpp_stage_create(ctypes.byref(c), ctypes.byref(self._h)))
        self.N = int(lib().zpp_stage_param_count(self._h))
        self.workspace_bytes = int(lib().zpp_stage_workspace_bytes(self._h))
        self.T = self.cfg.micro_batch * self.cfg.seq
        self.P = self.G = self.M = self.V = self.workspace = None
        if allocate:
            import torch
            self.act_dtype = torch.bfloat16 if self.cfg.compute_dtype == 1 else torch.float32
            dev = torch.device(device)
            self.P = torch.zeros(self.N, dtype=torch.float32, device=dev)
            self.G = torch.zeros_like(self.P)
            self.M = torch.zeros_like(self.P)
            self.V = torch.zeros_like(self.P)
            self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=dev)
            self.bind(self.P, self.G, self.M, self.V, self.workspace)

    def close(self):
        if self._h:
            lib().zpp_stage_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- host-only queries
    def layout(self):
        out = []
        name, off, r, c = ctypes.c_char_p(), ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
        for i in range(lib().zpp_stage_layout_size(self._h)):
            _check(lib().zpp_stage_param_layout(self._h, i, ctypes.byref(name), ctypes.byref(off), ctypes.byref(r),
                                                ctypes.byref(c)))
            out.append((name.value.decode(), off.value, r.value, c.value))
        return out

    def counters(self):
        a, b = ctypes.c_uint64(), ctypes.c_uint64()
        lib().zpp_stage_counters(self._h, ctypes.byref(a), ctypes.byref(b))
        return a.value, b.value

    # ---- binding and the hot path
    def bind(self, P, G, M, V, workspace):
        self.P, self.G, self.M, self.V, self.workspace = P, G, M, V, workspace
        _check(lib().zpp_stage_bind(self._h, P.data_ptr(), G.data_ptr(), M.data_ptr(), V.data_ptr(),
                                    workspace.data_ptr(), workspace.numel() * workspace.element_size()))

    def bind_raw(self, P, G, M, V, workspace, workspace_bytes):
        """Pointers as integers; no checks beyond the library's own (used by host-only tests)."""
        _check(lib().zpp_stage_bind(self._h, P, G, M, V, workspace, workspace_bytes))

    def materialize_params(self, stream=None):
        _check(lib().stage_materialize_params(self._h, _stream_ptr(stream)))

    def params_changed(self):
        _check(lib().zpp_stage_params_changed(self._h))

    def forward(self, mb: int, x, y=None, stream=None):
        import torch
        if y is None:
            y = torch.empty_like(x)
        _check(lib().stage_forward(self._h, mb, x.data_ptr(), y.data_ptr(), _stream_ptr(stream)))
        return y

    def backward(self, mb: int, dy, dx=None, stream=None):
        import torch
        if dx is None:
            dx = torch.empty_like(dy)
        _check(lib().stage_backward(self._h, mb, dy.data_ptr(), dx.data_ptr(), _stream_ptr(stream)))
        return dx

    def backward_accumulate(self, mb: int, dy, dx=None, scale: float = 1.0, stream=None):
        import torch
        if dx is None:
            dx = torch.empty_like(dy)
        _check(lib().stage_backward_accumulate(self._h, mb, dy.data_ptr(), dx.data_ptr(), scale,
                                               _stream_ptr(stream)))
        return dx

    def backward_input(self, mb: int, dy, dx=None, stream=None):
        import torch
        if dx is None:
            dx = torch.empty_like(dy)
        _check(lib().stage_backward_input(self._h, mb, dy.data_ptr(), dx.data_ptr(), _stream_ptr(stream)))
        return dx

    def backward_weight(self, mb: int, in_place: bool = False, scale: float = 1.0, stream=None):
        _check(lib().stage_backward_weight(self._h, mb, int(in_place), scale, _stream_ptr(stream)))

    def backward_weight_group(self, first: int, count: int, scale: float = 1.0, stream=None):
        _check(lib().stage_backward_weight_group(self._h, first, count, scale, _stream_ptr(stream)))

    def forward_group(self, first: int, count: int, x, y=None, stream=None):
        """x, y: [count * T, h], micro-batch first + k in rows [k*T, (k+1)*T)."""
        import torch
        if y is None:
            y = torch.empty_like(x)
        _check(lib().stage_forward_group(self._h, first, count, x.data_ptr(), y.data_ptr(), _stream_ptr(stream)))
        return y

    def backward_input_group(self, first: int, count: int, dy, dx=None, stream=None):
        import torch
        if dx is None:
            dx = torch.empty_like(dy)
        _check(lib().stage_backward_input_group(self._h, first, count, dy.data_ptr(), dx.data_ptr(),
                                                _stream_ptr(stream)))
        return dx

    def backward_accumulate_group(self, first: int, count: int, dy, dx=None, scale: float = 1.0, stream=None):
        import torch
        if dx is None:
            dx = torch.empty_like(dy)
        _check(lib().stage_backward_accumulate_group(self._h, first, count, dy.data_ptr(), dx.data_ptr(), scale,
                                                     _stream_ptr(stream)))
        return dx

    def accumulate_grads(self, mb: int, scale: float = 1.0, stream=None):
        _check(lib().stage_accumulate_grads(self._h, mb, scale, _stream_ptr(stream)))

    def adam_step(self, offset: int = 0, count: int | None = None, stream=None, **hp):
        a = _adam_struct(**hp)
        if count is None:
            count = self.N - offset
        _check(lib().shard_adam_step(self._h, offset, count, ctypes.byref(a), _stream_ptr(stream)))

    def decay_ranges(self, lr: float, weight_decay: float):
        """(offset, count, lr, weight_decay) tuples covering the shard: decay on matrices only."""
        n = lib().zpp_stage_decay_ranges(self._h, lr, weight_decay, None, 0)
        arr = (_AdamRange * n)()
        assert lib().zpp_stage_decay_ranges(self._h, lr, weight_decay, arr, n) == n
        return [(r.offset, r.count, r.lr, r.weight_decay) for r in arr]

    def adam_step_ranges(self, ranges, stream=None, **hp):
        """ranges: iterable of (offset, count, lr, weight_decay); hp as adam_step (its lr / weight_decay unused)."""
        ranges = list(ranges)
        arr = (_AdamRange * max(len(ranges), 1))(*[_AdamRange(*r) for r in ranges])
        a = _adam_struct(**hp)
        _check(lib().shard_adam_step_ranges(self._h, arr, len(ranges), ctypes.byref(a), _stream_ptr(stream)))

    def end_unit(self):
        _check(lib().zpp_stage_end_unit(self._h))

    def region(self, name: str, mb: int = 0, blk: int = 0):
        """torch view of a named workspace region (working copy, staging gradients, stash tensors)."""
        import torch
        p, n, e = ctypes.c_void_p(), ctypes.c_uint64(), ctypes.c_int32()
        _check(lib().zpp_stage_region(self._h, name.encode(), mb, blk, ctypes.byref(p), ctypes.byref(n),
                                      ctypes.byref(e)))
        off = p.value - self.workspace.data_ptr()
        raw = self.workspace[off:off + n.value * e.value]
        if e.value == 4:
            dt = torch.float32
        else:
            dt = torch.bfloat16
        return raw.view(dt)


class Device:
    """V stages of one configuration on one device (include/zpp_device.h).  With ``allocate=True`` it owns
    torch tensors for P, G, M, V (V * N elements, stage v at [v*N, (v+1)*N)) and the workspace."""

    def __init__(self, cfg, n_stages: int, prefetch: bool = True, device: str | None = "cuda:0",
                 allocate: bool = True, recompute=0, split_backward: int = 0):
        """recompute: one mode for all stages (0 none, 1 full, 2 selective) or a list with one mode per stage."""
        per_stage = list(recompute) if isinstance(recompute, (list, tuple)) else None
        self.cfg = cfg if isinstance(cfg, StageConfig) else StageConfig.from_shape(
            cfg, int(split_backward), 0 if per_stage is not None else int(recompute))
        self._h = ctypes.c_void_p()
        c = self.cfg._c()
        if per_stage is not None:
            if len(per_stage) != n_stages:
                raise ValueError("one recomputation mode per stage")
            modes = (ctypes.c_int32 * n_stages)(*[int(m) for m in per_stage])
            _check(lib().zpp_device_create_per_stage(ctypes.byref(c), n_stages, int(prefetch), modes,
                                                     ctypes.byref(self._h)))
        else:
            _check(lib().zpp_device_create(ctypes.byref(c), n_stages, int(prefetch), ctypes.byref(self._h)))
        self.n_stages = n_stages
        self.U = self.cfg.unit_mbs
        self.N_total = int(lib().zpp_device_param_count(self._h))
        self.N = self.N_total // n_stages
        self.workspace_bytes = int(lib().zpp_device_workspace_bytes(self._h))
        self.P = self.G = self.M = self.V = self.workspace = None
        if allocate:
            import torch
            self.act_dtype = torch.bfloat16 if self.cfg.compute_dtype == 1 else torch.float32
            dev = torch.device(device)
            self.P = torch.zeros(self.N_total, dtype=torch.float32, device=dev)
            self.G = torch.zeros_like(self.P)
            self.M = torch.zeros_like(self.P)
            self.V = torch.zeros_like(self.P)
            self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=dev)
            _check(lib().zpp_device_bind(self._h, self.P.data_ptr(), self.G.data_ptr(), self.M.data_ptr(),
                                         self.V.data_ptr(), self.workspace.data_ptr(), self.workspace_bytes))

    def close(self):
        if self._h:
            lib().zpp_device_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def memory_terms(self):
        a, b, c = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
        _check(lib().zpp_device_memory_terms(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
        return {"working_copies": a.value, "scratch": b.value, "stash": c.value}

    def bind_raw(self, P, G, M, V, workspace, workspace_bytes):
        _check(lib().zpp_device_bind(self._h, P, G, M, V, workspace, workspace_bytes))

    @staticmethod
    def _ptrs(tensors):
        arr = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
        return arr

    def forward_unit(self, xs, ys, stream=None, side_stream=None):
        """xs, ys: lists of V*U tensors, entry v*U + m for stage v and micro-batch m."""
        _check(lib().device_forward_unit(self._h, self._ptrs(xs), self._ptrs(ys), _stream_ptr(stream),
                                         None if side_stream is None else ctypes.c_void_p(side_stream.cuda_stream)))

    def backward_unit(self, dys, dxs, scale: float = 1.0, stream=None, side_stream=None):
        _check(lib().device_backward_unit(self._h, self._ptrs(dys), self._ptrs(dxs), scale, _stream_ptr(stream),
                                          None if side_stream is None else ctypes.c_void_p(side_stream.cuda_stream)))

    def adam_step(self, stream=None, **hp):
        a = _adam_struct(**hp)
        _check(lib().device_adam_step(self._h, ctypes.byref(a), _stream_ptr(stream)))

    def end_unit(self):
        _check(lib().zpp_device_end_unit(self._h))


# ---- cost model and planner (include/zpp_plan.h) ---------------------------------------------------
PP_METHODS = ["gpipe", "1f1b", "interleaved_1f1b", "zeropp", "zeropp_recompute"]


def plan_tp_comm(m: PlanModel) -> float:
    return lib().zpp_plan_tp_comm(ctypes.byref(m))


def plan_zeropp_comm(m: PlanModel, U: int) -> float:
    return lib().zpp_plan_zeropp_comm(ctypes.byref(m), U)


def plan_zeropp_wins(m: PlanModel, U: int) -> bool:
    return bool(lib().zpp_plan_zeropp_wins(ctypes.byref(m), U))


def plan_bubbles(m: PlanModel, U: int) -> float:
    return lib().zpp_plan_bubbles(ctypes.byref(m), U)


def plan_max_memory(m: PlanModel, U: int, V: int) -> dict:
    a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    tot = lib().zpp_plan_max_memory(ctypes.byref(m), U, V, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    return {"total": tot, "weights_partitioned": a.value, "weights_gathered": b.value, "activations": c.value}


def plan_pp_method(m: PlanModel, method: str, V: int = 1) -> dict:
    a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _check(lib().zpp_plan_pp_method(ctypes.byref(m), PP_METHODS.index(method), V, ctypes.byref(a), ctypes.byref(b),
                                    ctypes.byref(c)))
    return {"bubble_ratio": a.value, "weight_memory": b.value, "activation_memory": c.value}


def plan_choose(m: PlanModel, memory_limit: float) -> dict:
    c = _PlanChoice()
    _check(lib().zpp_plan_choose(ctypes.byref(m), memory_limit, ctypes.byref(c)))
    return {"U": c.U, "V": c.V, "memory": c.memory, "comm": c.comm, "bubbles": c.bubbles}


PROF_CLASSES = ["gemm", "attn_fwd", "attn_bwd", "accumulate", "adam", "materialize", "other", "gemm_dw"]


def profile_enable(on: bool):
    _check(lib().zpp_profile_enable(int(on)))


def profile_reset():
    lib().zpp_profile_reset()


def profile_read():
    """{class: (launches, total_ms, work, min_bytes)} for everything bracketed since the last reset."""
    out = {}
    n, ms, w, b = ctypes.c_uint64(), ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    for i, name in enumerate(PROF_CLASSES):
        _check(lib().zpp_profile_read(i, ctypes.byref(n), ctypes.byref(ms), ctypes.byref(w), ctypes.byref(b)))
        out[name] = (n.value, ms.value, w.value, b.value)
    return out


# ---- operator-level entry points (include/zpp_ops.h) ----------------------------------------------
GEMM_TILES = {"auto": -1, "256x256": 0, "128x128": 1, "256x128": 2, "128x256": 3}


def op_gemm_bf16_nt(A, B, C, bias=None, resid=None, tile="auto", stream=None, accumulate: bool = False):
    """C = A . B^T (+ bias) (+ resid); accumulate (float C only): C += A . B^T.  tile: a key of GEMM_TILES."""
    import torch
    if accumulate and C.dtype != torch.float32:
        raise ValueError("accumulate needs a float32 C")
    M, K = A.shape
    N = B.shape[0]
    _check(lib().zpp_op_gemm_bf16_nt(M, N, K, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), C.data_ptr(),
                                     C.stride(0), None if bias is None else bias.data_ptr(),
                                     None if resid is None else resid.data_ptr(),
                                     2 if accumulate else int(C.dtype == torch.float32), GEMM_TILES[tile],
                                     _stream_ptr(stream)))
    return C


def op_gemm_bf16_tt(A, B, C, stream=None, accumulate: bool = False):
    """C[M,N] = A^T . B with A [K, M] and B [K, N] (the weight-gradient product on token-major operands)."""
    import torch
    K, M = A.shape
    N = B.shape[1]
    _check(lib().zpp_op_gemm_bf16_tt(M, N, K, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), C.data_ptr(),
                                     C.stride(0), 2 if accumulate else int(C.dtype == torch.float32),
                                     _stream_ptr(stream)))
    return C


def op_gemm_bf16_tt_group(As, Bs, Cs, stream=None, accumulate: bool = False):
    """op_gemm_bf16_tt for several (A, B, C) with the same K and the same kind of C, as one launch."""
    import torch
    n = len(As)
    K = As[0].shape[0]
    if any(a.shape[0] != K or b.shape[0] != K for a, b in zip(As, Bs)) or any(c.dtype != Cs[0].dtype for c in Cs):
        raise ValueError("the products of a group share K and the output type")
    i64, ptr = ctypes.c_int64 * n, ctypes.c_void_p * n
    _check(lib().zpp_op_gemm_bf16_tt_group(
        n, i64(*[a.shape[1] for a in As]), i64(*[b.shape[1] for b in Bs]), K, ptr(*[a.data_ptr() for a in As]),
        i64(*[a.stride(0) for a in As]), ptr(*[b.data_ptr() for b in Bs]), i64(*[b.stride(0) for b in Bs]),
        ptr(*[c.data_ptr() for c in Cs]), i64(*[c.stride(0) for c in Cs]),
        2 if accumulate else int(Cs[0].dtype == torch.float32), _stream_ptr(stream)))
    return Cs


def op_gemm_bf16_nn(A, B, C, stream=None, accumulate: bool = False):
    """C[M,N] = A . B with A [M, K] and B [K, N] (the input-gradient product on the weights as stored)."""
    import torch
    M, K = A.shape
    N = B.shape[1]
    _check(lib().zpp_op_gemm_bf16_nn(M, N, K, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), C.data_ptr(),
                                     C.stride(0), 2 if accumulate else int(C.dtype == torch.float32),
                                     _stream_ptr(stream)))
    return C


def op_attention_fwd(qkv, attn, lse, b, seq, nh, d, impl=0, stream=None):
    import torch
    dt = 1 if qkv.dtype == torch.bfloat16 else 0
    _check(lib().zpp_op_attention_fwd(dt, impl, qkv.data_ptr(), attn.data_ptr(), lse.data_ptr(), b, seq, nh, d,
                                      _stream_ptr(stream)))


def op_attention_bwd(qkv, attn, dattn, lse, delta, dqkv, b, seq, nh, d, impl=0, stream=None):
    import torch
    dt = 1 if qkv.dtype == torch.bfloat16 else 0
    _check(lib().zpp_op_attention_bwd(dt, impl, qkv.data_ptr(), attn.data_ptr(), dattn.data_ptr(), lse.data_ptr(),
                                      delta.data_ptr(), dqkv.data_ptr(), b, seq, nh, d, _stream_ptr(stream)))


def op_attention_bwd_noalloc(qkv, attn, dattn, lse, dqkv, b, seq, nh, d, impl=0, stream=None):
    """As op_attention_bwd, scratch inside the library (no allocation anywhere in the call)."""
    import torch
    dt = 1 if qkv.dtype == torch.bfloat16 else 0
    _check(lib().zpp_op_attention_bwd_noalloc(dt, impl, qkv.data_ptr(), attn.data_ptr(), dattn.data_ptr(),
                                              lse.data_ptr(), dqkv.data_ptr(), b, seq, nh, d, _stream_ptr(stream)))


def op_flat_adam(P, M, V, G, stream=None, **hp):
    a = _adam_struct(**hp)
    _check(lib().zpp_op_flat_adam(P.data_ptr(), M.data_ptr(), V.data_ptr(), G.data_ptr(), P.numel(), ctypes.byref(a),
                                  _stream_ptr(stream)))


def op_flat_accumulate(G, S, scale=1.0, stream=None):
    _check(lib().zpp_op_flat_accumulate(G.data_ptr(), S.data_ptr(), G.numel(), scale, _stream_ptr(stream)))


def op_flat_materialize(P, W, stream=None):
    import torch
    _check(lib().zpp_op_flat_materialize(P.data_ptr(), W.data_ptr(), P.numel(), int(W.dtype == torch.bfloat16),
                                         _stream_ptr(stream)))
