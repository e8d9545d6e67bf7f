"""ctypes front end of the CPU oracle (``zpp_oracle.cpp``).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package.  It shares nothing
with the HIP path.

The oracle is the plain definition of what one pipeline stage computes over a
scheduling unit of U micro-batches (Sections 3.1 and 3.2 of the ZeroPP paper):
materialise the stage's weights once, run every micro-batch forward and
backward, sum the weight gradients over the micro-batches, take one Adam step
on the flat shard.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzpp_oracle.so")
_lib = None

P_, G_, M_, V_, W_, S_ = range(6)


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only; AVX2+FMA baseline so the binary runs on any recent x86-64)."""
    src = os.path.join(_HERE, "zpp_oracle.cpp")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(
            ["g++", "-O3", "-march=x86-64-v3", "-std=c++17", "-fopenmp", "-fPIC", "-shared",
             "-o", _LIB_PATH, src]
        )
    return _LIB_PATH


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("arch", ctypes.c_int32), ("n_blocks", ctypes.c_int32), ("hidden", ctypes.c_int32),
        ("n_heads", ctypes.c_int32), ("ffn", ctypes.c_int32), ("seq", ctypes.c_int32),
        ("micro_batch", ctypes.c_int32), ("unit_mbs", ctypes.c_int32), ("round_bf16", ctypes.c_int32),
        ("gelu_mode", ctypes.c_int32), ("norm_eps", ctypes.c_double), ("rope_base", ctypes.c_double),
    ]


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double
    cfgp = ctypes.POINTER(_Cfg)
    lib.oracle_stage_param_count.argtypes = [cfgp]
    lib.oracle_stage_param_count.restype = u64
    lib.oracle_stage_layout_size.argtypes = [cfgp]
    lib.oracle_stage_layout_size.restype = i32
    lib.oracle_stage_param_layout.argtypes = [cfgp, i32, ctypes.c_char_p, i32, ctypes.POINTER(u64),
                                              ctypes.POINTER(u64), ctypes.POINTER(u64)]
    lib.oracle_stage_param_layout.restype = i32
    lib.oracle_num_threads.restype = i32
    lib.oracle_set_num_threads.argtypes = [i32]
    lib.oracle_bf16_bits_rne.argtypes = [ctypes.c_float]
    lib.oracle_bf16_bits_rne.restype = ctypes.c_uint16
    lib.oracle_flat_materialize_bits.argtypes = [vp, vp, i64]
    lib.oracle_flat_materialize_bits.restype = None
    lib.oracle_flat_accumulate_f32.argtypes = [vp, vp, i64, dbl]
    lib.oracle_flat_accumulate_f32.restype = None
    lib.oracle_flat_adam_f32.argtypes = [vp, vp, vp, vp, i64, dbl, dbl, dbl, dbl, dbl, dbl, i32, i32, i32]
    lib.oracle_flat_adam_f32.restype = None
    for suf in ("f32", "f64"):
        def f(name):
            return getattr(lib, f"{name}_{suf}")
        f("oracle_stage_create").argtypes = [cfgp]
        f("oracle_stage_create").restype = vp
        f("oracle_stage_destroy").argtypes = [vp]
        f("oracle_stage_destroy").restype = None
        f("oracle_stage_buffer").argtypes = [vp, i32]
        f("oracle_stage_buffer").restype = vp
        f("oracle_stage_materialize_params").argtypes = [vp]
        f("oracle_stage_materialize_params").restype = None
        f("oracle_stage_forward").argtypes = [vp, i32, vp, vp]
        f("oracle_stage_forward").restype = None
        f("oracle_stage_backward").argtypes = [vp, i32, vp, vp]
        f("oracle_stage_backward").restype = None
        f("oracle_stage_accumulate_grads").argtypes = [vp, i32, dbl]
        f("oracle_stage_accumulate_grads").restype = None
        f("oracle_shard_adam_step").argtypes = [vp, u64, u64, dbl, dbl, dbl, dbl, dbl, dbl, i32, i32, i32]
        f("oracle_shard_adam_step").restype = None
        f("oracle_stage_release_stash").argtypes = [vp, i32]
        f("oracle_stage_release_stash").restype = None
        f("oracle_stage_stash").argtypes = [vp, i32, i32, ctypes.c_char_p, ctypes.POINTER(u64)]
        f("oracle_stage_stash").restype = vp
        f("oracle_layernorm_fwd").argtypes = [i64, i64, vp, vp, vp, dbl, vp, vp, vp]
        f("oracle_layernorm_bwd").argtypes = [i64, i64, vp, vp, vp, vp, vp, vp, vp]
        f("oracle_rmsnorm_fwd").argtypes = [i64, i64, vp, vp, dbl, vp, vp, vp]
        f("oracle_rmsnorm_bwd").argtypes = [i64, i64, vp, vp, vp, vp, vp, vp]
        f("oracle_linear_fwd").argtypes = [i64, i64, i64, vp, vp, vp, vp]
        f("oracle_linear_bwd_input").argtypes = [i64, i64, i64, vp, vp, vp]
        f("oracle_linear_bwd_weight").argtypes = [i64, i64, i64, vp, vp, vp, vp]
        f("oracle_rope").argtypes = [i64, i64, i64, i64, vp, dbl, i32]
        f("oracle_attention_fwd").argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp]
        f("oracle_attention_bwd").argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp]
        f("oracle_gelu").argtypes = [i64, vp, i32, vp, vp]
        for n in ("oracle_layernorm_fwd", "oracle_layernorm_bwd", "oracle_rmsnorm_fwd", "oracle_rmsnorm_bwd",
                  "oracle_linear_fwd", "oracle_linear_bwd_input", "oracle_linear_bwd_weight", "oracle_rope",
                  "oracle_attention_fwd", "oracle_attention_bwd", "oracle_gelu"):
            f(n).restype = None
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _mk_cfg(shape) -> _Cfg:
    """``shape`` is any object/dict with the StageShape fields."""
    g = (lambda k: shape[k]) if isinstance(shape, dict) else (lambda k: getattr(shape, k))
    return _Cfg(int(g("arch")), int(g("n_blocks")), int(g("hidden")), int(g("n_heads")), int(g("ffn")),
                int(g("seq")), int(g("micro_batch")), int(g("unit_mbs")), int(g("compute_dtype") == 1),
                int(g("gelu_mode")), float(g("norm_eps")), float(g("rope_base")))


def param_count(shape) -> int:
    c = _mk_cfg(shape)
    return int(_load().oracle_stage_param_count(ctypes.byref(c)))


def param_layout(shape):
    """List of (name, offset, rows, cols) of the stage's flat parameter layout."""
    lib = _load()
    c = _mk_cfg(shape)
    out = []
    buf = ctypes.create_string_buffer(128)
    off, r, cc = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
    for i in range(lib.oracle_stage_layout_size(ctypes.byref(c))):
        rc = lib.oracle_stage_param_layout(ctypes.byref(c), i, buf, 128, ctypes.byref(off), ctypes.byref(r),
                                           ctypes.byref(cc))
        assert rc == 0
        out.append((buf.value.decode(), off.value, r.value, cc.value))
    return out


def bf16_bits_rne(v: float) -> int:
    return int(_load().oracle_bf16_bits_rne(ctypes.c_float(v)))


def _flat_arg(a: np.ndarray, dtype) -> np.ndarray:
    assert a.dtype == dtype and a.flags.c_contiguous and a.ndim == 1
    return a


def flat_materialize_bits(P: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) of a float32 array, round to nearest even (the materialise pass)."""
    P = _flat_arg(P, np.float32)
    out = np.empty(P.size, np.uint16)
    _load().oracle_flat_materialize_bits(P.ctypes.data, out.ctypes.data, P.size)
    return out


def flat_accumulate(G: np.ndarray, S: np.ndarray, scale: float) -> None:
    """G <- G + scale * S in place over float32 arrays (the accumulate pass)."""
    G, S = _flat_arg(G, np.float32), _flat_arg(S, np.float32)
    assert G.size == S.size
    _load().oracle_flat_accumulate_f32(G.ctypes.data, S.ctypes.data, G.size, float(scale))


def flat_adam(P, M, V, G, *, lr, beta1, beta2, eps, weight_decay, grad_scale=1.0, step=1, decoupled_wd=1,
              zero_grad=0) -> None:
    """One Adam step in place over float32 arrays (the same routine OracleStage.adam runs on its shard)."""
    P, M, V, G = (_flat_arg(a, np.float32) for a in (P, M, V, G))
    assert P.size == M.size == V.size == G.size
    _load().oracle_flat_adam_f32(P.ctypes.data, M.ctypes.data, V.ctypes.data, G.ctypes.data, P.size, lr, beta1,
                                 beta2, eps, weight_decay, grad_scale, step, decoupled_wd, zero_grad)


def _np_dtype(dtype: str):
    return {"f32": np.float32, "f64": np.float64}[dtype]


def _ptr(a):
    return None if a is None else a.ctypes.data


class OracleStage:
    """One pipeline stage on the CPU, in fp32 ("f32") or fp64 ("f64")."""

    def __init__(self, shape, dtype: str = "f64"):
        self.lib = _load()
        self.dtype = dtype
        self.np_dtype = _np_dtype(dtype)
        self.shape = shape
        self.cfg = _mk_cfg(shape)
        self.h = self._f("oracle_stage_create")(ctypes.byref(self.cfg))
        self.N = param_count(shape)
        self.T = self.cfg.micro_batch * self.cfg.seq
        self.hidden = self.cfg.hidden

    def _f(self, name):
        return getattr(self.lib, f"{name}_{self.dtype}")

    def close(self):
        if self.h:
            self._f("oracle_stage_destroy")(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def buffer(self, which: int) -> np.ndarray:
        """numpy view (no copy) of P, G, M, V, W (working copy) or S (staging grads)."""
        p = self._f("oracle_stage_buffer")(self.h, which)
        ct = ctypes.c_float if self.dtype == "f32" else ctypes.c_double
        arr = np.ctypeslib.as_array(ctypes.cast(p, ctypes.POINTER(ct)), shape=(self.N,))
        return arr

    @property
    def P(self): return self.buffer(P_)
    @property
    def G(self): return self.buffer(G_)
    @property
    def M(self): return self.buffer(M_)
    @property
    def V(self): return self.buffer(V_)
    @property
    def W(self): return self.buffer(W_)
    @property
    def S(self): return self.buffer(S_)

    def layout(self):
        return param_layout(self.shape)

    def materialize(self):
        self._f("oracle_stage_materialize_params")(self.h)

    def forward(self, mb: int, x: np.ndarray) -> np.ndarray:
        x = np.ascontiguousarray(x, dtype=self.np_dtype).reshape(self.T, self.hidden)
        y = np.empty_like(x)
        self._f("oracle_stage_forward")(self.h, mb, x.ctypes.data, y.ctypes.data)
        return y

    def backward(self, mb: int, dy: np.ndarray) -> np.ndarray:
        dy = np.ascontiguousarray(dy, dtype=self.np_dtype).reshape(self.T, self.hidden)
        dx = np.empty_like(dy)
        self._f("oracle_stage_backward")(self.h, mb, dy.ctypes.data, dx.ctypes.data)
        return dx

    def accumulate(self, mb: int, scale: float = 1.0):
        self._f("oracle_stage_accumulate_grads")(self.h, mb, float(scale))

    def adam(self, offset=0, count=None, *, lr, beta1, beta2, eps, weight_decay, grad_scale=1.0, step=1,
             decoupled_wd=1, zero_grad=0):
        if count is None:
            count = self.N - offset
        self._f("oracle_shard_adam_step")(self.h, offset, count, lr, beta1, beta2, eps, weight_decay,
                                          grad_scale, step, decoupled_wd, zero_grad)

    def release_stash(self, mb: int):
        self._f("oracle_stage_release_stash")(self.h, mb)

    def stash(self, mb: int, blk: int, name: str) -> np.ndarray:
        n = ctypes.c_uint64()
        p = self._f("oracle_stage_stash")(self.h, mb, blk, name.encode(), ctypes.byref(n))
        if not p:
            raise KeyError(name)
        ct = ctypes.c_float if self.dtype == "f32" else ctypes.c_double
        return np.ctypeslib.as_array(ctypes.cast(p, ctypes.POINTER(ct)), shape=(n.value,))


class Ops:
    """Stand-alone operators of the oracle, for per-kernel parity and for pins."""

    def __init__(self, dtype: str = "f64"):
        self.lib = _load()
        self.dtype = dtype
        self.nd = _np_dtype(dtype)

    def _f(self, name):
        return getattr(self.lib, f"{name}_{self.dtype}")

    def _c(self, a):
        return np.ascontiguousarray(a, dtype=self.nd)

    def layernorm_fwd(self, x, gamma, beta, eps):
        x, gamma, beta = self._c(x), self._c(gamma), self._c(beta)
        T, h = x.shape
        xhat, rstd, n = np.empty_like(x), np.empty(T, self.nd), np.empty_like(x)
        self._f("oracle_layernorm_fwd")(T, h, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(xhat), _ptr(rstd), _ptr(n))
        return n, xhat, rstd

    def layernorm_bwd(self, dn, xhat, rstd, gamma):
        dn, xhat, rstd, gamma = self._c(dn), self._c(xhat), self._c(rstd), self._c(gamma)
        T, h = dn.shape
        dx, dg, db = np.empty_like(dn), np.empty(h, self.nd), np.empty(h, self.nd)
        self._f("oracle_layernorm_bwd")(T, h, _ptr(dn), _ptr(xhat), _ptr(rstd), _ptr(gamma), _ptr(dx), _ptr(dg), _ptr(db))
        return dx, dg, db

    def rmsnorm_fwd(self, x, gamma, eps):
        x, gamma = self._c(x), self._c(gamma)
        T, h = x.shape
        xhat, rinv, n = np.empty_like(x), np.empty(T, self.nd), np.empty_like(x)
        self._f("oracle_rmsnorm_fwd")(T, h, _ptr(x), _ptr(gamma), eps, _ptr(xhat), _ptr(rinv), _ptr(n))
        return n, xhat, rinv

    def rmsnorm_bwd(self, dn, xhat, rinv, gamma):
        dn, xhat, rinv, gamma = self._c(dn), self._c(xhat), self._c(rinv), self._c(gamma)
        T, h = dn.shape
        dx, dg = np.empty_like(dn), np.empty(h, self.nd)
        self._f("oracle_rmsnorm_bwd")(T, h, _ptr(dn), _ptr(xhat), _ptr(rinv), _ptr(gamma), _ptr(dx), _ptr(dg))
        return dx, dg

    def linear_fwd(self, x, W, b=None):
        x, W = self._c(x), self._c(W)
        b = None if b is None else self._c(b)
        T, i = x.shape
        o = W.shape[0]
        assert W.shape[1] == i
        y = np.empty((T, o), self.nd)
        self._f("oracle_linear_fwd")(T, i, o, _ptr(x), _ptr(W), _ptr(b), _ptr(y))
        return y

    def linear_bwd_input(self, dy, W):
        dy, W = self._c(dy), self._c(W)
        T, o = dy.shape
        i = W.shape[1]
        assert W.shape[0] == o
        dx = np.empty((T, i), self.nd)
        self._f("oracle_linear_bwd_input")(T, i, o, _ptr(dy), _ptr(W), _ptr(dx))
        return dx

    def linear_bwd_weight(self, dy, x):
        dy, x = self._c(dy), self._c(x)
        T, o = dy.shape
        i = x.shape[1]
        assert x.shape[0] == T
        dW, db = np.empty((o, i), self.nd), np.empty(o, self.nd)
        self._f("oracle_linear_bwd_weight")(T, i, o, _ptr(dy), _ptr(x), _ptr(dW), _ptr(db))
        return dW, db

    def rope(self, u, base=10000.0, sign=1):
        u = self._c(u).copy()
        b, nh, s, d = u.shape
        self._f("oracle_rope")(b, nh, s, d, _ptr(u), base, sign)
        return u

    def attention_fwd(self, q, k, v):
        q, k, v = self._c(q), self._c(k), self._c(v)
        b, nh, s, d = q.shape
        Pr, A = np.empty((b, nh, s, s), self.nd), np.empty_like(q)
        self._f("oracle_attention_fwd")(b, nh, s, d, _ptr(q), _ptr(k), _ptr(v), _ptr(Pr), _ptr(A))
        return A, Pr

    def attention_bwd(self, q, k, v, Pr, dA):
        q, k, v, Pr, dA = self._c(q), self._c(k), self._c(v), self._c(Pr), self._c(dA)
        b, nh, s, d = q.shape
        dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
        self._f("oracle_attention_bwd")(b, nh, s, d, _ptr(q), _ptr(k), _ptr(v), _ptr(Pr), _ptr(dA), _ptr(dq),
                                        _ptr(dk), _ptr(dv))
        return dq, dk, dv

    def gelu(self, u, mode=0):
        u = self._c(u)
        g, dg = np.empty_like(u), np.empty_like(u)
        self._f("oracle_gelu")(u.size, _ptr(u), mode, _ptr(g), _ptr(dg))
        return g, dg
