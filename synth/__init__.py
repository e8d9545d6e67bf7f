"""Seeded synthetic inputs for the ZeroPP stage hot path.

This module is shared by the CPU oracle's tests and by the GPU harness so that
both consume the same bytes.  It contains no arithmetic of the method: only the
workload table (shapes of the benchmark configurations), a counter-based normal
generator (implemented in ``zpp_synth.c``) and helpers that fill a flat
parameter buffer given a layout table supplied by the caller.

Recipe (every configuration): activations x ~ N(0, 1); upstream gradients
dy ~ N(0, std 1e-2); every matrix and bias ~ N(0, std 0.02); norm gains 1 and
norm offsets 0; Adam moments zero.  For bf16 configurations x and dy are
generated with the low 16 bits of the fp32 pattern cleared, so the values are
exactly representable in bf16 and both sides see identical numbers.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, asdict

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzpp_synth.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the generator with gcc (host code only)."""
    src = os.path.join(_HERE, "zpp_synth.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-std=c11", "-o", _LIB_PATH, src, "-lm"]
        )
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        u64 = ctypes.c_uint64
        lib.zpp_synth_normal_f32.argtypes = [u64, u64, u64, u64, ctypes.c_double, ctypes.c_double,
                                             ctypes.c_int, ctypes.c_void_p]
        lib.zpp_synth_normal_f32.restype = None
        lib.zpp_synth_normal_f64.argtypes = [u64, u64, u64, u64, ctypes.c_double, ctypes.c_double,
                                             ctypes.c_void_p]
        lib.zpp_synth_normal_f64.restype = None
        lib.zpp_synth_fill_f32.argtypes = [u64, ctypes.c_float, ctypes.c_void_p]
        lib.zpp_synth_fill_f32.restype = None
        _lib = lib
    return _lib


# --------------------------------------------------------------------------
# Workload table
# --------------------------------------------------------------------------
ARCH_GPT = 0
ARCH_LLAMA = 1
DTYPE_FP32 = 0
DTYPE_BF16 = 1


@dataclass(frozen=True)
class StageShape:
    """Shape of one pipeline stage and of one scheduling unit of U micro-batches."""
    name: str
    arch: int          # 0 GPT (pre-LN, biases, GeLU), 1 LLaMA (RMSNorm, RoPE, SwiGLU)
    n_blocks: int      # transformer blocks in the stage
    hidden: int        # h
    n_heads: int
    ffn: int           # f
    seq: int           # s
    micro_batch: int   # b
    unit_mbs: int      # U
    compute_dtype: int # 0 fp32 everywhere, 1 bf16 working copy / activations
    seed: int
    gelu_mode: int = 0
    norm_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def tokens(self) -> int:
        return self.micro_batch * self.seq

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    def as_dict(self):
        return asdict(self)

    def replace(self, **kw) -> "StageShape":
        d = asdict(self)
        d.update(kw)
        return StageShape(**d)


CONFIGS = {
    "cfg1_tiny_gpt_fp32": StageShape("cfg1_tiny_gpt_fp32", ARCH_GPT, 2, 256, 4, 1024, 128, 2, 4, DTYPE_FP32, 0),
    "cfg2_gpt_1p3b": StageShape("cfg2_gpt_1p3b", ARCH_GPT, 4, 2048, 16, 8192, 2048, 2, 8, DTYPE_BF16, 1),
    "cfg3_gpt_6p2b": StageShape("cfg3_gpt_6p2b", ARCH_GPT, 4, 4096, 32, 16384, 2048, 1, 16, DTYPE_BF16, 2),
    "cfg4_llama_13b": StageShape("cfg4_llama_13b", ARCH_LLAMA, 4, 5120, 40, 13824, 4096, 1, 8, DTYPE_BF16, 3),
    "cfg5_wide_gpt": StageShape("cfg5_wide_gpt", ARCH_GPT, 2, 8192, 64, 32768, 2048, 1, 32, DTYPE_BF16, 4),
}

# Adam hyper-parameters used by every configuration.
ADAM = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)

STREAM_X = 1
STREAM_DY = 2
STREAM_PARAM0 = 1000  # + index of the tensor in the stage's layout table


# --------------------------------------------------------------------------
# Generators
# --------------------------------------------------------------------------
def normal_f32(seed: int, stream: int, count: int, mean: float = 0.0, std: float = 1.0,
               first: int = 0, bf16_exact: bool = False, out: np.ndarray | None = None) -> np.ndarray:
    lib = _load()
    if out is None:
        out = np.empty(count, dtype=np.float32)
    assert out.dtype == np.float32 and out.flags.c_contiguous and out.size == count
    lib.zpp_synth_normal_f32(seed, stream, first, count, mean, std, int(bf16_exact), out.ctypes.data)
    return out


def normal_f64(seed: int, stream: int, count: int, mean: float = 0.0, std: float = 1.0,
               first: int = 0) -> np.ndarray:
    lib = _load()
    out = np.empty(count, dtype=np.float64)
    lib.zpp_synth_normal_f64(seed, stream, first, count, mean, std, out.ctypes.data)
    return out


def make_params(shape: StageShape, layout, out: np.ndarray | None = None,
                gain_jitter: float = 0.0) -> np.ndarray:
    """Fill a flat fp32 master buffer.

    ``layout`` is a list of (name, offset, rows, cols) supplied by whichever
    side is asking (each side owns its own layout code).  Tensors whose name
    ends in ``.gamma`` are set to 1 and ``.beta`` to 0 (or jittered around
    those values when ``gain_jitter`` > 0); all others are N(0, std 0.02).
    """
    total = max(off + r * c for _, off, r, c in layout)
    if out is None:
        out = np.empty(total, dtype=np.float32)
    assert out.size >= total
    for idx, (name, off, rows, cols) in enumerate(layout):
        n = rows * cols
        view = out[off:off + n]
        if name.endswith(".gamma"):
            if gain_jitter > 0:
                normal_f32(shape.seed, STREAM_PARAM0 + idx, n, 1.0, gain_jitter, out=view)
            else:
                _load().zpp_synth_fill_f32(n, 1.0, view.ctypes.data)
        elif name.endswith(".beta"):
            if gain_jitter > 0:
                normal_f32(shape.seed, STREAM_PARAM0 + idx, n, 0.0, gain_jitter, out=view)
            else:
                _load().zpp_synth_fill_f32(n, 0.0, view.ctypes.data)
        else:
            normal_f32(shape.seed, STREAM_PARAM0 + idx, n, 0.0, 0.02, out=view)
    return out


def make_x(shape: StageShape, mb: int) -> np.ndarray:
    """Input activations of micro-batch ``mb``: [b*s, h] fp32, N(0,1)."""
    n = shape.tokens * shape.hidden
    v = normal_f32(shape.seed, STREAM_X, n, 0.0, 1.0, first=mb * n,
                   bf16_exact=(shape.compute_dtype == DTYPE_BF16))
    return v.reshape(shape.tokens, shape.hidden)


def make_dy(shape: StageShape, mb: int) -> np.ndarray:
    """Upstream output gradient of micro-batch ``mb``: [b*s, h] fp32, N(0, std 1e-2)."""
    n = shape.tokens * shape.hidden
    v = normal_f32(shape.seed, STREAM_DY, n, 0.0, 1e-2, first=mb * n,
                   bf16_exact=(shape.compute_dtype == DTYPE_BF16))
    return v.reshape(shape.tokens, shape.hidden)
