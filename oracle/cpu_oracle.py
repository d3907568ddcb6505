"""ctypes front end of the C oracle (``dmr_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
CPU-baseline leg.  The GPU library and its Python binding never import this module, and this
module imports nothing from them.

Every function takes and returns numpy arrays that live in host memory; bf16 values travel as
``uint16`` bit patterns.  The arithmetic is all in the C file, which states the definitions
(format reading of Sec. 5.1 / App. E of the paper: 4-bit weights, 16-bit activations).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dmr_oracle.c")
_LIB = os.path.join(_HERE, "libdmr_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, OpenMP for the optional row-parallel loop)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-std=c99", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
               "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_bf16_to_f64.restype = ctypes.c_double
        lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
        lib.oracle_f64_to_bf16.restype = ctypes.c_uint16
        lib.oracle_f64_to_bf16.argtypes = [ctypes.c_double]
        lib.oracle_f32_to_bf16.restype = ctypes.c_uint16
        lib.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        lib.oracle_f32_to_bf16_array.restype = None
        lib.oracle_f32_to_bf16_array.argtypes = [i64, vp, vp]
        lib.oracle_f64_to_bf16_array.restype = None
        lib.oracle_f64_to_bf16_array.argtypes = [i64, vp, vp]
        lib.oracle_quantize.restype = i32
        lib.oracle_quantize.argtypes = [i64, i64, i64, vp, vp, vp, vp]
        lib.oracle_pack.restype = i32
        lib.oracle_pack.argtypes = [i64, i64, vp, vp]
        lib.oracle_unpack.restype = i32
        lib.oracle_unpack.argtypes = [i64, i64, vp, vp]
        lib.oracle_dequantize_exact.restype = i32
        lib.oracle_dequantize_exact.argtypes = [i64, i64, i64, vp, vp, vp, vp]
        lib.oracle_dequantize.restype = i32
        lib.oracle_dequantize.argtypes = [i64, i64, i64, vp, vp, vp, vp]
        lib.oracle_forward.restype = i32
        lib.oracle_forward.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, i32, i32]
        lib.oracle_forward_sampled.restype = i32
        lib.oracle_forward_sampled.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, i64, vp, vp, vp]
        lib.oracle_bf16_forward.restype = i32
        lib.oracle_bf16_forward.argtypes = [i64, i64, i64, vp, vp, vp, i32]
        lib.oracle_bf16_forward_sampled.restype = i32
        lib.oracle_bf16_forward_sampled.argtypes = [i64, i64, i64, vp, vp, i64, vp, vp, vp]
        lib.oracle_quantize_bits.restype = i32
        lib.oracle_quantize_bits.argtypes = [i64, i64, i64, i32, vp, vp, vp, vp]
        lib.oracle_pack3.restype = i32
        lib.oracle_pack3.argtypes = [i64, i64, vp, vp]
        lib.oracle_unpack3.restype = i32
        lib.oracle_unpack3.argtypes = [i64, i64, vp, vp]
        lib.oracle_dequantize_exact_bits.restype = i32
        lib.oracle_dequantize_exact_bits.argtypes = [i64, i64, i64, i32, vp, vp, vp, vp]
        lib.oracle_dequantize_bits.restype = i32
        lib.oracle_dequantize_bits.argtypes = [i64, i64, i64, i32, vp, vp, vp, vp]
        lib.oracle_forward_bits.restype = i32
        lib.oracle_forward_bits.argtypes = [i64, i64, i64, i32, i64, vp, vp, vp, vp, vp, i32]
        lib.oracle_rmsnorm.restype = i32
        lib.oracle_rmsnorm.argtypes = [i64, i64, vp, vp, ctypes.c_double, vp]
        lib.oracle_swiglu.restype = i32
        lib.oracle_swiglu.argtypes = [i64, i64, vp, vp]
        lib.oracle_max_threads.restype = i32
        lib.oracle_max_threads.argtypes = []
        _lib = lib
    return _lib


def _arr(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc < 0:
        raise ValueError(f"{what} rejected its arguments (code {rc})")
    return rc


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def bf16_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns (any shape) to float64."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f64_to_bf16(values) -> np.ndarray:
    """RNE rounding of float64 values (any shape) to bf16 bit patterns, done by the C code."""
    v = _arr(values, np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    _load().oracle_f64_to_bf16_array(v.size, _p(v), _p(out))
    return out


def f32_to_bf16(values) -> np.ndarray:
    v = _arr(values, np.float32)
    out = np.empty(v.shape, dtype=np.uint16)
    _load().oracle_f32_to_bf16_array(v.size, _p(v), _p(out))
    return out


def quantize(w, g: int):
    """fp32 weights [N][K] -> (q uint8 [N][K], s bf16 bits [N][K/g], z bf16 bits [N][K/g])."""
    w = _arr(w, np.float32)
    N, K = w.shape
    q = np.empty((N, K), dtype=np.uint8)
    s = np.empty((N, K // g), dtype=np.uint16)
    z = np.empty((N, K // g), dtype=np.uint16)
    _check(_load().oracle_quantize(K, N, g, _p(w), _p(q), _p(s), _p(z)), "oracle_quantize")
    return q, s, z


def pack(q) -> np.ndarray:
    q = _arr(q, np.uint8)
    N, K = q.shape
    out = np.empty((N, K // 8), dtype=np.uint32)
    _check(_load().oracle_pack(K, N, _p(q), _p(out)), "oracle_pack")
    return out


def unpack(qweight) -> np.ndarray:
    qweight = _arr(qweight, np.uint32)
    N, K8 = qweight.shape
    out = np.empty((N, K8 * 8), dtype=np.uint8)
    _check(_load().oracle_unpack(K8 * 8, N, _p(qweight), _p(out)), "oracle_unpack")
    return out


def _qsz(qweight, s, z, g):
    qweight = _arr(qweight, np.uint32)
    N, K8 = qweight.shape
    K = K8 * 8
    s = _arr(s, np.uint16, (N, K // g))
    z = _arr(z, np.uint16, (N, K // g))
    return qweight, s, z, N, K


def dequantize_exact(qweight, s, z, g: int) -> np.ndarray:
    qweight, s, z, N, K = _qsz(qweight, s, z, g)
    out = np.empty((N, K), dtype=np.float64)
    _check(_load().oracle_dequantize_exact(K, N, g, _p(qweight), _p(s), _p(z), _p(out)),
           "oracle_dequantize_exact")
    return out


def dequantize(qweight, s, z, g: int) -> np.ndarray:
    qweight, s, z, N, K = _qsz(qweight, s, z, g)
    out = np.empty((N, K), dtype=np.uint16)
    _check(_load().oracle_dequantize(K, N, g, _p(qweight), _p(s), _p(z), _p(out)),
           "oracle_dequantize")
    return out


def forward(qweight, s, z, g: int, x_bits, rounded_weights: bool = False, threads: int = 1):
    """y float64 [M][N]; with ``return_threads`` semantics folded in: returns (y, threads_used)."""
    qweight, s, z, N, K = _qsz(qweight, s, z, g)
    x_bits = _arr(x_bits, np.uint16)
    M = x_bits.shape[0]
    if x_bits.shape != (M, K):
        raise ValueError("x must be [M][K]")
    y = np.zeros((M, N), dtype=np.float64)
    used = _check(_load().oracle_forward(K, N, g, M, _p(qweight), _p(s), _p(z), _p(x_bits), _p(y),
                                         int(rounded_weights), int(threads)), "oracle_forward")
    return y, used


def forward_sampled(qweight, s, z, g: int, x_bits, ms, ns) -> np.ndarray:
    qweight, s, z, N, K = _qsz(qweight, s, z, g)
    x_bits = _arr(x_bits, np.uint16)
    M = x_bits.shape[0]
    ms = _arr(ms, np.int64)
    ns = _arr(ns, np.int64, ms.shape)
    out = np.empty(ms.shape, dtype=np.float64)
    _check(_load().oracle_forward_sampled(K, N, g, M, _p(qweight), _p(s), _p(z), _p(x_bits),
                                          ms.size, _p(ms), _p(ns), _p(out)),
           "oracle_forward_sampled")
    return out


def bf16_forward(w_bits, x_bits, threads: int = 1):
    w_bits = _arr(w_bits, np.uint16)
    N, K = w_bits.shape
    x_bits = _arr(x_bits, np.uint16)
    M = x_bits.shape[0]
    if x_bits.shape != (M, K):
        raise ValueError("x must be [M][K]")
    y = np.zeros((M, N), dtype=np.float64)
    used = _check(_load().oracle_bf16_forward(K, N, M, _p(w_bits), _p(x_bits), _p(y), int(threads)),
                  "oracle_bf16_forward")
    return y, used


def bf16_forward_sampled(w_bits, x_bits, ms, ns) -> np.ndarray:
    w_bits = _arr(w_bits, np.uint16)
    N, K = w_bits.shape
    x_bits = _arr(x_bits, np.uint16)
    M = x_bits.shape[0]
    ms = _arr(ms, np.int64)
    ns = _arr(ns, np.int64, ms.shape)
    out = np.empty(ms.shape, dtype=np.float64)
    _check(_load().oracle_bf16_forward_sampled(K, N, M, _p(w_bits), _p(x_bits), ms.size, _p(ms),
                                               _p(ns), _p(out)), "oracle_bf16_forward_sampled")
    return out


# ---- 3-bit variant (W3A16 group-128): 32 codes per three words ---------------------------------

def quantize_bits(w, g: int, bits: int):
    w = _arr(w, np.float32)
    N, K = w.shape
    q = np.empty((N, K), dtype=np.uint8)
    s = np.empty((N, K // g), dtype=np.uint16)
    z = np.empty((N, K // g), dtype=np.uint16)
    _check(_load().oracle_quantize_bits(K, N, g, bits, _p(w), _p(q), _p(s), _p(z)), "oracle_quantize_bits")
    return q, s, z


def pack3(q) -> np.ndarray:
    q = _arr(q, np.uint8)
    N, K = q.shape
    out = np.empty((N, K // 32 * 3), dtype=np.uint32)
    _check(_load().oracle_pack3(K, N, _p(q), _p(out)), "oracle_pack3")
    return out


def unpack3(qweight) -> np.ndarray:
    qweight = _arr(qweight, np.uint32)
    N, W = qweight.shape
    K = W // 3 * 32
    out = np.empty((N, K), dtype=np.uint8)
    _check(_load().oracle_unpack3(K, N, _p(qweight), _p(out)), "oracle_unpack3")
    return out


def _qsz3(qweight, s, z, g):
    qweight = _arr(qweight, np.uint32)
    N, W = qweight.shape
    K = W // 3 * 32
    return qweight, _arr(s, np.uint16, (N, K // g)), _arr(z, np.uint16, (N, K // g)), N, K


def dequantize_exact3(qweight, s, z, g: int) -> np.ndarray:
    qweight, s, z, N, K = _qsz3(qweight, s, z, g)
    out = np.empty((N, K), dtype=np.float64)
    _check(_load().oracle_dequantize_exact_bits(K, N, g, 3, _p(qweight), _p(s), _p(z), _p(out)),
           "oracle_dequantize_exact_bits")
    return out


def dequantize3(qweight, s, z, g: int) -> np.ndarray:
    qweight, s, z, N, K = _qsz3(qweight, s, z, g)
    out = np.empty((N, K), dtype=np.uint16)
    _check(_load().oracle_dequantize_bits(K, N, g, 3, _p(qweight), _p(s), _p(z), _p(out)),
           "oracle_dequantize_bits")
    return out


def forward3(qweight, s, z, g: int, x_bits, threads: int = 1):
    qweight, s, z, N, K = _qsz3(qweight, s, z, g)
    x_bits = _arr(x_bits, np.uint16)
    M = x_bits.shape[0]
    if x_bits.shape != (M, K):
        raise ValueError("x must be [M][K]")
    y = np.zeros((M, N), dtype=np.float64)
    used = _check(_load().oracle_forward_bits(K, N, g, 3, M, _p(qweight), _p(s), _p(z), _p(x_bits), _p(y),
                                              int(threads)), "oracle_forward_bits")
    return y, used


def rmsnorm(x_bits, gamma_bits, eps: float) -> np.ndarray:
    """bf16 [M][K], bf16 [K] -> bf16 [M][K]: x * gamma / sqrt(mean(x^2) + eps), one rounding at the end."""
    x_bits = _arr(x_bits, np.uint16)
    gamma_bits = _arr(gamma_bits, np.uint16)
    M, K = x_bits.shape
    if gamma_bits.shape != (K,):
        raise ValueError("gamma must be [K]")
    out = np.empty((M, K), dtype=np.uint16)
    _check(_load().oracle_rmsnorm(M, K, _p(x_bits), _p(gamma_bits), float(eps), _p(out)), "oracle_rmsnorm")
    return out


def swiglu(in_bits) -> np.ndarray:
    """bf16 [M][2I] (gate half, then up half) -> bf16 [M][I]: silu(gate) * up, one rounding at the end."""
    in_bits = _arr(in_bits, np.uint16)
    M, two_i = in_bits.shape
    if two_i % 2:
        raise ValueError("the last axis holds a gate half and an up half")
    out = np.empty((M, two_i // 2), dtype=np.uint16)
    _check(_load().oracle_swiglu(M, two_i // 2, _p(in_bits), _p(out)), "oracle_swiglu")
    return out
