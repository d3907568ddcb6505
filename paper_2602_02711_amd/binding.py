"""Python binding of ``include/dmr_qlinear.h``: argument marshalling only.

Every function has the name and meaning of the C entry point it calls; tensors are torch
tensors used as device memory (PyTorch supplies allocation and streams, nothing else) and all
arithmetic happens in the HIP kernels of ``libdmr_qlinear.so``.  There is no fallback: if the
library is missing or a call is refused, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdmr_qlinear.so")

DMR_OK = 0
DMR_ERR_NULL, DMR_ERR_SHAPE, DMR_ERR_ALIGN, DMR_ERR_WORKSPACE, DMR_ERR_UNSUPPORTED, DMR_ERR_HIP = range(1, 7)
DMR_OUT_BF16, DMR_OUT_FP32 = 0, 1

EXPORTS = (
    "dmr_qlinear_storage_bytes", "dmr_qlinear_workspace_bytes", "dmr_qlinear_bf16_workspace_bytes",
    "dmr_qlinear_create",
    "dmr_qlinear_dequantize", "dmr_qlinear_forward", "dmr_qlinear_bf16_forward",
    "dmr_qlinear_quantize", "dmr_qlinear_destroy", "dmr_qlinear_shape", "dmr_status_string",
    "dmr_probe_hbm_read", "dmr_qlinear_w3_storage_bytes", "dmr_qlinear_w3_workspace_bytes",
    "dmr_qlinear_w3_create", "dmr_qlinear_quantize_w3", "dmr_qlinear_bits", "dmr_qlinear_create_per_channel",
    "dmr_glue_rmsnorm", "dmr_glue_swiglu", "dmr_qlinear_fused_workspace_bytes",
    "dmr_qlinear_bf16_fused_workspace_bytes", "dmr_qlinear_forward_fused", "dmr_qlinear_bf16_forward_fused",
    "dmr_qlinear_kernel_path", "dmr_qlinear_forward_static", "dmr_probe_empty_launch",
    "dmr_qlinear_per_channel_storage_bytes",
)

DMR_PRO_NONE, DMR_PRO_RMSNORM, DMR_PRO_SWIGLU = 0, 1, 2
DMR_FMT_W4_G128, DMR_FMT_W4_PER_CHANNEL, DMR_FMT_W3_G128, DMR_FMT_BF16 = 0, 1, 2, 3


class DmrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        text = lib().dmr_status_string(status).decode()
        super().__init__(f"{where}: {text} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library, with prototypes set.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
        L.dmr_qlinear_storage_bytes.restype = sz
        L.dmr_qlinear_storage_bytes.argtypes = [i64, i64, i32]
        L.dmr_qlinear_workspace_bytes.restype = sz
        L.dmr_qlinear_workspace_bytes.argtypes = [i64, i64, i64]
        L.dmr_qlinear_bf16_workspace_bytes.restype = sz
        L.dmr_qlinear_bf16_workspace_bytes.argtypes = [i64, i64, i64]
        L.dmr_qlinear_create.restype = ctypes.c_int
        L.dmr_qlinear_create.argtypes = [ctypes.POINTER(vp), i64, i64, i32, vp, vp, vp, vp, sz, vp]
        L.dmr_qlinear_dequantize.restype = ctypes.c_int
        L.dmr_qlinear_dequantize.argtypes = [vp, vp, vp]
        L.dmr_qlinear_forward.restype = ctypes.c_int
        L.dmr_qlinear_forward.argtypes = [vp, vp, i64, vp, ctypes.c_int, vp, sz, vp]
        L.dmr_qlinear_forward_static.restype = ctypes.c_int
        L.dmr_qlinear_forward_static.argtypes = [vp, vp, i64, vp, ctypes.c_int, vp]
        L.dmr_qlinear_bf16_forward.restype = ctypes.c_int
        L.dmr_qlinear_bf16_forward.argtypes = [vp, vp, i64, i64, i64, vp, ctypes.c_int, vp, sz, vp]
        L.dmr_qlinear_quantize.restype = ctypes.c_int
        L.dmr_qlinear_quantize.argtypes = [i64, i64, i32, vp, vp, vp, vp, vp]
        L.dmr_qlinear_destroy.restype = None
        L.dmr_qlinear_destroy.argtypes = [vp]
        L.dmr_qlinear_shape.restype = ctypes.c_int
        L.dmr_qlinear_shape.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.dmr_qlinear_w3_storage_bytes.restype = sz
        L.dmr_qlinear_w3_storage_bytes.argtypes = [i64, i64, i32]
        L.dmr_qlinear_w3_workspace_bytes.restype = sz
        L.dmr_qlinear_w3_workspace_bytes.argtypes = [i64, i64, i64]
        L.dmr_qlinear_w3_create.restype = ctypes.c_int
        L.dmr_qlinear_w3_create.argtypes = [ctypes.POINTER(vp), i64, i64, i32, vp, vp, vp, vp, sz, vp]
        L.dmr_qlinear_quantize_w3.restype = ctypes.c_int
        L.dmr_qlinear_quantize_w3.argtypes = [i64, i64, i32, vp, vp, vp, vp, vp]
        L.dmr_qlinear_per_channel_storage_bytes.restype = sz
        L.dmr_qlinear_per_channel_storage_bytes.argtypes = [i64, i64]
        L.dmr_qlinear_create_per_channel.restype = ctypes.c_int
        L.dmr_qlinear_create_per_channel.argtypes = [ctypes.POINTER(vp), i64, i64, vp, vp, vp, sz, vp]
        L.dmr_qlinear_bits.restype = i32
        L.dmr_qlinear_bits.argtypes = [vp]
        L.dmr_probe_empty_launch.restype = ctypes.c_int
        L.dmr_probe_empty_launch.argtypes = [i32, i32, sz, vp]
        L.dmr_probe_hbm_read.restype = ctypes.c_int
        L.dmr_probe_hbm_read.argtypes = [vp, sz, vp, i32, vp]
        f32 = ctypes.c_float
        L.dmr_glue_rmsnorm.restype = ctypes.c_int
        L.dmr_glue_rmsnorm.argtypes = [vp, vp, f32, i64, i64, vp, vp]
        L.dmr_glue_swiglu.restype = ctypes.c_int
        L.dmr_glue_swiglu.argtypes = [vp, i64, i64, vp, vp]
        L.dmr_qlinear_fused_workspace_bytes.restype = sz
        L.dmr_qlinear_fused_workspace_bytes.argtypes = [vp, i64, ctypes.c_int, i32]
        L.dmr_qlinear_bf16_fused_workspace_bytes.restype = sz
        L.dmr_qlinear_bf16_fused_workspace_bytes.argtypes = [i64, i64, i64, ctypes.c_int, i32]
        L.dmr_qlinear_forward_fused.restype = ctypes.c_int
        L.dmr_qlinear_forward_fused.argtypes = [vp, ctypes.c_int, vp, vp, f32, vp, i64, vp, ctypes.c_int, vp, sz, vp]
        L.dmr_qlinear_bf16_forward_fused.restype = ctypes.c_int
        L.dmr_qlinear_bf16_forward_fused.argtypes = [vp, ctypes.c_int, vp, vp, f32, vp, i64, i64, i64, vp,
                                                     ctypes.c_int, vp, sz, vp]
        L.dmr_status_string.restype = ctypes.c_char_p
        L.dmr_status_string.argtypes = [ctypes.c_int]
        L.dmr_qlinear_kernel_path.restype = ctypes.c_char_p
        L.dmr_qlinear_kernel_path.argtypes = [ctypes.c_int, i64, i64, i64]
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != DMR_OK:
        raise DmrError(status, where)


def _dev(t: torch.Tensor, name: str, dtypes) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a tensor in device memory")
    if t.dtype not in dtypes:
        raise TypeError(f"{name} has dtype {t.dtype}, expected one of {dtypes}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


_BF16 = (torch.bfloat16, torch.int16, torch.uint16)
_U32 = (torch.int32, torch.uint32)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _out_code(dtype) -> int:
    if dtype == torch.bfloat16:
        return DMR_OUT_BF16
    if dtype == torch.float32:
        return DMR_OUT_FP32
    raise TypeError("output dtype must be torch.bfloat16 or torch.float32")


class Layer:
    """Host handle of one quantised Linear layer plus the storage tensor it points into."""

    def __init__(self, handle: int, storage: torch.Tensor, K: int, N: int, g: int, bits: int = 4):
        self.handle, self.storage, self.K, self.N, self.g, self.bits = handle, storage, K, N, g, bits

    def __del__(self):
        dmr_qlinear_destroy(self)


def dmr_qlinear_storage_bytes(K: int, N: int, g: int = 128) -> int:
    return int(lib().dmr_qlinear_storage_bytes(K, N, g))


def dmr_qlinear_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().dmr_qlinear_workspace_bytes(M, K, N))


def dmr_qlinear_bf16_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().dmr_qlinear_bf16_workspace_bytes(M, K, N))


def dmr_qlinear_create(qweight: torch.Tensor, scales: torch.Tensor, zeros: torch.Tensor, g: int = 128,
                       storage: torch.Tensor | None = None, stream=None) -> Layer:
    pq = _dev(qweight, "qweight", _U32)
    ps = _dev(scales, "scales", _BF16)
    pz = _dev(zeros, "zeros", _BF16)
    N, K8 = qweight.shape
    K = K8 * 8
    if g <= 0 or K % g or tuple(scales.shape) != (N, K // g) or tuple(zeros.shape) != (N, K // g):
        raise ValueError("scales and zeros must be [N][K/g]")
    need = dmr_qlinear_storage_bytes(K, N, g)
    if storage is None:
        storage = torch.empty(max(need, 16), dtype=torch.uint8, device=qweight.device)
    pst = _dev(storage, "storage", (torch.uint8,))
    handle = ctypes.c_void_p()
    _check(lib().dmr_qlinear_create(ctypes.byref(handle), K, N, g, pq, ps, pz, pst, storage.numel(),
                                    _stream(stream)), "dmr_qlinear_create")
    return Layer(handle.value, storage, K, N, g)


def dmr_qlinear_dequantize(layer: Layer, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((layer.N, layer.K), dtype=torch.bfloat16, device=layer.storage.device)
    po = _dev(out, "out", _BF16)
    if tuple(out.shape) != (layer.N, layer.K):
        raise ValueError("out must be [N][K]")
    _check(lib().dmr_qlinear_dequantize(layer.handle, po, _stream(stream)), "dmr_qlinear_dequantize")
    return out


def _workspace(workspace):
    if workspace is None:
        return None, 0
    return _dev(workspace, "workspace", (torch.uint8,)), workspace.numel()


def dmr_qlinear_forward(layer: Layer, x: torch.Tensor, out: torch.Tensor | None = None,
                        out_dtype=torch.bfloat16, workspace: torch.Tensor | None = None,
                        stream=None) -> torch.Tensor:
    px = _dev(x, "x", _BF16)
    if x.dim() != 2 or x.shape[1] != layer.K:
        raise ValueError("x must be [M][K]")
    M = x.shape[0]
    if out is None:
        out = torch.empty((M, layer.N), dtype=out_dtype, device=x.device)
    po = _dev(out, "out", (torch.bfloat16, torch.float32))
    if tuple(out.shape) != (M, layer.N):
        raise ValueError("out must be [M][N]")
    need = (dmr_qlinear_w3_workspace_bytes(M, layer.K, layer.N) if layer.bits == 3
            else dmr_qlinear_workspace_bytes(M, layer.K, layer.N))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)    # device memory only
    pw, wbytes = _workspace(workspace)
    _check(lib().dmr_qlinear_forward(layer.handle, px, M, po, _out_code(out.dtype), pw, wbytes,
                                     _stream(stream)), "dmr_qlinear_forward")
    return out


DMR_STATIC_SCRATCH_BYTES = 8 << 20


def dmr_qlinear_forward_static(layer: Layer, x: torch.Tensor, out: torch.Tensor | None = None,
                               out_dtype=torch.bfloat16, stream=None) -> torch.Tensor:
    """dmr_qlinear_forward on the library's own fixed scratch: no workspace is passed or allocated."""
    px = _dev(x, "x", _BF16)
    if x.dim() != 2 or x.shape[1] != layer.K:
        raise ValueError("x must be [M][K]")
    M = x.shape[0]
    if out is None:
        out = torch.empty((M, layer.N), dtype=out_dtype, device=x.device)
    po = _dev(out, "out", (torch.bfloat16, torch.float32))
    if tuple(out.shape) != (M, layer.N):
        raise ValueError("out must be [M][N]")
    _check(lib().dmr_qlinear_forward_static(layer.handle, px, M, po, _out_code(out.dtype), _stream(stream)),
           "dmr_qlinear_forward_static")
    return out


def dmr_qlinear_bf16_forward(w: torch.Tensor, x: torch.Tensor, out: torch.Tensor | None = None,
                             out_dtype=torch.bfloat16, workspace: torch.Tensor | None = None,
                             stream=None) -> torch.Tensor:
    pw_ = _dev(w, "w", _BF16)
    px = _dev(x, "x", _BF16)
    N, K = w.shape
    if x.dim() != 2 or x.shape[1] != K:
        raise ValueError("x must be [M][K]")
    M = x.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=x.device)
    po = _dev(out, "out", (torch.bfloat16, torch.float32))
    if tuple(out.shape) != (M, N):
        raise ValueError("out must be [M][N]")
    if workspace is None:
        need = dmr_qlinear_bf16_workspace_bytes(M, K, N)
        if need > 0:
            workspace = torch.empty(need, dtype=torch.uint8, device=x.device)    # device memory only
    pws, wbytes = _workspace(workspace)
    _check(lib().dmr_qlinear_bf16_forward(pw_, px, M, K, N, po, _out_code(out.dtype), pws, wbytes,
                                          _stream(stream)), "dmr_qlinear_bf16_forward")
    return out


def dmr_qlinear_quantize(w: torch.Tensor, g: int = 128, stream=None):
    """fp32 [N][K] in device memory -> (qweight int32 [N][K/8], scales bf16, zeros bf16 [N][K/g])."""
    pw_ = _dev(w, "w", (torch.float32,))
    N, K = w.shape
    if g <= 0 or K % g or K % 8:
        raise ValueError("K must be a multiple of g and of 8")
    qweight = torch.empty((N, K // 8), dtype=torch.int32, device=w.device)
    scales = torch.empty((N, K // g), dtype=torch.bfloat16, device=w.device)
    zeros = torch.empty((N, K // g), dtype=torch.bfloat16, device=w.device)
    _check(lib().dmr_qlinear_quantize(K, N, g, pw_, qweight.data_ptr(), scales.data_ptr(),
                                      zeros.data_ptr(), _stream(stream)), "dmr_qlinear_quantize")
    return qweight, scales, zeros


def dmr_qlinear_per_channel_storage_bytes(K: int, N: int) -> int:
    return int(lib().dmr_qlinear_per_channel_storage_bytes(K, N))


def dmr_qlinear_create_per_channel(qweight: torch.Tensor, scales: torch.Tensor,
                                   storage: torch.Tensor | None = None, stream=None) -> Layer:
    """Symmetric per-channel INT4: qweight [N][K/8], one bf16 scale per row, zero point 8."""
    pq = _dev(qweight, "qweight", _U32)
    ps = _dev(scales, "scales", _BF16)
    N, K8 = qweight.shape
    K = K8 * 8
    if scales.numel() != N:
        raise ValueError("scales must hold one value per row")
    need = dmr_qlinear_per_channel_storage_bytes(K, N)
    if storage is None:
        storage = torch.empty(max(need, 16), dtype=torch.uint8, device=qweight.device)
    pst = _dev(storage, "storage", (torch.uint8,))
    handle = ctypes.c_void_p()
    _check(lib().dmr_qlinear_create_per_channel(ctypes.byref(handle), K, N, pq, ps, pst, storage.numel(),
                                                _stream(stream)), "dmr_qlinear_create_per_channel")
    return Layer(handle.value, storage, K, N, K)


def dmr_qlinear_w3_storage_bytes(K: int, N: int, g: int = 128) -> int:
    return int(lib().dmr_qlinear_w3_storage_bytes(K, N, g))


def dmr_qlinear_w3_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().dmr_qlinear_w3_workspace_bytes(M, K, N))


def dmr_qlinear_w3_create(qweight3: torch.Tensor, scales: torch.Tensor, zeros: torch.Tensor, g: int = 128,
                          storage: torch.Tensor | None = None, stream=None) -> Layer:
    pq = _dev(qweight3, "qweight3", _U32)
    ps = _dev(scales, "scales", _BF16)
    pz = _dev(zeros, "zeros", _BF16)
    N, W = qweight3.shape
    if W % 3:
        raise ValueError("qweight3 must be [N][3K/32]")
    K = W // 3 * 32
    if g <= 0 or K % g or tuple(scales.shape) != (N, K // g) or tuple(zeros.shape) != (N, K // g):
        raise ValueError("scales and zeros must be [N][K/g]")
    need = dmr_qlinear_w3_storage_bytes(K, N, g)
    if storage is None:
        storage = torch.empty(max(need, 16), dtype=torch.uint8, device=qweight3.device)
    pst = _dev(storage, "storage", (torch.uint8,))
    handle = ctypes.c_void_p()
    _check(lib().dmr_qlinear_w3_create(ctypes.byref(handle), K, N, g, pq, ps, pz, pst, storage.numel(),
                                       _stream(stream)), "dmr_qlinear_w3_create")
    return Layer(handle.value, storage, K, N, g, bits=3)


def dmr_qlinear_quantize_w3(w: torch.Tensor, g: int = 128, stream=None):
    """fp32 [N][K] in device memory -> (qweight3 int32 [N][3K/32], scales bf16, zeros bf16 [N][K/g])."""
    pw_ = _dev(w, "w", (torch.float32,))
    N, K = w.shape
    if g <= 0 or K % g or K % 32:
        raise ValueError("K must be a multiple of g and of 32")
    qweight = torch.empty((N, K // 32 * 3), dtype=torch.int32, device=w.device)
    scales = torch.empty((N, K // g), dtype=torch.bfloat16, device=w.device)
    zeros = torch.empty((N, K // g), dtype=torch.bfloat16, device=w.device)
    _check(lib().dmr_qlinear_quantize_w3(K, N, g, pw_, qweight.data_ptr(), scales.data_ptr(),
                                         zeros.data_ptr(), _stream(stream)), "dmr_qlinear_quantize_w3")
    return qweight, scales, zeros


def dmr_probe_hbm_read(buf: torch.Tensor, sink: torch.Tensor, blocks: int, stream=None) -> None:
    pb = _dev(buf, "buf", (torch.uint8,))
    ps = _dev(sink, "sink", (torch.int32, torch.uint32))
    if sink.numel() < blocks * 256:
        raise ValueError("sink needs blocks * 256 words")
    _check(lib().dmr_probe_hbm_read(pb, buf.numel(), ps, blocks, _stream(stream)), "dmr_probe_hbm_read")


def dmr_probe_empty_launch(blocks: int, threads: int, lds_bytes: int = 0, stream=None) -> None:
    _check(lib().dmr_probe_empty_launch(blocks, threads, lds_bytes, _stream(stream)), "dmr_probe_empty_launch")


def dmr_qlinear_kernel_path(fmt: int, M: int, K: int, N: int) -> str:
    return lib().dmr_qlinear_kernel_path(fmt, M, K, N).decode()


def dmr_qlinear_destroy(layer: Layer) -> None:
    handle, layer.handle = getattr(layer, "handle", None), None
    if handle and _lib is not None:
        _lib.dmr_qlinear_destroy(handle)


# ---- decoder glue and fused forwards -------------------------------------------------------------

def dmr_glue_rmsnorm(x: torch.Tensor, gamma: torch.Tensor, eps: float, out: torch.Tensor | None = None,
                     stream=None) -> torch.Tensor:
    px, pg = _dev(x, "x", _BF16), _dev(gamma, "gamma", _BF16)
    M, K = x.shape
    if tuple(gamma.shape) != (K,):
        raise ValueError("gamma must be [K]")
    if out is None:
        out = torch.empty((M, K), dtype=torch.bfloat16, device=x.device)
    po = _dev(out, "out", _BF16)
    _check(lib().dmr_glue_rmsnorm(px, pg, float(eps), M, K, po, _stream(stream)), "dmr_glue_rmsnorm")
    return out


def dmr_glue_swiglu(gate_up: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    pi = _dev(gate_up, "gate_up", _BF16)
    M, two_i = gate_up.shape
    if two_i % 2:
        raise ValueError("gate_up must be [M][2 I]")
    if out is None:
        out = torch.empty((M, two_i // 2), dtype=torch.bfloat16, device=gate_up.device)
    po = _dev(out, "out", _BF16)
    _check(lib().dmr_glue_swiglu(pi, M, two_i // 2, po, _stream(stream)), "dmr_glue_swiglu")
    return out


def _fused_args(pro, inp, gamma, residual, K, N):
    pi = _dev(inp, "inp", _BF16)
    want = 2 * K if pro == DMR_PRO_SWIGLU else K
    if inp.dim() != 2 or inp.shape[1] != want:
        raise ValueError(f"inp must be [M][{want}]")
    M = inp.shape[0]
    pg = None
    if pro == DMR_PRO_RMSNORM:
        pg = _dev(gamma, "gamma", _BF16)
        if tuple(gamma.shape) != (K,):
            raise ValueError("gamma must be [K]")
    pr = None
    if residual is not None:
        pr = _dev(residual, "residual", _BF16)
        if tuple(residual.shape) != (M, N):
            raise ValueError("residual must be [M][N]")
    return pi, pg, pr, M


def dmr_qlinear_forward_fused(layer: Layer, pro: int, inp: torch.Tensor, gamma: torch.Tensor | None = None,
                              eps: float = 0.0, residual: torch.Tensor | None = None,
                              out: torch.Tensor | None = None, out_dtype=torch.bfloat16,
                              workspace: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    pi, pg, pr, M = _fused_args(pro, inp, gamma, residual, layer.K, layer.N)
    if out is None:
        out = torch.empty((M, layer.N), dtype=out_dtype, device=inp.device)
    po = _dev(out, "out", (torch.bfloat16, torch.float32))
    if tuple(out.shape) != (M, layer.N):
        raise ValueError("out must be [M][N]")
    if workspace is None:
        need = int(lib().dmr_qlinear_fused_workspace_bytes(layer.handle, M, pro, 1 if residual is not None else 0))
        if need > 0:
            workspace = torch.empty(need, dtype=torch.uint8, device=inp.device)    # device memory only
    pw, wbytes = _workspace(workspace)
    _check(lib().dmr_qlinear_forward_fused(layer.handle, pro, pi, pg, float(eps), pr, M, po, _out_code(out.dtype),
                                           pw, wbytes, _stream(stream)), "dmr_qlinear_forward_fused")
    return out


def dmr_qlinear_bf16_forward_fused(w: torch.Tensor, pro: int, inp: torch.Tensor, gamma: torch.Tensor | None = None,
                                   eps: float = 0.0, residual: torch.Tensor | None = None,
                                   out: torch.Tensor | None = None, out_dtype=torch.bfloat16,
                                   workspace: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    pw_ = _dev(w, "w", _BF16)
    N, K = w.shape
    pi, pg, pr, M = _fused_args(pro, inp, gamma, residual, K, N)
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=inp.device)
    po = _dev(out, "out", (torch.bfloat16, torch.float32))
    if tuple(out.shape) != (M, N):
        raise ValueError("out must be [M][N]")
    if workspace is None:
        need = int(lib().dmr_qlinear_bf16_fused_workspace_bytes(M, K, N, pro, 1 if residual is not None else 0))
        if need > 0:
            workspace = torch.empty(need, dtype=torch.uint8, device=inp.device)    # device memory only
    pws, wbytes = _workspace(workspace)
    _check(lib().dmr_qlinear_bf16_forward_fused(pw_, pro, pi, pg, float(eps), pr, M, K, N, po, _out_code(out.dtype),
                                                pws, wbytes, _stream(stream)), "dmr_qlinear_bf16_forward_fused")
    return out
