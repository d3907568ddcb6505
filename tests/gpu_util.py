"""Helpers of the GPU parity tests: move seeded numpy inputs to the device and results back."""
import numpy as np
import torch

from oracle import cpu_oracle as orc
from paper_2602_02711_amd import synth

DEV = "cuda:0"


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def u32_dev(words: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int32)).to(DEV)


def bits_host(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def quantized(seed: int, N: int, K: int, g: int = synth.GROUP):
    """Seeded fp32 weights quantised by the ORACLE: (w, words, s_bits, z_bits)."""
    w = synth.weights_f32(seed, N, K)
    q, s, z = orc.quantize(w, g)
    return w, orc.pack(q), s, z


def quantized3(seed: int, N: int, K: int, g: int = synth.GROUP):
    """The 3-bit variant: seeded fp32 weights quantised by the ORACLE: (w, words3, s_bits, z_bits)."""
    w = synth.weights_f32(seed, N, K)
    q, s, z = orc.quantize_bits(w, g, 3)
    return w, orc.pack3(q), s, z


def half_ulp_bf16(values: np.ndarray) -> np.ndarray:
    a = np.abs(values)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return 2.0 ** (e - 8)


def rel_err(y: np.ndarray, y_ref: np.ndarray) -> float:
    return float(np.max(np.abs(y.astype(np.float64) - y_ref)) / np.sqrt(np.mean(y_ref ** 2)))
