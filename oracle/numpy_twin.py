"""Second, independent statement of the oracle's definitions in numpy, for tiny shapes.

TEST INFRASTRUCTURE ONLY.  It exists so that the C oracle can be checked against something
that was written separately from it (different language, vectorised integer shifts instead of
loops, a bit-trick bf16 rounding instead of the frexp/nearbyint one, ``einsum`` instead of a
triple loop).  It imports neither the C oracle nor the GPU binding.

Definitions restated (format reading of the paper's W4A16 low-precision copy, Sec. 5.1 and
App. E): code j of word i of row n is weight k = 8i + j; w^ = (q - z) * s per group of g along
k; dequantize = RNE_bf16(w^); forward = x . w^T in fp64.
"""
import numpy as np


def bf16_bits_to_f64(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(values):
    """RNE fp32 -> bf16 by the add-half-and-truncate trick on the bit pattern (finite inputs)."""
    u = np.ascontiguousarray(values, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def f64_to_bf16_bits(values):
    """RNE fp64 -> bf16 in one step (normal range): scale so that one bf16 ulp is 1, rint, scale back."""
    v = np.asarray(values, dtype=np.float64)
    out = np.zeros(v.shape, dtype=np.float64)
    nz = v != 0
    e = np.floor(np.log2(np.abs(v[nz])))
    ulp = np.exp2(e - 7)
    out[nz] = np.rint(v[nz] / ulp) * ulp          # both scalings are exact (powers of two)
    return (out.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def unpack(qweight):
    qweight = np.asarray(qweight, dtype=np.uint32)
    shifts = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    return ((qweight[:, :, None] >> shifts) & 0xF).astype(np.uint8).reshape(qweight.shape[0], -1)


def pack(q):
    q = np.asarray(q, dtype=np.uint32).reshape(q.shape[0], -1, 8)
    shifts = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    return np.bitwise_or.reduce(q << shifts, axis=2).astype(np.uint32)


def dequantize_exact(qweight, s_bits, z_bits, g):
    q = unpack(qweight).astype(np.float64)
    s = np.repeat(bf16_bits_to_f64(s_bits), g, axis=1)
    z = np.repeat(bf16_bits_to_f64(z_bits), g, axis=1)
    return (q - z) * s


def dequantize(qweight, s_bits, z_bits, g):
    w = dequantize_exact(qweight, s_bits, z_bits, g)
    w32 = w.astype(np.float32)
    assert np.array_equal(w32.astype(np.float64), w), "w^ must be exact in fp32"
    return f32_to_bf16_bits(w32)


def forward(qweight, s_bits, z_bits, g, x_bits):
    return np.einsum("mk,nk->mn", bf16_bits_to_f64(x_bits), dequantize_exact(qweight, s_bits, z_bits, g))


def forward_group_sums(qweight, s_bits, z_bits, g, x_bits):
    """Same product regrouped as sum_G s_G (sum_{k in G} x_k q_k - z_G sum_{k in G} x_k)."""
    q = unpack(qweight).astype(np.float64)
    x = bf16_bits_to_f64(x_bits)
    N, K = q.shape
    M = x.shape[0]
    qg = q.reshape(N, K // g, g)
    xg = x.reshape(M, K // g, g)
    D = np.einsum("mGi,nGi->mnG", xg, qg)
    X = xg.sum(axis=2)
    s = bf16_bits_to_f64(s_bits)
    z = bf16_bits_to_f64(z_bits)
    return np.einsum("nG,mnG->mn", s, D - z[None, :, :] * X[:, None, :])


def bf16_forward(w_bits, x_bits):
    return np.einsum("mk,nk->mn", bf16_bits_to_f64(x_bits), bf16_bits_to_f64(w_bits))


# ---- 3-bit variant, written independently of the C code: the row is one little-endian bit stream


def unpack3(qweight):
    qweight = np.ascontiguousarray(qweight, dtype="<u4")
    N = qweight.shape[0]
    bits = np.unpackbits(qweight.view(np.uint8).reshape(N, -1), axis=1, bitorder="little")
    fields = bits.reshape(N, -1, 3).astype(np.uint8)
    return fields[:, :, 0] | (fields[:, :, 1] << 1) | (fields[:, :, 2] << 2)


def pack3(q):
    q = np.asarray(q, dtype=np.uint8)
    N = q.shape[0]
    bits = np.stack([(q >> b) & 1 for b in range(3)], axis=2).reshape(N, -1)
    return np.packbits(bits, axis=1, bitorder="little").view("<u4").reshape(N, -1)


def dequantize_exact3(qweight, s_bits, z_bits, g):
    q = unpack3(qweight).astype(np.float64)
    s = np.repeat(bf16_bits_to_f64(s_bits), g, axis=1)
    z = np.repeat(bf16_bits_to_f64(z_bits), g, axis=1)
    return (q - z) * s


def forward3(qweight, s_bits, z_bits, g, x_bits):
    return np.einsum("mk,nk->mn", bf16_bits_to_f64(x_bits), dequantize_exact3(qweight, s_bits, z_bits, g))


def rmsnorm(x_bits, gamma_bits, eps):
    x = bf16_bits_to_f64(x_bits)
    rms = np.sqrt((x * x).mean(axis=1, keepdims=True) + eps)
    with np.errstate(invalid="ignore", divide="ignore"):
        y = np.where(rms > 0, x * bf16_bits_to_f64(gamma_bits)[None, :] / rms, 0.0)
    return f64_to_bf16_bits(y)


def swiglu(in_bits):
    v = bf16_bits_to_f64(in_bits)
    half = v.shape[1] // 2
    gate, up = v[:, :half], v[:, half:]
    return f64_to_bf16_bits(gate / (1.0 + np.exp(-gate)) * up)
