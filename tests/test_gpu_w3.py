"""GPU parity of the 3-bit (W3A16 group-128) variant against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2602_02711_amd as dmr
from oracle import cpu_oracle as orc
from paper_2602_02711_amd import synth

from gpu_util import bf16_dev, bits_host, half_ulp_bf16, rel_err, u32_dev, quantized3

pytestmark = pytest.mark.gpu
G = synth.GROUP
TOL = 1e-2
THREADS = 16


def make_layer3(words, s, z):
    return dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)


@pytest.mark.parametrize("K,N", [(128, 16), (384, 48), (1920, 272), (4096, 4096)])
def test_w3_retile_then_dequantize_is_bit_exact(K, N):
    _, words, s, z = quantized3(7000 + K + N, N, K)
    got = bits_host(dmr.dmr_qlinear_dequantize(make_layer3(words, s, z)))
    assert np.array_equal(got, orc.dequantize3(words, s, z, G))


def test_w3_dequantize_all_codes_all_zero_points():
    N, K = 64, 256
    q = ((np.arange(K)[None, :] * 5 + 3 * np.arange(N)[:, None]) % 8).astype(np.uint8)
    words = orc.pack3(q)
    z = orc.f64_to_bf16(np.repeat((np.arange(N) % 8)[:, None], K // G, axis=1).astype(np.float64))
    s = synth.to_bf16_bits(np.abs(synth.weights_f32(5, N, K // G)) + np.float32(1e-3))
    got = bits_host(dmr.dmr_qlinear_dequantize(make_layer3(words, s, z)))
    assert np.array_equal(got, orc.dequantize3(words, s, z, G))


@pytest.mark.parametrize("K,N", [(1024, 1024), (384, 48), (4096, 6144)])
def test_w3_device_quantiser_matches_oracle_bit_for_bit(K, N):
    w = synth.weights_f32(7100 + K + N, N, K)
    if K == 384:
        w[0, :128] = 0.0
        w[1, :128] = np.abs(w[1, :128])
        w[2, 128:256] = -np.abs(w[2, 128:256])
    qw, s, z = dmr.dmr_qlinear_quantize_w3(torch.from_numpy(w).to("cuda:0"), G)
    torch.cuda.synchronize()
    q_ref, s_ref, z_ref = orc.quantize_bits(w, G, 3)
    assert np.array_equal(bits_host(s), s_ref)
    assert np.array_equal(bits_host(z), z_ref)
    assert np.array_equal(qw.cpu().numpy().view(np.uint32), orc.pack3(q_ref))


@pytest.mark.parametrize("K,N,M", [(1024, 1024, 1), (128, 16, 1), (384, 48, 1), (1920, 272, 1), (4096, 28672, 1),
                                   (14336, 4096, 1), (4096, 6144, 1), (1024, 1024, 5), (384, 48, 64),
                                   (1024, 400, 300), (384, 48, 2), (1920, 272, 7), (4096, 4112, 16), (4096, 28672, 8),
                                   (256, 4112, 3), (14336, 528, 4), (14336, 528, 12),
                                   # rollout batches beyond 16 rows: the register-unpack kernel with and without a split of K,
                                   # one and two weight tiles per wave, 1..4 row tiles, 8-wave workgroups above 64 rows
                                   (4096, 4096, 64), (14336, 4096, 40), (4096, 28672, 20), (2048, 1040, 128),
                                   (512, 4096, 200), (1024, 2064, 130), (640, 80, 17), (4096, 6144, 33),
                                   # wide layers at 17..64 rows: the wide-layer kernel (2, 3 and 4 row tiles, ragged last workgroup)
                                   (512, 16400, 24), (512, 16448, 40), (1024, 16384, 64)])
def test_w3_forward(K, N, M):
    _, words, s, z = quantized3(7200 + K + N, N, K)
    x = synth.activations_bf16(7201 + K + M, M, K)
    layer = make_layer3(words, s, z)
    xd = bf16_dev(x)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32)
    y16 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    y32, y16 = y32.cpu().numpy(), bits_host(y16)
    y_ref, _ = orc.forward3(words, s, z, G, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"w3 K={K} N={N} M={M}: max err {err:.3e} rms")
    assert err <= TOL
    assert np.array_equal(y16, orc.f32_to_bf16(y32))
    rms = np.sqrt(np.mean(y_ref ** 2))
    assert np.all(np.abs(orc.bf16_to_f64(y16) - y_ref) <= TOL * rms + half_ulp_bf16(y_ref))


def test_w3_one_hot_and_exact_cases():
    rng = np.random.default_rng(80)
    K, N = 512, 96
    _, words, s, z = quantized3(7300, N, K)
    layer = make_layer3(words, s, z)
    # M = 1 one-hot activations reproduce single dequantised weights bit for bit
    wq = orc.dequantize3(words, s, z, G)
    for k in (0, 31, 32, 127, 128, 300, 511):
        x = np.zeros((1, K))
        x[0, k] = 1.0
        y16 = bits_host(dmr.dmr_qlinear_forward(layer, bf16_dev(orc.f64_to_bf16(x)), out_dtype=torch.bfloat16))
        assert np.array_equal(y16[0], wq[:, k]), k
    # power-of-two scales and small-integer activations: exact in any summation order
    q = rng.integers(0, 8, size=(N, K), dtype=np.uint8)
    s2 = orc.f64_to_bf16(2.0 ** rng.integers(-4, 3, size=(N, K // G)).astype(np.float64))
    z2 = orc.f64_to_bf16(rng.integers(0, 8, size=(N, K // G)).astype(np.float64))
    words2 = orc.pack3(q)
    layer2 = make_layer3(words2, s2, z2)
    for M in (1, 9):
        x = orc.f64_to_bf16(rng.integers(-8, 9, size=(M, K)).astype(np.float64))
        y32 = dmr.dmr_qlinear_forward(layer2, bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
        y_ref, _ = orc.forward3(words2, s2, z2, G, x)
        assert np.array_equal(y32.astype(np.float64), y_ref), M


# ------------------------------------------------------------------ per-channel symmetric W4 (g = K, z = 8)

@pytest.mark.parametrize("K,N,M", [(1024, 1024, 1), (384, 48, 7), (4096, 4096, 1), (1920, 272, 33), (512, 256, 200),
                                   (512, 1024, 6400),      # large enough for the tiled GEMM
                                   # one case per kernel class that reads the row's single scale word: streaming (2..16),
                                   # k-sliced panels, wide-layer, its variant for odd group counts, rollout batch with K
                                   # split, and the direct-from-L2 kernel that very long decode rows fall back to
                                   (4096, 4096, 16), (14336, 528, 8), (512, 16400, 24), (640, 16400, 40), (2048, 1024, 64),
                                   (32768, 64, 1), (4096, 28672, 1)])
def test_per_channel_symmetric_layer(K, N, M):
    rng = np.random.default_rng(90 + K + M)
    q = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    s_row = synth.to_bf16_bits(np.abs(synth.weights_f32(91 + K, N, 1)) + np.float32(2e-3))       # [N][1]
    z_row = orc.f64_to_bf16(np.full((N, 1), 8.0))
    words = orc.pack(q)
    layer = dmr.dmr_qlinear_create_per_channel(u32_dev(words), bf16_dev(s_row.reshape(N)))
    assert layer.g == K
    # half a byte per weight and one scale word per row, nothing per group
    assert dmr.dmr_qlinear_per_channel_storage_bytes(K, N) == N * K // 2 + 4 * N
    assert layer.storage.numel() == max(N * K // 2 + 4 * N, 16)
    # the oracle takes any group size that divides K: one group per row, zero point 8
    assert np.array_equal(bits_host(dmr.dmr_qlinear_dequantize(layer)), orc.dequantize(words, s_row, z_row, K))
    x = synth.activations_bf16(92 + K, M, K)
    y32 = dmr.dmr_qlinear_forward(layer, bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward(words, s_row, z_row, K, x, threads=THREADS)
    assert rel_err(y32, y_ref) <= TOL
