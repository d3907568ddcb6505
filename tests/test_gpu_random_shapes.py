"""GPU parity on seeded random shapes: every (K, N, M) drawn here goes through whatever kernel the
dispatch picks for it (GEMV, streaming, panel, rollout-batch, tiled GEMMs, for all three formats and the
bf16 twin) and is compared with the CPU oracle element by element, to the same bar as the fixed cases:
max|y - y_ref| <= 1e-2 rms(y_ref) on the fp32 output, the bf16 output the RNE rounding of that
accumulator.  The point is the boundaries between kernels (row counts, ragged last tiles, odd group
counts) that the hand-picked cases may not sit on."""
import numpy as np
import pytest
import torch

import paper_2602_02711_amd as dmr
from oracle import cpu_oracle as orc
from paper_2602_02711_amd import synth

from gpu_util import bf16_dev, bits_host, quantized, quantized3, rel_err, u32_dev

pytestmark = pytest.mark.gpu
G = synth.GROUP
TOL = 1e-2
THREADS = 16


def draw_cases(seed, count, max_macs):
    rng = np.random.default_rng(seed)
    m_choices = [1, 2, 3, 5, 8, 9, 15, 16, 17, 24, 31, 32, 33, 47, 48, 49, 63, 64, 65, 96, 127, 128, 129, 200, 257, 384, 511]
    cases = []
    while len(cases) < count:
        K = G * int(rng.integers(1, 41))
        N = 16 * int(rng.integers(1, 301))
        if rng.random() < 0.3:
            N = 16 * int(rng.integers(1024, 1100))          # wide layers: >= 1024 row tiles
        M = int(rng.choice(m_choices))
        if M * K * N <= max_macs:
            cases.append((K, N, M))
    return cases


CASES4 = draw_cases(2602_02711, 40, 6e8)
CASES3 = draw_cases(2602_02712, 16, 3e8)
CASESB = draw_cases(2602_02713, 24, 6e8)


@pytest.mark.parametrize("K,N,M", CASES4)
def test_random_shapes_int4(K, N, M):
    _, words, s, z = quantized(9000 + K + N + M, N, K)
    x = synth.activations_bf16(9001 + K + N + M, M, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    xd = bf16_dev(x)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.bfloat16))
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"int4 ({K},{N}) M={M}: max err {err:.3e} rms")
    assert err <= TOL
    assert np.array_equal(y16, orc.f32_to_bf16(y32))


@pytest.mark.parametrize("K,N,M", CASES3)
def test_random_shapes_w3(K, N, M):
    _, words, s, z = quantized3(9100 + K + N + M, N, K)
    x = synth.activations_bf16(9101 + K + N + M, M, K)
    layer = dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    xd = bf16_dev(x)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.bfloat16))
    y_ref, _ = orc.forward3(words, s, z, G, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"w3 ({K},{N}) M={M}: max err {err:.3e} rms")
    assert err <= TOL
    assert np.array_equal(y16, orc.f32_to_bf16(y32))


@pytest.mark.parametrize("K,N,M", CASESB)
def test_random_shapes_bf16(K, N, M):
    w = synth.to_bf16_bits(synth.weights_f32(9200 + K + N + M, N, K))
    x = synth.activations_bf16(9201 + K + N + M, M, K)
    wd, xd = bf16_dev(w), bf16_dev(x)
    y32 = dmr.dmr_qlinear_bf16_forward(wd, xd, out_dtype=torch.float32).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_bf16_forward(wd, xd, out_dtype=torch.bfloat16))
    y_ref, _ = orc.bf16_forward(w, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"bf16 ({K},{N}) M={M}: max err {err:.3e} rms")
    assert err <= TOL
    assert np.array_equal(y16, orc.f32_to_bf16(y32))
