"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer / bit work (re-tiling, dequantize, quantise, exact special cases) is compared
bit for bit; floating-point forwards within max|y - y_ref| <= 1e-2 rms(y_ref) on the fp32 output
(the bound concerns fp32 accumulation), and the bf16 output must be the RNE rounding of that same
accumulator (its own half-ulp can exceed 1e-2 rms for |y| >= 4, so it gets that half-ulp added).
"""
import numpy as np
import pytest
import torch

import paper_2602_02711_amd as dmr
from oracle import cpu_oracle as orc
from paper_2602_02711_amd import synth

from gpu_util import bf16_dev, bits_host, half_ulp_bf16, quantized, rel_err, u32_dev

pytestmark = pytest.mark.gpu
G = synth.GROUP
TOL = 1e-2
THREADS = 16


def make_layer(words, s, z):
    return dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)


def forward_both(layer, x_bits):
    xd = bf16_dev(x_bits)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32)
    y16 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    return y32.cpu().numpy(), bits_host(y16)


def check_forward(y32, y16_bits, y_ref, where):
    err = rel_err(y32, y_ref)
    print(f"{where}: max err {err:.3e} rms")
    assert err <= TOL, where
    # bf16 output: the rounding of the same accumulator, bit for bit
    assert np.array_equal(y16_bits, orc.f32_to_bf16(y32)), where
    rms = np.sqrt(np.mean(y_ref ** 2))
    y16 = orc.bf16_to_f64(y16_bits)
    assert np.all(np.abs(y16 - y_ref) <= TOL * rms + half_ulp_bf16(y_ref)), where


# ------------------------------------------------------------------ layout, bit-exact

@pytest.mark.parametrize("K,N", [(1024, 1024), (128, 16), (384, 48), (1920, 272), (4096, 4096)])
def test_retile_then_dequantize_is_bit_exact(K, N):
    _, words, s, z = quantized(1000 + K + N, N, K)
    layer = make_layer(words, s, z)
    got = bits_host(dmr.dmr_qlinear_dequantize(layer))
    assert np.array_equal(got, orc.dequantize(words, s, z, G))


def test_dequantize_all_codes_all_zero_points():
    # every (q, z) pair appears: rows use z = row % 16, codes cycle along k
    N, K = 64, 256
    q = (np.arange(K)[None, :] + 3 * np.arange(N)[:, None]) % 16
    words = orc.pack(q.astype(np.uint8))
    z = orc.f64_to_bf16(np.repeat((np.arange(N) % 16)[:, None], K // G, axis=1).astype(np.float64))
    s = synth.to_bf16_bits(np.abs(synth.weights_f32(5, N, K // G)) + np.float32(1e-3))
    got = bits_host(dmr.dmr_qlinear_dequantize(make_layer(words, s, z)))
    assert np.array_equal(got, orc.dequantize(words, s, z, G))


@pytest.mark.parametrize("K,N", [(1024, 1024), (384, 48), (4096, 6144)])
def test_device_quantiser_matches_oracle_bit_for_bit(K, N):
    w = synth.weights_f32(2000 + K + N, N, K)
    if K == 384:
        w[0, :128] = 0.0           # all-zero group -> s = 1
        w[1, :128] = np.abs(w[1, :128])        # all-positive group -> z = 0
        w[2, 128:256] = -np.abs(w[2, 128:256])  # all-negative group -> z = 15
    qw, s, z = dmr.dmr_qlinear_quantize(torch.from_numpy(w).to("cuda:0"), G)
    torch.cuda.synchronize()
    q_ref, s_ref, z_ref = orc.quantize(w, G)
    assert np.array_equal(bits_host(s), s_ref)
    assert np.array_equal(bits_host(z), z_ref)
    assert np.array_equal(qw.cpu().numpy().view(np.uint32), orc.pack(q_ref))


# ------------------------------------------------------------------ decode / skinny forward

@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 48, 49, 63, 64])
def test_forward_small_shape_all_skinny_m(M):
    _, K, N = synth.SMALL_SHAPE
    _, words, s, z = quantized(synth.seed_for(0, 0, 0), N, K)
    x = synth.activations_bf16(synth.seed_for(0, 0, 1) + M, M, K)
    y32, y16 = forward_both(make_layer(words, s, z), x)
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"small M={M}")


@pytest.mark.parametrize("K,N,M", [(128, 16, 1), (384, 48, 7), (1920, 272, 20), (640, 16, 64), (256, 4112, 3),
                                   (1920, 272, 7), (128, 16, 16), (4096, 4112, 16), (14336, 528, 4),
                                   (14336, 528, 5), (1920, 8208, 2), (14336, 528, 16), (14336, 272, 9),
                                   (7168, 1040, 13), (14464, 64, 16)])
def test_forward_ragged_shapes(K, N, M):
    _, words, s, z = quantized(3000 + K + N, N, K)
    x = synth.activations_bf16(3001 + K + N, M, K)
    y32, y16 = forward_both(make_layer(words, s, z), x)
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"ragged K={K} N={N} M={M}")


@pytest.mark.parametrize("idx", range(4))
@pytest.mark.parametrize("M", [1, 8, 64])
def test_forward_decode_shapes(idx, M):
    name, K, N = synth.SWEEP_SHAPES[idx]
    cfg = 1 if M == 1 else 2
    _, words, s, z = quantized(synth.seed_for(cfg, idx, 0), N, K)
    x = synth.activations_bf16(synth.seed_for(cfg, idx, 1), M, K)
    y32, y16 = forward_both(make_layer(words, s, z), x)
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"{name} M={M}")


@pytest.mark.parametrize("M", [1, 16, 40, 64, 200])
def test_one_hot_activations_reproduce_dequantize_bit_for_bit(M):
    K, N = 512, 96
    _, words, s, z = quantized(4000 + M, N, K)
    layer = make_layer(words, s, z)
    ks = (np.arange(M) * 37 + 5) % K
    x = np.zeros((M, K))
    x[np.arange(M), ks] = 1.0
    y16 = bits_host(dmr.dmr_qlinear_forward(layer, bf16_dev(orc.f64_to_bf16(x)), out_dtype=torch.bfloat16))
    wq = orc.dequantize(words, s, z, G)
    assert np.array_equal(y16, wq[:, ks].T)
    assert np.array_equal(y16, bits_host(dmr.dmr_qlinear_dequantize(layer))[:, ks].T)


@pytest.mark.parametrize("M", [1, 5, 33, 64, 130])
def test_power_of_two_scales_small_integer_activations_are_exact(M):
    rng = np.random.default_rng(50 + M)
    K, N = 768, 80
    q = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    s = orc.f64_to_bf16(2.0 ** rng.integers(-4, 3, size=(N, K // G)).astype(np.float64))
    z = orc.f64_to_bf16(rng.integers(0, 16, size=(N, K // G)).astype(np.float64))
    x = orc.f64_to_bf16(rng.integers(-8, 9, size=(M, K)).astype(np.float64))
    words = orc.pack(q)
    y32 = dmr.dmr_qlinear_forward(make_layer(words, s, z), bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward(words, s, z, G, x)
    assert np.array_equal(y32.astype(np.float64), y_ref)      # any summation order is exact here


@pytest.mark.parametrize("N,M", [(64, 1), (64, 64), (64, 130), (1024, 6400)])
def test_zero_point_only_weights_give_zero(N, M):
    # q == z everywhere, so w^ == 0 and y == 0.  With small-integer activations every partial sum of the
    # streaming paths is exact and they must return exactly 0.  With Gaussian activations they form
    # sum x (128+q) - (128+z) sum x from two separately rounded fp32 sums, so they are only required to stay
    # four orders of magnitude below the size of an ordinary output (the 1e-2 bar is 100x looser still).
    # The tiled kernel for 256 rows and more carries its running sum from one group's scale to the next with a
    # rounded ratio, so the same looser requirement holds for it whatever the activations.
    rng = np.random.default_rng(60)
    K = 512
    zc = rng.integers(0, 16, size=(N, K // G))
    q = np.repeat(zc, G, axis=1).astype(np.uint8)
    s_f32 = np.abs(synth.weights_f32(61, N, K // G)) + np.float32(1e-3)
    s = synth.to_bf16_bits(s_f32)
    z = orc.f64_to_bf16(zc.astype(np.float64))
    layer = make_layer(orc.pack(q), s, z)
    ordinary = float(s_f32.mean()) * 4.6 * np.sqrt(K)         # rms of x . w^ for codes spread over 0..15, x ~ N(0, 1)
    rescaling = dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N).endswith("_rescale")
    assert rescaling == (M == 6400)
    xi = orc.f64_to_bf16(rng.integers(-8, 9, size=(M, K)).astype(np.float64))
    y_int = dmr.dmr_qlinear_forward(layer, bf16_dev(xi), out_dtype=torch.float32)
    if rescaling:
        assert float(y_int.abs().max()) <= 1e-4 * 4.9 * ordinary          # integers -8..8: rms 4.9
    else:
        assert torch.count_nonzero(y_int).item() == 0
    x = synth.activations_bf16(62, M, K)
    y32 = dmr.dmr_qlinear_forward(layer, bf16_dev(x), out_dtype=torch.float32)
    assert float(y32.abs().max()) <= 1e-4 * ordinary


def test_forward_is_deterministic_and_m0_is_a_no_op():
    name, K, N = synth.SWEEP_SHAPES[0]
    _, words, s, z = quantized(7, N, K)
    layer = make_layer(words, s, z)
    x = bf16_dev(synth.activations_bf16(8, 8, K))
    runs = [dmr.dmr_qlinear_forward(layer, x, out_dtype=torch.float32).clone() for _ in range(3)]
    assert torch.equal(runs[0], runs[1]) and torch.equal(runs[0], runs[2])
    empty = torch.empty((0, K), dtype=torch.bfloat16, device="cuda:0")
    assert dmr.dmr_qlinear_forward(layer, empty).shape == (0, N)


# ------------------------------------------------------------------ prefill (MFMA tiles)

def sample_pairs(M, N, seed):
    rng = np.random.default_rng(seed)
    rows = sorted({0, 1, 15, 16, 31, 32, 63, 64, 127, 128, 255, 256, M // 2, M - 2, M - 1} & set(range(M)))
    cols = sorted({0, 1, 15, 16, 63, 64, 127, 128, N // 2, N - 129, N - 17, N - 1} & set(range(N)))
    ms = [m for m in rows for _ in cols] + list(rng.integers(0, M, 4096))
    ns = [n for _ in rows for n in cols] + list(rng.integers(0, N, 4096))
    return np.array(ms, dtype=np.int64), np.array(ns, dtype=np.int64)


def test_prefill_full_check_m512_attn_out():
    name, K, N = synth.SWEEP_SHAPES[0]
    M = 512
    _, words, s, z = quantized(synth.seed_for(3, 0, 0), N, K)
    x = synth.activations_bf16(synth.seed_for(3, 0, 1), M, K)
    y32, y16 = forward_both(make_layer(words, s, z), x)
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"prefill {name} M={M}")


@pytest.mark.parametrize("K,N,M", [(256, 144, 65), (384, 128, 129), (1024, 400, 300), (128, 16, 1000)])
def test_prefill_ragged_shapes(K, N, M):
    _, words, s, z = quantized(5000 + K + N, N, K)
    x = synth.activations_bf16(5001 + K + N, M, K)
    y32, y16 = forward_both(make_layer(words, s, z), x)
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"prefill ragged K={K} N={N} M={M}")


@pytest.mark.parametrize("K,N,M", [(1024, 1024, 65), (4096, 4096, 100), (512, 272, 130), (1792, 512, 96),
                                   (1024, 4096, 200), (2048, 1040, 257), (4096, 6144, 384)])
def test_forward_rollout_batch_sizes(K, N, M):
    # 64 < M <= 512: row blocks of 96 / 128, ragged column blocks, K split over workgroups (also with an
    # odd number of groups per split) and the partial-sum pass
    _, words, s, z = quantized(7000 + K + N + M, N, K)
    x = synth.activations_bf16(7001 + K + N + M, M, K)
    y32, y16 = forward_both(make_layer(words, s, z), x)
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"rollout batch ({K},{N}) M={M}")


@pytest.mark.parametrize("K,N,M", [(512, 16400, 17), (1536, 16400, 33), (1024, 16512, 48), (1536, 16528, 64),
                                   (2560, 16384, 20), (640, 16400, 40)])
def test_forward_wide_layers_small_batches(K, N, M):
    # 17 <= M <= 64 on layers of >= 1024 weight tiles: chunked activation panels in LDS (one chunk, an odd
    # and an even number of chunks), 2..4 row tiles with a ragged last one, a ragged last column block; five
    # groups (not a multiple of the chunk): the pre-pass kernel that re-orders the activations in memory
    _, words, s, z = quantized(7500 + K + N + M, N, K)
    x = synth.activations_bf16(7501 + K + N + M, M, K)
    y32, y16 = forward_both(make_layer(words, s, z), x)
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"wide layer ({K},{N}) M={M}")


@pytest.mark.parametrize("idx,M", [(1, 512), (2, 2048), (3, 2048), (0, 8192), (2, 512), (2, 450)])
def test_prefill_sampled_outputs_at_full_size(idx, M):
    name, K, N = synth.SWEEP_SHAPES[idx]
    _, words, s, z = quantized(synth.seed_for(3, idx, 0), N, K)
    x = synth.activations_bf16(synth.seed_for(3, idx, 1), M, K)
    y32 = dmr.dmr_qlinear_forward(make_layer(words, s, z), bf16_dev(x), out_dtype=torch.float32)
    ms, ns = sample_pairs(M, N, 9 + idx)
    got = y32[torch.from_numpy(ms).to("cuda:0"), torch.from_numpy(ns).to("cuda:0")].cpu().numpy()
    ref = orc.forward_sampled(words, s, z, G, x, ms, ns)
    err = float(np.max(np.abs(got - ref)) / np.sqrt(np.mean(ref ** 2)))
    print(f"prefill {name} M={M}: sampled max err {err:.3e} rms over {len(ms)} outputs")
    assert err <= TOL


# ------------------------------------------------------------------ bf16 twin

def bf16_both(w_bits, x_bits):
    wd, xd = bf16_dev(w_bits), bf16_dev(x_bits)
    y32 = dmr.dmr_qlinear_bf16_forward(wd, xd, out_dtype=torch.float32)
    y16 = dmr.dmr_qlinear_bf16_forward(wd, xd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    return y32.cpu().numpy(), bits_host(y16)


@pytest.mark.parametrize("K,N,M", [(1024, 1024, 1), (1024, 1024, 13), (384, 48, 64), (1920, 272, 33),
                                   (4096, 4096, 1), (14336, 4096, 8), (4096, 6144, 64),
                                   (256, 144, 65), (1024, 400, 300), (4096, 4096, 512),
                                   (1024, 1024, 17), (1024, 1024, 100), (512, 272, 130), (1792, 512, 96),
                                   (4096, 4096, 200), (2048, 1040, 257), (1920, 272, 2), (384, 48, 5),
                                   (4096, 4112, 16), (4096, 28672, 4), (4096, 6144, 9), (128, 16, 16),
                                   (1024, 16400, 12), (4096, 28672, 16), (256, 16384, 9)])
def test_bf16_forward(K, N, M):
    w = synth.to_bf16_bits(synth.weights_f32(6000 + K + N, N, K))
    x = synth.activations_bf16(6001 + K + M, M, K)
    y32, y16 = bf16_both(w, x)
    y_ref, _ = orc.bf16_forward(w, x, threads=THREADS)
    check_forward(y32, y16, y_ref, f"bf16 K={K} N={N} M={M}")


def test_bf16_forward_small_integers_exact():
    rng = np.random.default_rng(70)
    K, N = 512, 64
    for M in (1, 20, 64, 150):
        w = orc.f64_to_bf16(rng.integers(-16, 17, size=(N, K)).astype(np.float64))
        x = orc.f64_to_bf16(rng.integers(-8, 9, size=(M, K)).astype(np.float64))
        y32, _ = bf16_both(w, x)
        y_ref, _ = orc.bf16_forward(w, x)
        assert np.array_equal(y32.astype(np.float64), y_ref), M


@pytest.mark.parametrize("M", [1, 8, 40, 300])
def test_int4_vocabulary_sized_layer_sampled(M):
    # the largest N of the model (8016 weight tiles): every kernel class at a grid far beyond the decoder layers'
    name, K, N = synth.LM_HEAD
    _, words, s, z = quantized(synth.seed_for(4, 5, 0), N, K)
    x = synth.activations_bf16(synth.seed_for(4, 5, 1) + M, M, K)
    y32 = dmr.dmr_qlinear_forward(make_layer(words, s, z), bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    ms, ns = sample_pairs(M, N, 77 + M)
    y_ref = orc.forward_sampled(words, s, z, G, x, ms, ns)
    err = float(np.max(np.abs(y32[ms, ns].astype(np.float64) - y_ref)) / np.sqrt(np.mean(y_ref ** 2)))
    print(f"int4 {name}-sized layer M={M}: sampled max err {err:.3e} rms over {len(ms)} outputs")
    assert err <= TOL


def test_bf16_lm_head_shape_sampled():
    name, K, N = synth.LM_HEAD
    w = synth.to_bf16_bits(synth.weights_f32(synth.seed_for(4, 4, 0), N, K))
    x = synth.activations_bf16(synth.seed_for(4, 4, 1), 1, K)
    y32 = dmr.dmr_qlinear_bf16_forward(bf16_dev(w), bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.bf16_forward(w, x, threads=THREADS)
    assert rel_err(y32, y_ref) <= TOL
