"""Pins of the CPU oracle to things other than itself (no GPU).

Each test fixes the oracle to a hand-worked value, a closed form, an invariant, a special case
that reduces to integer arithmetic, or to a separately written numpy statement of the same
definitions, chosen so that a plausible mistake (dropped zero point, wrong nibble order,
transposed operand, rounding toward zero, scale applied per row instead of per group) fails
at least one of them.
"""
import itertools

import numpy as np
import pytest

from oracle import cpu_oracle as orc
from oracle import numpy_twin as twin
from paper_2602_02711_amd import synth


def _f(strs):
    return np.array([float(s) for s in strs], dtype=np.float64)


def _h(strs):
    return np.array([int(s, 16) for s in strs], dtype=np.uint64)


# ------------------------------------------------------------------ bf16 rounding

def test_bf16_rounding_known_values():
    # 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7: goes to even; 1 + 3*2^-8 ties up to even.
    cases = {
        1.0: 0x3F80, -2.0: 0xC000, 0.0: 0x0000, 1.0 + 2.0 ** -8: 0x3F80,
        1.0 + 3 * 2.0 ** -8: 0x3F82, 1.0 + 2.0 ** -8 + 2.0 ** -20: 0x3F81,
        0.2: 0x3E4D, 255.5: 0x4380, 3.0e38: 0x7F62, 3.4e38: 0x7F80, 2.0 ** -133: 0x0001,
        2.0 ** -134: 0x0000, 3 * 2.0 ** -134: 0x0002,
    }
    for value, bits in cases.items():
        assert int(orc.f64_to_bf16(np.array([value]))[0]) == bits, value
        assert int(orc.f64_to_bf16(np.array([-value]))[0]) == (bits ^ 0x8000), -value


def test_bf16_round_trip_all_finite_patterns():
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    finite = (bits & 0x7F80) != 0x7F80
    vals = orc.bf16_to_f64(bits[finite])
    assert np.array_equal(orc.f64_to_bf16(vals), bits[finite])


def test_bf16_rounding_is_nearest_on_random_doubles():
    rng = np.random.default_rng(7)
    v = rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))
    b = orc.f64_to_bf16(v)
    r = orc.bf16_to_f64(b)
    up = orc.bf16_to_f64((b + 1).astype(np.uint16))
    dn = orc.bf16_to_f64((b - 1).astype(np.uint16))
    assert np.all(np.abs(r - v) <= np.abs(up - v))
    assert np.all(np.abs(r - v) <= np.abs(dn - v))
    # and it agrees with the independent bit-trick rounding wherever the value is exact in fp32
    v32 = v.astype(np.float32)
    assert np.array_equal(orc.f32_to_bf16(v32), twin.f32_to_bf16_bits(v32))
    assert np.array_equal(synth.to_bf16_bits(v32), orc.f32_to_bf16(v32))


# ------------------------------------------------------------------ hand-worked examples

def test_handworked_4x8(golden):
    gd = golden("handworked_4x8.txt")
    w = np.stack([_f(gd[f"w_row{r}"]) for r in range(4)]).astype(np.float32)
    x = _f(gd["x"])
    q, s, z = orc.quantize(w, 8)
    assert np.array_equal(s[:, 0].astype(np.uint64), _h(gd["scale_bits"]))
    assert np.array_equal(orc.bf16_to_f64(s)[:, 0], _f(gd["scale"]))
    assert np.array_equal(orc.bf16_to_f64(z)[:, 0], _f(gd["zero"]))
    for r in range(4):
        assert np.array_equal(q[r].astype(np.float64), _f(gd[f"q_row{r}"])), r
    words = orc.pack(q)
    assert np.array_equal(words[:, 0].astype(np.uint64), _h(gd["words"]))
    w_hat = orc.dequantize_exact(words, s, z, 8)
    # power-of-two scales reproduce rows 0..2 exactly; row 3 is the printed exact product
    assert np.array_equal(w_hat[:3], w[:3].astype(np.float64))
    assert np.array_equal(w_hat[3], _f(gd["what_row3"]))
    wb = orc.dequantize(words, s, z, 8)
    for r in range(4):
        assert np.array_equal(wb[r].astype(np.uint64), _h(gd[f"wbf16_bits_row{r}"])), r
    xb = orc.f64_to_bf16(x)[None, :]
    assert np.array_equal(orc.bf16_to_f64(xb)[0], x)
    y, _ = orc.forward(words, s, z, 8, xb)
    assert np.array_equal(y[0], _f(gd["y_ref"]))
    y_bw, _ = orc.forward(words, s, z, 8, xb, rounded_weights=True)
    assert y_bw[0, 3] == float(gd["y_rounded_weights_row3"][0])
    assert np.array_equal(y_bw[0, :3], y[0, :3])
    assert np.array_equal(orc.f64_to_bf16(y[0]).astype(np.uint64), _h(gd["y_bf16_bits"]))
    # group-sum form, by hand: s * (sum x q - z * sum x)
    sx = x.sum()
    sxq = _f(gd["sum_x_q"])
    assert np.array_equal(_f(gd["scale"]) * (sxq - _f(gd["zero"]) * sx), _f(gd["y_ref"]))
    assert np.array_equal((q.astype(np.float64) * x).sum(axis=1), sxq)


def test_handworked_2x2(golden):
    gd = golden("handworked_2x2.txt")
    # embed in the smallest packed shape: K=8 with six zero-activation columns
    q = np.zeros((2, 8), dtype=np.uint8)
    q[0, :2] = _f(gd["q_row0"])
    q[1, :2] = _f(gd["q_row1"])
    q[:, 2:] = 9                         # irrelevant codes: their activations are 0
    s = orc.f64_to_bf16(_f(gd["scale"]))[:, None]
    z = orc.f64_to_bf16(_f(gd["zero"]))[:, None]
    x = np.zeros((2, 8))
    x[0, :2] = _f(gd["x_row0"])
    x[1, :2] = _f(gd["x_row1"])
    words = orc.pack(q)
    w_hat = orc.dequantize_exact(words, s, z, 8)
    assert np.array_equal(w_hat[0, :2], _f(gd["what_row0"]))
    assert np.array_equal(w_hat[1, :2], _f(gd["what_row1"]))
    y, _ = orc.forward(words, s, z, 8, orc.f64_to_bf16(x))
    assert np.array_equal(y[0], _f(gd["y_row0"]))
    assert np.array_equal(y[1], _f(gd["y_row1"]))


# ------------------------------------------------------------------ packing

def test_pack_unpack_bijection():
    rng = np.random.default_rng(11)
    q = rng.integers(0, 16, size=(13, 64), dtype=np.uint8)
    assert np.array_equal(orc.unpack(orc.pack(q)), q)
    words = rng.integers(0, 2 ** 32, size=(9, 24), dtype=np.uint64).astype(np.uint32)
    assert np.array_equal(orc.pack(orc.unpack(words)), words)
    for c in range(16):
        qc = np.full((3, 16), c, dtype=np.uint8)
        assert np.all(orc.pack(qc) == np.uint32(c * 0x11111111))
        assert np.array_equal(orc.unpack(orc.pack(qc)), qc)


def test_nibble_order_is_little_first_along_k():
    # code j of the word sits at bits [4j, 4j+4): a single 1 in position k sets bit 4*(k%8)
    for k in range(16):
        q = np.zeros((1, 16), dtype=np.uint8)
        q[0, k] = 1
        words = orc.pack(q)
        assert int(words[0, k // 8]) == 1 << (4 * (k % 8))
        assert int(words[0, 1 - k // 8]) == 0


def test_pack_rejects_codes_above_15():
    q = np.zeros((1, 8), dtype=np.uint8)
    q[0, 3] = 16
    with pytest.raises(ValueError):
        orc.pack(q)


# ------------------------------------------------------------------ special cases with exact answers

def _random_qsz(rng, N, K, g, pow2_scales=False):
    q = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    z = rng.integers(0, 16, size=(N, K // g)).astype(np.float64)
    if pow2_scales:
        s = 2.0 ** rng.integers(-8, 3, size=(N, K // g)).astype(np.float64)
    else:
        s = np.abs(rng.standard_normal((N, K // g))) * 0.01 + 1e-3
    return q, orc.f64_to_bf16(s), orc.f64_to_bf16(z)


def test_zero_point_only_gives_exact_zero():
    rng = np.random.default_rng(3)
    N, K, g = 6, 256, 128
    _, s, z = _random_qsz(rng, N, K, g)
    q = np.repeat(orc.bf16_to_f64(z), g, axis=1).astype(np.uint8)      # q == z everywhere
    words = orc.pack(q)
    assert np.all(orc.dequantize(words, s, z, g) == 0)
    x = synth.activations_bf16(5, 3, K)
    y, _ = orc.forward(words, s, z, g, x)
    assert np.all(y == 0.0) and not np.any(np.signbit(y))


def test_integer_special_case_matches_int64_matmul():
    # z = 8, s = 1, small-integer activations: forward is the integer product x . (q-8)^T
    rng = np.random.default_rng(5)
    N, K, g, M = 24, 512, 128, 5
    q = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    s = orc.f64_to_bf16(np.ones((N, K // g)))
    z = orc.f64_to_bf16(np.full((N, K // g), 8.0))
    xi = rng.integers(-8, 9, size=(M, K))
    y, _ = orc.forward(orc.pack(q), s, z, g, orc.f64_to_bf16(xi.astype(np.float64)))
    expect = xi.astype(np.int64) @ (q.astype(np.int64) - 8).T
    assert np.array_equal(y, expect.astype(np.float64))


def test_power_of_two_scales_are_exact_in_any_summation_order():
    rng = np.random.default_rng(6)
    N, K, g, M = 16, 384, 128, 4
    q, s, z = _random_qsz(rng, N, K, g, pow2_scales=True)
    xi = rng.integers(-8, 9, size=(M, K)).astype(np.float64)
    words = orc.pack(q)
    y, _ = orc.forward(words, s, z, g, orc.f64_to_bf16(xi))
    # exact rational check through integers: y * 2^8 is an integer
    sg = np.repeat(orc.bf16_to_f64(s), g, axis=1)
    zg = np.repeat(orc.bf16_to_f64(z), g, axis=1)
    w_int = ((q.astype(np.int64) - zg.astype(np.int64)) * (sg * 256).astype(np.int64))
    expect = (xi.astype(np.int64) @ w_int.T).astype(np.float64) / 256.0
    assert np.array_equal(y, expect)
    # reversed summation order (permute k within the row) gives the same bits
    perm = rng.permutation(g)
    qp = q.reshape(N, K // g, g)[:, :, perm].reshape(N, K)
    xp = xi.reshape(M, K // g, g)[:, :, perm].reshape(M, K)
    y2, _ = orc.forward(orc.pack(qp), s, z, g, orc.f64_to_bf16(xp))
    assert np.array_equal(y, y2)


def test_one_hot_activation_selects_dequantized_weight():
    rng = np.random.default_rng(8)
    N, K, g = 12, 256, 128
    q, s, z = _random_qsz(rng, N, K, g)
    words = orc.pack(q)
    ks = [0, 1, 7, 8, 127, 128, 200, 255]
    x = np.zeros((len(ks), K))
    x[np.arange(len(ks)), ks] = 1.0
    y, _ = orc.forward(words, s, z, g, orc.f64_to_bf16(x))
    w_hat = orc.dequantize_exact(words, s, z, g)
    assert np.array_equal(y, w_hat[:, ks].T)
    assert np.array_equal(orc.f64_to_bf16(y), orc.dequantize(words, s, z, g)[:, ks].T)


def test_scaling_and_row_permutation_invariants():
    rng = np.random.default_rng(9)
    N, K, g, M = 10, 256, 128, 3
    q, s, z = _random_qsz(rng, N, K, g)
    words = orc.pack(q)
    x = synth.activations_bf16(21, M, K)
    y, _ = orc.forward(words, s, z, g, x)
    x4 = orc.f64_to_bf16(orc.bf16_to_f64(x) * 4.0)
    y4, _ = orc.forward(words, s, z, g, x4)
    assert np.array_equal(y4, 4.0 * y)
    p = rng.permutation(N)
    yp, _ = orc.forward(words[p], s[p], z[p], g, x)
    assert np.array_equal(yp, y[:, p])


def test_groups_use_their_own_scale_and_zero():
    # one row, two groups with different (s, z): activations that touch only group 1
    K, g = 256, 128
    q = np.full((1, K), 10, dtype=np.uint8)
    s = orc.f64_to_bf16(np.array([[0.5, 0.25]]))
    z = orc.f64_to_bf16(np.array([[2.0, 6.0]]))
    x = np.zeros((1, K))
    x[0, 130] = 1.0
    y, _ = orc.forward(orc.pack(q), s, z, g, orc.f64_to_bf16(x))
    assert y[0, 0] == (10 - 6) * 0.25
    x[0, 3] = 2.0
    y, _ = orc.forward(orc.pack(q), s, z, g, orc.f64_to_bf16(x))
    assert y[0, 0] == (10 - 6) * 0.25 + 2.0 * (10 - 2) * 0.5


# ------------------------------------------------------------------ independent twin, brute force

@pytest.mark.parametrize("N,K,g", [(1, 8, 8), (3, 16, 8), (5, 64, 32), (16, 128, 128),
                                   (64, 256, 128), (7, 256, 64), (33, 96, 32)])
def test_numpy_twin_agrees_on_tiny_shapes(N, K, g):
    rng = np.random.default_rng(100 + N + K)
    q, s, z = _random_qsz(rng, N, K, g)
    words = orc.pack(q)
    assert np.array_equal(words, twin.pack(q))
    assert np.array_equal(orc.unpack(words), twin.unpack(words))
    assert np.array_equal(orc.dequantize_exact(words, s, z, g), twin.dequantize_exact(words, s, z, g))
    assert np.array_equal(orc.dequantize(words, s, z, g), twin.dequantize(words, s, z, g))
    x = synth.activations_bf16(300 + K, 4, K)
    y, _ = orc.forward(words, s, z, g, x)
    yt = twin.forward(words, s, z, g, x)
    scale = np.sqrt(np.mean(yt ** 2)) + 1e-30
    assert np.max(np.abs(y - yt)) <= 1e-12 * scale * np.sqrt(K)
    yg = twin.forward_group_sums(words, s, z, g, x)
    assert np.max(np.abs(y - yg)) <= 1e-11 * scale * np.sqrt(K)
    ms = np.array([0, 3, 1, 2], dtype=np.int64)
    ns = np.array([0, N - 1, N // 2, 0], dtype=np.int64)
    assert np.array_equal(orc.forward_sampled(words, s, z, g, x, ms, ns), y[ms, ns])


def test_dequantize_exhaustive_codes_zeros_scales():
    # every (q, z) pair with a spread of bf16 scales: D4 and D5 against integer arithmetic
    scales_bits = np.array([0x3C00, 0x3C01, 0x3C7F, 0x3BFF, 0x3E4D, 0x3F80, 0x3D23, 0x0080, 0x3AAB],
                           dtype=np.uint16)
    for sb in scales_bits:
        s_val = float(orc.bf16_to_f64(np.array([sb]))[0])
        for zc in range(16):
            q = np.arange(16, dtype=np.uint8)[None, :]
            s = np.array([[sb, sb]], dtype=np.uint16)
            z = orc.f64_to_bf16(np.full((1, 2), float(zc)))
            words = orc.pack(q)
            w_hat = orc.dequantize_exact(words, s, z, 8)[0]
            assert np.array_equal(w_hat, (np.arange(16) - zc) * s_val)
            wb = orc.bf16_to_f64(orc.dequantize(words, s, z, 8)[0])
            # nearest: error at most half a bf16 ulp of the result, 2^(floor(log2|w^|) - 8)
            nz = w_hat != 0
            half_ulp = 2.0 ** (np.floor(np.log2(np.abs(w_hat[nz]))) - 8)
            assert np.all(np.abs(wb[nz] - w_hat[nz]) <= half_ulp)
            assert np.all(wb[~nz] == 0)


def test_bf16_forward_against_einsum_and_integers():
    rng = np.random.default_rng(12)
    N, K, M = 9, 200, 3
    w = synth.to_bf16_bits(synth.weights_f32(77, N, K))
    x = synth.activations_bf16(78, M, K)
    y, _ = orc.bf16_forward(w, x)
    yt = twin.bf16_forward(w, x)
    assert np.max(np.abs(y - yt)) <= 1e-12 * np.sqrt(np.mean(yt ** 2)) * np.sqrt(K)
    wi = rng.integers(-100, 100, size=(N, K))
    xi = rng.integers(-100, 100, size=(M, K))
    yi, _ = orc.bf16_forward(orc.f64_to_bf16(wi.astype(float)), orc.f64_to_bf16(xi.astype(float)))
    assert np.array_equal(yi, (xi @ wi.T).astype(np.float64))
    ms = np.array([0, 2], dtype=np.int64)
    ns = np.array([8, 1], dtype=np.int64)
    assert np.array_equal(orc.bf16_forward_sampled(w, x, ms, ns), y[ms, ns])


# ------------------------------------------------------------------ quantiser

def test_quantizer_error_bound_and_code_range():
    N, K, g = 32, 1024, 128
    w = synth.weights_f32(synth.seed_for(0, 0, 0), N, K)
    q, s, z = orc.quantize(w, g)
    assert q.max() <= 15
    zf = orc.bf16_to_f64(z)
    assert np.all((zf >= 0) & (zf <= 15) & (zf == np.rint(zf)))
    sf = np.repeat(orc.bf16_to_f64(s), g, axis=1)
    w_hat = orc.dequantize_exact(orc.pack(q), s, z, g)
    err = np.abs(w_hat - w.astype(np.float64))
    # closed form: half a step wherever the unclamped code fits, plus the clamped excess
    unclamped = np.rint(w.astype(np.float64) / sf) + np.repeat(zf, g, axis=1)
    excess = np.maximum(unclamped - 15, 0) + np.maximum(-unclamped, 0)
    assert np.all(err <= sf * (0.5 + excess) * (1 + 1e-12))
    # the scale is the bf16 rounding of range/15: within 2^-8 relative of it
    wg = w.reshape(N, K // g, g).astype(np.float64)
    rng_ = np.maximum(wg.max(axis=2), 0) - np.minimum(wg.min(axis=2), 0)
    assert np.all(np.abs(orc.bf16_to_f64(s) - rng_ / 15) <= (rng_ / 15) * 2.0 ** -8)
    # both extreme codes are (nearly always) used: the range is covered
    assert np.mean(q.reshape(N, K // g, g).max(axis=2) >= 14) > 0.99
    assert np.mean(q.reshape(N, K // g, g).min(axis=2) <= 1) > 0.99


def test_quantizer_degenerate_groups():
    w = np.zeros((2, 16), dtype=np.float32)
    w[1, :8] = 3.0                                    # constant positive group
    q, s, z = orc.quantize(w, 8)
    assert np.all(q[0] == 0) and np.all(orc.bf16_to_f64(s)[0] == 1.0) and np.all(orc.bf16_to_f64(z)[0] == 0)
    assert np.all(q[1, :8] == 15) and orc.bf16_to_f64(s)[1, 0] == 0.2001953125 and orc.bf16_to_f64(z)[1, 0] == 0
    assert np.array_equal(orc.dequantize_exact(orc.pack(q), s, z, 8)[0], np.zeros(16))
    assert np.all(z == 0x0000)                       # the zero point 0 is +0, never -0


def test_threads_do_not_change_results():
    N, K, g, M = 40, 256, 128, 2
    w = synth.weights_f32(1, N, K)
    q, s, z = orc.quantize(w, g)
    x = synth.activations_bf16(2, M, K)
    y1, used1 = orc.forward(orc.pack(q), s, z, g, x, threads=1)
    y4, used4 = orc.forward(orc.pack(q), s, z, g, x, threads=4)
    assert used1 == 1 and used4 == 4
    assert np.array_equal(y1, y4)


def test_synth_is_seeded_and_shaped():
    a = synth.weights_f32(synth.seed_for(1, 2, 0), 8, 256)
    b = synth.weights_f32(synth.seed_for(1, 2, 0), 8, 256)
    assert np.array_equal(a, b) and a.dtype == np.float32
    assert abs(float(a.std()) - 0.02) < 0.002
    x = synth.activations_bf16(synth.seed_for(1, 2, 1), 2, 4096)
    assert x.dtype == np.uint16 and abs(float(orc.bf16_to_f64(x).std()) - 1.0) < 0.05
    assert len({synth.seed_for(c, s, r) for c, s, r in itertools.product(range(5), range(4), range(2))}) == 40


# ------------------------------------------------------------------ 3-bit variant (W3A16 g128)

def test_w3_handworked_packing(golden):
    gd = golden("handworked_w3_pack.txt")
    q = np.stack([_f(gd[f"q_row{r}"]) for r in range(3)]).astype(np.uint8)
    words = orc.pack3(q)
    for r in range(3):
        assert np.array_equal(words[r].astype(np.uint64), _h(gd[f"words_row{r}"])), r
    assert np.array_equal(orc.unpack3(words), q)


def test_w3_handworked_quantizer(golden):
    # the 3-bit quantiser against values worked by hand (ties, a scale that rounds up in bf16, a forced zero
    # end point): a wrong divisor (range / 15), a wrong rounding of the scale or of the codes fails here
    gd = golden("handworked_w3_quant.txt")
    w = np.stack([_f(gd[f"w_row{r}"]) for r in range(3)]).astype(np.float32)
    q, s, z = orc.quantize_bits(w, 8, 3)
    assert np.array_equal(s.reshape(3).astype(np.uint64), _h(gd["s_bits"]))
    assert np.array_equal(orc.bf16_to_f64(z).reshape(3), _f(gd["z"]))
    for r in range(3):
        assert np.array_equal(q[r].astype(np.float64), _f(gd[f"q_row{r}"])), r
    # K = 8 is below one packed run of 32 codes, so the exact weights are formed here from the definition
    w_hat = (q.astype(np.float64) - orc.bf16_to_f64(z)) * orc.bf16_to_f64(s)
    assert np.array_equal(w_hat[1], _f(gd["what_row1"]))
    assert np.array_equal(w_hat[2], w[2].astype(np.float64))          # power-of-two scale, no tie: exact
    # the same rows through the packed path (padded to one run of 32 codes with zero weights)
    w32 = np.zeros((3, 32), dtype=np.float32)
    w32[:, :8] = w
    q32, s32, z32 = orc.quantize_bits(w32, 32, 3)
    assert np.array_equal(q32[:, :8], q) and np.array_equal(s32, s) and np.array_equal(z32, z)
    assert np.array_equal(orc.dequantize_exact3(orc.pack3(q32), s32, z32, 32)[:, :8], w_hat)


def test_w3_pack_bijection_and_twin():
    rng = np.random.default_rng(31)
    q = rng.integers(0, 8, size=(11, 160), dtype=np.uint8)
    words = orc.pack3(q)
    assert words.shape == (11, 15)
    assert np.array_equal(orc.unpack3(words), q)
    assert np.array_equal(twin.pack3(q), words)
    assert np.array_equal(twin.unpack3(words), q)
    raw = rng.integers(0, 2 ** 32, size=(5, 9), dtype=np.uint64).astype(np.uint32)
    assert np.array_equal(orc.pack3(orc.unpack3(raw)), raw)
    bad = q.copy()
    bad[0, 3] = 8
    with pytest.raises(ValueError):
        orc.pack3(bad)


def test_w3_quantizer_dequantize_forward():
    N, K, g, M = 24, 256, 128, 3
    w = synth.weights_f32(41, N, K)
    q, s, z = orc.quantize_bits(w, g, 3)
    assert q.max() <= 7
    zf, sf = orc.bf16_to_f64(z), np.repeat(orc.bf16_to_f64(s), g, axis=1)
    assert np.all((zf >= 0) & (zf <= 7) & (zf == np.rint(zf)))
    words = orc.pack3(q)
    w_hat = orc.dequantize_exact3(words, s, z, g)
    # closed form: half a step (steps are range / 7 now), plus the clamped excess
    unclamped = np.rint(w.astype(np.float64) / sf) + np.repeat(zf, g, axis=1)
    excess = np.maximum(unclamped - 7, 0) + np.maximum(-unclamped, 0)
    assert np.all(np.abs(w_hat - w) <= sf * (0.5 + excess) * (1 + 1e-12))
    assert np.array_equal(w_hat, twin.dequantize_exact3(words, s, z, g))
    assert np.array_equal(orc.dequantize3(words, s, z, g), twin.f32_to_bf16_bits(w_hat.astype(np.float32)))
    x = synth.activations_bf16(42, M, K)
    y, _ = orc.forward3(words, s, z, g, x)
    yt = twin.forward3(words, s, z, g, x)
    assert np.max(np.abs(y - yt)) <= 1e-12 * np.sqrt(np.mean(yt ** 2)) * np.sqrt(K)
    # integer special case: z = 4, s = 1 -> x . (q - 4)^T in int64
    rng = np.random.default_rng(43)
    xi = rng.integers(-8, 9, size=(M, K))
    one = orc.f64_to_bf16(np.ones((N, K // g)))
    four = orc.f64_to_bf16(np.full((N, K // g), 4.0))
    yi, _ = orc.forward3(words, one, four, g, orc.f64_to_bf16(xi.astype(np.float64)))
    assert np.array_equal(yi, (xi @ (q.astype(np.int64) - 4).T).astype(np.float64))
    # the 4-bit entry point is the bits = 4 case of the general one
    q4a, s4a, z4a = orc.quantize(w, g)
    q4b, s4b, z4b = orc.quantize_bits(w, g, 4)
    assert np.array_equal(q4a, q4b) and np.array_equal(s4a, s4b) and np.array_equal(z4a, z4b)


# ------------------------------------------------------------------ decoder glue (RMSNorm, SwiGLU)

def test_glue_handworked(golden):
    gd = golden("handworked_glue.txt")
    x = _h(gd["rmsnorm_x"]).astype(np.uint16)[None, :]
    gamma = _h(gd["rmsnorm_gamma"]).astype(np.uint16)
    assert np.array_equal(orc.rmsnorm(x, gamma, 0.0)[0], _h(gd["rmsnorm_out"]).astype(np.uint16))
    gu = _h(gd["swiglu_in"]).astype(np.uint16)[None, :]
    assert np.array_equal(orc.swiglu(gu)[0], _h(gd["swiglu_out"]).astype(np.uint16))


def test_rmsnorm_closed_forms_and_invariances():
    rng = np.random.default_rng(41)
    K = 96
    one = orc.f64_to_bf16(np.ones(K))
    # a constant row has rms |c|: the result is sign(c) exactly
    for c in (0.75, -3.0, 1e-3):
        x = orc.f64_to_bf16(np.full((1, K), c))
        assert np.array_equal(orc.bf16_to_f64(orc.rmsnorm(x, one, 0.0))[0], np.full(K, np.sign(c)))
    x = synth.activations_bf16(42, 5, K)
    gamma = orc.f64_to_bf16(rng.uniform(0.5, 2.0, K))
    y = orc.rmsnorm(x, gamma, 0.0)
    # scaling the row by a power of two changes nothing (eps = 0)
    x4 = orc.f64_to_bf16(orc.bf16_to_f64(x) * 4.0)
    assert np.array_equal(orc.rmsnorm(x4, gamma, 0.0), y)
    # with gamma = 1 the output has unit mean square up to the bf16 rounding of each element
    y1 = orc.bf16_to_f64(orc.rmsnorm(x, one, 0.0))
    assert np.all(np.abs((y1 ** 2).mean(axis=1) - 1.0) < 2.0 ** -7)
    # gamma multiplies element-wise: a one-hot gamma keeps exactly that element
    hot = np.zeros(K)
    hot[7] = 1.0
    yh = orc.bf16_to_f64(orc.rmsnorm(x, orc.f64_to_bf16(hot), 0.0))
    assert np.array_equal(yh[:, 7], y1[:, 7]) and np.count_nonzero(np.delete(yh, 7, axis=1)) == 0
    # eps enters under the root: a zero row stays zero, and a huge eps shrinks the row by sqrt(eps)
    assert np.count_nonzero(orc.rmsnorm(np.zeros((1, K), np.uint16), gamma, 1e-6)) == 0
    assert np.count_nonzero(orc.rmsnorm(np.zeros((1, K), np.uint16), gamma, 0.0)) == 0
    big = orc.bf16_to_f64(orc.rmsnorm(x, one, 2.0 ** 20))
    ref = orc.bf16_to_f64(x) / np.sqrt((orc.bf16_to_f64(x) ** 2).mean(axis=1, keepdims=True) + 2.0 ** 20)
    assert np.all(np.abs(big - ref) <= np.abs(ref) * 2.0 ** -8)
    assert np.array_equal(twin.rmsnorm(x, gamma, 1e-5), orc.rmsnorm(x, gamma, 1e-5))
    with pytest.raises(ValueError):
        orc.rmsnorm(x, gamma[:-1], 0.0)


def test_swiglu_closed_forms():
    rng = np.random.default_rng(43)
    I = 64
    g = orc.bf16_to_f64(synth.activations_bf16(44, 3, I)) * 3.0
    u = orc.bf16_to_f64(synth.activations_bf16(45, 3, I))
    def run(gate, up):
        return orc.bf16_to_f64(orc.swiglu(np.concatenate([orc.f64_to_bf16(gate), orc.f64_to_bf16(up)], axis=1)))
    g, u = orc.bf16_to_f64(orc.f64_to_bf16(g)), orc.bf16_to_f64(orc.f64_to_bf16(u))
    assert np.count_nonzero(run(np.zeros_like(g), u)) == 0          # silu(0) = 0
    assert np.count_nonzero(run(g, np.zeros_like(u))) == 0
    # silu(a) - silu(-a) = a: with up = 1 the two results differ by the gate, up to their roundings
    p, n = run(g, np.ones_like(u)), run(-g, np.ones_like(u))
    assert np.all(np.abs(p - n - g) <= (np.abs(p) + np.abs(n)) * 2.0 ** -8 + 1e-30)
    # far in the tails silu is the identity resp. zero
    assert np.array_equal(run(np.full((1, I), 32.0), u[:1]), u[:1] * 32.0)
    assert np.all(np.abs(run(np.full((1, I), -40.0), u[:1])) < 1e-14)
    # the up half scales linearly by powers of two
    assert np.array_equal(run(g, u * 8.0), run(g, u) * 8.0)
    # the halves are (gate | up), not interleaved and not swapped
    packed = np.concatenate([orc.f64_to_bf16(g), orc.f64_to_bf16(u)], axis=1)
    assert np.array_equal(twin.swiglu(packed), orc.swiglu(packed))
    swapped = np.concatenate([orc.f64_to_bf16(u), orc.f64_to_bf16(g)], axis=1)
    assert not np.array_equal(orc.swiglu(swapped), orc.swiglu(packed))
    with pytest.raises(ValueError):
        orc.swiglu(packed[:, :-1])
