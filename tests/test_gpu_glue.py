"""GPU parity of the decoder glue and of the forwards that fuse it, through the C ABI, against the CPU
oracle.  The glue rounds to bf16 once, from fp32 on the GPU and from fp64 in the oracle: an element may
land on the other side of a rounding boundary, so outputs are required to agree bit for bit on at least
99.8 % of the elements and to differ by one bf16 ulp at most elsewhere.  Fused forwards are compared
with the oracle's composition (glue, forward in fp64, residual) to the usual 1e-2 rms on the fp32
output; at M = 1 the fused kernel must also agree with the library's own unfused composition."""
import numpy as np
import pytest
import torch

import paper_2602_02711_amd as dmr
from oracle import cpu_oracle as orc
from paper_2602_02711_amd import synth

from gpu_util import bf16_dev, bits_host, quantized, rel_err, u32_dev

pytestmark = pytest.mark.gpu
G = synth.GROUP
TOL = 1e-2
EPS = 1e-6


def close_bf16(dev_bits, ref_bits, where):
    d = dev_bits.astype(np.int32) - ref_bits.astype(np.int32)
    assert np.all(np.abs(d) <= 1), where                     # neighbours in bf16 (same sign, same binade or next)
    frac = np.count_nonzero(d) / d.size
    print(f"{where}: {frac:.2e} of the elements one ulp apart")
    assert frac <= 2e-3, where


def gamma_bits(seed, K):
    rng = np.random.default_rng(seed)
    return orc.f64_to_bf16(rng.uniform(0.5, 1.5, K))


@pytest.mark.parametrize("M,K", [(1, 4096), (1, 128), (3, 1000 * 8), (40, 4096), (2, 14336)])
def test_rmsnorm_kernel(M, K):
    x = synth.activations_bf16(8000 + M + K, M, K)
    x[0, :8] = orc.f64_to_bf16(np.array([37.0, -50.0, 0, 0, 1e-3, 2.0, -2.0, 64.0]))   # outliers, zeros
    gm = gamma_bits(8001 + K, K)
    y = bits_host(dmr.dmr_glue_rmsnorm(bf16_dev(x), bf16_dev(gm), EPS))
    close_bf16(y, orc.rmsnorm(x, gm, EPS), f"rmsnorm M={M} K={K}")


def test_rmsnorm_kernel_special_rows():
    K = 256
    gm = gamma_bits(1, K)
    zero = np.zeros((1, K), np.uint16)
    assert np.count_nonzero(bits_host(dmr.dmr_glue_rmsnorm(bf16_dev(zero), bf16_dev(gm), 0.0))) == 0
    const = orc.f64_to_bf16(np.full((1, K), -0.75))
    one = orc.f64_to_bf16(np.ones(K))
    y = orc.bf16_to_f64(bits_host(dmr.dmr_glue_rmsnorm(bf16_dev(const), bf16_dev(one), 0.0)))
    assert np.array_equal(y, np.full((1, K), -1.0))


@pytest.mark.parametrize("M,I", [(1, 14336), (1, 8), (5, 1024), (33, 14336)])
def test_swiglu_kernel(M, I):
    gu = synth.activations_bf16(8100 + M + I, M, 2 * I)
    gu[0, :4] = orc.f64_to_bf16(np.array([0.0, 30.0, -30.0, 8.0]))
    y = bits_host(dmr.dmr_glue_swiglu(bf16_dev(gu)))
    close_bf16(y, orc.swiglu(gu), f"swiglu M={M} I={I}")


def oracle_chain(pro, inp, gm, forward):
    if pro == dmr.DMR_PRO_RMSNORM:
        return forward(orc.rmsnorm(inp, gm, EPS))
    if pro == dmr.DMR_PRO_SWIGLU:
        return forward(orc.swiglu(inp))
    return forward(inp)


CASES = [(dmr.DMR_PRO_RMSNORM, 4096, 6144, False), (dmr.DMR_PRO_RMSNORM, 4096, 4096, True),
         (dmr.DMR_PRO_SWIGLU, 14336, 4096, True), (dmr.DMR_PRO_SWIGLU, 1024, 272, False),
         (dmr.DMR_PRO_NONE, 4096, 4096, True), (dmr.DMR_PRO_RMSNORM, 1024, 1024, True),
         (dmr.DMR_PRO_RMSNORM, 512, 16400, True)]       # wide layer: the bf16 streaming kernel at M = 12


@pytest.mark.parametrize("M", [1, 5, 16, 40])
@pytest.mark.parametrize("pro,K,N,with_res", CASES)
def test_fused_forward_int4(pro, K, N, with_res, M):
    _, words, s, z = quantized(8200 + K + N, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    width = 2 * K if pro == dmr.DMR_PRO_SWIGLU else K
    inp = synth.activations_bf16(8201 + K + M, M, width)
    gm = gamma_bits(8202 + K, K)
    res = synth.activations_bf16(8203 + N + M, M, N) if with_res else None
    kw = dict(gamma=bf16_dev(gm) if pro == dmr.DMR_PRO_RMSNORM else None, eps=EPS,
              residual=bf16_dev(res) if with_res else None)
    y32 = dmr.dmr_qlinear_forward_fused(layer, pro, bf16_dev(inp), out_dtype=torch.float32, **kw).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_forward_fused(layer, pro, bf16_dev(inp), out_dtype=torch.bfloat16, **kw))
    y_ref = oracle_chain(pro, inp, gm, lambda xb: orc.forward(words, s, z, G, xb, threads=16)[0])
    if with_res:
        y_ref = y_ref + orc.bf16_to_f64(res)
    err = rel_err(y32, y_ref)
    print(f"fused int4 pro={pro} ({K},{N}) M={M} res={with_res}: max err {err:.3e} rms")
    assert err <= TOL
    assert np.array_equal(y16, orc.f32_to_bf16(y32))          # bf16 output = one rounding of the same fp32 value


@pytest.mark.parametrize("pro,with_res", [(dmr.DMR_PRO_RMSNORM, True), (dmr.DMR_PRO_SWIGLU, False)])
def test_fused_forward_int4_at_a_prefill_size(pro, with_res):
    # M large enough for the tiled kernel, whose own workspace (zero-point operands, rescale factors) sits behind the
    # glue output and the fp32 result in the caller's workspace
    K, N, M = 256, 2192, 2200
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N) == "w4_gemm256x128_rescale"
    _, words, s, z = quantized(8250 + K + N, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    width = 2 * K if pro == dmr.DMR_PRO_SWIGLU else K
    inp = synth.activations_bf16(8251 + K + M, M, width)
    gm = gamma_bits(8252 + K, K)
    res = synth.activations_bf16(8253 + N + M, M, N) if with_res else None
    kw = dict(gamma=bf16_dev(gm) if pro == dmr.DMR_PRO_RMSNORM else None, eps=EPS,
              residual=bf16_dev(res) if with_res else None)
    y32 = dmr.dmr_qlinear_forward_fused(layer, pro, bf16_dev(inp), out_dtype=torch.float32, **kw).cpu().numpy()
    y_ref = oracle_chain(pro, inp, gm, lambda xb: orc.forward(words, s, z, G, xb, threads=16)[0])
    if with_res:
        y_ref = y_ref + orc.bf16_to_f64(res)
    err = rel_err(y32, y_ref)
    print(f"fused int4 pro={pro} ({K},{N}) M={M} res={with_res}: max err {err:.3e} rms")
    assert err <= TOL


@pytest.mark.parametrize("M", [1, 8])
@pytest.mark.parametrize("pro,K,N,with_res", CASES)
def test_fused_kernels_match_unfused_composition(pro, K, N, with_res, M):
    # The fused streaming kernels against glue kernel + plain forward + residual of the same library.  The sum
    # of squares is reduced in a different order, so a normalised activation may differ by one bf16 ulp;
    # the outputs must agree far below the parity tolerance.
    _, words, s, z = quantized(8300 + K + N, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    width = 2 * K if pro == dmr.DMR_PRO_SWIGLU else K
    inp = bf16_dev(synth.activations_bf16(8301 + K, M, width))
    gm = bf16_dev(gamma_bits(8302 + K, K))
    res = bf16_dev(synth.activations_bf16(8303 + N, M, N)) if with_res else None
    fused = dmr.dmr_qlinear_forward_fused(layer, pro, inp, gamma=gm, eps=EPS, residual=res, out_dtype=torch.float32)
    x = inp
    if pro == dmr.DMR_PRO_RMSNORM:
        x = dmr.dmr_glue_rmsnorm(inp, gm, EPS)
    if pro == dmr.DMR_PRO_SWIGLU:
        x = dmr.dmr_glue_swiglu(inp)
    plain = dmr.dmr_qlinear_forward(layer, x, out_dtype=torch.float32)
    if with_res:
        plain = plain + res.float()
    rms = plain.pow(2).mean().sqrt().item()
    assert (fused - plain).abs().max().item() <= 1e-3 * rms


@pytest.mark.parametrize("M", [1, 12])
@pytest.mark.parametrize("pro,K,N,with_res", CASES)
def test_fused_forward_bf16(pro, K, N, with_res, M):
    w = synth.to_bf16_bits(synth.weights_f32(8400 + K + N, N, K))
    width = 2 * K if pro == dmr.DMR_PRO_SWIGLU else K
    inp = synth.activations_bf16(8401 + K + M, M, width)
    gm = gamma_bits(8402 + K, K)
    res = synth.activations_bf16(8403 + N + M, M, N) if with_res else None
    kw = dict(gamma=bf16_dev(gm) if pro == dmr.DMR_PRO_RMSNORM else None, eps=EPS,
              residual=bf16_dev(res) if with_res else None)
    y32 = dmr.dmr_qlinear_bf16_forward_fused(bf16_dev(w), pro, bf16_dev(inp), out_dtype=torch.float32, **kw).cpu().numpy()
    y_ref = oracle_chain(pro, inp, gm, lambda xb: orc.bf16_forward(w, xb, threads=16)[0])
    if with_res:
        y_ref = y_ref + orc.bf16_to_f64(res)
    err = rel_err(y32, y_ref)
    print(f"fused bf16 pro={pro} ({K},{N}) M={M} res={with_res}: max err {err:.3e} rms")
    assert err <= TOL


def test_fused_forward_w3_layer_takes_the_composition():
    K, N, M = 1024, 256, 3
    w = synth.weights_f32(8500, N, K)
    q, s, z = orc.quantize_bits(w, G, 3)
    words = orc.pack3(q)
    layer = dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    inp = synth.activations_bf16(8501, M, K)
    gm = gamma_bits(8502, K)
    y32 = dmr.dmr_qlinear_forward_fused(layer, dmr.DMR_PRO_RMSNORM, bf16_dev(inp), gamma=bf16_dev(gm), eps=EPS,
                                        out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward3(words, s, z, G, orc.rmsnorm(inp, gm, EPS))
    assert rel_err(y32, y_ref) <= TOL
