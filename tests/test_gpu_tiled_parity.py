"""GPU parity of the tiled MFMA GEMMs (prefill sizes) and of the paths that only large or unusual shapes
reach, through the C ABI against the CPU oracle.  Every case asserts which kernel class the dispatch
picks for it (dmr_qlinear_kernel_path, the same host arithmetic the forward uses), so that a change of
a crossover cannot silently move a case off the kernel it is meant to cover.

Bars as elsewhere: max|y - y_ref| <= 1e-2 rms(y_ref) on the fp32 output; where the oracle cannot afford
the whole output, sampled outputs (tile-edge rows and columns plus random pairs) with the rms taken over
the sample.  The raw ratio is printed for every case.
"""
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
DEV = "cuda:0"


def sample_pairs(M, N, seed):
    """First / last rows and columns of every tile size in use (16, 64, 128, 256) plus 4096 random pairs."""
    rng = np.random.default_rng(seed)
    rows = sorted({0, 1, 15, 16, 31, 32, 63, 64, 127, 128, 255, 256, 257, M // 2, M - 257, M - 129, M - 2, M - 1}
                  & set(range(M)))
    cols = sorted({0, 1, 15, 16, 63, 64, 127, 128, 255, 256, N // 2, N - 257, N - 129, N - 17, N - 1} & set(range(N)))
    ms = [m for m in rows for _ in cols] + list(rng.integers(0, M, 4096))
    ns = [n for _ in rows for n in cols] + list(rng.integers(0, N, 4096))
    return np.array(ms, dtype=np.int64), np.array(ns, dtype=np.int64)


def sampled_err(y32, ms, ns, ref):
    got = y32[torch.from_numpy(ms).to(DEV), torch.from_numpy(ns).to(DEV)].cpu().numpy().astype(np.float64)
    return float(np.max(np.abs(got - ref)) / np.sqrt(np.mean(ref ** 2)))


# ------------------------------------------------------------------ bf16 twin, tiled kernels

@pytest.mark.parametrize("K,N,M,path", [
    (4096, 28672, 2048, "bf16_gemm256"),       # 8 x 112 tiles of 256: the widest layer of the prefill config
    (4096, 4096, 8192, "bf16_gemm256"),        # 32 x 16 tiles of 256
    (4096, 4096, 1024, "bf16_gemm128_dma"),    # 256 workgroups of 128 x 128, direct-to-LDS operand loads
    (512, 4096, 4224, "bf16_gemm128"),         # K < 1024: register-staged 128 x 128 kernel, 1056 workgroups
])
def test_bf16_prefill_sampled_at_full_size(K, N, M, path):
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_BF16, M, K, N) == path
    w = synth.to_bf16_bits(synth.weights_f32(8100 + K + N, N, K))
    x = synth.activations_bf16(8101 + K + M, M, K)
    y32 = dmr.dmr_qlinear_bf16_forward(bf16_dev(w), bf16_dev(x), out_dtype=torch.float32)
    ms, ns = sample_pairs(M, N, 11 + M)
    err = sampled_err(y32, ms, ns, orc.bf16_forward_sampled(w, x, ms, ns))
    print(f"{path} ({K},{N}) M={M}: sampled max err {err:.3e} rms over {len(ms)} outputs")
    assert err <= TOL


@pytest.mark.parametrize("K,N,M,path", [
    (256, 2192, 1100, "bf16_gemm128"),         # 9 x 18 workgroups, ragged last row and column tiles
    (1024, 2192, 1100, "bf16_gemm128_dma"),    # the same grid on the direct-to-LDS kernel
    (256, 3840, 3584, "bf16_gemm256"),         # 14 x 15 = 210 tiles of 256: one round of the big kernel
    (384, 3856, 3500, "bf16_gemm256"),         # 14 x 16 = 224 tiles, ragged last row and column tiles, 3 groups
])
def test_bf16_tiled_gemm_full_output(K, N, M, path):
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_BF16, M, K, N) == path
    w = synth.to_bf16_bits(synth.weights_f32(8200 + K + N, N, K))
    x = synth.activations_bf16(8201 + K + M, M, K)
    wd, xd = bf16_dev(w), bf16_dev(x)
    y32 = dmr.dmr_qlinear_bf16_forward(wd, xd, out_dtype=torch.float32).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_bf16_forward(wd, xd, out_dtype=torch.bfloat16))
    y_ref, _ = orc.bf16_forward(w, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"{path} ({K},{N}) M={M}: max err {err:.3e} rms, all {M * N} outputs")
    assert err <= TOL
    assert np.array_equal(y16, orc.f32_to_bf16(y32))


def test_bf16_tiled_gemms_small_integers_exact():
    # integer weights and activations: every product and partial sum is exact, so each tiled kernel must
    # return the oracle's value bit for bit whatever its summation order
    rng = np.random.default_rng(83)
    for K, N, M, path in [(256, 2192, 1100, "bf16_gemm128"), (1024, 2192, 1100, "bf16_gemm128_dma"),
                          (256, 3840, 3584, "bf16_gemm256")]:
        assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_BF16, M, K, N) == path
        w = orc.f64_to_bf16(rng.integers(-16, 17, size=(N, K)).astype(np.float64))
        x = orc.f64_to_bf16(rng.integers(-8, 9, size=(M, K)).astype(np.float64))
        y32 = dmr.dmr_qlinear_bf16_forward(bf16_dev(w), bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
        y_ref, _ = orc.bf16_forward(w, x, threads=THREADS)
        assert np.array_equal(y32.astype(np.float64), y_ref), path


# ------------------------------------------------------------------ INT4, tiled kernels, whole output

@pytest.mark.parametrize("K,N,M,path", [
    (1024, 3840, 3584, "w4_gemm256_rescale"),        # 14 x 15 tiles of 256 on eight waves
    (1152, 3856, 3500, "w4_gemm256_rescale"),        # ragged last tiles, an odd number of groups
    (256, 3840, 3584, "w4_gemm256_rescale"),         # short rows, 1.4e7 outputs: where weights rounded to bf16 were seen to miss the bound
    (256, 2192, 2200, "w4_gemm256x128_rescale"),     # 9 x 18 tiles of 256 x 128 on four waves, two groups only
    (1152, 2192, 2200, "w4_gemm256x128_rescale"),    # the same grid, nine groups, ragged in both directions
    (128, 2192, 2200, "w4_gemm256x128_rescale"),     # a single group: nothing to rescale, the zero-point loop is one step
    (256, 19200, 200, "w4_gemm256x128_rescale"),     # fewer than 256 rows on a very wide layer: a half-empty row tile
    (128, 112, 40000, "w4_gemm256x128_rescale"),     # one column tile, not even full (7 row tiles of 16), 157 row blocks
    (256, 272, 45100, "w4_gemm256_rescale"),         # two column tiles of 256, the second with 16 columns; ragged rows
    (1152, 2064, 1500, "w4_gemm128_rescale"),        # 12 x 17 tiles of 128 x 128 (at most 256 of them: one round), ragged both ways
    (128, 4096, 520, "w4_gemm128_rescale"),          # 5 x 32 tiles, a single group, 8 rows in the last row tile
])
def test_int4_tiled_gemm_full_output(K, N, M, path):
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N) == path
    _, words, s, z = quantized(8300 + K + N, N, K)
    x = synth.activations_bf16(8301 + K + M, M, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    xd = bf16_dev(x)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.bfloat16))
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"{path} ({K},{N}) M={M}: max err {err:.3e} rms, all {M * N} outputs")
    # the codes stay exact, so only fp32 accumulation is left: far inside the bound
    assert err <= 1e-4
    assert np.array_equal(y16, orc.f32_to_bf16(y32))


def _one_zero_scale_per_32_rows(s):
    """Scales with group 0 of every 32nd row set to zero: every block of 32 rows is flagged, so the whole output comes
    from the 128 x 128 kernel that serves the blocks the rescaling kernel declines."""
    out = s.copy()
    out[::32, 0] = 0
    return out


def test_int4_one_hot_rows_through_the_tiled_gemms():
    # One-hot rows: output m, n is the single weight w^[n][m] = s (q - z).
    # 128 x 128 kernel (every column block flagged; 200 rows of the identity): one exact fp32 product rounded once, so
    # the bf16 output must equal dmr_qlinear_dequantize bit for bit.
    K, N, M = 256, 19200, 200
    _, words, s, z = quantized(8400 + K, N, K)
    s = _one_zero_scale_per_32_rows(s)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    x = torch.eye(K, dtype=torch.bfloat16, device=DEV)[:M].contiguous()
    y16 = dmr.dmr_qlinear_forward(layer, x, out_dtype=torch.bfloat16)
    wq = dmr.dmr_qlinear_dequantize(layer)
    # (compared as values: a zero scale dequantises (q - z) < 0 to -0, a sum that starts at +0 ends at +0)
    assert torch.equal(y16, wq.t()[:M].contiguous())
    assert np.array_equal(bits_host(wq), orc.dequantize(words, s, z, G))
    # rescaling kernels: the weight comes out as s_last (prod of scale ratios) (16 + q) - s (16 + z), a handful of fp32
    # roundings from s (q - z); each output is checked against the exact weight on its own, relative to the largest
    # term of that difference
    for K, N, path in [(2304, 2304, "w4_gemm256x128_rescale"), (3584, 3840, "w4_gemm256_rescale"),
                       (1536, 2048, "w4_gemm128_rescale")]:
        M = K
        assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N) == path
        _, words, s, z = quantized(8400 + K, N, K)
        layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
        y32 = dmr.dmr_qlinear_forward(layer, torch.eye(K, dtype=torch.bfloat16, device=DEV), out_dtype=torch.float32)
        exact = orc.dequantize_exact(words, s, z, G)                       # [N][K] fp64
        scale = np.repeat(orc.bf16_to_f64(s), G, axis=1)                   # [N][K]
        dev = np.abs(y32.cpu().numpy().astype(np.float64).T - exact) / (31.0 * np.abs(scale))
        print(f"{path} one-hot ({K},{N}): max deviation {dev.max():.3e} of the largest term")
        assert dev.max() <= 2e-5, path


@pytest.mark.parametrize("K,N,M", [(1024, 3840, 3584), (1152, 2192, 1100)])
def test_int4_128_tile_kernel_whole_output(K, N, M):
    # the kernel with a per-group tile, reached through flags on every block of 32 rows, on its own merits
    _, words, s, z = quantized(8300 + K + N, N, K)
    s = _one_zero_scale_per_32_rows(s)
    x = synth.activations_bf16(8301 + K + M, M, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    y32 = dmr.dmr_qlinear_forward(layer, bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"128 x 128 exact kernel ({K},{N}) M={M}: max err {err:.3e} rms, all {M * N} outputs")
    assert err <= 1e-4


def test_int4_tiled_gemm_very_long_rows_sampled():
    # K = 32768: 256 groups, i.e. 255 rescales of the running sum and a zero-point loop of 48 k steps; N = 528 leaves the
    # last column tile mostly empty
    K, N, M = 32768, 528, 8192
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N) == "w4_gemm256x128_rescale"
    _, words, s, z = quantized(8350, N, K)
    x = synth.activations_bf16(8351, M, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    y32 = dmr.dmr_qlinear_forward(layer, bf16_dev(x), out_dtype=torch.float32)
    ms, ns = sample_pairs(M, N, 8352)
    err = sampled_err(y32, ms, ns, orc.forward_sampled(words, s, z, G, x, ms, ns))
    print(f"w4_gemm256x128_rescale ({K},{N}) M={M}: sampled max err {err:.3e} rms over {len(ms)} outputs")
    assert err <= 1e-4


def _scales_with(s, rows_groups, bits):
    out = s.copy()
    for (n, g) in rows_groups:
        out[n, g] = bits
    return out


@pytest.mark.parametrize("K,N,M,path", [(1152, 2192, 2200, "w4_gemm256x128_rescale"), (1152, 3856, 3500, "w4_gemm256_rescale"),
                                        (1152, 2064, 1500, "w4_gemm128_rescale")])
def test_int4_tiled_gemm_scales_that_cannot_be_rescaled(K, N, M, path):
    # A zero scale, a subnormal one and a row whose scales span 2^41: the running rescale of the tiled kernels
    # cannot carry them, so their column blocks must come from the 128 x 128 kernel behind it, all others from the
    # fast kernel, and the output must be the oracle's everywhere.
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N) == path
    _, words, s, z = quantized(8300 + K + N, N, K)
    x = synth.activations_bf16(8301 + K + M, M, K)
    xd = bf16_dev(x)
    s2 = _scales_with(s, [(200, 3), (N - 1, 0)], 0x0000)                     # zero
    s2 = _scales_with(s2, [(700, 8)], 0x0040)                               # subnormal
    s2 = _scales_with(s2, [(1500, 1)], 0x5000)                              # 2^33 next to 2^-6-sized neighbours
    s2 = _scales_with(s2, [(1500, 5)], 0x2B80)                              # 2^-40
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s2), bf16_dev(z), G)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward(words, s2, z, G, x, threads=THREADS)
    assert np.all(np.isfinite(y32))
    # column by column (the columns with the huge scale dwarf the rms of the whole output)
    rms_col = np.sqrt(np.mean(y_ref ** 2, axis=0))
    err = np.max(np.abs(y32.astype(np.float64) - y_ref) / np.maximum(rms_col, 1e-30))
    print(f"{path} with scales it declines ({K},{N}) M={M}: max err {err:.3e} of the column rms")
    assert err <= 1e-4


@pytest.mark.parametrize("K,N,M,path", [(256, 3840, 3584, "w4_gemm256_rescale"), (1024, 1024, 6400, "w4_gemm256x128_rescale"),
                                        (512, 2064, 1500, "w4_gemm128_rescale")])
def test_per_channel_layer_through_the_tiled_gemms(K, N, M, path):
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_PER_CHANNEL, M, K, N) == path
    rng = np.random.default_rng(8700 + K + M)
    q = rng.integers(0, 16, size=(N, K), dtype=np.uint8)
    s_row = synth.to_bf16_bits(np.abs(synth.weights_f32(8701 + K, N, 1)) + np.float32(2e-3))       # [N][1]
    z_row = orc.f64_to_bf16(np.full((N, 1), 8.0))
    words = orc.pack(q)
    layer = dmr.dmr_qlinear_create_per_channel(u32_dev(words), bf16_dev(s_row.reshape(N)))
    x = synth.activations_bf16(8702 + K, M, K)
    y32 = dmr.dmr_qlinear_forward(layer, bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward(words, s_row, z_row, K, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"per-channel {path} ({K},{N}) M={M}: max err {err:.3e} rms")
    assert err <= 1e-4


@pytest.mark.parametrize("K,N,M,path", [(512, 2064, 1500, "w4_gemm128_rescale"), (512, 2192, 2200, "w4_gemm256x128_rescale"),
                                        (512, 3856, 3500, "w4_gemm256_rescale")])
def test_int4_tiled_gemm_same_bits_every_time(K, N, M, path):
    # no atomics and a fixed order of additions: the output must not depend on the run, on what the workspace held
    # before the call, or on whether the launches are replayed from a graph
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N) == path
    _, words, s, z = quantized(8800 + K + N, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    xd = bf16_dev(synth.activations_bf16(8801 + K + M, M, K))
    need = dmr.dmr_qlinear_workspace_bytes(M, K, N)
    torch.cuda.synchronize()
    first = None
    for fill in (0x00, 0xFF, 0x7F, 0xAA, 0x00):
        ws = torch.full((need,), fill, dtype=torch.uint8, device=DEV)
        y = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
        dmr.dmr_qlinear_forward(layer, xd, out=y, workspace=ws)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(y).any()) and not bool((y == 7.0).any())     # every output written, no poison
        if first is None:
            first = y.clone()
        assert torch.equal(y, first), hex(fill)
    stream = torch.cuda.Stream()
    ws = torch.empty((need,), dtype=torch.uint8, device=DEV)
    y = torch.empty((M, N), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        dmr.dmr_qlinear_forward(layer, xd, out=y, workspace=ws)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(3):
                dmr.dmr_qlinear_forward(layer, xd, out=y, workspace=ws)
        for _ in range(4):
            y.fill_(7.0)
            graph.replay()
            stream.synchronize()
            assert torch.equal(y, first)
    torch.cuda.synchronize()


def test_int4_tiled_gemm_refuses_a_short_workspace():
    K, N, M = 256, 2192, 2200
    need = dmr.dmr_qlinear_workspace_bytes(M, K, N)
    assert need > 0                       # zero-point operands, rescale factors, flags
    _, words, s, z = quantized(8300 + K + N, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    xd = bf16_dev(synth.activations_bf16(8301 + K + M, M, K))
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    y = torch.full((M, N), 7.0, dtype=torch.float32, device=DEV)
    lib = dmr.binding.lib()
    for pws, nbytes in ((None, 0), (ws.data_ptr(), need - 1)):
        st = lib.dmr_qlinear_forward(layer.handle, xd.data_ptr(), M, y.data_ptr(), dmr.DMR_OUT_FP32, pws, nbytes,
                                     torch.cuda.current_stream().cuda_stream)
        assert st == dmr.binding.DMR_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
    # a workspace full of NaN bit patterns must not leak into the result (every word that is read is written first)
    ws.fill_(0xFF)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32, workspace=ws)
    y_again = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32)
    assert torch.equal(y32, y_again) and bool(torch.isfinite(y32).all())


# ------------------------------------------------------------------ prefill config: every (M, shape) cell, sampled

@pytest.mark.parametrize("idx", range(4))
@pytest.mark.parametrize("M", [512, 2048, 8192])
def test_prefill_config_cells_sampled(idx, M):
    name, K, N = synth.SWEEP_SHAPES[idx]
    w, words, s, z = quantized(synth.seed_for(3, idx, 0), N, K)
    x = synth.activations_bf16(synth.seed_for(3, idx, 1), M, K)
    ms, ns = sample_pairs(M, N, 21 + idx + M)
    xd = bf16_dev(x)
    p4 = dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N)
    y32 = dmr.dmr_qlinear_forward(dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G), xd,
                                  out_dtype=torch.float32)
    err4 = sampled_err(y32, ms, ns, orc.forward_sampled(words, s, z, G, x, ms, ns))
    del y32
    wb = synth.to_bf16_bits(w)
    p16 = dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_BF16, M, K, N)
    y32 = dmr.dmr_qlinear_bf16_forward(bf16_dev(wb), xd, out_dtype=torch.float32)
    err16 = sampled_err(y32, ms, ns, orc.bf16_forward_sampled(wb, x, ms, ns))
    print(f"prefill {name} M={M}: INT4 [{p4}] {err4:.3e} rms, bf16 [{p16}] {err16:.3e} rms over {len(ms)} outputs")
    assert err4 <= TOL and err16 <= TOL


# ------------------------------------------------------------------ 3-bit layers at prefill sizes

@pytest.mark.parametrize("K,N,M,path", [
    (512, 4096, 1200, "w3_gemm256x128_rescale"),
    (1152, 2192, 2200, "w3_gemm256x128_rescale"),    # nine groups, ragged in both directions
    (256, 3840, 3584, "w3_gemm256_rescale"),
    (1152, 3856, 3500, "w3_gemm256_rescale"),
    (256, 19200, 200, "w3_gemm256x128_rescale"),     # fewer than 256 rows on a very wide layer: a half-empty row tile
    (1152, 2064, 1500, "w3_gemm128_rescale"),        # 12 x 17 tiles of 128 x 128, ragged both ways
])
def test_w3_prefill_size(K, N, M, path):
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W3_G128, M, K, N) == path
    assert (dmr.dmr_qlinear_w3_workspace_bytes(M, K, N) > 0) == path.endswith("_rescale")
    _, words, s, z = quantized3(8500 + K + N, N, K)
    x = synth.activations_bf16(8501 + K + M, M, K)
    layer = dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    xd = bf16_dev(x)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.bfloat16))
    y_ref, _ = orc.forward3(words, s, z, G, x, threads=THREADS)
    err = rel_err(y32, y_ref)
    print(f"{path} ({K},{N}) M={M}: max err {err:.3e} rms, all {M * N} outputs")
    assert err <= 1e-4                      # exact codes: only fp32 accumulation is left
    assert np.array_equal(y16, orc.f32_to_bf16(y32))


def test_w3_one_hot_rows_through_the_tiled_gemms():
    # as for 4 bits: bit for bit on the 128 x 128 kernel (every block flagged), to a few fp32 roundings on the rescaling one
    K, N, M = 256, 19200, 200
    _, words, s, z = quantized3(8550, N, K)
    s = _one_zero_scale_per_32_rows(s)
    layer = dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    x = torch.eye(K, dtype=torch.bfloat16, device=DEV)[:M].contiguous()
    y16 = dmr.dmr_qlinear_forward(layer, x, out_dtype=torch.bfloat16)
    wq = dmr.dmr_qlinear_dequantize(layer)
    assert torch.equal(y16, wq.t()[:M].contiguous())
    assert np.array_equal(bits_host(wq), orc.dequantize3(words, s, z, G))
    K, N = 2304, 2304
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W3_G128, K, K, N) == "w3_gemm256x128_rescale"
    _, words, s, z = quantized3(8551, N, K)
    layer = dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    y32 = dmr.dmr_qlinear_forward(layer, torch.eye(K, dtype=torch.bfloat16, device=DEV), out_dtype=torch.float32)
    exact = orc.dequantize_exact3(words, s, z, G)
    scale = np.repeat(orc.bf16_to_f64(s), G, axis=1)
    dev = np.abs(y32.cpu().numpy().astype(np.float64).T - exact) / (23.0 * np.abs(scale))
    assert dev.max() <= 2e-5


def test_w3_128_tile_kernel_whole_output():
    K, N, M = 1152, 2192, 1100
    _, words, s, z = quantized3(8570, N, K)
    s = _one_zero_scale_per_32_rows(s)
    x = synth.activations_bf16(8571, M, K)
    layer = dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    y32 = dmr.dmr_qlinear_forward(layer, bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward3(words, s, z, G, x, threads=THREADS)
    assert rel_err(y32, y_ref) <= 1e-4


def test_w3_tiled_gemm_scales_that_cannot_be_rescaled():
    K, N, M = 1152, 2192, 2200
    _, words, s, z = quantized3(8560, N, K)
    x = synth.activations_bf16(8561, M, K)
    s2 = s.copy()
    s2[200, 3] = 0x0000
    s2[1500, 1] = 0x5000
    layer = dmr.dmr_qlinear_w3_create(u32_dev(words), bf16_dev(s2), bf16_dev(z), G)
    y32 = dmr.dmr_qlinear_forward(layer, bf16_dev(x), out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward3(words, s2, z, G, x, threads=THREADS)
    rms_col = np.sqrt(np.mean(y_ref ** 2, axis=0))
    err = np.max(np.abs(y32.astype(np.float64) - y_ref) / np.maximum(rms_col, 1e-30))
    assert np.all(np.isfinite(y32)) and err <= 1e-4


# ------------------------------------------------------------------ decode rows too long for the M = 1 kernels

def test_decode_very_long_rows_take_the_fallbacks():
    # K = 32768: the activations exceed the LDS budget of the decode kernels, so M = 1 goes to the
    # direct-from-L2 kernel (4 bits, bf16) and to the rollout-batch kernel with K split (3 bits, whose
    # workspace the size query must report)
    K, N = 32768, 528
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, 1, K, N) == "w4_skinny"
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W3_G128, 1, K, N) == "w3_mid"
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_BF16, 1, K, N) == "bf16_skinny"
    x = synth.activations_bf16(8601, 1, K)
    xd = bf16_dev(x)
    w, words, s, z = quantized(8600, N, K)
    y32 = dmr.dmr_qlinear_forward(dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G), xd,
                                  out_dtype=torch.float32).cpu().numpy()
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    assert rel_err(y32, y_ref) <= TOL
    _, words3, s3, z3 = quantized3(8600, N, K)
    layer3 = dmr.dmr_qlinear_w3_create(u32_dev(words3), bf16_dev(s3), bf16_dev(z3), G)
    need = dmr.dmr_qlinear_w3_workspace_bytes(1, K, N)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    y32 = dmr.dmr_qlinear_forward(layer3, xd, out_dtype=torch.float32, workspace=ws).cpu().numpy()
    y_ref3, _ = orc.forward3(words3, s3, z3, G, x, threads=THREADS)
    assert rel_err(y32, y_ref3) <= TOL
    # a missing or short workspace is refused before anything is launched
    y = torch.full((1, N), 7.0, dtype=torch.float32, device=DEV)
    lib = dmr.binding.lib()
    for pws, nbytes in ((None, 0), (ws.data_ptr(), need - 1)):
        st = lib.dmr_qlinear_forward(layer3.handle, xd.data_ptr(), 1, y.data_ptr(), dmr.DMR_OUT_FP32, pws, nbytes,
                                     torch.cuda.current_stream().cuda_stream)
        assert st == dmr.binding.DMR_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
    wb = synth.to_bf16_bits(w)
    yb = dmr.dmr_qlinear_bf16_forward(bf16_dev(wb), xd, out_dtype=torch.float32).cpu().numpy()
    yb_ref, _ = orc.bf16_forward(wb, x, threads=THREADS)
    assert rel_err(yb, yb_ref) <= TOL


# ------------------------------------------------------------------ rollout-batch config at M = 4, 16

@pytest.mark.parametrize("idx", range(4))
@pytest.mark.parametrize("M", [4, 16])
def test_rollout_config_cells(idx, M):
    name, K, N = synth.SWEEP_SHAPES[idx]
    w, words, s, z = quantized(synth.seed_for(2, idx, 0), N, K)
    x = synth.activations_bf16(synth.seed_for(2, idx, 1) + M, M, K)
    xd = bf16_dev(x)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    y32 = dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.float32).cpu().numpy()
    y16 = bits_host(dmr.dmr_qlinear_forward(layer, xd, out_dtype=torch.bfloat16))
    y_ref, _ = orc.forward(words, s, z, G, x, threads=THREADS)
    err4 = rel_err(y32, y_ref)
    assert np.array_equal(y16, orc.f32_to_bf16(y32))
    wb = synth.to_bf16_bits(w)
    yb = dmr.dmr_qlinear_bf16_forward(bf16_dev(wb), xd, out_dtype=torch.float32).cpu().numpy()
    yb_ref, _ = orc.bf16_forward(wb, x, threads=THREADS)
    err16 = rel_err(yb, yb_ref)
    print(f"{name} M={M}: INT4 [{dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, M, K, N)}] {err4:.3e} rms, "
          f"bf16 [{dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_BF16, M, K, N)}] {err16:.3e} rms")
    assert err4 <= TOL and err16 <= TOL


# ------------------------------------------------------------------ mixed routed step: both copies at once

@pytest.mark.parametrize("m_high", [3, 6, 11])
def test_mixed_routed_step_two_streams(m_high):
    # One decision step of a group of 16 rollouts (Sec. 4.3): the router sends m_high of them to the bf16 copy
    # and the rest to the INT4 copy; the two copies' layers run concurrently on two streams into disjoint
    # rows of the same output.  Each half is checked against its own oracle, and against the same call run
    # alone (bit for bit: concurrency must not change a result).
    G_ROLL = 16
    m_low = G_ROLL - m_high
    s_low, s_high = torch.cuda.Stream(), torch.cuda.Stream()      # both at the default priority
    layers = []
    for idx, (name, K, N) in enumerate(synth.SWEEP_SHAPES):
        w, words, s, z = quantized(synth.seed_for(2, idx, 0) + 7, N, K)
        x = synth.activations_bf16(synth.seed_for(2, idx, 1) + 7, G_ROLL, K)
        wb = synth.to_bf16_bits(w)
        layers.append((name, K, N, words, s, z, wb, x,
                       dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G), bf16_dev(wb), bf16_dev(x),
                       torch.full((G_ROLL, N), float("nan"), dtype=torch.float32, device=DEV)))
    torch.cuda.synchronize()
    for rep in range(3):
        for (_, _, _, _, _, _, _, _, layer, wbd, xd, y) in layers:
            y.fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(s_low):
            for (_, _, _, _, _, _, _, _, layer, wbd, xd, y) in layers:
                dmr.dmr_qlinear_forward(layer, xd[:m_low], out=y[:m_low])
        with torch.cuda.stream(s_high):
            for (_, _, _, _, _, _, _, _, layer, wbd, xd, y) in layers:
                dmr.dmr_qlinear_bf16_forward(wbd, xd[m_low:], out=y[m_low:])
        torch.cuda.synchronize()
        for (name, K, N, words, s, z, wb, x, layer, wbd, xd, y) in layers:
            alone_low = dmr.dmr_qlinear_forward(layer, xd[:m_low], out_dtype=torch.float32)
            alone_high = dmr.dmr_qlinear_bf16_forward(wbd, xd[m_low:], out_dtype=torch.float32)
            torch.cuda.synchronize()
            assert torch.equal(y[:m_low], alone_low) and torch.equal(y[m_low:], alone_high), (name, rep)
            if rep == 0:
                yl, _ = orc.forward(words, s, z, G, x[:m_low], threads=THREADS)
                yh, _ = orc.bf16_forward(wb, x[m_low:], threads=THREADS)
                got = y.cpu().numpy()
                el, eh = rel_err(got[:m_low], yl), rel_err(got[m_low:], yh)
                print(f"mixed step {name}: {m_low} rows INT4 {el:.3e} rms, {m_high} rows bf16 {eh:.3e} rms")
                assert el <= TOL and eh <= TOL
