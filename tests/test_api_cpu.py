"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, answers the size queries, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

from paper_2602_02711_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000        # a 16-byte aligned address that is never dereferenced by a rejected call


@pytest.fixture(scope="module")
def lib():
    return binding.lib()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "dmr_qlinear.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dmr_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_size_queries(lib):
    # 0.5 byte per weight + 4 bytes per (row, group of 128)
    assert lib.dmr_qlinear_storage_bytes(4096, 4096, 128) == 4096 * 4096 // 2 + 4096 * 32 * 4
    assert lib.dmr_qlinear_storage_bytes(1024, 1024, 128) == 1024 * 512 + 1024 * 8 * 4
    assert lib.dmr_qlinear_storage_bytes(1000, 1024, 128) == 0
    assert lib.dmr_qlinear_storage_bytes(1024, 1000, 128) == 0
    assert lib.dmr_qlinear_storage_bytes(1024, 1024, 64) == 0
    assert lib.dmr_qlinear_workspace_bytes(1, 4096, 4096) == 0
    assert lib.dmr_qlinear_workspace_bytes(16, 4096, 4096) == 0
    # 16 < M <= 64 on a wide layer: activation panels in LDS, no workspace; when the group count is not a
    # multiple of four: activations in MFMA operand order (4 KiB per group and row tile) plus their group sums
    assert lib.dmr_qlinear_workspace_bytes(64, 4096, 28672) == 0
    assert lib.dmr_qlinear_workspace_bytes(17, 4096, 28672) == 0
    assert lib.dmr_qlinear_workspace_bytes(64, 4224, 28672) == 33 * 4 * (4096 + 64)
    # rollout batches on layers too small to fill the chip: fp32 partials of a 4-way (8-way) split of K
    assert lib.dmr_qlinear_workspace_bytes(64, 4096, 4096) == 4 * 64 * 4096 * 4
    assert lib.dmr_qlinear_workspace_bytes(17, 4096, 4096) == 4 * 17 * 4096 * 4
    assert lib.dmr_qlinear_workspace_bytes(65, 4096, 4096) == 4 * 65 * 4096 * 4
    assert lib.dmr_qlinear_workspace_bytes(8, 14336, 4096) == 4 * 8 * 4096 * 4    # rows exceed LDS: four k slices
    # enough column blocks: no split
    assert lib.dmr_qlinear_workspace_bytes(128, 4096, 28672) == 0
    # the tiled GEMM (more than 128 rows here): zero-point operands, rescale factors and flags
    assert lib.dmr_qlinear_workspace_bytes(200, 4096, 28672) > 200 * 192 * 2 + 28672 * 192 * 2
    assert lib.dmr_qlinear_workspace_bytes(600, 4096, 28672) > 600 * 192 * 2 + 28672 * 192 * 2
    # the bf16 twin splits K under the same rule
    assert lib.dmr_qlinear_bf16_workspace_bytes(1, 4096, 4096) == 0
    assert lib.dmr_qlinear_bf16_workspace_bytes(8, 4096, 4096) == 0
    assert lib.dmr_qlinear_bf16_workspace_bytes(16, 4096, 4096) == 4 * 16 * 4096 * 4
    assert lib.dmr_qlinear_bf16_workspace_bytes(64, 4096, 4096) == 4 * 64 * 4096 * 4
    assert lib.dmr_qlinear_bf16_workspace_bytes(128, 4096, 28672) == 0
    assert lib.dmr_qlinear_bf16_workspace_bytes(128, 4096, 4096) == 4 * 128 * 4096 * 4
    assert lib.dmr_qlinear_bf16_workspace_bytes(600, 4096, 28672) == 0


def test_status_strings(lib):
    seen = {lib.dmr_status_string(i) for i in range(7)}
    assert len(seen) == 7 and all(s for s in seen)
    assert lib.dmr_status_string(99)


def _create(lib, K, N, g, q=FAKE, s=FAKE, z=FAKE, st=FAKE, st_bytes=1 << 40, out=True):
    h = ctypes.c_void_p(0xDEAD)
    rc = lib.dmr_qlinear_create(ctypes.byref(h) if out else None, K, N, g, q, s, z, st, st_bytes, None)
    return rc, h.value


def test_create_rejects_bad_arguments_without_touching_hip(lib):
    assert _create(lib, 1024, 1024, 128, out=False)[0] == binding.DMR_ERR_NULL
    for K, N, g, want in [(0, 1024, 128, binding.DMR_ERR_SHAPE), (1024, -16, 128, binding.DMR_ERR_SHAPE),
                          (1000, 1024, 128, binding.DMR_ERR_SHAPE), (1024, 1000, 128, binding.DMR_ERR_SHAPE),
                          (1024, 1024, 0, binding.DMR_ERR_SHAPE), (1024, 1024, 100, binding.DMR_ERR_SHAPE),
                          (1024, 1024, 64, binding.DMR_ERR_UNSUPPORTED),
                          (1024, 1024, 1024, binding.DMR_ERR_UNSUPPORTED)]:
        rc, h = _create(lib, K, N, g)
        assert rc == want, (K, N, g)
        assert h is None                       # *out is cleared on failure
    assert _create(lib, 1024, 1024, 128, q=None)[0] == binding.DMR_ERR_NULL
    assert _create(lib, 1024, 1024, 128, s=None)[0] == binding.DMR_ERR_NULL
    assert _create(lib, 1024, 1024, 128, z=None)[0] == binding.DMR_ERR_NULL
    assert _create(lib, 1024, 1024, 128, st=None)[0] == binding.DMR_ERR_NULL
    assert _create(lib, 1024, 1024, 128, q=FAKE + 4)[0] == binding.DMR_ERR_ALIGN
    assert _create(lib, 1024, 1024, 128, st=FAKE + 8)[0] == binding.DMR_ERR_ALIGN
    need = lib.dmr_qlinear_storage_bytes(1024, 1024, 128)
    assert _create(lib, 1024, 1024, 128, st_bytes=need - 1)[0] == binding.DMR_ERR_WORKSPACE


def test_forward_and_friends_reject_bad_arguments(lib):
    assert lib.dmr_qlinear_forward(None, FAKE, 1, FAKE, 0, None, 0, None) == binding.DMR_ERR_NULL
    assert lib.dmr_qlinear_dequantize(None, FAKE, None) == binding.DMR_ERR_NULL
    assert lib.dmr_qlinear_shape(None, None, None, None) == binding.DMR_ERR_NULL
    lib.dmr_qlinear_destroy(None)             # NULL-safe
    bf = lib.dmr_qlinear_bf16_forward
    assert bf(FAKE, FAKE, 1, 1000, 1024, FAKE, 0, None, 0, None) == binding.DMR_ERR_SHAPE
    assert bf(FAKE, FAKE, -1, 1024, 1024, FAKE, 0, None, 0, None) == binding.DMR_ERR_SHAPE
    assert bf(FAKE, FAKE, 1, 1024, 1024, FAKE, 7, None, 0, None) == binding.DMR_ERR_UNSUPPORTED
    assert bf(FAKE, FAKE, 0, 1024, 1024, FAKE, 0, None, 0, None) == binding.DMR_OK   # M == 0: nothing to do
    assert bf(None, FAKE, 1, 1024, 1024, FAKE, 0, None, 0, None) == binding.DMR_ERR_NULL
    assert bf(FAKE, None, 1, 1024, 1024, FAKE, 0, None, 0, None) == binding.DMR_ERR_NULL
    assert bf(FAKE, FAKE, 1, 1024, 1024, None, 0, None, 0, None) == binding.DMR_ERR_NULL
    assert bf(FAKE, FAKE + 2, 1, 1024, 1024, FAKE, 0, None, 0, None) == binding.DMR_ERR_ALIGN
    qz = lib.dmr_qlinear_quantize
    assert qz(1024, 1024, 128, None, FAKE, FAKE, FAKE, None) == binding.DMR_ERR_NULL
    assert qz(1024, 1024, 32, FAKE, FAKE, FAKE, FAKE, None) == binding.DMR_ERR_UNSUPPORTED
    assert qz(1024, 8, 128, FAKE, FAKE, FAKE, FAKE, None) == binding.DMR_ERR_SHAPE


def test_measurement_aids_reject_bad_arguments(lib):
    # both probes check everything before their first HIP call
    pe = lib.dmr_probe_empty_launch
    for blocks, threads, lds in ((0, 256, 0), (1 << 21, 256, 0), (256, 0, 0), (256, 100, 0), (256, 2048, 0), (256, 256, 65 * 1024)):
        assert pe(blocks, threads, lds, None) == binding.DMR_ERR_SHAPE
    pr = lib.dmr_probe_hbm_read
    assert pr(None, 1 << 20, FAKE, 256, None) == binding.DMR_ERR_NULL
    assert pr(FAKE, 1 << 20, None, 256, None) == binding.DMR_ERR_NULL
    assert pr(FAKE, 0, FAKE, 256, None) == binding.DMR_ERR_SHAPE
    assert pr(FAKE, (1 << 20) + 8, FAKE, 256, None) == binding.DMR_ERR_SHAPE
    assert pr(FAKE, 1 << 20, FAKE, 0, None) == binding.DMR_ERR_SHAPE
    assert pr(FAKE + 4, 1 << 20, FAKE, 256, None) == binding.DMR_ERR_ALIGN


def test_glue_and_fused_forwards_reject_bad_arguments(lib):
    rn, sw = lib.dmr_glue_rmsnorm, lib.dmr_glue_swiglu
    assert rn(FAKE, FAKE, 1e-6, 1, 1001, FAKE, None) == binding.DMR_ERR_SHAPE          # K not a multiple of 8
    assert rn(FAKE, FAKE, 1e-6, -1, 1024, FAKE, None) == binding.DMR_ERR_SHAPE
    assert rn(FAKE, FAKE, -1.0, 1, 1024, FAKE, None) == binding.DMR_ERR_UNSUPPORTED
    assert rn(FAKE, FAKE, 1e-6, 0, 1024, FAKE, None) == binding.DMR_OK
    assert rn(FAKE, None, 1e-6, 1, 1024, FAKE, None) == binding.DMR_ERR_NULL
    assert rn(FAKE + 8, FAKE, 1e-6, 1, 1024, FAKE, None) == binding.DMR_ERR_ALIGN
    assert sw(FAKE, 1, 12, FAKE, None) == binding.DMR_ERR_SHAPE
    assert sw(None, 1, 16, FAKE, None) == binding.DMR_ERR_NULL
    assert sw(FAKE, 1, 16, FAKE + 2, None) == binding.DMR_ERR_ALIGN
    ff = lib.dmr_qlinear_forward_fused
    assert ff(None, 1, FAKE, FAKE, 1e-6, None, 1, FAKE, 0, FAKE, 1 << 30, None) == binding.DMR_ERR_NULL
    bf = lib.dmr_qlinear_bf16_forward_fused
    ok_ws = (FAKE, 1 << 30)
    assert bf(FAKE, 1, FAKE, FAKE, 1e-6, None, 1, 1000, 1024, FAKE, 0, *ok_ws, None) == binding.DMR_ERR_SHAPE
    assert bf(FAKE, 3, FAKE, FAKE, 1e-6, None, 1, 1024, 1024, FAKE, 0, *ok_ws, None) == binding.DMR_ERR_UNSUPPORTED
    assert bf(FAKE, 1, FAKE, None, 1e-6, None, 1, 1024, 1024, FAKE, 0, *ok_ws, None) == binding.DMR_ERR_NULL   # gamma
    assert bf(FAKE, 2, FAKE, None, 0.0, FAKE + 4, 1, 1024, 1024, FAKE, 0, *ok_ws, None) == binding.DMR_ERR_ALIGN
    assert bf(FAKE, 1, FAKE, FAKE, 1e-6, None, 0, 1024, 1024, FAKE, 0, None, 0, None) == binding.DMR_OK
    # a prologue or a residual needs the workspace the query names
    q = lib.dmr_qlinear_bf16_fused_workspace_bytes
    assert q(1, 4096, 4096, 0, 0) == 0
    assert q(1, 4096, 4096, 1, 0) == 8192 and q(1, 4096, 4096, 0, 1) == 16384
    assert q(5, 4096, 4096, 2, 1) == 5 * 4096 * 2 + 5 * 4096 * 4 + lib.dmr_qlinear_bf16_workspace_bytes(5, 4096, 4096)
    assert bf(FAKE, 1, FAKE, FAKE, 1e-6, None, 1, 4096, 4096, FAKE, 0, None, 0, None) == binding.DMR_ERR_WORKSPACE
    assert bf(FAKE, 1, FAKE, FAKE, 1e-6, None, 1, 4096, 4096, FAKE, 0, FAKE, 100, None) == binding.DMR_ERR_WORKSPACE
    assert lib.dmr_qlinear_fused_workspace_bytes(None, 1, 1, 0) == 0


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(TypeError):
        binding.dmr_qlinear_bf16_forward(torch.zeros(16, 128, dtype=torch.bfloat16),
                                         torch.zeros(1, 128, dtype=torch.bfloat16))


def test_w3_size_query_and_kernel_paths(lib):
    q3 = lib.dmr_qlinear_w3_workspace_bytes
    # shapes the library does not take get no workspace answer
    assert q3(8, 1000, 4096) == 0 and q3(8, 4096, 1000) == 0 and q3(0, 4096, 4096) == 0
    # decode and 2..16 rows of the decoder layers: native streaming kernels, no scratch
    assert q3(1, 4096, 4096) == 0 and q3(1, 14336, 4096) == 0 and q3(16, 4096, 28672) == 0
    # a decode row too long for the GEMV's LDS budget: the rollout-batch kernel with K split, whose fp32
    # partials need the workspace; the query must say so (the forward refuses a smaller one)
    path = lib.dmr_qlinear_kernel_path
    assert path(binding.DMR_FMT_W3_G128, 1, 32768, 528) == b"w3_mid"
    need = q3(1, 32768, 528)
    assert need > 0 and need % (528 * 4) == 0
    assert path(binding.DMR_FMT_W3_G128, 1, 4096, 4096) == b"w3_gemv"
    # the rollout-batch sizes share the 4-bit plan
    assert q3(64, 4096, 4096) == lib.dmr_qlinear_workspace_bytes(64, 4096, 4096)
    # the tiled kernels, with the 4-bit kernels' workspace
    assert path(binding.DMR_FMT_W3_G128, 200, 256, 19200) == b"w3_gemm256x128_rescale"
    assert path(binding.DMR_FMT_W3_G128, 1200, 512, 4096) == b"w3_gemm256x128_rescale"
    assert path(binding.DMR_FMT_W3_G128, 8192, 4096, 28672) == b"w3_gemm256_rescale"
    assert q3(1200, 512, 4096) == lib.dmr_qlinear_workspace_bytes(1200, 512, 4096) > 0
    # the kernel classes of the four decoder shapes at the sizes of the benchmark configurations
    assert path(binding.DMR_FMT_W4_G128, 1, 4096, 28672) == b"w4_gemv"
    assert path(binding.DMR_FMT_W4_G128, 8, 14336, 4096) == b"w4_panel"
    assert path(binding.DMR_FMT_W4_G128, 64, 4096, 28672) == b"w4_wide"
    assert path(binding.DMR_FMT_W4_G128, 64, 4096, 4096) == b"w4_mid"
    assert path(binding.DMR_FMT_W4_G128, 8192, 4096, 28672) == b"w4_gemm256_rescale"
    assert path(binding.DMR_FMT_W4_G128, 2048, 4096, 4096) == b"w4_gemm256x128_rescale"     # 128 tiles of 256 x 256 only
    assert path(binding.DMR_FMT_W4_PER_CHANNEL, 6400, 512, 1024) == b"w4_gemm256x128_rescale"
    assert path(binding.DMR_FMT_W4_G128, 200, 256, 19200) == b"w4_gemm256x128_rescale"      # a half-empty row tile
    assert path(binding.DMR_FMT_W4_G128, 1024, 4096, 4096) == b"w4_gemm128_rescale"         # 256 blocks of 128 x 128: one round
    assert path(binding.DMR_FMT_W3_G128, 768, 14336, 4096) == b"w3_gemm128_rescale"
    assert path(binding.DMR_FMT_W4_G128, 512, 4096, 4096) == b"w4_mid"                      # 128 blocks: too few
    # the 256-row kernels keep their zero-point operands, rescale factors and flags in the workspace
    G_n, KP = 4096 // 128, 192
    need = lib.dmr_qlinear_workspace_bytes(8192, 4096, 28672)
    assert need >= 8192 * KP * 2 + 28672 * KP * 2 + 28672 * (G_n + 1) * 4 + (28672 // 32) * 4
    assert need <= 1.01 * (8192 * KP * 2 + 28672 * KP * 2 + 28672 * (G_n + 1) * 4 + (28672 // 32) * 4) + 2048
    assert lib.dmr_qlinear_workspace_bytes(200, 256, 19200) > 0
    assert path(binding.DMR_FMT_W4_G128, 1, 32768, 528) == b"w4_skinny"
    assert path(binding.DMR_FMT_BF16, 1, 32768, 528) == b"bf16_skinny"
    assert path(binding.DMR_FMT_BF16, 512, 4096, 4096) == b"bf16_mid"          # exactly 128 workgroups: not tiled yet
    assert path(binding.DMR_FMT_BF16, 1024, 4096, 4096) == b"bf16_gemm128_dma"
    assert path(binding.DMR_FMT_BF16, 8192, 4096, 4096) == b"bf16_gemm256"
    assert path(binding.DMR_FMT_W4_G128, 4, 1000, 4096) == b"none"
