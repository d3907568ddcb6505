"""dmr_qlinear_forward_static (the forward on the library's own fixed scratch, for callers that cannot
allocate) against dmr_qlinear_forward with a caller workspace: same kernels, so the outputs must agree bit
for bit, on calls in a row that share the scratch, the later ones with smaller inputs."""
import numpy as np
import pytest
import torch

import paper_2602_02711_amd as dmr
from oracle import cpu_oracle as orc
from paper_2602_02711_amd import binding, synth

from gpu_util import bf16_dev, quantized, quantized3, rel_err, u32_dev

pytestmark = pytest.mark.gpu
G = synth.GROUP
DEV = "cuda:0"


def test_forward_static_matches_forward_on_consecutive_calls():
    K, N = 4096, 4096
    _, words, s, z = quantized(9700, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    # 64 rows: K split four ways, 4 MiB of fp32 partials; then 17 rows (1 MiB) on the same scratch; then a
    # smaller layer, a 3-bit layer, and a decode row that needs no scratch at all
    calls = [(layer, 64), (layer, 17)]
    _, w2, s2, z2 = quantized(9701, 1024, 1024)
    calls.append((dmr.dmr_qlinear_create(u32_dev(w2), bf16_dev(s2), bf16_dev(z2), G), 40))
    _, w3, s3, z3 = quantized3(9702, 4096, 4096)
    calls.append((dmr.dmr_qlinear_w3_create(u32_dev(w3), bf16_dev(s3), bf16_dev(z3), G), 33))
    calls.append((layer, 1))
    # the tiled path keeps its zero-point operands, factors and flags there: a layer with one zero scale (its
    # 32 columns are flagged and go to the second kernel), then the clean layer, whose flags must read clear
    Kt, Nt = 1024, 16384
    _, wt, st, zt = quantized(9703, Nt, Kt)
    sf = st.copy()
    sf[70, 3] = 0
    flagged = dmr.dmr_qlinear_create(u32_dev(wt), bf16_dev(sf), bf16_dev(zt), G)
    clean = dmr.dmr_qlinear_create(u32_dev(wt), bf16_dev(st), bf16_dev(zt), G)
    calls += [(flagged, 300), (clean, 260)]
    assert dmr.dmr_qlinear_kernel_path(dmr.DMR_FMT_W4_G128, 260, Kt, Nt).endswith("_rescale")
    xs = [bf16_dev(synth.activations_bf16(9710 + i, M, L.K)) for i, (L, M) in enumerate(calls)]
    outs = [torch.full((M, L.N), float("nan"), dtype=torch.float32, device=DEV) for L, M in calls]
    want = []
    for (L, M), x in zip(calls, xs):
        need = (dmr.dmr_qlinear_w3_workspace_bytes(M, L.K, L.N) if L.bits == 3
                else dmr.dmr_qlinear_workspace_bytes(M, L.K, L.N))
        assert need <= binding.DMR_STATIC_SCRATCH_BYTES
        want.append(dmr.dmr_qlinear_forward(L, x, out_dtype=torch.float32))
    assert dmr.dmr_qlinear_workspace_bytes(64, K, N) == 4 * 64 * N * 4      # the first call really uses the scratch
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for (L, M), x, y in zip(calls, xs, outs):                 # back to back on one stream, no sync in between
        dmr.dmr_qlinear_forward_static(L, x, out=y)
    assert torch.cuda.memory_allocated() == before            # the binding brought no workspace either
    torch.cuda.synchronize()
    for i, (y, w) in enumerate(zip(outs, want)):
        assert torch.equal(y, w), i
    # and the first result is right, not merely equal to its twin
    y_ref, _ = orc.forward(words, s, z, G, synth.activations_bf16(9710, 64, K), threads=16)
    assert rel_err(outs[0].cpu().numpy(), y_ref) <= 1e-2
    # bf16 output through the same path
    y16 = dmr.dmr_qlinear_forward_static(layer, xs[1], out_dtype=torch.bfloat16)
    assert torch.equal(y16, dmr.dmr_qlinear_forward(layer, xs[1], out_dtype=torch.bfloat16))


def test_forward_static_refuses_what_exceeds_its_scratch():
    K, N, M = 4096, 6144, 128
    assert dmr.dmr_qlinear_workspace_bytes(M, K, N) > binding.DMR_STATIC_SCRATCH_BYTES
    _, words, s, z = quantized(9720, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    x = bf16_dev(synth.activations_bf16(9721, M, K))
    y = torch.full((M, N), 3.0, dtype=torch.float32, device=DEV)
    with pytest.raises(dmr.DmrError) as err:
        dmr.dmr_qlinear_forward_static(layer, x, out=y)
    assert err.value.status == binding.DMR_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())                             # refused before anything was launched
    lib = binding.lib()
    assert lib.dmr_qlinear_forward_static(None, x.data_ptr(), M, y.data_ptr(), 1, None) == binding.DMR_ERR_NULL
    assert lib.dmr_qlinear_forward_static(layer.handle, x.data_ptr(), 0, y.data_ptr(), 1, None) == binding.DMR_OK
