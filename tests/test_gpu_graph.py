"""HIP-graph capture of the forwards (how bench.py launches them): every replay must reproduce the
eager result bit for bit, also with eager work of the same library between the replays and with the
kernels that use a workspace (split of K and its reduction pass, the activation pre-pass)."""
import pytest
import torch

import paper_2602_02711_amd as dmr
from paper_2602_02711_amd import synth

from gpu_util import bf16_dev, quantized, u32_dev

pytestmark = pytest.mark.gpu
G = synth.GROUP


@pytest.mark.parametrize("K,N,M", [(4096, 4096, 1), (4096, 4096, 8), (1024, 1024, 40), (4096, 4096, 128),
                                   (4096, 28672, 48), (512, 1024, 6400), (4096, 28672, 16), (14336, 4096, 8),
                                   (1024, 6400, 4000), (2048, 4096, 1024)])
def test_graph_replays_match_eager(K, N, M):
    _, words, s, z = quantized(9000 + K + N, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    wb = bf16_dev(synth.to_bf16_bits(synth.weights_f32(9001 + K + N, N, K)))
    xs = [bf16_dev(synth.activations_bf16(9002 + i, M, K)) for i in range(2)]
    x = xs[0].clone()
    ws4 = torch.empty(max(dmr.dmr_qlinear_workspace_bytes(M, K, N), 16), dtype=torch.uint8, device="cuda:0")
    ws16 = torch.empty(max(dmr.dmr_qlinear_bf16_workspace_bytes(M, K, N), 16), dtype=torch.uint8, device="cuda:0")
    y4 = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    y16 = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    eager = []
    for xi in xs:
        eager.append((dmr.dmr_qlinear_forward(layer, xi, out_dtype=torch.float32).clone(),
                      dmr.dmr_qlinear_bf16_forward(wb, xi, out_dtype=torch.float32).clone()))
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()        # what ran on the default stream so far shares buffers with what follows
    with torch.cuda.stream(stream):
        dmr.dmr_qlinear_forward(layer, x, out=y4, workspace=ws4)            # warm-up outside the capture
        dmr.dmr_qlinear_bf16_forward(wb, x, out=y16, workspace=ws16)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            dmr.dmr_qlinear_forward(layer, x, out=y4, workspace=ws4)
            dmr.dmr_qlinear_bf16_forward(wb, x, out=y16, workspace=ws16)
        for rep in range(4):
            x.copy_(xs[rep % 2])                                           # new input, same buffers
            y4.fill_(float("nan"))
            y16.fill_(float("nan"))
            graph.replay()
            stream.synchronize()
            assert torch.equal(y4, eager[rep % 2][0]), rep
            assert torch.equal(y16, eager[rep % 2][1]), rep
            # eager work of the library between replays, sharing the workspace
            other = dmr.dmr_qlinear_forward(layer, xs[(rep + 1) % 2], out_dtype=torch.float32, workspace=ws4)
            stream.synchronize()
            assert torch.equal(other, eager[(rep + 1) % 2][0]), rep


def test_graph_replays_fused_chain_link():
    K, N = 4096, 4096
    _, words, s, z = quantized(9100, N, K)
    layer = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
    gamma = bf16_dev(synth.to_bf16_bits(1.0 + 5.0 * synth.weights_f32(9101, 1, K)).reshape(K))
    x = bf16_dev(synth.activations_bf16(9102, 1, K))
    res = bf16_dev(synth.activations_bf16(9103, 1, N))
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    y = torch.empty((1, N), dtype=torch.bfloat16, device="cuda:0")
    want = dmr.dmr_qlinear_forward_fused(layer, dmr.DMR_PRO_RMSNORM, x, gamma=gamma, eps=1e-6, residual=res,
                                         workspace=ws).clone()
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()        # what ran on the default stream so far shares buffers with what follows
    with torch.cuda.stream(stream):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            dmr.dmr_qlinear_forward_fused(layer, dmr.DMR_PRO_RMSNORM, x, gamma=gamma, eps=1e-6, residual=res, out=y,
                                          workspace=ws)
        for rep in range(3):
            y.zero_()
            graph.replay()
            stream.synchronize()
            assert torch.equal(y, want), rep
