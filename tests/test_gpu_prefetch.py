"""The decode-step hint dmr_qlinear_set_next must change nothing but timing: an M = 1 forward of a layer with a
named successor (plain and fused) returns bit for bit what it returns without one, for every pairing of the
decoder's layer shapes, a successor of another format, and the layer named as its own successor; and the result
matches the oracle."""
import numpy as np
import pytest
import torch

import paper_2602_02711_amd as dmr
from oracle import cpu_oracle as orc
from paper_2602_02711_amd import synth

from gpu_util import bf16_dev, quantized, quantized3, rel_err, u32_dev

pytestmark = pytest.mark.gpu
G = synth.GROUP


def test_successor_hint_leaves_results_unchanged():
    shapes = list(synth.SWEEP_SHAPES) + [("small", 1024, 1024), ("odd", 640, 272)]
    layers, xs, refs = [], [], []
    for i, (name, K, N) in enumerate(shapes):
        _, words, s, z = quantized(9800 + i, N, K)
        layers.append(dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G))
        x = synth.activations_bf16(9850 + i, 1, K)
        xs.append(bf16_dev(x))
        refs.append(orc.forward(words, s, z, G, x, threads=16)[0])
    _, w3, s3, z3 = quantized3(9890, 1024, 1024)
    other = dmr.dmr_qlinear_w3_create(u32_dev(w3), bf16_dev(s3), bf16_dev(z3), G)
    plain = [dmr.dmr_qlinear_forward(L, x, out_dtype=torch.float32).clone() for L, x in zip(layers, xs)]
    for L, y, ref in zip(layers, plain, refs):
        assert rel_err(y.cpu().numpy(), ref) <= 1e-2
    gamma = bf16_dev(synth.to_bf16_bits(1.0 + 5.0 * synth.weights_f32(9891, 1, 4096)).reshape(4096))
    res = bf16_dev(synth.activations_bf16(9892, 1, 4096))
    fused_plain = dmr.dmr_qlinear_forward_fused(layers[0], dmr.DMR_PRO_RMSNORM, xs[0], gamma=gamma, eps=1e-6,
                                                residual=res, out_dtype=torch.float32).clone()
    for i, L in enumerate(layers):
        for nxt in layers + [other, L]:
            dmr.dmr_qlinear_set_next(L, nxt)
            for rep in range(2):
                y = dmr.dmr_qlinear_forward(L, xs[i], out_dtype=torch.float32)
                assert torch.equal(y, plain[i]), (shapes[i][0], rep)
            if i == 0:
                yf = dmr.dmr_qlinear_forward_fused(L, dmr.DMR_PRO_RMSNORM, xs[0], gamma=gamma, eps=1e-6, residual=res,
                                                   out_dtype=torch.float32)
                assert torch.equal(yf, fused_plain)
        dmr.dmr_qlinear_set_next(L, None)
        assert torch.equal(dmr.dmr_qlinear_forward(L, xs[i], out_dtype=torch.float32), plain[i])
    # more rows than one: the hint is ignored
    dmr.dmr_qlinear_set_next(layers[0], layers[1])
    x8 = bf16_dev(synth.activations_bf16(9893, 8, 4096))
    a = dmr.dmr_qlinear_forward(layers[0], x8, out_dtype=torch.float32)
    dmr.dmr_qlinear_set_next(layers[0], None)
    assert torch.equal(a, dmr.dmr_qlinear_forward(layers[0], x8, out_dtype=torch.float32))
