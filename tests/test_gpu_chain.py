"""GPU parity of the persistent decode chain (one resident grid runs the Linear layers of a step in order,
grid barriers between them) through the C ABI.  Each stage is one fused M = 1 forward, so the chain is
checked (a) stage by stage against the CPU oracle's composition, feeding the oracle the activations the
device itself produced for the earlier stages (a bf16 residual stream amplifies one-ulp differences over
many layers, so the oracle does not run the chain open loop), and (b) end to end against the library's own
per-stage launches, which compute the same values up to the order of the fp32 additions over k."""
import numpy as np
import pytest
import torch

import paper_2602_02711_amd as dmr
from oracle import cpu_oracle as orc
from paper_2602_02711_amd import synth

from gpu_util import bf16_dev, bits_host, half_ulp_bf16, quantized, u32_dev

pytestmark = pytest.mark.gpu
G = synth.GROUP
TOL = 1e-2
EPS = 1e-6
R, S, NONE = dmr.DMR_PRO_RMSNORM, dmr.DMR_PRO_SWIGLU, dmr.DMR_PRO_NONE


def gamma_bits(seed, K):
    rng = np.random.default_rng(seed)
    return orc.f64_to_bf16(rng.uniform(0.5, 1.5, K))


class Block:
    """A decoder block's four Linear layers (hidden H, MLP width I, fused qkv width Q) on one set of buffers."""

    def __init__(self, seed, H, I, Q, layers):
        self.H, self.I, self.Q = H, I, Q
        self.host, self.dev, self.gam = [], [], []
        for li in range(layers):
            shapes = {"qkv": (H, Q), "attn_out": (H, H), "gate_up": (H, 2 * I), "down": (I, H)}
            hl, dl = {}, {}
            for si, (name, (K, N)) in enumerate(shapes.items()):
                _, words, s, z = quantized(seed + 10 * li + si, N, K)
                hl[name] = (words, s, z)
                dl[name] = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)
            self.host.append(hl)
            self.dev.append(dl)
            self.gam.append((gamma_bits(seed + 10 * li + 7, H), gamma_bits(seed + 10 * li + 8, H)))
        self.h0 = synth.activations_bf16(seed + 999, 1, H)
        dev = "cuda"
        self.buf = {"h": [torch.empty((1, H), dtype=torch.bfloat16, device=dev) for _ in range(2 * layers + 1)],
                    "qkv": [torch.empty((1, Q), dtype=torch.bfloat16, device=dev) for _ in range(layers)],
                    "gu": [torch.empty((1, 2 * I), dtype=torch.bfloat16, device=dev) for _ in range(layers)]}
        self.gdev = [(bf16_dev(a), bf16_dev(b)) for a, b in self.gam]

    def stages(self):
        """Every stage writes a buffer of its own, so that all intermediate activations can be read back."""
        out = []
        for li, L in enumerate(self.dev):
            h, h1, h2 = self.buf["h"][2 * li], self.buf["h"][2 * li + 1], self.buf["h"][2 * li + 2]
            qkv, gu = self.buf["qkv"][li], self.buf["gu"][li]
            g1, g2 = self.gdev[li]
            attn = qkv[:, :self.H]                              # attention stand-in: the q slice
            out.append(dict(layer=L["qkv"], pro=R, inp=h, gamma=g1, eps=EPS, out=qkv, name=("qkv", li)))
            out.append(dict(layer=L["attn_out"], pro=NONE, inp=attn, residual=h, out=h1, name=("attn_out", li)))
            out.append(dict(layer=L["gate_up"], pro=R, inp=h1, gamma=g2, eps=EPS, out=gu, name=("gate_up", li)))
            out.append(dict(layer=L["down"], pro=S, inp=gu, residual=h1, out=h2, name=("down", li)))
        return out

    def reset(self):
        for group in self.buf.values():
            for t in group:
                t.fill_(float("nan"))
        self.buf["h"][0].copy_(bf16_dev(self.h0))


def run_per_stage(stages):
    for st in stages:
        dmr.dmr_qlinear_forward_fused(st["layer"], st["pro"], st["inp"], gamma=st.get("gamma"), eps=st.get("eps", 0.0),
                                      residual=st.get("residual"), out=st["out"])


def oracle_stage(block, st):
    name, li = st["name"]
    words, s, z = block.host[li][name]
    inp = bits_host(st["inp"])
    if st["pro"] == R:
        g = block.gam[li][0 if name == "qkv" else 1]
        x = orc.rmsnorm(inp, g, EPS)
    elif st["pro"] == S:
        x = orc.swiglu(inp)
    else:
        x = inp
    y = orc.forward(words, s, z, G, x, threads=16)[0]
    if st.get("residual") is not None:
        y = y + orc.bf16_to_f64(bits_host(st["residual"]))
    return y


# (H, I, Q, layers): tile counts below, at and above the 256 workgroups of the grid, ragged against them
# (Q / 16 = 136, 2 I / 16 = 344), k slices of 1, 2 and 3.5 groups per wave, several passes through the ring.
SHAPES = [(2048, 2816, 2176, 2), (4096, 7168, 6144, 1), (2048, 2048, 2048, 3)]


@pytest.mark.parametrize("H,I,Q,layers", SHAPES)
def test_chain_against_oracle_and_per_stage_launches(H, I, Q, layers):
    block = Block(9100 + H + I, H, I, Q, layers)
    stages = block.stages()
    chain = dmr.dmr_chain_create(stages)
    block.reset()
    dmr.dmr_chain_forward(chain)
    assert not dmr.dmr_chain_timed_out(chain)
    got = [bits_host(st["out"]).copy() for st in stages]
    for st, y in zip(stages, got):                      # closed loop: the oracle sees the device's own inputs
        y_ref = oracle_stage(block, st)
        rms = np.sqrt(np.mean(y_ref ** 2))
        # the fp32 result within the parity tolerance, then one rounding to bf16 (half an ulp of the value)
        excess = np.abs(orc.bf16_to_f64(y) - y_ref) - half_ulp_bf16(y_ref) * 1.01
        print(f"chain stage {st['name']} ({st['layer'].K},{st['layer'].N}): max err beyond the rounding "
              f"{max(excess.max(), 0.0) / rms:.3e} rms")
        assert excess.max() <= TOL * rms, st["name"]
    block.reset()
    run_per_stage(stages)
    torch.cuda.synchronize()
    ref_final = stages[-1]["out"].float()
    rms = ref_final.pow(2).mean().sqrt().item()
    diff = (torch.from_numpy(orc.bf16_to_f64(got[-1])).to(ref_final.device).float() - ref_final).abs().max().item()
    print(f"chain vs per-stage launches, final hidden state: max diff {diff / rms:.3e} rms")
    assert diff <= 3e-2 * rms


def test_chain_repeated_and_in_a_graph():
    block = Block(9300, 2048, 2816, 2176, 2)
    stages = block.stages()
    chain = dmr.dmr_chain_create(stages)
    block.reset()
    dmr.dmr_chain_forward(chain)
    torch.cuda.synchronize()
    first = [bits_host(st["out"]).copy() for st in stages]
    for _ in range(3):                                  # deterministic: same bits every time
        block.reset()
        dmr.dmr_chain_forward(chain)
        torch.cuda.synchronize()
        assert all(np.array_equal(bits_host(st["out"]), f) for st, f in zip(stages, first))
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        dmr.dmr_chain_forward(chain, stream)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            dmr.dmr_chain_forward(chain, stream)
            dmr.dmr_chain_forward(chain, stream)
    for _ in range(3):
        block.reset()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(np.array_equal(bits_host(st["out"]), f) for st, f in zip(stages, first))
    assert not dmr.dmr_chain_timed_out(chain)


def test_chain_time_out_path_drains():
    # a barrier that gives up at the first unsuccessful poll: the launch must still end, with the flag set
    block = Block(9400, 2048, 2048, 2048, 2)
    chain = dmr.dmr_chain_create(block.stages())
    dmr.dmr_chain_set_spin_limit(chain, 0)
    block.reset()
    dmr.dmr_chain_forward(chain)
    torch.cuda.synchronize()
    assert dmr.dmr_chain_timed_out(chain)


def test_chain_rejects_what_it_does_not_take():
    _, words, s, z = quantized(9500, 64, 1024)
    small = dmr.dmr_qlinear_create(u32_dev(words), bf16_dev(s), bf16_dev(z), G)      # K = 1024: under 16 groups
    x = torch.zeros((1, 1024), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((1, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(dmr.DmrError) as e:
        dmr.dmr_chain_create([dict(layer=small, pro=NONE, inp=x, out=y)])
    assert e.value.status == 5
    with pytest.raises(dmr.DmrError):
        dmr.dmr_chain_create([])
