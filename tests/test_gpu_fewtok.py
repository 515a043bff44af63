"""GPU parity of the few-token (M <= 16) streaming path: forward and input gradient at 1, 4 and 16
tokens on LLaMA-65B-shaped linears (every output element is checked), plus ragged small shapes."""
import numpy as np
import pytest
import torch

from gpu_util import dev_bf16, download_quant, host_bits, upload_quant
from test_gpu_linear import _check, _run_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,h,o,r", [(1, 64, 64, 0), (3, 192, 320, 16), (7, 448, 192, 32), (16, 1024, 1024, 16),
                                      (5, 2048, 64, 64), (16, 64, 2048, 64), (2, 4160, 4224, 16), (9, 320, 448, 256),
                                      (16, 2112, 8256, 144)])
def test_fewtok_small_shapes(oracle, synth, M, h, o, r):
    import paper_2305_14314_amd as ql
    L = synth.make_layer(0, 0, M=M, h=h, o=o, r=max(r, 16))
    _run_case(oracle, ql, L, f"few M={M} h={h} o={o} r={r}", with_lora=r > 0)


@pytest.mark.parametrize("layer", [0, 4, 6])
def test_fewtok_65b_shapes(oracle, synth, layer):
    """Workload 4: 65B-shaped linears at 1, 4 and 16 tokens, forward and dX, all outputs checked."""
    import paper_2305_14314_amd as ql
    cfg = synth.CONFIGS[4]
    h, o = cfg["linears"][layer]
    r, s = cfg["r"], cfg["alpha"] / cfg["r"]
    Wd = synth.normal_f32_device((h, o), synth.SIGMA_W, synth.tensor_seed(4, layer, "W"))
    Wq = ql.qlora_nf4_quantize(Wd)
    del Wd
    q = download_quant(Wq)
    What = oracle.nf4_dequant(q)
    hL1 = synth.normal_bf16((h, r), cfg["sigma_l"], synth.tensor_seed(4, layer, "L1"))
    hL2 = synth.normal_bf16((r, o), cfg["sigma_l"], synth.tensor_seed(4, layer, "L2"))
    L1, L2 = dev_bf16(hL1), dev_bf16(hL2)
    for M in cfg["M"]:
        print(f"case 65b layer{layer} M={M}: h={h} o={o}", flush=True)
        hX = synth.normal_bf16((M, h), 1.0, synth.tensor_seed(4, layer, "X") + M)
        hdY = synth.normal_bf16((M, o), 1.0, synth.tensor_seed(4, layer, "dY") + M)
        Y = ql.qlora_linear_fwd(dev_bf16(hX), Wq, L1, L2, s)
        dX, _, _ = ql.qlora_linear_bwd(dev_bf16(hdY), None, Wq, L1, L2, s, need_dL=False)
        torch.cuda.synchronize()
        _check(host_bits(Y), oracle.linear_fwd(hX, What, hL1, hL2, s), f"M={M} Y")
        _check(host_bits(dX), oracle.linear_bwd_dx(hdY, What, hL1, hL2, s), f"M={M} dX")


def test_fewtok_graph_replay(synth):
    """The few-token path under HIP graph capture (how a decode loop would run it): every replay, with eager
    work and synchronisations in between, reproduces the eager result bit for bit."""
    import paper_2305_14314_amd as ql
    M, h, o, r, s = 4, 2048, 2304, 16, 0.5
    W = synth.normal_f32_device((h, o), synth.SIGMA_W, 99)
    Wq = ql.qlora_nf4_quantize(W)
    L1 = dev_bf16(synth.normal_bf16((h, r), 0.05, 100))
    L2 = dev_bf16(synth.normal_bf16((r, o), 0.05, 101))
    X = dev_bf16(synth.normal_bf16((M, h), 1.0, 102))
    dY = dev_bf16(synth.normal_bf16((M, o), 1.0, 103))
    ws = ql.workspace_alloc(max(ql.qlora_linear_fwd_sizes(M, h, o, r), ql.qlora_linear_bwd_sizes(M, h, o, r)))
    hdr = ql.binding.WORKSPACE_HEADER_BYTES
    Y0 = ql.qlora_linear_fwd(X, Wq, L1, L2, s, workspace=ws)
    dX0, _, _ = ql.qlora_linear_bwd(dY, None, Wq, L1, L2, s, need_dL=False, workspace=ws)
    torch.cuda.synchronize()
    Y = torch.empty_like(Y0)
    dX = torch.empty_like(dX0)

    def step():
        ql.qlora_linear_fwd(X, Wq, L1, L2, s, Y=Y, workspace=ws)
        ql.qlora_linear_bwd(dY, None, Wq, L1, L2, s, dX=dX, need_dL=False, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for it in range(4):
        Y.fill_(0)
        dX.fill_(0)
        ws[hdr:].random_(0, 255)                             # stale contents behind the counter header must not matter
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), Y0.view(torch.int16)), f"replay {it}: Y differs"
        assert torch.equal(dX.view(torch.int16), dX0.view(torch.int16)), f"replay {it}: dX differs"
        assert int(ws[:hdr].max()) == 0, "arrival counters are not back at zero"


def test_fewtok_counters_reset_and_repeat(oracle, synth):
    """Repeated calls on one workspace, shapes and ranks changing in between (so slab and split counts differ):
    every call starts from, and returns to, a zero counter header, and results are reproducible bit for bit."""
    import paper_2305_14314_amd as ql
    hdr = ql.binding.WORKSPACE_HEADER_BYTES
    shapes = [(16, 1024, 1024, 16), (1, 4160, 4224, 64), (5, 192, 8256, 0), (16, 1024, 1024, 16), (3, 8256, 192, 32)]
    ws = ql.workspace_alloc(max(max(ql.qlora_linear_fwd_sizes(M, h, o, r), ql.qlora_linear_bwd_sizes(M, h, o, r))
                                for M, h, o, r in shapes))
    first = {}
    for rep in range(2):
        for si, (M, h, o, r) in enumerate(shapes):
            print(f"case repeat rep={rep} M={M} h={h} o={o} r={r}", flush=True)
            W = synth.normal_f32_device((h, o), synth.SIGMA_W, 500 + si)
            Wq = ql.qlora_nf4_quantize(W)
            L1 = dev_bf16(synth.normal_bf16((h, r), 0.05, 600 + si)) if r else None
            L2 = dev_bf16(synth.normal_bf16((r, o), 0.05, 700 + si)) if r else None
            X = dev_bf16(synth.normal_bf16((M, h), 1.0, 800 + si))
            dY = dev_bf16(synth.normal_bf16((M, o), 1.0, 900 + si))
            Y = ql.qlora_linear_fwd(X, Wq, L1, L2, 0.25, workspace=ws)
            dX, _, _ = ql.qlora_linear_bwd(dY, None, Wq, L1, L2, 0.25, need_dL=False, workspace=ws)
            torch.cuda.synchronize()
            assert int(ws[:hdr].max()) == 0, "arrival counters are not back at zero"
            key = (si, "Y"), (si, "dX")
            if rep == 0:
                first[key[0]], first[key[1]] = Y.clone(), dX.clone()
            else:
                assert torch.equal(Y.view(torch.int16), first[key[0]].view(torch.int16))
                assert torch.equal(dX.view(torch.int16), first[key[1]].view(torch.int16))
