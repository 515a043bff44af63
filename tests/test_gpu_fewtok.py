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


@pytest.mark.parametrize("M,n", [(1, 3), (5, 3), (16, 3), (3, 1), (8, 4), (16, 2)])
def test_multi_layer_forward_small(oracle, synth, M, n):
    """Several layers on one input in one launch: one to four layers of different widths, one of them without an
    adapter, one with rank 64; every output element against the oracle; the counter header is zero afterwards."""
    import paper_2305_14314_amd as ql
    h = 1024
    outs, ranks, ss = [1024, 320, 2304, 64][:n], [16, 0, 64, 32][:n], [0.5, 1.0, 0.25, 2.0][:n]
    hX = synth.normal_bf16((M, h), 1.0, 4000 + M)
    X = dev_bf16(hX)
    Wqs, L1s, L2s, refs = [], [], [], []
    for l, (o, r) in enumerate(zip(outs, ranks)):
        W = synth.normal_f32((h, o), synth.SIGMA_W, 4100 + l)
        q = oracle.nf4_quantize(W)
        Wqs.append(upload_quant(q))
        hL1 = synth.normal_bf16((h, r), 0.05, 4200 + l) if r else None
        hL2 = synth.normal_bf16((r, o), 0.05, 4300 + l) if r else None
        L1s.append(dev_bf16(hL1) if r else None)
        L2s.append(dev_bf16(hL2) if r else None)
        refs.append(oracle.linear_fwd(hX, oracle.nf4_dequant(q), hL1, hL2, ss[l]))
    ws = ql.workspace_alloc(ql.qlora_linear_fwd_multi_sizes(M, h, outs, ranks))
    print(f"case multi M={M} h={h} o={outs} r={ranks}", flush=True)
    Ys = ql.qlora_linear_fwd_multi(X, Wqs, L1s, L2s, ss, workspace=ws)
    torch.cuda.synchronize()
    for l in range(len(outs)):
        _check(host_bits(Ys[l]), refs[l], f"multi M={M} layer {l} Y")
    assert int(ws[:ql.binding.WORKSPACE_HEADER_BYTES].max()) == 0, "arrival counters are not back at zero"
    # twice in a row on the same workspace: bit for bit the same
    Ys2 = ql.qlora_linear_fwd_multi(X, Wqs, L1s, L2s, ss, workspace=ws)
    torch.cuda.synchronize()
    for a, b in zip(Ys, Ys2):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_multi_layer_forward_many_tokens_is_the_single_layer_path(synth):
    """Above 16 tokens the layers run one after the other through qlora_linear_fwd: identical bits."""
    import paper_2305_14314_amd as ql
    M, h, outs, ranks, ss = 96, 512, [512, 192], [16, 32], [0.5, 2.0]
    X = dev_bf16(synth.normal_bf16((M, h), 1.0, 5000))
    Wqs = [ql.qlora_nf4_quantize(synth.normal_f32_device((h, o), synth.SIGMA_W, 5100 + l)) for l, o in enumerate(outs)]
    L1s = [dev_bf16(synth.normal_bf16((h, r), 0.05, 5200 + l)) for l, r in enumerate(ranks)]
    L2s = [dev_bf16(synth.normal_bf16((r, o), 0.05, 5300 + l)) for l, (r, o) in enumerate(zip(ranks, outs))]
    Ys = ql.qlora_linear_fwd_multi(X, Wqs, L1s, L2s, ss)
    torch.cuda.synchronize()
    for l in range(2):
        Y1 = ql.qlora_linear_fwd(X, Wqs[l], L1s[l], L2s[l], ss[l])
        torch.cuda.synchronize()
        assert torch.equal(Ys[l].view(torch.int16), Y1.view(torch.int16))


@pytest.mark.parametrize("group", ["qkv", "gate_up"])
def test_multi_layer_forward_65b_groups(oracle, synth, group):
    """The groups of a 65B-shaped decoder block that share their input -- q / k / v (3 x 8192 x 8192) and gate / up
    (2 x 8192 x 22016) -- at 1 and 16 tokens, r = 64: every output element of every layer against the oracle."""
    import paper_2305_14314_amd as ql
    cfg = synth.CONFIGS[4]
    r, s = cfg["r"], cfg["alpha"] / cfg["r"]
    h, o, n = (8192, 8192, 3) if group == "qkv" else (8192, 22016, 2)
    Wqs, Whats, hL1, hL2 = [], [], [], []
    for l in range(n):
        Wd = synth.normal_f32_device((h, o), synth.SIGMA_W, 6000 + 10 * l + (0 if group == "qkv" else 5))
        Wqs.append(ql.qlora_nf4_quantize(Wd))
        del Wd
        Whats.append(oracle.nf4_dequant(download_quant(Wqs[-1])))
        hL1.append(synth.normal_bf16((h, r), cfg["sigma_l"], 6100 + l))
        hL2.append(synth.normal_bf16((r, o), cfg["sigma_l"], 6200 + l))
    L1s, L2s = [dev_bf16(a) for a in hL1], [dev_bf16(a) for a in hL2]
    for M in (1, 16):
        print(f"case multi {group} M={M}", flush=True)
        hX = synth.normal_bf16((M, h), 1.0, 6300 + M)
        Ys = ql.qlora_linear_fwd_multi(dev_bf16(hX), Wqs, L1s, L2s, [s] * n)
        torch.cuda.synchronize()
        for l in range(n):
            _check(host_bits(Ys[l]), oracle.linear_fwd(hX, Whats[l], hL1[l], hL2[l], s), f"{group} M={M} layer {l} Y")
