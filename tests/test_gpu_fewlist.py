"""GPU parity of the few-token list kernels (one persistent launch for several independent layers): forward and
input gradient against the fp64 oracle, every output element; the counter header's protocol (back to zero, dirty
headers reported, the hand-over path of the output stage); HIP-graph replay."""
import numpy as np
import pytest
import torch

from gpu_util import dev_bf16, download_quant, host_bits, upload_quant
from test_gpu_linear import _check

pytestmark = pytest.mark.gpu

HDR = 16384


def _make_list(oracle, synth, M, shapes, seed):
    """shapes: [(h, o, r)]; returns device and host operands of every layer plus the oracle's dequantised weights."""
    layers = []
    for l, (h, o, r) in enumerate(shapes):
        W = synth.normal_f32((h, o), synth.SIGMA_W, seed + 10 * l)
        q = oracle.nf4_quantize(W)
        hL1 = synth.normal_bf16((h, r), 0.05, seed + 10 * l + 1) if r else None
        hL2 = synth.normal_bf16((r, o), 0.05, seed + 10 * l + 2) if r else None
        hX = synth.normal_bf16((M, h), 1.0, seed + 10 * l + 3)
        hdY = synth.normal_bf16((M, o), 1.0, seed + 10 * l + 4)
        layers.append(dict(h=h, o=o, r=r, Wq=upload_quant(q), What=oracle.nf4_dequant(q), hL1=hL1, hL2=hL2, hX=hX, hdY=hdY,
                           L1=dev_bf16(hL1) if r else None, L2=dev_bf16(hL2) if r else None, X=dev_bf16(hX),
                           dY=dev_bf16(hdY), s=[0.5, 1.0, 0.25, 2.0][l % 4]))
    return layers


def _run_list(ql, layers, backward, ws=None):
    ins = [y["dY"] if backward else y["X"] for y in layers]
    fn = ql.qlora_linear_bwd_list if backward else ql.qlora_linear_fwd_list
    return fn(ins, [y["Wq"] for y in layers], [y["L1"] for y in layers], [y["L2"] for y in layers],
              [y["s"] for y in layers], workspace=ws)


def _check_list(oracle, layers, outs, backward, tag):
    for l, (y, got) in enumerate(zip(layers, outs)):
        if backward:
            ref = oracle.linear_bwd_dx(y["hdY"], y["What"], y["hL1"], y["hL2"], y["s"])
        else:
            ref = oracle.linear_fwd(y["hX"], y["What"], y["hL1"], y["hL2"], y["s"])
        _check(host_bits(got), ref, f"{tag} layer {l} {'dX' if backward else 'Y'}")


SMALL = [
    (1, [(64, 64, 0)]),
    (3, [(192, 320, 16), (448, 192, 32)]),
    (8, [(1024, 1024, 16), (1024, 320, 0), (1024, 2304, 64), (1024, 64, 32)]),
    (9, [(320, 448, 256), (2048, 64, 64)]),
    (16, [(64, 2048, 64), (2112, 8256, 144), (4160, 4224, 16)]),
    (5, [(512, 512, 16)] * 8),
    (16, [(8256, 192, 32), (192, 8256, 0), (1088, 1088, 48)]),
]


@pytest.mark.parametrize("case", range(len(SMALL)))
@pytest.mark.parametrize("backward", [False, True])
def test_list_small_shapes(oracle, synth, case, backward):
    """Lists of one to eight layers with different shapes, ranks (some without an adapter) and scales, ragged
    against the 256-wide slabs and the 16-row / 128-column units: every output element; the header is zero afterwards
    and the status word clear; a second call on the same workspace gives the same bits."""
    import paper_2305_14314_amd as ql
    M, shapes = SMALL[case]
    layers = _make_list(oracle, synth, M, shapes, 7000 + 100 * case)
    ws = ql.workspace_alloc(ql.qlora_linear_list_sizes(M, [s[0] for s in shapes], [s[1] for s in shapes],
                                                       [s[2] for s in shapes], backward))
    print(f"case list {'bwd' if backward else 'fwd'} M={M} shapes={shapes}", flush=True)
    outs = _run_list(ql, layers, backward, ws)
    torch.cuda.synchronize()
    _check_list(oracle, layers, outs, backward, f"list M={M}")
    assert int(ws[:HDR].max()) == 0, "arrival words are not back at zero"
    assert ql.qlora_workspace_check(ws)
    ws[HDR:].random_(0, 255)                                  # stale contents behind the header must not matter
    outs2 = _run_list(ql, layers, backward, ws)
    torch.cuda.synchronize()
    for a, b in zip(outs, outs2):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("M", [1, 16])
def test_list_65b_block(oracle, synth, M):
    """Workload 4 as one list: the seven linears of a 65B-shaped block (r = 64) at 1 and 16 tokens, forward and input
    gradient, every output element of every layer against the oracle."""
    import paper_2305_14314_amd as ql
    cfg = synth.CONFIGS[4]
    r, s = cfg["r"], cfg["alpha"] / cfg["r"]
    layers = []
    for l, (h, o) in enumerate(cfg["linears"]):
        Wd = synth.normal_f32_device((h, o), synth.SIGMA_W, synth.tensor_seed(4, l, "W") + 77)
        Wq = ql.qlora_nf4_quantize(Wd)
        del Wd
        hL1 = synth.normal_bf16((h, r), cfg["sigma_l"], synth.tensor_seed(4, l, "L1") + 77)
        hL2 = synth.normal_bf16((r, o), cfg["sigma_l"], synth.tensor_seed(4, l, "L2") + 77)
        hX = synth.normal_bf16((M, h), 1.0, synth.tensor_seed(4, l, "X") + 77 + M)
        hdY = synth.normal_bf16((M, o), 1.0, synth.tensor_seed(4, l, "dY") + 77 + M)
        layers.append(dict(h=h, o=o, r=r, Wq=Wq, What=None, hL1=hL1, hL2=hL2, hX=hX, hdY=hdY, L1=dev_bf16(hL1),
                           L2=dev_bf16(hL2), X=dev_bf16(hX), dY=dev_bf16(hdY), s=s))
    print(f"case list 65b block M={M}", flush=True)
    Ys = _run_list(ql, layers, False)
    dXs = _run_list(ql, layers, True)
    torch.cuda.synchronize()
    for l, y in enumerate(layers):                            # one layer's dequantised weight at a time on the host
        What = oracle.nf4_dequant(download_quant(y["Wq"]))
        _check(host_bits(Ys[l]), oracle.linear_fwd(y["hX"], What, y["hL1"], y["hL2"], s), f"65b list M={M} layer {l} Y")
        _check(host_bits(dXs[l]), oracle.linear_bwd_dx(y["hdY"], What, y["hL1"], y["hL2"], s), f"65b list M={M} layer {l} dX")
        del What


@pytest.mark.parametrize("config,M", [(1, 4), (2, 16)])
def test_list_7b_13b_blocks(oracle, synth, config, M):
    """The seven linears of the 7B- and 13B-shaped blocks (d = 4096 / 5120, ffn = 11008 / 13824: 43 and 54 slabs, the
    contraction of `down` ragged against the 1024-element adapter chunks) as one list, forward and input gradient, every
    output element."""
    import paper_2305_14314_amd as ql
    cfg = synth.CONFIGS[config]
    r, s = cfg["r"], cfg["alpha"] / cfg["r"]
    layers = []
    for l, (h, o) in enumerate(cfg["linears"]):
        Wd = synth.normal_f32_device((h, o), synth.SIGMA_W, synth.tensor_seed(config, l, "W") + 55)
        Wq = ql.qlora_nf4_quantize(Wd)
        del Wd
        hL1 = synth.normal_bf16((h, r), cfg["sigma_l"], synth.tensor_seed(config, l, "L1") + 55)
        hL2 = synth.normal_bf16((r, o), cfg["sigma_l"], synth.tensor_seed(config, l, "L2") + 55)
        hX = synth.normal_bf16((M, h), 1.0, synth.tensor_seed(config, l, "X") + 55 + M)
        hdY = synth.normal_bf16((M, o), 1.0, synth.tensor_seed(config, l, "dY") + 55 + M)
        layers.append(dict(h=h, o=o, r=r, Wq=Wq, What=None, hL1=hL1, hL2=hL2, hX=hX, hdY=hdY, L1=dev_bf16(hL1),
                           L2=dev_bf16(hL2), X=dev_bf16(hX), dY=dev_bf16(hdY), s=s))
    print(f"case list {cfg['name']} M={M}", flush=True)
    Ys = _run_list(ql, layers, False)
    dXs = _run_list(ql, layers, True)
    torch.cuda.synchronize()
    for l, y in enumerate(layers):
        What = oracle.nf4_dequant(download_quant(y["Wq"]))
        _check(host_bits(Ys[l]), oracle.linear_fwd(y["hX"], What, y["hL1"], y["hL2"], s), f"{cfg['name']} M={M} layer {l} Y")
        _check(host_bits(dXs[l]), oracle.linear_bwd_dx(y["hdY"], What, y["hL1"], y["hL2"], s), f"{cfg['name']} M={M} layer {l} dX")
        del What


@pytest.mark.parametrize("backward", [False, True])
def test_list_output_stage_handed_to_the_adapter(oracle, synth, backward):
    """Poll limit 0: a slab's last contributor never waits for the adapter's partial sums, so wherever they are not in
    yet the adapter's workgroups run the output stage.  Same bits as the default path, header back at zero."""
    import paper_2305_14314_amd as ql
    M, shapes = 4, [(2048, 2304, 64), (1024, 512, 16), (512, 4096, 32)]
    layers = _make_list(oracle, synth, M, shapes, 8100)
    ws = ql.workspace_alloc(ql.qlora_linear_list_sizes(M, [s[0] for s in shapes], [s[1] for s in shapes],
                                                       [s[2] for s in shapes], backward))
    ref = _run_list(ql, layers, backward, ws)
    torch.cuda.synchronize()
    _check_list(oracle, layers, ref, backward, "default polls")
    try:
        ql.qlora_fewtok_poll_limit(0)
        print(f"case list poll limit 0 {'bwd' if backward else 'fwd'}", flush=True)
        for rep in range(3):
            got = _run_list(ql, layers, backward, ws)
            torch.cuda.synchronize()
            for a, b in zip(ref, got):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"rep {rep}"
            assert int(ws[:HDR].max()) == 0
            assert ql.qlora_workspace_check(ws)
    finally:
        ql.qlora_fewtok_poll_limit(64)


@pytest.mark.parametrize("dirt", ["big count", "one bit", "foreign tag", "handshake"])
def test_list_dirty_header_is_reported(oracle, synth, dirt):
    """A counter header that is not zero on entry: every kernel still exits, the status word is raised and
    qlora_workspace_check reports it; after qlora_workspace_init the same call is right again."""
    import paper_2305_14314_amd as ql
    M, shapes = 2, [(1024, 1024, 16), (2048, 512, 32)]
    layers = _make_list(oracle, synth, M, shapes, 8200)
    ws = ql.workspace_alloc(ql.qlora_linear_list_sizes(M, [s[0] for s in shapes], [s[1] for s in shapes],
                                                       [s[2] for s in shapes], False))
    words = ws[:HDR].view(torch.int32)
    assert ql.qlora_workspace_check(ws)
    if dirt == "big count":
        words[1] = 0x00ffffff
    elif dirt == "one bit":
        words[0] = 1                                          # as if contributor 0 of slab 0 had arrived already
    elif dirt == "foreign tag":
        words[2] = (0x7f << 24) | 2
    else:
        words[2048 + 1] = 1 << 22                             # an adapter item that this layer does not have
    torch.cuda.synchronize()
    print(f"case list dirty header: {dirt}", flush=True)
    _run_list(ql, layers, False, ws)                          # launches and completes normally
    torch.cuda.synchronize()
    assert not ql.qlora_workspace_check(ws), "the dirty header went unnoticed"
    ql.qlora_workspace_init(ws)
    assert ql.qlora_workspace_check(ws)
    outs = _run_list(ql, layers, False, ws)
    torch.cuda.synchronize()
    _check_list(oracle, layers, outs, False, "after init")
    assert ql.qlora_workspace_check(ws)


def test_list_graph_replay(synth):
    """Both list kernels captured in one HIP graph: every replay, with eager work and synchronisations in between,
    reproduces the eager result bit for bit and leaves the header zero."""
    import paper_2305_14314_amd as ql
    M, shapes = 4, [(2048, 2304, 16), (1024, 1024, 64), (2304, 512, 0)]
    Wqs = [ql.qlora_nf4_quantize(synth.normal_f32_device((h, o), synth.SIGMA_W, 8300 + l)) for l, (h, o, r) in enumerate(shapes)]
    L1s = [dev_bf16(synth.normal_bf16((h, r), 0.05, 8310 + l)) if r else None for l, (h, o, r) in enumerate(shapes)]
    L2s = [dev_bf16(synth.normal_bf16((r, o), 0.05, 8320 + l)) if r else None for l, (h, o, r) in enumerate(shapes)]
    Xs = [dev_bf16(synth.normal_bf16((M, h), 1.0, 8330 + l)) for l, (h, o, r) in enumerate(shapes)]
    dYs = [dev_bf16(synth.normal_bf16((M, o), 1.0, 8340 + l)) for l, (h, o, r) in enumerate(shapes)]
    ss = [0.5, 0.25, 1.0]
    hs, os_, rs = [s[0] for s in shapes], [s[1] for s in shapes], [s[2] for s in shapes]
    ws = ql.workspace_alloc(max(ql.qlora_linear_list_sizes(M, hs, os_, rs, False), ql.qlora_linear_list_sizes(M, hs, os_, rs, True)))
    Y0 = ql.qlora_linear_fwd_list(Xs, Wqs, L1s, L2s, ss, workspace=ws)
    dX0 = ql.qlora_linear_bwd_list(dYs, Wqs, L1s, L2s, ss, workspace=ws)
    torch.cuda.synchronize()
    Ys = [torch.empty_like(a) for a in Y0]
    dXs = [torch.empty_like(a) for a in dX0]

    def step():
        ql.qlora_linear_fwd_list(Xs, Wqs, L1s, L2s, ss, Ys=Ys, workspace=ws)
        ql.qlora_linear_bwd_list(dYs, Wqs, L1s, L2s, ss, dXs=dXs, workspace=ws)

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
        for t in Ys + dXs:
            t.fill_(0)
        ws[HDR:].random_(0, 255)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(Y0 + dX0, Ys + dXs):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {it}"
        assert int(ws[:HDR].max()) == 0, "arrival words are not back at zero"


def test_list_many_tokens_is_the_single_layer_path(synth):
    """Above 16 tokens the layers run one after the other through qlora_linear_fwd / qlora_linear_bwd: identical bits."""
    import paper_2305_14314_amd as ql
    M, shapes = 80, [(512, 512, 16), (256, 192, 32)]
    Wqs = [ql.qlora_nf4_quantize(synth.normal_f32_device((h, o), synth.SIGMA_W, 8400 + l)) for l, (h, o, r) in enumerate(shapes)]
    L1s = [dev_bf16(synth.normal_bf16((h, r), 0.05, 8410 + l)) for l, (h, o, r) in enumerate(shapes)]
    L2s = [dev_bf16(synth.normal_bf16((r, o), 0.05, 8420 + l)) for l, (h, o, r) in enumerate(shapes)]
    Xs = [dev_bf16(synth.normal_bf16((M, h), 1.0, 8430 + l)) for l, (h, o, r) in enumerate(shapes)]
    dYs = [dev_bf16(synth.normal_bf16((M, o), 1.0, 8440 + l)) for l, (h, o, r) in enumerate(shapes)]
    ss = [0.5, 2.0]
    Ys = ql.qlora_linear_fwd_list(Xs, Wqs, L1s, L2s, ss)
    dXs = ql.qlora_linear_bwd_list(dYs, Wqs, L1s, L2s, ss)
    torch.cuda.synchronize()
    for l in range(2):
        Y1 = ql.qlora_linear_fwd(Xs[l], Wqs[l], L1s[l], L2s[l], ss[l])
        dX1, _, _ = ql.qlora_linear_bwd(dYs[l], None, Wqs[l], L1s[l], L2s[l], ss[l], need_dL=False)
        torch.cuda.synchronize()
        assert torch.equal(Ys[l].view(torch.int16), Y1.view(torch.int16))
        assert torch.equal(dXs[l].view(torch.int16), dX1.view(torch.int16))
