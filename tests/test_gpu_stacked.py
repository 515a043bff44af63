"""GPU parity of qlora_linear_fwd_stacked: several layers on one input, one matrix product (dequantised weights stacked
along the outputs, adapters block-diagonal in the second contraction segment).  Every layer's output columns are
compared with oracle.linear_fwd of that layer alone (Eq. 5 per layer), so a leak of one layer's adapter into another
layer's columns, a wrong column offset or a wrong scale fails."""
import numpy as np
import pytest
import torch

from gpu_util import dev_bf16, download_quant, host_bits, upload_quant
from test_gpu_linear import _check

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,n", [(1, 2), (16, 3), (17, 3), (100, 4), (300, 3), (257, 1), (600, 2)])
def test_stacked_forward_small(oracle, synth, M, n):
    """One to four layers of different widths and ranks (one without an adapter, one with rank 80: padded to 128
    columns of the shared segment); all outputs; the [hi | lo] pair of X L1 of every layer with an adapter."""
    import paper_2305_14314_amd as ql
    h = 704
    outs, ranks, ss = [1024, 320, 2304, 64][:n], [16, 0, 80, 32][:n], [0.5, 1.0, 0.25, 2.0][:n]
    hX = synth.normal_bf16((M, h), 1.0, 7000 + M)
    Wqs, L1s, L2s, refs, hL1s = [], [], [], [], []
    for l, (o, r) in enumerate(zip(outs, ranks)):
        q = oracle.nf4_quantize(synth.normal_f32((h, o), synth.SIGMA_W, 7100 + l))
        Wqs.append(upload_quant(q))
        hL1 = synth.normal_bf16((h, r), 0.05, 7200 + l) if r else None
        hL2 = synth.normal_bf16((r, o), 0.05, 7300 + l) if r else None
        hL1s.append(hL1)
        L1s.append(dev_bf16(hL1) if r else None)
        L2s.append(dev_bf16(hL2) if r else None)
        refs.append(oracle.linear_fwd(hX, oracle.nf4_dequant(q), hL1, hL2, ss[l]))
    print(f"case stacked M={M} h={h} o={outs} r={ranks}", flush=True)
    Ts = [torch.empty((M, 2 * r), dtype=torch.bfloat16, device="cuda") if r else None for r in ranks]
    nbytes = ql.qlora_linear_fwd_stacked_sizes(M, h, outs, ranks)
    ws = ql.workspace_alloc(nbytes)
    ws[ql.binding.WORKSPACE_HEADER_BYTES:].fill_(0x7F)          # stale contents: NaN-ish bf16 everywhere
    Y = ql.qlora_linear_fwd_stacked(dev_bf16(hX), Wqs, L1s, L2s, ss, T_saves=Ts, workspace=ws)
    torch.cuda.synchronize()
    assert Y.shape == (M, sum(outs))
    Yh, n0 = host_bits(Y), 0
    for l, o in enumerate(outs):
        _check(Yh[:, n0:n0 + o], refs[l], f"stacked M={M} layer {l} Y")
        n0 += o
        if ranks[l]:
            # the saved pair is X L1 as hi + lo, 16 significant bits
            from gpu_util import bits_f64
            t = host_bits(Ts[l])
            got = bits_f64(t[:, :ranks[l]]) + bits_f64(t[:, ranks[l]:])
            want = bits_f64(hX) @ bits_f64(hL1s[l])
            assert np.abs(got - want).max() <= 2.0 ** -14 * np.abs(want).max() + 1e-6
    assert int(ws[:ql.binding.WORKSPACE_HEADER_BYTES].max()) == 0   # the counter header is not touched
    with pytest.raises(ql.QloraError) as e:
        ql.qlora_linear_fwd_stacked(dev_bf16(hX), Wqs, L1s, L2s, ss, workspace=ws[:nbytes - 256])
    assert e.value.status == -4


@pytest.mark.parametrize("group", ["qkv", "gate_up"])
def test_stacked_forward_65b_groups(oracle, synth, group):
    """q / k / v (3 x 8192 x 8192) and gate / up (2 x 8192 x 22016) of a 65B-shaped block at 4096 tokens, r = 64:
    sampled token rows and sampled columns of every layer."""
    import paper_2305_14314_amd as ql
    cfg = synth.CONFIGS[3]
    M, r, s = cfg["M"], cfg["r"], cfg["alpha"] / cfg["r"]
    h, o, n = (8192, 8192, 3) if group == "qkv" else (8192, 22016, 2)
    Wqs, Whats, hL1, hL2 = [], [], [], []
    for l in range(n):
        Wd = synth.normal_f32_device((h, o), synth.SIGMA_W, 8000 + 10 * l + (0 if group == "qkv" else 5))
        Wqs.append(ql.qlora_nf4_quantize(Wd))
        del Wd
        Whats.append(oracle.nf4_dequant(download_quant(Wqs[-1])))
        hL1.append(synth.normal_bf16((h, r), cfg["sigma_l"], 8100 + l))
        hL2.append(synth.normal_bf16((r, o), cfg["sigma_l"], 8200 + l))
    L1s, L2s = [dev_bf16(a) for a in hL1], [dev_bf16(a) for a in hL2]
    ss = [s * (l + 1) for l in range(n)]                        # a different scale per layer
    print(f"case stacked {group} M={M}", flush=True)
    hX = synth.normal_bf16((M, h), 1.0, 8300)
    Y = ql.qlora_linear_fwd_stacked(dev_bf16(hX), Wqs, L1s, L2s, ss)
    torch.cuda.synchronize()
    Yh = host_bits(Y)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, M // 2, M - 256, M - 1],
                                     np.random.default_rng(7).integers(0, M, 8)])).astype(np.int64)
    cols = np.array([0, 255, 256, o // 2 + 3, o - 256, o - 1], np.int64)
    for l in range(n):
        _check(Yh[rows, l * o:(l + 1) * o], oracle.linear_fwd(hX, Whats[l], hL1[l], hL2[l], ss[l], rows=rows),
               f"{group} layer {l} rows")
        _check(Yh[:, l * o + cols], oracle.linear_fwd(hX, Whats[l], hL1[l], hL2[l], ss[l], cols=cols),
               f"{group} layer {l} cols")


@pytest.mark.parametrize("M,n", [(1, 2), (16, 3), (17, 3), (100, 4), (300, 3), (257, 1)])
def test_stacked_backward_small(oracle, synth, M, n):
    """dX is the SUM of the layers' input gradients (each from oracle.linear_bwd_dx on its own columns of dY), and
    every layer's dL1 / dL2 are its own (oracle.linear_bwd_dl); with T saved by the stacked forward and recomputed."""
    import paper_2305_14314_amd as ql
    from gpu_util import bits_f64
    h = 704
    outs, ranks, ss = [1024, 320, 2304, 64][:n], [16, 0, 80, 32][:n], [0.5, 1.0, 0.25, 2.0][:n]
    hX = synth.normal_bf16((M, h), 1.0, 9000 + M)
    hdY = synth.normal_bf16((M, sum(outs)), 1.0, 9050 + M)
    Wqs, L1s, L2s, ref_dx, ref_dl, n0 = [], [], [], 0.0, [], 0
    for l, (o, r) in enumerate(zip(outs, ranks)):
        q = oracle.nf4_quantize(synth.normal_f32((h, o), synth.SIGMA_W, 9100 + l))
        Wqs.append(upload_quant(q))
        hL1 = synth.normal_bf16((h, r), 0.05, 9200 + l) if r else None
        hL2 = synth.normal_bf16((r, o), 0.05, 9300 + l) if r else None
        L1s.append(dev_bf16(hL1) if r else None)
        L2s.append(dev_bf16(hL2) if r else None)
        dYl = np.ascontiguousarray(hdY[:, n0:n0 + o])
        ref_dx = ref_dx + oracle.linear_bwd_dx(dYl, oracle.nf4_dequant(q), hL1, hL2, ss[l])
        ref_dl.append(oracle.linear_bwd_dl(dYl, hX, hL1, hL2, ss[l]) if r else None)
        n0 += o
    print(f"case stacked bwd M={M} h={h} o={outs} r={ranks}", flush=True)
    X, dY = dev_bf16(hX), dev_bf16(hdY)
    Ts = [torch.empty((M, 2 * r), dtype=torch.bfloat16, device="cuda") if r else None for r in ranks]
    ql.qlora_linear_fwd_stacked(X, Wqs, L1s, L2s, ss, T_saves=Ts)
    nbytes = ql.qlora_linear_bwd_stacked_sizes(M, h, outs, ranks)
    ws = ql.workspace_alloc(nbytes)
    ws[ql.binding.WORKSPACE_HEADER_BYTES:].fill_(0x7F)
    for saved in (Ts, None):
        dX, dL1s, dL2s = ql.qlora_linear_bwd_stacked(dY, X, Wqs, L1s, L2s, ss, T_saveds=saved, workspace=ws)
        torch.cuda.synchronize()
        _check(host_bits(dX), ref_dx, f"stacked bwd M={M} dX (T {'saved' if saved else 'recomputed'})")
        for l, r in enumerate(ranks):
            if r:
                _check(host_bits(dL1s[l]), ref_dl[l][0], f"stacked bwd M={M} layer {l} dL1", few_terms=M < 64)
                _check(host_bits(dL2s[l]), ref_dl[l][1], f"stacked bwd M={M} layer {l} dL2", few_terms=M < 64)
            else:
                assert dL1s[l] is None and dL2s[l] is None
    # input gradient only: X is not needed
    dX2, _, _ = ql.qlora_linear_bwd_stacked(dY, None, Wqs, L1s, L2s, ss, need_dL=False, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(dX2.view(torch.int16), dX.view(torch.int16))
    with pytest.raises(ql.QloraError) as e:
        ql.qlora_linear_bwd_stacked(dY, X, Wqs, L1s, L2s, ss, workspace=ws[:nbytes - 256])
    assert e.value.status == -4


def test_stacked_backward_65b_qkv(oracle, synth):
    """q / k / v of a 65B-shaped block at 4096 tokens: dX (the sum of three input gradients, contraction over 24576
    outputs and 192 rank columns) on sampled rows and columns."""
    import paper_2305_14314_amd as ql
    cfg = synth.CONFIGS[3]
    M, r, s = cfg["M"], cfg["r"], cfg["alpha"] / cfg["r"]
    h, o, n = 8192, 8192, 3
    Wqs, Whats, hL1, hL2 = [], [], [], []
    for l in range(n):
        Wd = synth.normal_f32_device((h, o), synth.SIGMA_W, 9500 + 10 * l)
        Wqs.append(ql.qlora_nf4_quantize(Wd))
        del Wd
        Whats.append(oracle.nf4_dequant(download_quant(Wqs[-1])))
        hL1.append(synth.normal_bf16((h, r), cfg["sigma_l"], 9600 + l))
        hL2.append(synth.normal_bf16((r, o), cfg["sigma_l"], 9700 + l))
    L1s, L2s = [dev_bf16(a) for a in hL1], [dev_bf16(a) for a in hL2]
    ss = [s, 2 * s, 3 * s]
    hdY = synth.normal_bf16((M, n * o), 1.0, 9800)
    print(f"case stacked bwd qkv M={M}", flush=True)
    dX, _, _ = ql.qlora_linear_bwd_stacked(dev_bf16(hdY), None, Wqs, L1s, L2s, ss, need_dL=False)
    torch.cuda.synchronize()
    dXh = host_bits(dX)
    rows = np.array([0, 255, 256, M // 2, M - 1], np.int64)
    cols = np.array([0, 255, 256, h // 2 + 3, h - 1], np.int64)
    ref_r, ref_c = 0.0, 0.0
    for l in range(n):
        dYl = np.ascontiguousarray(hdY[:, l * o:(l + 1) * o])
        ref_r = ref_r + oracle.linear_bwd_dx(dYl, Whats[l], hL1[l], hL2[l], ss[l], rows=rows)
        ref_c = ref_c + oracle.linear_bwd_dx(dYl, Whats[l], hL1[l], hL2[l], ss[l], cols=cols)
    _check(dXh[rows], ref_r, "qkv dX rows")
    _check(dXh[:, cols], ref_c, "qkv dX cols")
