"""GPU parity of LoRA dropout on the adapter's input: Y, dX, dL1 and dL2 against the fp64 oracle with the same
seeded keep-mask, with an adapter strong enough that a misplaced mask bit, a missing 1/(1-p) or an uncorrected
input gradient is far outside the tolerance; the degenerate masks; and the plain path recovered bit for bit."""
import numpy as np
import pytest
import torch

from gpu_util import dev_bf16, host_bits, upload_quant
from test_gpu_linear import _check

pytestmark = pytest.mark.gpu


def _layer(oracle, synth, M, h, o, r, seed, sigma_l=0.05):
    q = oracle.nf4_quantize(synth.normal_f32((h, o), synth.SIGMA_W, seed))
    L = dict(M=M, h=h, o=o, r=r, q=q, What=oracle.nf4_dequant(q), Wq=upload_quant(q),
             X=synth.normal_bf16((M, h), 1.0, seed + 1), dY=synth.normal_bf16((M, o), 1.0, seed + 2),
             L1=synth.normal_bf16((h, r), sigma_l, seed + 3), L2=synth.normal_bf16((r, o), sigma_l, seed + 4))
    for k in ("X", "dY", "L1", "L2"):
        L["d" + k] = dev_bf16(L[k])
    return L


def _mask(M, h, p, seed):
    """Seeded keep-mask: host boolean matrix and the device bit mask (bit e % 8 of byte e // 8, 1 = kept)."""
    keep = np.random.default_rng(seed).random((M, h)) >= p
    bits = np.packbits(keep.reshape(-1), bitorder="little")
    return keep, torch.from_numpy(bits).cuda()


@pytest.mark.parametrize("M,h,o,r,p", [(300, 448, 576, 32, 0.1), (17, 128, 320, 64, 0.05), (5, 192, 64, 16, 0.5),
                                        (513, 256, 192, 128, 0.1), (1024, 1024, 1024, 64, 0.05),
                                        (200, 512, 448, 144, 0.1), (1, 64, 64, 16, 0.25)])
def test_dropout_forward_backward(oracle, synth, M, h, o, r, p):
    import paper_2305_14314_amd as ql
    s = 1.0
    L = _layer(oracle, synth, M, h, o, r, 8000 + M)
    keep, dmask = _mask(M, h, p, 8100 + M)
    D = oracle.dropout_multipliers(keep, p)
    print(f"case dropout M={M} h={h} o={o} r={r} p={p}", flush=True)
    T = torch.empty((M, 2 * r), dtype=torch.bfloat16, device="cuda")
    Y = ql.qlora_linear_fwd_dropout(L["dX"], L["Wq"], L["dL1"], L["dL2"], s, dmask, p, T_save=T)
    dX, dL1, dL2 = ql.qlora_linear_bwd_dropout(L["ddY"], L["dX"], L["Wq"], L["dL1"], L["dL2"], s, dmask, p, T_saved=T)
    torch.cuda.synchronize()
    few = M < 64
    _check(host_bits(Y), oracle.linear_fwd(L["X"], L["What"], L["L1"], L["L2"], s, D=D), "Y")
    ref_dx = oracle.linear_bwd_dx(L["dY"], L["What"], L["L1"], L["L2"], s, D=D)
    _check(host_bits(dX), ref_dx, "dX")
    # the adapter is strong enough for the checks above to see a mistake in the mask handling
    plain_dx = oracle.linear_bwd_dx(L["dY"], L["What"], L["L1"], L["L2"], s)
    assert np.abs(plain_dx - ref_dx).max() > 10 * 2e-2 * np.sqrt((ref_dx ** 2).mean())
    r1, r2 = oracle.linear_bwd_dl(L["dY"], L["X"], L["L1"], L["L2"], s, D=D)
    _check(host_bits(dL1), r1, "dL1", few_terms=few)
    _check(host_bits(dL2), r2, "dL2", few_terms=few)
    # gradient checkpointing (X L1 recomputed under the mask) and fp32 accumulation
    a1 = torch.zeros((h, r), dtype=torch.float32, device="cuda")
    a2 = torch.zeros((r, o), dtype=torch.float32, device="cuda")
    dXb, _, _ = ql.qlora_linear_bwd_dropout(L["ddY"], L["dX"], L["Wq"], L["dL1"], L["dL2"], s, dmask, p, T_saved=None,
                                            dL1_acc=a1, dL2_acc=a2)
    torch.cuda.synchronize()
    assert torch.equal(dXb, dX)
    for got, ref, tag in ((a1, r1, "dL1 acc"), (a2, r2, "dL2 acc")):
        err = np.abs(got.cpu().numpy().astype(np.float64) - ref).max()
        rms = np.sqrt((ref ** 2).mean())
        print(f"  {tag}: max|err|/rms = {err / rms:.2e}", flush=True)
        assert err <= 2e-4 * rms, tag


def test_dropout_degenerate_masks(oracle, synth):
    """Nothing dropped at p = 0 is the plain layer bit for bit; everything dropped removes the adapter from Y and dX
    and leaves zero adapter gradients.  (A dropped element of dX is rounded twice -- the product writes it with the
    adapter's term, which is then taken off -- so with EVERY element dropped the adapter has the strength of the
    paper's workloads here, sigma 0.01, not the exaggerated one of the parity cases.)"""
    import paper_2305_14314_amd as ql
    M, h, o, r, s = 300, 448, 576, 32, 0.5
    L = _layer(oracle, synth, M, h, o, r, 8200, sigma_l=0.01)
    ones = torch.full((M * h // 8,), 255, dtype=torch.uint8, device="cuda")
    zeros = torch.zeros((M * h // 8,), dtype=torch.uint8, device="cuda")
    Y0 = ql.qlora_linear_fwd(L["dX"], L["Wq"], L["dL1"], L["dL2"], s)
    g0 = ql.qlora_linear_bwd(L["ddY"], L["dX"], L["Wq"], L["dL1"], L["dL2"], s)
    Y1 = ql.qlora_linear_fwd_dropout(L["dX"], L["Wq"], L["dL1"], L["dL2"], s, ones, 0.0)
    g1 = ql.qlora_linear_bwd_dropout(L["ddY"], L["dX"], L["Wq"], L["dL1"], L["dL2"], s, ones, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(Y0.view(torch.int16), Y1.view(torch.int16))
    for a, b in zip(g0, g1):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    Y2 = ql.qlora_linear_fwd_dropout(L["dX"], L["Wq"], L["dL1"], L["dL2"], s, zeros, 0.5)
    dX2, dL1, dL2 = ql.qlora_linear_bwd_dropout(L["ddY"], L["dX"], L["Wq"], L["dL1"], L["dL2"], s, zeros, 0.5)
    torch.cuda.synchronize()
    _check(host_bits(Y2), oracle.linear_fwd(L["X"], L["What"], None, None, s), "all dropped Y")
    _check(host_bits(dX2), oracle.linear_bwd_dx(L["dY"], L["What"], None, None, s), "all dropped dX")
    assert int(dL1.view(torch.int16).abs().max()) == 0 and int(dL2.view(torch.int16).abs().max()) == 0
    # without an adapter the mask is not needed at all
    Y3 = ql.qlora_linear_fwd_dropout(L["dX"], L["Wq"], None, None, s, None, 0.1)
    torch.cuda.synchronize()
    _check(host_bits(Y3), oracle.linear_fwd(L["X"], L["What"], None, None, s), "r = 0 Y")


def test_dropout_full_size_sampled(oracle, synth):
    """A 65B-shaped 8192 x 8192 linear at the benchmark's 4096 tokens, p = 0.05, r = 64: Y and dX on sampled token
    rows (the mask bits of those rows decide which elements lose the adapter's gradient), dL1 and dL2 in full."""
    import paper_2305_14314_amd as ql
    from gpu_util import download_quant
    cfg = synth.CONFIGS[3]
    h, o = cfg["linears"][0]
    M, r, s, p = cfg["M"], cfg["r"], cfg["alpha"] / cfg["r"], 0.05
    print(f"case dropout full size: M={M} h={h} o={o} r={r} p={p}", flush=True)
    Wq = ql.qlora_nf4_quantize(synth.normal_f32_device((h, o), synth.SIGMA_W, 8300))
    What = oracle.nf4_dequant(download_quant(Wq))
    hX, hdY = synth.normal_bf16((M, h), 1.0, 8301), synth.normal_bf16((M, o), 1.0, 8302)
    hL1, hL2 = synth.normal_bf16((h, r), 0.03, 8303), synth.normal_bf16((r, o), 0.03, 8304)
    X, dY, L1, L2 = dev_bf16(hX), dev_bf16(hdY), dev_bf16(hL1), dev_bf16(hL2)
    keep, dmask = _mask(M, h, p, 8305)
    D = oracle.dropout_multipliers(keep, p)
    T = torch.empty((M, 2 * r), dtype=torch.bfloat16, device="cuda")
    Y = ql.qlora_linear_fwd_dropout(X, Wq, L1, L2, s, dmask, p, T_save=T)
    dX, dL1, dL2 = ql.qlora_linear_bwd_dropout(dY, X, Wq, L1, L2, s, dmask, p, T_saved=T)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 255, 256, M // 2, M - 256, M - 1],
                                     np.random.default_rng(83).integers(0, M, 10)])).astype(np.int64)
    _check(host_bits(Y)[rows], oracle.linear_fwd(hX, What, hL1, hL2, s, rows=rows, D=D), "Y rows")
    ref_dx = oracle.linear_bwd_dx(hdY, What, hL1, hL2, s, rows=rows, D=D)
    _check(host_bits(dX)[rows], ref_dx, "dX rows")
    plain = oracle.linear_bwd_dx(hdY, What, hL1, hL2, s, rows=rows)
    assert np.abs(plain - ref_dx).max() > 5 * 2e-2 * np.sqrt((ref_dx ** 2).mean())      # the mask matters here
    r1, r2 = oracle.linear_bwd_dl(hdY, hX, hL1, hL2, s, D=D)
    _check(host_bits(dL1), r1, "dL1")
    _check(host_bits(dL2), r2, "dL2")
