"""The large-token backward product with the weight decoded inside the GEMM (qlora_bwd_fused_dequant(1)) against the
oracle and against the two-kernel form (dequantise, then multiply).

Both forms build the same bf16 weight tiles, so without an adapter dX must be the same bits; with one, the adapter
term enters the fp32 sum first instead of last and the outputs may differ by one bf16 rounding."""
import numpy as np
import pytest
import torch

from gpu_util import bits_f64, dev_bf16, host_bits, upload_quant

pytestmark = pytest.mark.gpu

TOL = 2e-2


@pytest.fixture()
def fused():
    import paper_2305_14314_amd as ql
    prev = ql.qlora_bwd_fused_dequant(1)
    yield ql
    ql.qlora_bwd_fused_dequant(prev)


def _dx(ql, mode, dY, X, Wq, L1, L2, s):
    ql.qlora_bwd_fused_dequant(mode)
    dX, _, _ = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s)
    torch.cuda.synchronize()
    return dX


# h = 64 .. 1024 rows of W (the output columns of the product, ragged against the 256-wide tiles), o = 64 .. 1536: 1 to
# 32 K-steps (shorter and longer than the prefetch ring and the unrolled loop), ranks below and at 64, none, and 128
# (two adapter steps: that call takes the two-kernel form whatever the mode)
@pytest.mark.parametrize("M,h,o,r", [(256, 1024, 1024, 16), (300, 448, 576, 32), (17, 128, 320, 64), (65, 64, 64, 0),
                                      (513, 256, 192, 64), (257, 320, 1536, 0), (40, 704, 128, 16), (1024, 512, 832, 64),
                                      (33, 320, 64, 16), (128, 960, 2048, 64),
                                      (96, 384, 256, 128)])
def test_fused_backward_matches(oracle, synth, fused, M, h, o, r):
    ql = fused
    print(f"fused bwd: M {M} h {h} o {o} r {r}", flush=True)
    L = synth.make_layer(0, 0, M=M, h=h, o=o, r=max(r, 1))
    q = oracle.nf4_quantize(L["W"])
    What = oracle.nf4_dequant(q)
    Wq = upload_quant(q)
    X, dY = dev_bf16(L["X"]), dev_bf16(L["dY"])
    L1 = dev_bf16(L["L1"]) if r else None
    L2 = dev_bf16(L["L2"]) if r else None
    a = _dx(ql, 0, dY, X, Wq, L1, L2, L["s"])
    b = _dx(ql, 1, dY, X, Wq, L1, L2, L["s"])
    ref = oracle.linear_bwd_dx(L["dY"], What, L["L1"] if r else None, L["L2"] if r else None, L["s"])
    rms = np.sqrt((ref ** 2).mean())
    for tag, got in (("two kernels", a), ("fused", b)):
        err = np.abs(bits_f64(host_bits(got)).reshape(ref.shape) - ref).max()
        print(f"  {tag}: max|err|/rms = {err / rms:.4f}", flush=True)
        assert err <= TOL * rms, tag
    ga, gb = bits_f64(host_bits(a)), bits_f64(host_bits(b))
    if r == 0:
        assert torch.equal(a, b)
    else:
        assert np.all(np.abs(ga - gb) <= 2.0 ** -7 * np.abs(ga) + 1e-4 * rms)   # one bf16 step; fp32 sum order near zero
    # a second call with the mode still set gives the same bits (no state is carried between calls)
    assert torch.equal(_dx(ql, 1, dY, X, Wq, L1, L2, L["s"]), b)


@pytest.mark.parametrize("dtype_name", ["FP4_E2M1", "INT4"])
def test_fused_backward_other_types_and_plain_constants(oracle, synth, fused, dtype_name):
    """The other 4-bit data types (their table goes through the same lookup) and weights without Double Quantization."""
    ql = fused
    M, h, o, r = 130, 320, 384, 16
    L = synth.make_layer(0, 0, M=M, h=h, o=o, r=r)
    W = torch.from_numpy(L["W"]).cuda()
    X, dY, L1, L2 = dev_bf16(L["X"]), dev_bf16(L["dY"]), dev_bf16(L["L1"]), dev_bf16(L["L2"])
    for dq in (True, False):
        print(f"fused bwd: {dtype_name} dq {dq}", flush=True)
        Wq = ql.qlora_quantize_4bit(W, getattr(ql, dtype_name), dq_blocksize=256 if dq else 0)
        a = _dx(ql, 0, dY, X, Wq, L1, L2, L["s"])
        b = _dx(ql, 1, dY, X, Wq, L1, L2, L["s"])
        ga, gb = bits_f64(host_bits(a)), bits_f64(host_bits(b))
        assert np.all(np.abs(ga - gb) <= 2.0 ** -7 * np.abs(ga) + 1e-4 * np.sqrt((ga ** 2).mean()))
        # without the adapter the two forms are the same bits
        a0 = _dx(ql, 0, dY, X, Wq, None, None, 0.0)
        b0 = _dx(ql, 1, dY, X, Wq, None, None, 0.0)
        assert torch.equal(a0, b0)


def test_fused_backward_under_dropout_and_accumulation(synth, fused):
    """The other callers of the backward product: LoRA dropout (the input-gradient fix-up runs behind either form) and
    fp32 gradient accumulation; both forms against each other."""
    ql = fused
    M, h, o, r = 200, 384, 512, 32
    L = synth.make_layer(0, 0, M=M, h=h, o=o, r=r)
    Wq = ql.qlora_nf4_quantize(torch.from_numpy(L["W"]).cuda())
    X, dY, L1, L2 = dev_bf16(L["X"]), dev_bf16(L["dY"]), dev_bf16(L["L1"]), dev_bf16(L["L2"])
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    mask = ql.pack_keep_mask(torch.rand((M, h), device="cuda", generator=gen) >= 0.1)
    res = {}
    for mode in (0, 1):
        ql.qlora_bwd_fused_dequant(mode)
        dX, dL1, dL2 = ql.qlora_linear_bwd_dropout(dY, X, Wq, L1, L2, L["s"], mask, 0.1)
        a1 = torch.zeros((h, r), dtype=torch.float32, device="cuda")
        a2 = torch.zeros((r, o), dtype=torch.float32, device="cuda")
        dXa = ql.qlora_linear_bwd_acc(dY, X, Wq, L1, L2, L["s"], dL1_acc=a1, dL2_acc=a2)
        torch.cuda.synchronize()
        res[mode] = (dX, dL1, dL2, dXa, a1, a2)
    for k in (1, 2, 4, 5):                                    # the adapter gradients do not pass through the product
        assert torch.equal(res[0][k], res[1][k])
    for k in (0, 3):
        ga, gb = bits_f64(host_bits(res[0][k])), bits_f64(host_bits(res[1][k]))
        assert np.all(np.abs(ga - gb) <= 2.0 ** -7 * np.abs(ga) + 1e-4 * np.sqrt((ga ** 2).mean()))
