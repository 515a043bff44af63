"""GPU parity for the other 4-bit data types of the paper's comparison (Int4, Float4 E2M1, Float4 E3M0): the same
kernels with another 16-value table.  Quantisation and dequantisation bit-exact against the oracle (ties and
duplicate values included), the linear layer within the GEMM tolerance on both the large-GEMM and the few-token
path."""
import numpy as np
import pytest
import torch

from gpu_util import code_to_flat, dev_bf16, dev_f32, host_bits, host_u8, host_u32, upload_quant
from test_gpu_linear import _check

pytestmark = pytest.mark.gpu

KINDS = [("fp4_e2m1", 1), ("fp4_e3m0", 2), ("int4", 3), ("nf3", 5), ("nf2", 6)]


def _cases(oracle, synth, kind):
    yield "normal", synth.normal_f32((257, 192), 0.02, 9000)
    yield "unit-normal", synth.normal_f32((64, 512), 1.0, 9001)
    w = synth.normal_f32((128, 256), 0.02, 9002)
    w.reshape(-1)[:64 * 3] = 0.0                                          # all-zero blocks
    yield "zero-blocks", w
    # every decision point of the table, and its fp32 neighbours, in blocks whose absmax is exactly 1
    t = oracle.codebook4(kind).astype(np.float64)
    mids = ((t[:-1] + t[1:]) / 2).astype(np.float32)
    pts = np.concatenate([mids, np.nextafter(mids, np.float32(2)), np.nextafter(mids, np.float32(-2)), t.astype(np.float32)])
    flat = np.zeros((4 * 64,), np.float32)
    flat[:len(pts)] = pts
    flat[63::64] = 1.0                                                    # absmax 1 in every block
    yield "decision-points", flat.reshape(1, -1).copy()


@pytest.mark.parametrize("kind,dtype", KINDS)
def test_quantize_dequant_bit_exact(oracle, synth, kind, dtype):
    import paper_2305_14314_amd as ql
    table = oracle.codebook4(kind)
    assert np.array_equal(np.array(ql.qlora_codebook_4bit(dtype), np.float32).view(np.uint32), table.view(np.uint32))
    for tag, W in _cases(oracle, synth, kind):
        print("case", kind, tag, W.shape, flush=True)
        q = oracle.nf4_quantize(W, table=table)
        Wq = ql.qlora_quantize_4bit(dev_f32(W), dtype)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host_u8(Wq.packed), q["packed"], err_msg=f"{kind} {tag}: packed")
        assert host_u32(Wq.mean)[0] == np.float32(q["mean"]).view(np.uint32)
        np.testing.assert_array_equal(host_u32(Wq.c1), q["c1"].view(np.uint32))
        np.testing.assert_array_equal(code_to_flat(host_u8(Wq.code), Wq.rows, Wq.cols), q["code"])
        got = host_bits(ql.qlora_nf4_dequant(Wq))
        np.testing.assert_array_equal(got, oracle.nf4_dequant(q), err_msg=f"{kind} {tag}: dequantised bf16")


@pytest.mark.parametrize("kind,dtype", KINDS)
@pytest.mark.parametrize("M,h,o,r", [(300, 448, 576, 32), (5, 192, 320, 16), (16, 1024, 1024, 64)])
def test_linear_other_types(oracle, synth, kind, dtype, M, h, o, r):
    """Forward and backward on a weight of another data type: M = 300 takes the dequantise + GEMM path, M = 5 and 16
    the few-token streaming kernels (8- and 16-token variants), all against the oracle on its own dequantised weight."""
    import paper_2305_14314_amd as ql
    s = 0.5
    table = oracle.codebook4(kind)
    q = oracle.nf4_quantize(synth.normal_f32((h, o), synth.SIGMA_W, 9100 + M), table=table)
    What = oracle.nf4_dequant(q)
    Wq = upload_quant(q)
    Wq.dtype = dtype
    hX, hdY = synth.normal_bf16((M, h), 1.0, 9101), synth.normal_bf16((M, o), 1.0, 9102)
    hL1, hL2 = synth.normal_bf16((h, r), 0.05, 9103), synth.normal_bf16((r, o), 0.05, 9104)
    X, dY, L1, L2 = dev_bf16(hX), dev_bf16(hdY), dev_bf16(hL1), dev_bf16(hL2)
    print(f"case {kind} linear M={M} h={h} o={o} r={r}", flush=True)
    Y = ql.qlora_linear_fwd(X, Wq, L1, L2, s)
    dX, dL1, dL2 = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s)
    Ym = ql.qlora_linear_fwd_multi(X, [Wq, Wq], [L1, None], [L2, None], [s, 1.0])
    torch.cuda.synchronize()
    _check(host_bits(Y), oracle.linear_fwd(hX, What, hL1, hL2, s), f"{kind} Y")
    _check(host_bits(dX), oracle.linear_bwd_dx(hdY, What, hL1, hL2, s), f"{kind} dX")
    r1, r2 = oracle.linear_bwd_dl(hdY, hX, hL1, hL2, s)
    _check(host_bits(dL1), r1, f"{kind} dL1", few_terms=M < 64)
    _check(host_bits(dL2), r2, f"{kind} dL2", few_terms=M < 64)
    _check(host_bits(Ym[0]), oracle.linear_fwd(hX, What, hL1, hL2, s), f"{kind} multi Y0")
    _check(host_bits(Ym[1]), oracle.linear_fwd(hX, What, None, None, 1.0), f"{kind} multi Y1")
    # the table matters: the same codes read as NF4 are far from this reference
    Wq.dtype = 0
    Ynf4 = ql.qlora_linear_fwd(X, Wq, None, None, s)
    torch.cuda.synchronize()
    ref = oracle.linear_fwd(hX, What, None, None, s)
    got = (host_bits(Ynf4).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.abs(got - ref).max() > 10 * 2e-2 * np.sqrt((ref ** 2).mean())


@pytest.mark.parametrize("kind,dtype", [("nf4", 0), ("int4", 3)])
def test_without_double_quantization(oracle, synth, kind, dtype):
    """dq_blocksize = 0: the fp32 constants are kept (4.5 bit per parameter).  Quantise and dequantise bit-exact; the
    linear layer at 300 and at 5 tokens (the latter through the large-GEMM path: the streaming kernels read
    double-quantised constants) against the oracle; the several-layers forward refuses such a weight at few tokens."""
    import paper_2305_14314_amd as ql
    table = oracle.codebook4(kind)
    h, o, r, s = 448, 576, 32, 0.5
    W = synth.normal_f32((h, o), synth.SIGMA_W, 9200)
    q = oracle.nf4_quantize(W, dq_blocksize=0, table=table)
    Wq = ql.qlora_nf4_quantize(dev_f32(W), dq_blocksize=0, dtype=dtype)
    torch.cuda.synchronize()
    assert Wq.dq_blocksize == 0 and Wq.code.numel() == 0 and Wq.nbytes * 8 / (h * o) == 4.5
    np.testing.assert_array_equal(host_u8(Wq.packed), q["packed"])
    np.testing.assert_array_equal(host_u32(Wq.c1), q["c2"].view(np.uint32))
    What = oracle.nf4_dequant(q)
    np.testing.assert_array_equal(host_bits(ql.qlora_nf4_dequant(Wq)), What)
    hL1, hL2 = synth.normal_bf16((h, r), 0.05, 9201), synth.normal_bf16((r, o), 0.05, 9202)
    L1, L2 = dev_bf16(hL1), dev_bf16(hL2)
    for M in (300, 5):
        print(f"case no-DQ {kind} M={M}", flush=True)
        hX, hdY = synth.normal_bf16((M, h), 1.0, 9203 + M), synth.normal_bf16((M, o), 1.0, 9204 + M)
        X, dY = dev_bf16(hX), dev_bf16(hdY)
        Y = ql.qlora_linear_fwd(X, Wq, L1, L2, s)
        dX, dL1, dL2 = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s)
        torch.cuda.synchronize()
        _check(host_bits(Y), oracle.linear_fwd(hX, What, hL1, hL2, s), f"no-DQ {kind} M={M} Y")
        _check(host_bits(dX), oracle.linear_bwd_dx(hdY, What, hL1, hL2, s), f"no-DQ {kind} M={M} dX")
        r1, r2 = oracle.linear_bwd_dl(hdY, hX, hL1, hL2, s)
        _check(host_bits(dL1), r1, "dL1", few_terms=M < 64)
        _check(host_bits(dL2), r2, "dL2", few_terms=M < 64)
    ws = ql.workspace_alloc(ql.qlora_linear_dropout_sizes(5, h, o, r)[0])
    with pytest.raises(ql.QloraError) as e:
        ql.qlora_linear_fwd_multi(X, [Wq], [L1], [L2], [s], workspace=ws)
    assert e.value.status == -3


def _int8_cases(synth):
    yield "normal", synth.normal_f32((257, 192), 0.02, 9300)
    yield "unit-normal", synth.normal_f32((64, 512), 1.0, 9301)
    w = synth.normal_f32((128, 256), 0.02, 9302)
    w.reshape(-1)[:64 * 3] = 0.0                                          # all-zero blocks
    w.reshape(-1)[64 * 5:64 * 6] *= np.float32(1e-36)                     # 127 / absmax overflows fp32: zeros
    yield "zero-and-tiny-blocks", w
    # blocks with absmax 127 (c = 1): every half-integer and its fp32 neighbours, both signs -> ties to even
    k = np.arange(0, 42, dtype=np.float32) * 3 + 0.5
    pts = np.concatenate([k, np.nextafter(k, np.float32(1e9)), np.nextafter(k, np.float32(-1e9))])
    pts = np.concatenate([pts, -pts])
    flat = np.zeros((5 * 64,), np.float32)
    idx = np.arange(len(pts))
    flat[idx + idx // 63] = pts                                           # 63 points per block, the last slot stays free
    flat[63::64] = 127.0
    yield "ties", flat.reshape(1, -1).copy()


@pytest.mark.parametrize("dq_blocksize", [256, 0])
def test_int8_quantize_dequant_bit_exact(oracle, synth, dq_blocksize):
    """Eq. 1 / Eq. 2 with 8-bit integers: the bytes, the constants (double-quantised or kept) and the dequantised bf16
    weights equal the oracle's bit for bit; the 4-bit entry points refuse the type."""
    import paper_2305_14314_amd as ql
    for tag, W in _int8_cases(synth):
        print("case int8", tag, W.shape, "dq", dq_blocksize, flush=True)
        q = oracle.int8_quantize(W, dq_blocksize=dq_blocksize)
        Wq = ql.qlora_quantize_int8(dev_f32(W), dq_blocksize=dq_blocksize)
        torch.cuda.synchronize()
        assert Wq.dtype == ql.INT8 and Wq.packed.numel() == W.size
        np.testing.assert_array_equal(host_u8(Wq.packed).view(np.int8), q["q8"], err_msg=f"int8 {tag}: bytes")
        if dq_blocksize:
            assert host_u32(Wq.mean)[0] == np.float32(q["mean"]).view(np.uint32)
            np.testing.assert_array_equal(host_u32(Wq.c1), q["c1"].view(np.uint32))
            np.testing.assert_array_equal(code_to_flat(host_u8(Wq.code), Wq.rows, Wq.cols), q["code"])
        else:
            np.testing.assert_array_equal(host_u32(Wq.c1), q["c2"].view(np.uint32))
        np.testing.assert_array_equal(host_bits(ql.qlora_nf4_dequant(Wq)), oracle.int8_dequant(q),
                                      err_msg=f"int8 {tag}: dequantised bf16")
    with pytest.raises(ql.QloraError) as e:
        ql.qlora_codebook_4bit(ql.INT8)
    assert e.value.status == -3
    bits = 8 + (8 / 64 + 32 / (64 * 256) if dq_blocksize else 0.5)
    assert abs(Wq.nbytes * 8 / W.size - bits) < 1e-3 + (32 + 32) / W.size


@pytest.mark.parametrize("dq_blocksize", [256, 0])
@pytest.mark.parametrize("M,h,o,r", [(300, 448, 576, 32), (5, 192, 320, 16)])
def test_int8_linear(oracle, synth, dq_blocksize, M, h, o, r):
    """Forward and backward on an Int8 weight (dequantise + GEMM at any token count; the transposed dequantisation
    feeds the forward product, the plain one the backward) against the oracle on its own dequantised weight."""
    import paper_2305_14314_amd as ql
    s = 0.5
    W = synth.normal_f32((h, o), synth.SIGMA_W, 9310 + M)
    q = oracle.int8_quantize(W, dq_blocksize=dq_blocksize)
    What = oracle.int8_dequant(q)
    Wq = ql.qlora_quantize_int8(dev_f32(W), dq_blocksize=dq_blocksize)
    hX, hdY = synth.normal_bf16((M, h), 1.0, 9311), synth.normal_bf16((M, o), 1.0, 9312)
    hL1, hL2 = synth.normal_bf16((h, r), 0.05, 9313), synth.normal_bf16((r, o), 0.05, 9314)
    X, dY, L1, L2 = dev_bf16(hX), dev_bf16(hdY), dev_bf16(hL1), dev_bf16(hL2)
    print(f"case int8 linear M={M} h={h} o={o} r={r} dq={dq_blocksize}", flush=True)
    Y = ql.qlora_linear_fwd(X, Wq, L1, L2, s)
    dX, dL1, dL2 = ql.qlora_linear_bwd(dY, X, Wq, L1, L2, s)
    torch.cuda.synchronize()
    _check(host_bits(Y), oracle.linear_fwd(hX, What, hL1, hL2, s), "int8 Y")
    _check(host_bits(dX), oracle.linear_bwd_dx(hdY, What, hL1, hL2, s), "int8 dX")
    r1, r2 = oracle.linear_bwd_dl(hdY, hX, hL1, hL2, s)
    _check(host_bits(dL1), r1, "int8 dL1", few_terms=M < 64)
    _check(host_bits(dL2), r2, "int8 dL2", few_terms=M < 64)
    if M <= 16:
        ws = ql.workspace_alloc(ql.qlora_linear_dropout_sizes(M, h, o, r)[0])
        with pytest.raises(ql.QloraError) as e:
            ql.qlora_linear_fwd_multi(X, [Wq], [L1], [L2], [s], workspace=ws)
        assert e.value.status == -3
