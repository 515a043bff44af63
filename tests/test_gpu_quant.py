"""GPU parity: NF4 quantise (with Double Quantization) and doubleDequant against the CPU oracle.
Bit-exact on packed nibbles, 8-bit codes, c1, the mean and the dequantised bf16 weights."""
import numpy as np
import pytest
import torch

from gpu_util import code_to_flat, dev_f32, host_bits, host_u8, host_u32, upload_quant

pytestmark = pytest.mark.gpu


def _compare_quant(oracle, W_host, Wq, tag):
    q = oracle.nf4_quantize(W_host)
    np.testing.assert_array_equal(host_u8(Wq.packed), q["packed"], err_msg=f"{tag}: packed nibbles")
    assert host_u32(Wq.mean)[0] == np.float32(q["mean"]).view(np.uint32), f"{tag}: mean"
    np.testing.assert_array_equal(host_u32(Wq.c1), q["c1"].view(np.uint32), err_msg=f"{tag}: c1")
    np.testing.assert_array_equal(code_to_flat(host_u8(Wq.code), Wq.rows, Wq.cols), q["code"], err_msg=f"{tag}: c2 codes")
    return q


def _cases(synth):
    rng = np.random.default_rng(11)
    base = synth.make_layer(0, 0)["W"]                       # 1024 x 1024, N(0, 0.02)
    yield "config0", base
    yield "one-block", synth.normal_f32((1, 64), 0.02, 21)
    yield "three-blocks", synth.normal_f32((3, 64), 0.02, 22)
    yield "ragged-257x192", synth.normal_f32((257, 192), 0.02, 23)        # 771 blocks: 3 full runs + 3
    yield "ragged-1000x320", synth.normal_f32((1000, 320), 0.02, 24)
    w = synth.normal_f32((512, 512), 0.02, 25)
    w *= rng.uniform(0.5, 2.0, (1, 512)).astype(np.float32)               # per-column scale
    out = rng.random(w.shape) < 1e-3
    w[out] *= 10.0                                                        # outliers
    yield "outliers", w
    z = synth.normal_f32((256, 256), 0.02, 26)
    z.reshape(-1)[:64 * 5] = 0.0                                          # all-zero blocks
    z.reshape(-1)[64 * 300:64 * 300 + 64 * 256] = 0.0                     # an all-zero run of constants
    yield "zero-blocks", z
    yield "all-zero", np.zeros((64, 128), np.float32)
    yield "constant", np.full((64, 128), 0.37, np.float32)
    big = synth.normal_f32((128, 256), 1.0, 27)
    big.reshape(-1, 64)[::3] *= np.float32(1e30)
    big.reshape(-1, 64)[1::3] *= np.float32(1e-30)
    yield "wide-range", big
    tiny = synth.normal_f32((64, 256), 1.0, 28) * np.float32(1e-39)       # subnormal inputs
    yield "subnormal", tiny.astype(np.float32)


def test_quantize_dequant_bit_exact(oracle, synth):
    import paper_2305_14314_amd as ql
    for tag, W in _cases(synth):
        print("case", tag, W.shape, flush=True)
        Wd = dev_f32(W)
        Wq = ql.qlora_nf4_quantize(Wd)
        Wq2 = ql.qlora_nf4_quantize(Wd)                                   # run-to-run determinism
        torch.cuda.synchronize()
        q = _compare_quant(oracle, W, Wq, tag)
        assert torch.equal(Wq.packed, Wq2.packed) and torch.equal(Wq.code, Wq2.code)
        assert torch.equal(Wq.c1, Wq2.c1) and torch.equal(Wq.mean, Wq2.mean)
        got = host_bits(ql.qlora_nf4_dequant(Wq))
        np.testing.assert_array_equal(got, oracle.nf4_dequant(q), err_msg=f"{tag}: dequantised bf16")


def test_dequant_of_oracle_artefacts(oracle, synth):
    """Dequantise buffers produced by the oracle's quantiser: isolates the dequant kernel."""
    import paper_2305_14314_amd as ql
    W = synth.normal_f32((320, 448), 0.02, 31)
    q = oracle.nf4_quantize(W)
    # exercise every 8-bit code, not only those the data happens to produce
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 256, q["code"].size).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x7E
    q["code"] = codes
    got = host_bits(ql.qlora_nf4_dequant(upload_quant(q)))
    np.testing.assert_array_equal(got, oracle.nf4_dequant(q))


@pytest.mark.parametrize("shape", [(4096, 11008), (5120, 13824), (8192, 22016)])
def test_quantize_full_size(oracle, synth, shape):
    """LLaMA-shaped tensors drawn on the device, copied back for the oracle."""
    import paper_2305_14314_amd as ql
    print("case full-size", shape, flush=True)
    Wd = synth.normal_f32_device(shape, synth.SIGMA_W, 1000 + shape[0])
    Wq = ql.qlora_nf4_quantize(Wd)
    Wh = ql.qlora_nf4_dequant(Wq)
    torch.cuda.synchronize()
    q = _compare_quant(oracle, Wd.cpu().numpy(), Wq, str(shape))
    np.testing.assert_array_equal(host_bits(Wh), oracle.nf4_dequant(q))
    assert Wq.nbytes * 8 / (shape[0] * shape[1]) < 4.127 + 1e-3            # Section 3 footprint


def test_argument_errors_launch_nothing():
    import paper_2305_14314_amd as ql
    W = torch.zeros((4, 96), dtype=torch.float32, device="cuda")            # cols not a multiple of 64
    with pytest.raises(ql.QloraError) as e:
        ql.qlora_nf4_quantize(W)
    assert e.value.status == -2
    with pytest.raises(ql.QloraError) as e:
        ql.qlora_nf4_quantize(torch.zeros((4, 128), dtype=torch.float32, device="cuda"), blocksize=128)
    assert e.value.status == -3
