"""k-bit storage of NF3 / NF2 codes (qlora_kbit_pack / qlora_kbit_unpack) against oracle/kbit.py: the stream bit for
bit, the container restored bit for bit, and the dequantised weight of a packed-then-unpacked tensor identical to the
oracle's dequantisation with the k-bit table."""
import numpy as np
import pytest
import torch

import oracle
from oracle import kbit
import paper_2305_14314_amd as ql
from gpu_util import download_quant, host_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k,dtype", [(3, ql.NF3), (2, ql.NF2)])
@pytest.mark.parametrize("shape", [(1, 64), (3, 192), (64, 64), (320, 448), (1000, 1088), (4096, 11008)])
def test_pack_unpack_bit_exact(k, dtype, shape):
    h, o = shape
    print(f"kbit: k {k} shape {h} x {o}", flush=True)
    W = torch.from_numpy((np.random.default_rng(h + o + k).standard_normal((h, o)) * 0.02).astype(np.float32)).cuda()
    Wq = ql.qlora_quantize_4bit(W, dtype)
    q = download_quant(Wq)
    codes = kbit.codes_of_packed4(q["packed"])
    assert int(codes.max()) < (1 << k)
    stream = ql.qlora_kbit_pack(Wq)
    torch.cuda.synchronize()
    assert stream.numel() == h * o * k // 8 == ql.qlora_kbit_sizes(h, o, k)
    assert np.array_equal(stream.cpu().numpy(), kbit.kbit_pack(codes, k))
    ref_w = ql.qlora_nf4_dequant(Wq).clone()
    keep = Wq.packed.clone()
    Wq.packed.fill_(0xEE)                                      # the container is transient: rebuilt from the stream
    ql.qlora_kbit_unpack(stream, Wq)
    torch.cuda.synchronize()
    assert torch.equal(Wq.packed, keep)
    assert np.array_equal(Wq.packed.cpu().numpy(), kbit.packed4_of_codes(kbit.kbit_unpack(stream.cpu().numpy(), k, h * o)))
    got = ql.qlora_nf4_dequant(Wq)
    assert torch.equal(got.view(torch.int16), ref_w.view(torch.int16))
    if h * o <= 1 << 21:                                       # against the oracle's dequantisation with the k-bit table
        table = oracle.nfk_derive(k).astype(np.float32)
        qo = oracle.nf4_quantize(W.cpu().numpy(), table=table)
        assert np.array_equal(qo["packed"], q["packed"])
        want = oracle.nf4_dequant(qo)
        assert np.array_equal(host_bits(got), want)


def test_upper_bits_are_dropped_and_arguments_checked():
    h, o = 4, 64
    packed4 = torch.full((h * o // 2,), 0xFF, dtype=torch.uint8, device="cuda")      # code 15 everywhere
    L = ql.lib()
    import ctypes
    for k in (2, 3):
        out = torch.zeros(h * o * k // 8, dtype=torch.uint8, device="cuda")
        assert L.qlora_kbit_pack(ctypes.c_void_p(packed4.data_ptr()), h, o, k, ctypes.c_void_p(out.data_ptr()), None) == 0
        torch.cuda.synchronize()
        assert int(out.min()) == 0xFF                          # 2^k - 1 in every field
        back = torch.zeros_like(packed4)
        assert L.qlora_kbit_unpack(ctypes.c_void_p(out.data_ptr()), h, o, k, ctypes.c_void_p(back.data_ptr()), None) == 0
        torch.cuda.synchronize()
        want = ((1 << k) - 1) * 0x11
        assert int(back.min()) == want and int(back.max()) == want
    p = ctypes.c_void_p(packed4.data_ptr())
    assert L.qlora_kbit_pack(p, h, o, 4, p, None) == -3
    assert L.qlora_kbit_pack(p, h, 96, 3, p, None) in (-2, -3)
    assert L.qlora_kbit_pack(None, h, o, 3, p, None) == -1
    assert L.qlora_kbit_unpack(ctypes.c_void_p(packed4.data_ptr() + 4), h, o, 3, p, None) == -5
