"""The entry point that allocates nothing (qlora_nf4_quantize_static, for callers that cannot call hipMalloc): its
results are those of qlora_nf4_quantize bit for bit, on two calls in a row (the second on a smaller tensor, so the
shared device array still holds the first call's constants), and sizes beyond its limit are refused."""
import ctypes

import pytest
import torch

import paper_2305_14314_amd as q
from paper_2305_14314_amd import synth

pytestmark = pytest.mark.gpu


def _same(a: q.NF4Weight, b: q.NF4Weight):
    assert torch.equal(a.packed, b.packed)
    assert torch.equal(a.code, b.code)
    assert torch.equal(a.c1.view(torch.int32), b.c1.view(torch.int32))
    assert torch.equal(a.mean.view(torch.int32), b.mean.view(torch.int32))


@pytest.mark.parametrize("dq", [256, 0])
def test_static_scratch_matches_the_scratch_argument(dq):
    dev = torch.device("cuda:0")
    for seed, (h, o) in enumerate([(1024, 2752), (320, 192)]):        # the second call is the smaller one
        print(f"static quantise: dq {dq} shape {h} x {o}", flush=True)
        W = torch.from_numpy(synth.normal_f32((h, o), 0.02, seed=40 + seed)).to(dev)
        ref = q.qlora_nf4_quantize(W, dq_blocksize=dq)
        out = q.nf4_alloc(h, o, dev, dq_blocksize=dq)
        for t in (out.packed, out.code, out.c1, out.mean):
            t.view(torch.uint8).fill_(0xA5)
        before = torch.cuda.memory_allocated(dev)
        q.qlora_nf4_quantize_static(W, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(dev) == before
        if dq == 0:
            out.mean.copy_(ref.mean)                                   # not written without Double Quantization
        _same(out, ref)


def test_static_scratch_rejects_sizes_beyond_its_limit():
    dev = torch.device("cuda:0")
    L = q.lib()
    dummy = torch.zeros(64, dtype=torch.float32, device=dev)
    rows, cols = 1 << 15, (1 << 13) + 64                               # one column group over 2^28 weights
    assert rows * cols > q.STATIC_QUANT_MAX_WEIGHTS
    p = ctypes.c_void_p(dummy.data_ptr())
    st = L.qlora_nf4_quantize_static(p, rows, cols, 64, 256, p, p, p, p, None)
    assert st == -4, st                                                # QLORA_ERR_WORKSPACE, before any launch
    assert b"WORKSPACE" in L.qlora_status_string(st)
