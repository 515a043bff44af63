"""GPU parity of the few-token (M <= 16) streaming path: forward and input gradient at 1, 4 and 16
tokens on LLaMA-65B-shaped linears (every output element is checked), plus ragged small shapes."""
import numpy as np
import pytest
import torch

from gpu_util import dev_bf16, host_bits, upload_quant
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
    q = dict(packed=Wq.packed.cpu().numpy(), code=Wq.code.cpu().numpy(), c1=Wq.c1.cpu().numpy(),
             mean=np.float32(Wq.mean.cpu().numpy()[0]), rows=h, cols=o, blocksize=64, dq_blocksize=256)
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
