"""Helpers shared by the GPU parity tests (host <-> device plumbing only)."""
import numpy as np
import torch


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def dev_bf16(bits):
    """uint16 bf16 bit patterns -> bf16 device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16))
    return t.view(torch.bfloat16).cuda()


def host_bits(t):
    """bf16 device tensor -> uint16 bit patterns on the host."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_u8(t):
    return t.detach().cpu().numpy()


def host_u32(t):
    """fp32 device tensor -> its bit patterns."""
    return t.detach().cpu().numpy().view(np.uint32)


def bits_f64(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def upload_quant(q):
    """Oracle quantisation result (host dict) -> NF4Weight on the device."""
    from paper_2305_14314_amd import NF4Weight
    return NF4Weight(q["rows"], q["cols"], torch.from_numpy(q["packed"]).cuda(), torch.from_numpy(q["code"]).cuda(),
                     torch.from_numpy(q["c1"]).cuda(), torch.tensor([q["mean"]], dtype=torch.float32).cuda())
