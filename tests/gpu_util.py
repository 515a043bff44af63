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


def code_positions(rows, cols, blocksize=64):
    """Storage position, in the library's c2_code buffer, of every block of the flattened (row-major) order.

    The oracle keeps one code per block in flattened order; the library stores the same codes column-group-major
    (groups of 4 blocks = 256 columns, group after group, row after row inside a group).  This is the index map
    between the two -- a permutation, no arithmetic of the method."""
    bpr = cols // blocksize
    row = np.repeat(np.arange(rows, dtype=np.int64), bpr)
    blk = np.tile(np.arange(bpr, dtype=np.int64), rows)
    grp = blk // 4
    width = np.minimum(4, bpr - 4 * grp)
    return 4 * rows * grp + row * width + blk % 4


def code_to_flat(code_lib, rows, cols):
    """Library-order code bytes -> flattened block order (what the oracle holds)."""
    return np.asarray(code_lib)[code_positions(rows, cols)]


def code_from_flat(code_flat, rows, cols):
    """Flattened block order -> library storage order."""
    out = np.empty_like(np.asarray(code_flat))
    out[code_positions(rows, cols)] = code_flat
    return out


def download_quant(Wq):
    """NF4Weight on the device -> host dict in the oracle's conventions (codes in flattened block order)."""
    return dict(packed=Wq.packed.cpu().numpy(), code=code_to_flat(Wq.code.cpu().numpy(), Wq.rows, Wq.cols),
                c1=Wq.c1.cpu().numpy(), mean=np.float32(Wq.mean.cpu().numpy()[0]), rows=Wq.rows, cols=Wq.cols,
                blocksize=64, dq_blocksize=256)


def upload_quant(q):
    """Oracle quantisation result (host dict) -> NF4Weight on the device."""
    from paper_2305_14314_amd import NF4Weight
    code = code_from_flat(q["code"], q["rows"], q["cols"])
    return NF4Weight(q["rows"], q["cols"], torch.from_numpy(q["packed"]).cuda(), torch.from_numpy(code).cuda(),
                     torch.from_numpy(q["c1"]).cuda(), torch.tensor([q["mean"]], dtype=torch.float32).cuda())
