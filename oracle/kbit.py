"""CPU oracle for the k-bit storage of NormalFloat codes with k < 4 (plain numpy).

TEST INFRASTRUCTURE ONLY, like the rest of ``oracle/``.

Section 3 of the paper constructs the k-bit NormalFloat data type for general k (2^k values); a weight stored with it
costs k bits plus the constants' 8/64 + 32/(64 * 256) = 0.127 bits.  The paper does not say how the k-bit codes lie in
memory.  The format here (the exchange format between this oracle and the library, like the nibble order of the 4-bit
types): the codes of the flattened (row-major) weight form one bit stream, code i in bits [k i, k i + k) of it, and bit b
of the stream is bit b % 8 of byte b // 8 (little-endian throughout).  For k = 2 a byte holds 4 codes, for k = 3 three
bytes hold 8 codes, for k = 4 this is the nibble order of the 4-bit types.
"""
from __future__ import annotations

import numpy as np


def codes_of_packed4(packed4) -> np.ndarray:
    """The codes (one uint8 each) of a 4-bit container: element 2i in bits 3:0 of byte i, element 2i+1 in bits 7:4."""
    p = np.asarray(packed4, dtype=np.uint8).ravel()
    out = np.empty(2 * p.size, np.uint8)
    out[0::2] = p & 15
    out[1::2] = p >> 4
    return out


def kbit_pack(codes, k: int) -> np.ndarray:
    """codes: integers in [0, 2^k), their number a multiple of 8.  Returns the k * len / 8 bytes of the bit stream."""
    c = np.asarray(codes, dtype=np.uint8).ravel()
    assert 1 <= k <= 4 and c.size % 8 == 0 and (c.size == 0 or int(c.max()) < (1 << k))
    bits = (c[:, None] >> np.arange(k, dtype=np.uint8)[None, :]) & 1        # code i -> its k bits, lowest first
    return np.packbits(bits.ravel(), bitorder="little")


def kbit_unpack(stream, k: int, count: int) -> np.ndarray:
    """The first `count` codes of a bit stream written by kbit_pack."""
    bits = np.unpackbits(np.asarray(stream, dtype=np.uint8).ravel(), bitorder="little")[: k * count].reshape(count, k)
    return (bits << np.arange(k, dtype=np.uint8)[None, :]).sum(axis=1).astype(np.uint8)


def packed4_of_codes(codes) -> np.ndarray:
    return kbit_pack(codes, 4)


def bits_per_param(k: int, blocksize: int = 64, dq_blocksize: int = 256) -> float:
    """Footprint of a k-bit weight with Double Quantization (Section 3's 4.127 for k = 4)."""
    return k + 8 / blocksize + 32 / (blocksize * dq_blocksize)
