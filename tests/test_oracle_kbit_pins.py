"""Pins of the k-bit packing oracle (oracle/kbit.py): hand-written byte patterns, the 4-bit case against the nibble
order every other test uses, round trips, the footprint formula of Section 3 extended to k bits."""
import numpy as np
import pytest

import oracle
from oracle import kbit


def test_hand_written_streams():
    # k = 2: codes 1, 2, 3, 0 -> bits 01 10 11 00 from bit 0 upward -> 0b00111001
    assert kbit.kbit_pack([1, 2, 3, 0, 0, 0, 0, 1], 2).tolist() == [0b00111001, 0b01000000]
    # k = 3: codes 0..7 -> stream bit 3i+j = bit j of i: 000 100 010 110 001 101 011 111 (lowest bit first)
    # bytes: bits 0-7 = 0,0,0,1,0,0,0,1 -> 0x88; bits 8-15 = 0,1,1,0,0,0,1,1 -> 0xC6; bits 16-23 = 0,1,0,1,1,1,1,1 -> 0xFA
    assert kbit.kbit_pack(list(range(8)), 3).tolist() == [0x88, 0xC6, 0xFA]
    assert kbit.kbit_pack([7] * 8, 3).tolist() == [0xFF] * 3
    assert kbit.kbit_pack([3] * 8, 2).tolist() == [0xFF] * 2
    # the same through integer arithmetic: the stream is sum(code_i << (k i))
    rng = np.random.default_rng(0)
    for k in (2, 3, 4):
        c = rng.integers(0, 1 << k, 64)
        want = sum(int(v) << (k * i) for i, v in enumerate(c)).to_bytes(8 * k, "little")
        assert bytes(kbit.kbit_pack(c, k)) == want


def test_four_bits_is_the_nibble_order():
    W = np.random.default_rng(1).standard_normal((64, 128)).astype(np.float32)
    q = oracle.nf4_quantize(W)
    codes = kbit.codes_of_packed4(q["packed"])
    assert np.array_equal(kbit.kbit_pack(codes, 4), q["packed"])
    assert codes[0] == (q["packed"][0] & 15) and codes[1] == (q["packed"][0] >> 4)


@pytest.mark.parametrize("k", [2, 3])
def test_round_trip_and_footprint(k):
    W = (np.random.default_rng(2 + k).standard_normal((128, 192)) * 0.02).astype(np.float32)
    q = oracle.nf4_quantize(W, table=oracle.nfk_derive(k).astype(np.float32))
    codes = kbit.codes_of_packed4(q["packed"])
    assert int(codes.max()) == (1 << k) - 1 and int(codes.min()) == 0        # codes >= 2^k never occur
    s = kbit.kbit_pack(codes, k)
    assert s.size == W.size * k // 8
    assert np.array_equal(kbit.kbit_unpack(s, k, W.size), codes)
    assert np.array_equal(kbit.packed4_of_codes(kbit.kbit_unpack(s, k, W.size)), q["packed"])
    total_bits = 8 * (s.size + q["code"].size + 4 * q["c1"].size)
    assert total_bits / W.size == pytest.approx(kbit.bits_per_param(k), abs=0.01)
    assert kbit.bits_per_param(4) == 4 + 8 / 64 + 32 / (64 * 256)              # Section 3: 4.127
