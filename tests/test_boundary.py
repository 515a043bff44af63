"""Host-only checks of the C-ABI boundary: the library loads, exports every declared entry
point, and rejects bad arguments with a status code before any HIP call (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2305_14314_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    return binding.lib()


def test_every_declared_symbol_is_exported(L):
    text = open(os.path.join(ROOT, "include", "qlora.h")).read()
    declared = set(re.findall(r"\b(qlora_[a-z0-9_]+)\s*\(", text))
    assert {"qlora_nf4_quantize", "qlora_nf4_dequant", "qlora_linear_fwd", "qlora_linear_bwd"} <= declared
    for name in declared:
        assert hasattr(L, name), f"{name} declared in qlora.h but not exported"
    from paper_2305_14314_amd import binding
    assert declared == set(binding.EXPORTS)


def test_status_strings(L):
    for st in range(-6, 1):
        assert L.qlora_status_string(st).startswith(b"QLORA_")


def test_sizes_follow_the_footprint_formula(L):
    from paper_2305_14314_amd import qlora_nf4_sizes
    pb, cb, c1b, sb = qlora_nf4_sizes(8192, 22016)
    P = 8192 * 22016
    assert (pb, cb, c1b) == (P // 2, P // 64, 4 * P // (64 * 256))
    assert (pb + cb + c1b) * 8 / P == 4 + 8 / 64 + 32 / (64 * 256)      # Section 3: 4.127 bit/param
    assert sb >= 4 * P // 64


def test_bad_arguments_are_rejected_on_the_host(L):
    from paper_2305_14314_amd import QloraError, qlora_nf4_sizes
    from paper_2305_14314_amd.binding import qlora_nf4_view
    for args, st in [((0, 64), -2), ((4, 96), -2), ((4, 64, 32, 256), -3), ((4, 64, 64, 128), -3), ((-1, 64), -2)]:
        with pytest.raises(QloraError) as e:
            qlora_nf4_sizes(*args)
        assert e.value.status == st
    fake = ctypes.c_void_p(0x1000)                # never dereferenced: validation fails first
    assert L.qlora_nf4_quantize(None, 4, 64, 64, 256, fake, fake, fake, fake, fake, 1 << 20, None) == -1
    assert L.qlora_nf4_quantize(fake, 4, 64, 64, 256, fake, fake, fake, fake, fake, 8, None) == -4
    assert L.qlora_nf4_quantize(ctypes.c_void_p(0x1004), 4, 64, 64, 256, fake, fake, fake, fake, fake,
                                1 << 20, None) == -5
    assert L.qlora_nf4_dequant(None, fake, None) == -1
    v = qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 4, 96, 64, 256)
    assert L.qlora_nf4_dequant(ctypes.byref(v), fake, None) == -2
    v = qlora_nf4_view(0x1000, 0, 0x1000, 0x1000, 4, 128, 64, 256)
    assert L.qlora_nf4_dequant(ctypes.byref(v), fake, None) == -1
