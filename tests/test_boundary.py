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
    for st in range(-7, 1):
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


def test_linear_arguments_are_rejected_on_the_host(L):
    from paper_2305_14314_amd import QloraError, qlora_linear_bwd_sizes, qlora_linear_fwd_sizes
    from paper_2305_14314_amd.binding import WORKSPACE_HEADER_BYTES, qlora_nf4_view
    # shapes: in/out features multiples of 64, rank a multiple of 16 up to 256, at least one token
    for fn in (qlora_linear_fwd_sizes, qlora_linear_bwd_sizes):
        for args, st in [((0, 64, 64, 0), -2), ((4, 96, 64, 0), -3), ((4, 64, 96, 0), -3), ((4, 64, 64, 8), -3),
                         ((4, 64, 64, 272), -3), ((4, 64, 64, -16), -2)]:
            with pytest.raises(QloraError) as e:
                fn(*args)
            assert e.value.status == st
        # every workspace starts with the counter header, whichever path the token count selects
        assert fn(1, 64, 64, 0) > WORKSPACE_HEADER_BYTES and fn(4096, 64, 64, 16) > WORKSPACE_HEADER_BYTES
    fake = ctypes.c_void_p(0x1000)                # never dereferenced: validation fails first
    v = qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256)
    big = 1 << 30
    f = L.qlora_linear_fwd
    assert f(None, ctypes.byref(v), None, None, 1.0, 4, 0, fake, None, fake, big, None) == -1          # X
    assert f(fake, ctypes.byref(v), None, None, 1.0, 4, 0, None, None, fake, big, None) == -1          # Y
    assert f(fake, ctypes.byref(v), None, None, 1.0, 4, 0, fake, None, None, big, None) == -1          # workspace
    assert f(fake, ctypes.byref(v), None, fake, 1.0, 4, 16, fake, None, fake, big, None) == -1         # L1 with r > 0
    assert f(fake, ctypes.byref(v), None, None, 1.0, 4, 0, fake, None, fake, 64, None) == -4           # too small
    assert f(ctypes.c_void_p(0x1008), ctypes.byref(v), None, None, 1.0, 4, 0, fake, None, fake, big, None) == -5
    b = L.qlora_linear_bwd
    assert b(None, None, ctypes.byref(v), None, None, 1.0, 4, 0, None, fake, None, None, fake, big, None) == -1   # dY
    assert b(fake, None, ctypes.byref(v), fake, fake, 1.0, 4, 16, None, fake, fake, None, fake, big, None) == -1  # dL1 needs X
    assert b(fake, None, ctypes.byref(v), None, None, 1.0, 4, 0, None, fake, None, None, fake, 64, None) == -4
    a = L.qlora_linear_bwd_acc                    # same checks; the gradient outputs are fp32 accumulators
    assert a(None, None, ctypes.byref(v), None, None, 1.0, 4, 0, None, fake, None, None, fake, big, None) == -1
    assert a(fake, None, ctypes.byref(v), fake, fake, 1.0, 4, 16, None, fake, fake, None, fake, big, None) == -1  # needs X
    assert a(fake, fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, None, fake, ctypes.c_void_p(0x1004), None, fake, big, None) == -5
    w = L.qlora_workspace_init
    assert w(None, big, None) == -1
    assert w(fake, WORKSPACE_HEADER_BYTES - 1, None) == -4
    assert w(ctypes.c_void_p(0x1004), big, None) == -5


def test_multi_layer_arguments_are_rejected_on_the_host(L):
    """The several-layers-on-one-input forward validates before any HIP call: layer count, every layer's shape,
    one common number of input features, pointers, alignment and workspace size."""
    from paper_2305_14314_amd import QloraError, qlora_linear_fwd_multi_sizes, qlora_linear_fwd_sizes
    from paper_2305_14314_amd.binding import WORKSPACE_HEADER_BYTES, qlora_nf4_view
    for args, st in [((4, 64, [], []), -2), ((4, 64, [64] * 5, [0] * 5), -2), ((4, 64, [64, 96], [0, 0]), -3),
                     ((4, 64, [64, 64], [0, 8]), -3), ((0, 64, [64], [0]), -2)]:
        with pytest.raises(QloraError) as e:
            qlora_linear_fwd_multi_sizes(*args)
        assert e.value.status == st
    assert qlora_linear_fwd_multi_sizes(4, 64, [64, 128], [0, 16]) > WORKSPACE_HEADER_BYTES
    # many tokens: the layers run one after the other in one workspace of the largest single-layer size
    assert qlora_linear_fwd_multi_sizes(300, 64, [64, 128], [0, 16]) == max(qlora_linear_fwd_sizes(300, 64, 64, 0),
                                                                              qlora_linear_fwd_sizes(300, 64, 128, 16))
    fake = ctypes.c_void_p(0x1000)
    big = 1 << 30
    n = 2
    views = (qlora_nf4_view * n)(qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256),
                                 qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 64, 64, 256))
    ptrs = lambda *v: (ctypes.c_void_p * n)(*v)
    s, r0, r16 = (ctypes.c_float * n)(1.0, 1.0), (ctypes.c_int32 * n)(0, 0), (ctypes.c_int32 * n)(0, 16)
    f = L.qlora_linear_fwd_multi
    ok_y = ptrs(0x1000, 0x1000)
    assert f(None, n, views, None, None, s, 4, r0, ok_y, fake, big, None) == -1                         # X
    assert f(fake, n, views, None, None, s, 4, r0, ptrs(0x1000, None), fake, big, None) == -1           # Y[1]
    assert f(fake, n, views, None, None, s, 4, r16, ok_y, fake, big, None) == -1                        # L1 with r > 0
    assert f(fake, n, views, ptrs(None, 0x1000), ptrs(None, None), s, 4, r16, ok_y, fake, big, None) == -1
    assert f(fake, 0, views, None, None, s, 4, r0, ok_y, fake, big, None) == -2
    assert f(fake, 5, views, None, None, s, 4, r0, ok_y, fake, big, None) == -2
    assert f(fake, n, views, None, None, s, 4, r0, ok_y, fake, 64, None) == -4                          # too small
    assert f(fake, n, views, None, None, s, 4, r0, ptrs(0x1000, 0x1008), fake, big, None) == -5
    views[1].rows = 192                                                                                # another h
    assert f(fake, n, views, None, None, s, 4, r0, ok_y, fake, big, None) == -2


def test_dropout_arguments_are_rejected_on_the_host(L):
    """LoRA-dropout calls: the rate must lie in [0, 1), the mask is required exactly when there is an adapter, and
    the workspace is the large-GEMM one whatever the number of tokens."""
    from paper_2305_14314_amd import qlora_linear_bwd_sizes, qlora_linear_dropout_sizes, qlora_linear_fwd_sizes
    from paper_2305_14314_amd.binding import qlora_nf4_view
    fake = ctypes.c_void_p(0x1000)
    v = qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256)
    big = 1 << 30
    f = L.qlora_linear_fwd_dropout
    assert f(fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, 1.0, fake, None, fake, big, None) == -2      # p = 1
    assert f(fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, -0.1, fake, None, fake, big, None) == -2
    assert f(fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, float("nan"), fake, None, fake, big, None) == -2
    assert f(fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, None, 0.1, fake, None, fake, big, None) == -1      # mask
    assert f(None, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, 0.1, fake, None, fake, big, None) == -1      # X
    assert f(fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, 0.1, fake, None, fake, 64, None) == -4
    b = L.qlora_linear_bwd_dropout
    assert b(fake, fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, 1.5, None, fake, None, None, None, None, fake, big, None) == -2
    assert b(fake, fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, None, 0.1, None, fake, None, None, None, None, fake, big, None) == -1
    assert b(fake, None, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, 0.1, None, fake, fake, None, None, None, fake, big, None) == -1  # dL1 needs X
    assert b(fake, fake, ctypes.byref(v), fake, fake, 1.0, 4, 16, fake, 0.1, None, fake, None, None, None, None, fake, 64, None) == -4
    # 4 tokens: the plain calls would stream (small workspace), the dropout calls dequantise the whole weight; the
    # plain size queries know no data type and report a size that serves both plans (an 8-bit or not double-quantised
    # weight takes the dequantise plan at any M)
    fb, bb = qlora_linear_dropout_sizes(4, 1024, 1024, 16)
    assert fb >= 2 * 1024 * 1024 and bb >= 2 * 1024 * 1024
    assert qlora_linear_fwd_sizes(4, 1024, 1024, 16) >= fb and qlora_linear_bwd_sizes(4, 1024, 1024, 16) >= bb
    assert qlora_linear_dropout_sizes(300, 1024, 1024, 16) == (qlora_linear_fwd_sizes(300, 1024, 1024, 16),
                                                                qlora_linear_bwd_sizes(300, 1024, 1024, 16))
    # no adapter, nothing to drop: the dropout calls are the plain ones, streaming kernels included (small workspace)
    f0, b0 = qlora_linear_dropout_sizes(4, 1024, 1024, 0)
    assert f0 < 1024 * 1024 and b0 < 1024 * 1024
    assert f0 <= qlora_linear_fwd_sizes(4, 1024, 1024, 0) and b0 <= qlora_linear_bwd_sizes(4, 1024, 1024, 0)


def test_data_type_tables_and_their_validation(L, oracle):
    """The library's tables of the 4-bit data types equal the oracle's bit for bit (host call, no GPU), unknown
    types are refused, and a view carries its type."""
    import numpy as np
    from paper_2305_14314_amd import qlora_codebook_4bit
    from paper_2305_14314_amd.binding import QloraError, qlora_nf4_view
    for name, dtype in (("nf4", 0), ("fp4_e2m1", 1), ("fp4_e3m0", 2), ("int4", 3), ("nf3", 5), ("nf2", 6)):
        mine = np.array(qlora_codebook_4bit(dtype), np.float32)
        assert np.array_equal(mine.view(np.uint32), oracle.codebook4(name).view(np.uint32)), name
    for bad in (-1, 4, 7):
        with pytest.raises(QloraError) as e:
            qlora_codebook_4bit(bad)
        assert e.value.status == -3
    fake = ctypes.c_void_p(0x1000)
    assert L.qlora_codebook_4bit(0, None) == -1
    assert L.qlora_quantize_4bit(fake, 4, 64, 64, 256, 7, fake, fake, fake, fake, fake, 1 << 20, None) == -3
    assert L.qlora_quantize_4bit(None, 4, 64, 64, 256, 1, fake, fake, fake, fake, fake, 1 << 20, None) == -1
    v = qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256, 7, 0)
    assert L.qlora_nf4_dequant(ctypes.byref(v), fake, None) == -3
    # Int8 is a data type of a view, but has no table and is not a 4-bit type
    assert L.qlora_quantize_4bit(fake, 4, 64, 64, 256, 4, fake, fake, fake, fake, fake, 1 << 20, None) == -3
    v = qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256, 4, 0)
    assert L.qlora_nf4_dequant(ctypes.byref(v), None, None) == -1           # the view passes, the output is missing
    v = qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256)       # eight fields: NF4
    assert v.dtype == 0


def test_int8_sizes_and_validation(L):
    """8-bit integers: one byte per weight, the constants as for the 4-bit types (8.127 bit per parameter with Double
    Quantization, 8.5 without); argument checks of the quantise call (host only: every call stops at validation)."""
    from paper_2305_14314_amd import INT8, qlora_nf4_sizes, qlora_quant_sizes
    from paper_2305_14314_amd.binding import QloraError
    P = 8192 * 8192
    pb, cb, c1b, sb = qlora_quant_sizes(8192, 8192, 64, 256, INT8)
    assert (pb, cb, c1b) == (P, P // 64, 4 * P // (64 * 256)) and sb == qlora_nf4_sizes(8192, 8192)[3]
    assert abs((pb + cb + c1b) * 8 / P - 8.127) < 1e-3
    pb, cb, c1b, _ = qlora_quant_sizes(8192, 8192, 64, 0, INT8)
    assert (pb + cb + c1b) * 8 / P == 8.5
    assert qlora_quant_sizes(8192, 8192, 64, 256, 0) == qlora_nf4_sizes(8192, 8192, 64, 256)
    with pytest.raises(QloraError) as e:
        qlora_quant_sizes(64, 64, 64, 256, 7)
    assert e.value.status == -3
    assert qlora_quant_sizes(8192, 8192, 64, 256, 5) == qlora_nf4_sizes(8192, 8192, 64, 256)   # NF3: 4-bit containers
    fake = ctypes.c_void_p(0x1000)
    q = L.qlora_quantize_int8
    assert q(None, 4, 64, 64, 256, fake, fake, fake, fake, fake, 1 << 20, None) == -1
    assert q(fake, 4, 64, 64, 256, None, fake, fake, fake, fake, 1 << 20, None) == -1
    assert q(fake, 4, 64, 64, 256, fake, None, fake, fake, fake, 1 << 20, None) == -1
    assert q(fake, 4, 64, 64, 0, fake, None, fake, None, fake, 8, None) == -4        # no DQ: code / mean may be NULL
    assert q(fake, 4, 60, 64, 256, fake, fake, fake, fake, fake, 1 << 20, None) == -2
    assert q(fake, 4, 64, 32, 256, fake, fake, fake, fake, fake, 1 << 20, None) == -3
    assert q(fake, 4, 64, 64, 256, fake, fake, fake, fake, fake, 8, None) == -4
    assert q(ctypes.c_void_p(0x1004), 4, 64, 64, 256, fake, fake, fake, fake, fake, 1 << 20, None) == -5


def test_sizes_without_double_quantization(L):
    """dq_blocksize = 0: no code bytes, one fp32 constant per block (4.5 bit per parameter, Section 3), and a view
    needs only its packed indices and constants."""
    from paper_2305_14314_amd import qlora_nf4_sizes
    from paper_2305_14314_amd.binding import qlora_nf4_view
    pb, cb, c1b, sb = qlora_nf4_sizes(8192, 8192, 64, 0)
    P = 8192 * 8192
    assert (pb, cb, c1b) == (P // 2, 0, 4 * P // 64) and (pb + cb + c1b) * 8 / P == 4.5
    fake = ctypes.c_void_p(0x1000)
    v = qlora_nf4_view(0x1000, None, 0x1000, None, 128, 128, 64, 0)
    assert L.qlora_nf4_dequant(ctypes.byref(v), None, None) == -1            # the view passes, the output is missing
    v = qlora_nf4_view(0x1000, None, None, None, 128, 128, 64, 0)
    assert L.qlora_nf4_dequant(ctypes.byref(v), fake, None) == -1            # the constants are still required
    # no code / mean buffers needed: the call gets past the NULL checks and stops at the (deliberately) small scratch
    assert L.qlora_nf4_quantize(fake, 4, 64, 64, 0, fake, None, fake, None, fake, 8, None) == -4


def test_constant_storage_order_is_a_permutation_that_keeps_groups_together():
    """The 8-bit constants are stored column-group-major (include/qlora.h).  The index map used by the parity
    tests and the one the binding offers agree, are permutations, and put the <= 4 constants of one row and one
    256-column group side by side -- for widths that are and are not multiples of 256 columns."""
    import numpy as np
    import torch
    from gpu_util import code_from_flat, code_positions, code_to_flat
    from paper_2305_14314_amd import NF4Weight
    for rows, cols in [(1, 64), (3, 256), (5, 320), (7, 704), (64, 22016 // 43)]:
        bpr = cols // 64
        pos = code_positions(rows, cols)
        assert sorted(pos.tolist()) == list(range(rows * bpr))
        flat = np.arange(rows * bpr, dtype=np.int64)
        lib_order = code_from_flat(flat, rows, cols)
        assert np.array_equal(code_to_flat(lib_order, rows, cols), flat)
        for r in range(rows):
            for g in range((bpr + 3) // 4):
                w = min(4, bpr - 4 * g)
                p0 = pos[r * bpr + 4 * g]
                assert p0 == 4 * rows * g + r * w                       # the formula of the header
                assert np.array_equal(pos[r * bpr + 4 * g:r * bpr + 4 * g + w], p0 + np.arange(w))
        codes = torch.from_numpy((lib_order % 251).astype(np.uint8))
        Wq = NF4Weight(rows, cols, None, codes, None, None)
        assert np.array_equal(Wq.code_flat().numpy(), (flat % 251).astype(np.uint8))


def test_header_is_plain_c_and_the_library_links_from_c(L, tmp_path):
    """include/qlora.h compiles as C99 with -pedantic, and a C program linked against the library gets the footprint
    of Section 3, a data-type table and a status string through the host-only entry points (no GPU touched)."""
    import shutil
    import subprocess
    from paper_2305_14314_amd import binding
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "abi.c"
    src.write_text('#include "qlora.h"\n#include <stdio.h>\n'
                   'int main(void) {\n'
                   '  size_t pb = 0, cb = 0, c1b = 0, sb = 0;\n'
                   '  float t[16];\n'
                   '  qlora_status a = qlora_nf4_sizes(8192, 22016, 64, 256, &pb, &cb, &c1b, &sb);\n'
                   '  qlora_status b = qlora_codebook_4bit(QLORA_FP4_E3M0, t);\n'
                   '  printf("%d %lu %lu %lu %d %g %g %s\\n", (int)a, (unsigned long)pb, (unsigned long)cb, (unsigned long)c1b,\n'
                   '         (int)b, t[9], t[15], qlora_status_string(QLORA_ERR_ALIGN));\n'
                   '  return 0;\n}\n')
    exe = tmp_path / "abi"
    libdir = os.path.dirname(binding.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-lqlora_hip", f"-Wl,-rpath,{libdir}",
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(maxsplit=7)
    P = 8192 * 22016
    assert out[:7] == ["0", str(P // 2), str(P // 64), str(4 * P // (64 * 256)), "0", "0.015625", "1"]
    assert out[7].startswith("QLORA_ERR_ALIGN")


def test_list_and_header_arguments_are_rejected_on_the_host(L):
    """The persistent list calls, the header check and the poll limit validate before any HIP call."""
    from paper_2305_14314_amd import QloraError, qlora_linear_list_sizes
    from paper_2305_14314_amd.binding import LIST_MAX, WORKSPACE_HEADER_BYTES, qlora_nf4_view
    assert LIST_MAX == 8
    assert qlora_linear_list_sizes(4, [64, 128], [64, 64], [0, 16]) > WORKSPACE_HEADER_BYTES
    assert qlora_linear_list_sizes(4, [64, 128], [64, 64], [0, 16], backward=True) > WORKSPACE_HEADER_BYTES
    for args, st in [((4, [], [], []), -2), ((4, [64] * 9, [64] * 9, [0] * 9), -2), ((4, [64], [96], [0]), -3),
                     ((0, [64], [64], [0]), -2), ((4, [64], [64], [8]), -3)]:
        with pytest.raises(QloraError) as e:
            qlora_linear_list_sizes(*args)
        assert e.value.status == st, args
    fake, big, n = ctypes.c_void_p(0x1000), 1 << 30, 2
    views = (qlora_nf4_view * n)(qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256),
                                 qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 64, 128, 64, 256))
    ptrs = lambda *v: (ctypes.c_void_p * n)(*v)
    s, r0, r16 = (ctypes.c_float * n)(1.0, 1.0), (ctypes.c_int32 * n)(0, 0), (ctypes.c_int32 * n)(0, 16)
    ok = ptrs(0x1000, 0x1000)
    for f in (L.qlora_linear_fwd_list, L.qlora_linear_bwd_list):
        assert f(n, None, views, None, None, s, 4, r0, ok, fake, big, None) == -1                      # inputs
        assert f(n, ptrs(0x1000, None), views, None, None, s, 4, r0, ok, fake, big, None) == -1        # input 1
        assert f(n, ok, views, None, None, s, 4, r0, ptrs(None, 0x1000), fake, big, None) == -1        # output 0
        assert f(n, ok, views, None, None, s, 4, r16, ok, fake, big, None) == -1                       # adapter of layer 1
        assert f(n, ok, views, None, None, s, 4, r0, ok, None, big, None) == -1                        # workspace
        assert f(0, ok, views, None, None, s, 4, r0, ok, fake, big, None) == -2
        assert f(9, ok, views, None, None, s, 4, r0, ok, fake, big, None) == -2
        assert f(n, ok, views, None, None, s, 0, r0, ok, fake, big, None) == -2
        assert f(n, ok, views, None, None, s, 4, r0, ok, fake, 64, None) == -4                         # too small
        assert f(n, ok, views, None, None, s, 4, r0, ptrs(0x1000, 0x1008), fake, big, None) == -5
    # the header check: arguments first (it would synchronise the stream and read the status word otherwise)
    assert L.qlora_workspace_check(None, big, None) == -1
    assert L.qlora_workspace_check(fake, WORKSPACE_HEADER_BYTES - 1, None) == -4
    assert L.qlora_status_string(-7).startswith(b"QLORA_ERR_STATE")
    L.qlora_fewtok_poll_limit(-5)                              # clamped, no error path
    L.qlora_fewtok_poll_limit(64)


def test_optimizer_arguments_are_rejected_on_the_host(L):
    from paper_2305_14314_amd.binding import qlora_adam_config
    fake = ctypes.c_void_p(0x1000)
    cfg = qlora_adam_config(1e-4, 0.9, 0.999, 1e-8, 0.0, 1.0, 0.3, 1, 0, 0)
    f = L.qlora_adam_step
    assert f(fake, fake, fake, fake, None, 64, None, None, None) == -1                                  # no config
    assert f(None, fake, fake, fake, None, 64, ctypes.byref(cfg), None, None) == -1
    assert f(fake, fake, fake, None, None, 64, ctypes.byref(cfg), None, None) == -1
    assert f(fake, fake, fake, fake, None, -1, ctypes.byref(cfg), None, None) == -2
    assert f(ctypes.c_void_p(0x1004), fake, fake, fake, None, 64, ctypes.byref(cfg), None, None) == -5
    assert f(fake, fake, fake, fake, ctypes.c_void_p(0x1004), 64, ctypes.byref(cfg), None, None) == -5  # bf16 copy
    assert f(fake, fake, fake, fake, None, 64, ctypes.byref(cfg), ctypes.c_void_p(0x1004), None) == -5  # norm
    assert f(None, None, None, None, None, 0, ctypes.byref(cfg), None, None) == 0                       # empty: nothing to do
    for field, bad in (("step", 0), ("beta1", 1.0), ("beta2", -0.1), ("eps", -1.0), ("lr", float("nan")), ("reserved", 1)):
        c = qlora_adam_config(1e-4, 0.9, 0.999, 1e-8, 0.0, 1.0, 0.3, 1, 0, 0)
        setattr(c, field, bad)
        assert f(fake, fake, fake, fake, None, 64, ctypes.byref(c), None, None) in (-2, -3), field
    g = L.qlora_grad_sqnorm
    assert g(None, 64, fake, None) == -1 and g(fake, 64, None, None) == -1
    assert g(fake, -1, fake, None) == -2 and g(None, 0, None, None) == 0
    assert g(ctypes.c_void_p(0x1004), 64, fake, None) == -5 and g(fake, 64, ctypes.c_void_p(0x1004), None) == -5
    # the static-scratch quantiser: its size limit is checked before anything else touches the device
    q = L.qlora_nf4_quantize_static
    assert q(fake, 1 << 15, (1 << 13) + 64, 64, 256, fake, fake, fake, fake, None) == -4
    assert q(None, 64, 64, 64, 256, fake, fake, fake, fake, None) == -1
    assert q(fake, 64, 96, 64, 256, fake, fake, fake, fake, None) in (-2, -3)


def test_stacked_arguments_are_rejected_on_the_host(L):
    """One matrix product for the layers that share an input, forward and backward: validation before any HIP call."""
    from paper_2305_14314_amd import (QloraError, qlora_linear_bwd_stacked_sizes, qlora_linear_fwd_sizes,
                                      qlora_linear_fwd_stacked_sizes)
    from paper_2305_14314_amd.binding import qlora_nf4_view
    for fn in (qlora_linear_fwd_stacked_sizes, qlora_linear_bwd_stacked_sizes):
        for args, st in [((4, 64, [], []), -2), ((4, 64, [64] * 5, [0] * 5), -2), ((4, 64, [64, 96], [0, 0]), -3),
                         ((4, 64, [64, 64], [0, 8]), -3), ((0, 64, [64], [0]), -2)]:
            with pytest.raises(QloraError) as e:
                fn(*args)
            assert e.value.status == st
    # the stacked weight: (sum o) x (h + sum of padded ranks) bf16 values, plus the small buffers
    M, h, outs, ranks = 300, 1024, [1024, 512], [16, 80]
    assert qlora_linear_fwd_stacked_sizes(M, h, outs, ranks) >= 2 * sum(outs) * (h + 64 + 128)
    assert qlora_linear_bwd_stacked_sizes(M, h, outs, ranks) >= 2 * sum(outs) * h + 2 * h * (64 + 128)
    assert qlora_linear_fwd_stacked_sizes(M, h, [1024], [16]) <= qlora_linear_fwd_sizes(M, h, 1024, 16) + 4096
    fake, big, n = ctypes.c_void_p(0x1000), 1 << 34, 2
    views = (qlora_nf4_view * n)(qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 128, 64, 256),
                                 qlora_nf4_view(0x1000, 0x1000, 0x1000, 0x1000, 128, 64, 64, 256))
    ptrs = lambda *v: (ctypes.c_void_p * n)(*v)
    s, r0, r16 = (ctypes.c_float * n)(1.0, 1.0), (ctypes.c_int32 * n)(0, 0), (ctypes.c_int32 * n)(0, 16)
    f = L.qlora_linear_fwd_stacked
    assert f(None, n, views, None, None, s, 4, r0, fake, None, fake, big, None) == -1                       # X
    assert f(fake, n, views, None, None, s, 4, r0, None, None, fake, big, None) == -1                       # Y
    assert f(fake, n, views, None, None, s, 4, r16, fake, None, fake, big, None) == -1                      # L1 with r > 0
    assert f(fake, 0, views, None, None, s, 4, r0, fake, None, fake, big, None) == -2
    assert f(fake, 5, views, None, None, s, 4, r0, fake, None, fake, big, None) == -2
    assert f(fake, n, views, None, None, s, 4, r0, fake, None, fake, 64, None) == -4
    assert f(fake, n, views, None, None, s, 4, r0, ctypes.c_void_p(0x1008), None, fake, big, None) == -5
    assert f(fake, n, views, None, None, s, 4, r0, fake, ptrs(0x1000, 0x1008), fake, big, None) == -5       # T_save[1]
    b = L.qlora_linear_bwd_stacked
    assert b(None, fake, n, views, None, None, s, 4, r0, None, fake, None, None, fake, big, None) == -1     # dY
    assert b(fake, fake, n, views, None, None, s, 4, r0, None, None, None, None, fake, big, None) == -1     # dX
    assert b(fake, None, n, views, ptrs(None, 0x1000), ptrs(None, 0x1000), s, 4, r16, None, fake,
             ptrs(None, 0x1000), None, fake, big, None) == -1                                               # dL1 needs X
    assert b(fake, None, n, views, ptrs(None, 0x1000), ptrs(None, 0x1000), s, 4, r16, None, fake, None, None, fake, 64,
             None) == -4
    assert b(fake, fake, n, views, None, None, s, 4, r0, None, ctypes.c_void_p(0x1004), None, None, fake, big, None) == -5
    views[1].rows = 192                                                                                     # another h
    assert f(fake, n, views, None, None, s, 4, r0, fake, None, fake, big, None) == -2
    assert b(fake, fake, n, views, None, None, s, 4, r0, None, fake, None, None, fake, big, None) == -2


def test_kbit_arguments_are_rejected_on_the_host(L):
    from paper_2305_14314_amd import qlora_kbit_sizes
    assert qlora_kbit_sizes(8192, 22016, 3) == 8192 * 22016 * 3 // 8
    assert qlora_kbit_sizes(64, 64, 2) == 1024
    # with the constants: 3.127 and 2.127 bits per parameter (Section 3's formula with k in place of 4)
    P = 8192 * 22016
    assert (qlora_kbit_sizes(8192, 22016, 3) + P // 64 + 4 * P // (64 * 256)) * 8 / P == 3 + 8 / 64 + 32 / (64 * 256)
    fake = ctypes.c_void_p(0x1000)
    out = ctypes.c_size_t()
    assert L.qlora_kbit_sizes(64, 64, 4, ctypes.byref(out)) == -3
    assert L.qlora_kbit_sizes(64, 64, 3, None) == -1
    assert L.qlora_kbit_sizes(64, 96, 3, ctypes.byref(out)) == -2
    for f in (L.qlora_kbit_pack, L.qlora_kbit_unpack):
        assert f(None, 64, 64, 3, fake, None) == -1 and f(fake, 64, 64, 3, None, None) == -1
        assert f(fake, 64, 64, 1, fake, None) == -3 and f(fake, 0, 64, 3, fake, None) == -2
        assert f(ctypes.c_void_p(0x1008), 64, 64, 3, fake, None) == -5
        assert f(fake, 64, 64, 2, ctypes.c_void_p(0x1004), None) == -5
