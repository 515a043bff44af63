"""Pins for the CPU oracle: everything here checks the oracle against something
other than itself -- values the paper prints, closed forms, invariants, library
routines on special cases, exact rational arithmetic, brute force on tiny inputs.
No GPU needed."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_table():
    vals = []
    with open(os.path.join(GOLD, "nf4_appendix_e.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                vals.append(line)
    return vals


def _bf16_bits(a):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def _bf16_f64(b):
    return (np.asarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- codebook

def test_nf4_table_is_the_printed_one(oracle):
    printed = _read_table()
    tab = oracle.nf4_table()
    assert len(printed) == 16
    for s, v in zip(printed, tab):
        # the printed decimal is the shortest form of a double that is exactly the fp32 entry
        assert float(s) == float(v) and repr(float(v)) == s, (s, v)


def test_nf4_table_structure(oracle):
    tab = oracle.nf4_table().astype(np.float64)
    assert np.all(np.diff(tab) > 0)
    assert tab[0] == -1.0 and tab[15] == 1.0 and tab[7] == 0.0
    assert (tab < 0).sum() == 7 and (tab > 0).sum() == 8


def test_nf4_table_from_normal_quantiles(oracle):
    # Section 3: asymmetric construction from N(0,1) quantiles, normalised to [-1, 1].
    p_max = 1.0 - 0.5 * (1.0 / 32.0 + 1.0 / 30.0)
    derived = oracle.nf4_derive(p_max)
    tab = oracle.nf4_table().astype(np.float64)
    assert np.abs(derived - tab).max() <= 2e-7
    assert derived[7] == 0.0 and derived[0] == -1.0 and derived[15] == 1.0
    # a wrong split (8 negative / 7 positive steps) must not fit
    wrong = -oracle.nf4_derive(p_max)[::-1]
    assert np.abs(wrong - tab).max() > 1e-2


def test_normal_quantile_against_library(oracle):
    from scipy.stats import norm
    for p in [1e-6, 0.01, 0.25, 0.5, 0.75, 0.9677083, 0.999]:
        assert abs(oracle.normal_quantile(p) - norm.ppf(p)) < 1e-11


# ----------------------------------------------------------------------------- index assignment

def test_index_is_nearest_value_bruteforce(oracle):
    tab = oracle.nf4_table()
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.uniform(-1, 1, 4000), tab.astype(np.float64),
                         [0.0, -0.0, 1.0000001, -1.0000001, 1e-30, -1e-30]]).astype(np.float32)
    for x in xs:
        d = [abs(Fraction(float(x)) - Fraction(float(q))) for q in tab]
        best = min(d)
        winners = [j for j in range(16) if d[j] == best]
        got = oracle.nf4_index(x)
        assert got == winners[0], (x, got, winners)       # lower index on an exact tie


def test_index_ties_and_monotone(oracle):
    tab = oracle.nf4_table()
    n_ties = 0
    for j in range(15):
        mid = (Fraction(float(tab[j])) + Fraction(float(tab[j + 1]))) / 2
        m32 = np.float32(float(mid))
        if Fraction(float(m32)) == mid:                     # representable midpoint: a real tie
            n_ties += 1
            assert oracle.nf4_index(m32) == j
            assert oracle.nf4_index(np.nextafter(m32, np.float32(2))) == j + 1
        else:
            lo = m32 if Fraction(float(m32)) < mid else np.nextafter(m32, np.float32(-2))
            assert oracle.nf4_index(lo) == j
            assert oracle.nf4_index(np.nextafter(lo, np.float32(2))) == j + 1
    assert n_ties == 6                                      # six of the 15 midpoints are fp32 numbers
    xs = np.sort(np.random.default_rng(2).uniform(-1.1, 1.1, 2000).astype(np.float32))
    idx = [oracle.nf4_index(x) for x in xs]
    assert all(a <= b for a, b in zip(idx, idx[1:]))
    assert oracle.nf4_index(np.float32(0.0)) == 7 and oracle.nf4_index(np.float32(-0.0)) == 7


# ----------------------------------------------------------------------------- roundings

def test_bf16_rne_against_library(oracle):
    rng = np.random.default_rng(3)
    vals = np.concatenate([
        rng.standard_normal(3000).astype(np.float32),
        (rng.standard_normal(500) * 1e-20).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 1.0 + 2**-8, 1.0 + 3 * 2**-8, 3.3895314e38,
                  -2.5, 65280.0, 65408.0, 65535.9], np.float32)])
    want = _bf16_bits(vals)
    got = np.array([oracle.bf16_rne(v) for v in vals], np.uint16)
    np.testing.assert_array_equal(got, want)


def test_e4m3_decode_against_library(oracle):
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for c in range(256):
        v = oracle.e4m3_value(c)
        if c & 0x7F == 0x7F:
            assert np.isnan(v) and np.isnan(lib[c])
        else:
            assert v == lib[c], (c, v, lib[c])
    assert oracle.e4m3_value(0x7E) == 448.0 and oracle.e4m3_value(0x01) == 2.0 ** -9
    finite = {oracle.e4m3_value(c) for c in range(256) if c & 0x7F != 0x7F}
    assert len(finite) == 253                               # +0 and -0 coincide


def test_e4m3_encode_against_library(oracle):
    rng = np.random.default_rng(4)
    mags = np.array([oracle.e4m3_value(c) for c in range(0x7F)], np.float64)
    mids = (mags[:-1] + mags[1:]) / 2                       # every tie point of the format
    zs = np.concatenate([rng.uniform(-448, 448, 4000), rng.uniform(-1, 1, 2000), rng.uniform(-0.02, 0.02, 2000),
                         mags, -mags, mids, -mids, np.nextafter(mids.astype(np.float32), 0),
                         np.nextafter(mids.astype(np.float32), 1000)]).astype(np.float32)
    zs = zs[np.abs(zs) <= 448]
    lib = torch.from_numpy(zs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    for z, w in zip(zs, lib):
        got = oracle.e4m3_encode(z)
        if (w & 0x7F) == 0:
            assert got == 0, (z, got)                       # zero is always 0x00, never 0x80
        else:
            assert got == w, (z, got, w)
    # every finite value is a fixed point
    for c in range(256):
        if c & 0x7F not in (0x7F, 0):
            assert oracle.e4m3_encode(oracle.e4m3_value(c)) == c


def test_e4m3_saturates(oracle):
    for z, want in [(448.0, 0x7E), (449.0, 0x7E), (1e9, 0x7E), (-448.00003, 0xFE), (-3e38, 0xFE), (463.9, 0x7E)]:
        assert oracle.e4m3_encode(z) == want


def test_e4m3_unit_table(oracle):
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue
        exact = Fraction(oracle.e4m3_value(c)) / 448
        u = oracle.e4m3_unit(c)
        # correctly rounded fp32 quotient: no fp32 neighbour is closer
        for nb in (np.nextafter(u, np.float32(-9)), np.nextafter(u, np.float32(9))):
            assert abs(Fraction(float(u)) - exact) <= abs(Fraction(float(nb)) - exact)
    assert oracle.e4m3_unit(0x7E) == 1.0 and oracle.e4m3_unit(0xFE) == -1.0 and oracle.e4m3_unit(0) == 0.0


# ----------------------------------------------------------------------------- quantize invariants

def _round_f32(fr: Fraction) -> np.float32:
    c = np.float32(float(fr))
    cands = [c, np.nextafter(c, np.float32(-np.inf)), np.nextafter(c, np.float32(np.inf))]
    best = min(cands, key=lambda v: (abs(Fraction(float(v)) - fr), int(np.float32(v).view(np.uint32)) & 1))
    return np.float32(best)


def _unpack(packed):
    out = np.empty(packed.size * 2, np.uint8)
    out[0::2] = packed & 15
    out[1::2] = packed >> 4
    return out


@pytest.fixture(scope="module")
def small_q(oracle, synth):
    W = synth.normal_f32((128, 512), 0.02, 77)
    return W, oracle.nf4_quantize(W)


def test_footprint_matches_paper(oracle, small_q):
    gold = {}
    with open(os.path.join(GOLD, "dq_footprint.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                gold[k] = float(v)
    W, q = small_q
    P = W.size
    const_bits = (q["code"].nbytes * 8 + q["c1"].nbytes * 8) / P
    assert const_bits == 8 / 64 + 32 / (64 * 256)
    assert round(const_bits, 3) == gold["bits_double_quant"]
    assert round(q["c2"].nbytes * 8 / P, 3) == gold["bits_fp32_constants"]
    assert round(q["c2"].nbytes * 8 / P - const_bits, 3) == gold["bits_saved"]
    assert (q["packed"].nbytes * 8) / P == 4.0
    assert (q["packed"].nbytes + q["code"].nbytes + q["c1"].nbytes) * 8 / P == 4.126953125


def test_blocks_are_contiguous_slices(oracle, small_q):
    W, q = small_q
    W2 = W.copy()
    flat = W2.reshape(-1)
    b = 37
    flat[64 * b:64 * (b + 1)] *= 3.0                        # touch one block only
    q2 = oracle.nf4_quantize(W2)
    c2a, c2b = q["c2"], q2["c2"]
    changed = np.nonzero(c2a != c2b)[0]
    np.testing.assert_array_equal(changed, [b])
    assert c2b[b] == np.abs(flat[64 * b:64 * (b + 1)]).max()
    # scaling a block by a constant leaves its NF4 indices essentially unchanged
    ia, ib = _unpack(q["packed"]), _unpack(q2["packed"])
    other = np.ones(ia.size, bool)
    other[64 * b:64 * (b + 1)] = False
    np.testing.assert_array_equal(ia[other], ib[other])


def test_absmax_and_zero_elements(oracle, small_q):
    W, q = small_q
    idx = _unpack(q["packed"]).reshape(-1, 64)
    blocks = W.reshape(-1, 64)
    np.testing.assert_array_equal(q["c2"], np.abs(blocks).max(axis=1))
    am = np.abs(blocks).argmax(axis=1)
    rows = np.arange(blocks.shape[0])
    top = idx[rows, am]
    sign = blocks[rows, am] > 0
    np.testing.assert_array_equal(top, np.where(sign, 15, 0))
    Z = W.copy()
    Z.reshape(-1)[:64] = 0.0                                # an all-zero block
    Z.reshape(-1)[100] = 0.0
    qz = oracle.nf4_quantize(Z)
    iz = _unpack(qz["packed"])
    assert np.all(iz[:64] == 7) and iz[100] == 7 and qz["c2"][0] == 0.0


def test_round_trip_error_bound(oracle, small_q):
    W, q = small_q
    tab = oracle.nf4_table().astype(np.float64)
    idx = _unpack(q["packed"]).reshape(-1, 64)
    xh = W.reshape(-1, 64).astype(np.float64) / q["c2"][:, None].astype(np.float64)
    err = np.abs(xh - tab[idx])
    half_gap = np.diff(tab).max() / 2
    assert abs(half_gap - 0.1519036) < 1e-6                 # largest gap is -1 -> -0.696
    assert err.max() <= half_gap + 1e-6
    # idx is the nearest value wherever xh is not within rounding distance of a midpoint
    near = np.abs(xh[..., None] - tab).argmin(-1)
    mids = (tab[:-1] + tab[1:]) / 2
    safe = np.abs(xh[..., None] - mids).min(-1) > 1e-6
    np.testing.assert_array_equal(idx[safe], near[safe])
    rel_rms = np.sqrt(((xh - tab[idx]) ** 2).mean() / (xh ** 2).mean())
    assert 0.07 < rel_rms < 0.12                            # ~0.09 for normal data, statistical sanity


def test_packing_low_nibble_first(oracle):
    W = np.zeros((1, 64), np.float32)
    W[0, 0] = -1.0      # idx 0 (absmax element, negative)
    W[0, 1] = 1.0       # idx 15
    W[0, 2] = 0.5       # xhat 0.5 -> between 0.4407 (12) and 0.5626 (13): nearest 12
    q = oracle.nf4_quantize(W)
    assert q["packed"][0] == (0 | (15 << 4))
    assert q["packed"][1] == (12 | (7 << 4))


def test_mean_is_exactly_rounded(oracle):
    rng = np.random.default_rng(5)
    cases = [np.abs(rng.standard_normal(64 * 300)).astype(np.float32) * 0.05]
    wide = np.abs(rng.standard_normal(64 * 40)).astype(np.float32)
    wide[::64] *= np.float32(2.0) ** rng.integers(-60, 60, wide[::64].size).astype(np.float32)
    cases.append(wide)                                      # no fp64 running sum is exact here
    tiny = (np.abs(rng.standard_normal(64 * 8)) * 1e-41).astype(np.float32)  # subnormal constants
    cases.append(tiny)
    for flat in cases:
        W = flat.reshape(-1, 64)
        q = oracle.nf4_quantize(W)
        c2 = np.abs(W).max(axis=1)
        exact = sum((Fraction(float(v)) for v in c2), Fraction(0)) / len(c2)
        assert q["mean"] == _round_f32(exact), (q["mean"], float(exact))


def test_double_quant_invariants(oracle, small_q):
    W, q = small_q
    c2, mean = q["c2"], q["mean"]
    assert np.all(c2 > 0)
    c2p = (c2 - mean).astype(np.float32)                    # fp32 subtraction
    assert abs(c2p.astype(np.float64).sum()) < 1e-6 * len(c2)
    nb = len(q["c1"])
    for B in range(nb):
        seg = c2p[256 * B:256 * (B + 1)]
        assert q["c1"][B] == np.abs(seg).max()
        codes = q["code"][256 * B:256 * (B + 1)]
        assert np.any((codes & 0x7F) == 0x7E)               # the super-block maximum uses the full range
        unit = np.array([oracle.e4m3_unit(c) for c in codes], np.float64)
        y = seg.astype(np.float64) / q["c1"][B]
        bound = np.maximum(np.abs(y) * 2.0 ** -4, 2.0 ** -10 / 448) + 1e-6
        assert np.all(np.abs(y - unit) <= bound)


def test_dequant_against_library_pieces(oracle, small_q):
    W, q = small_q
    bits, c2hat = oracle.nf4_dequant(q, return_c2hat=True)
    # constants: library E4M3 decode, then the two fp32 steps in numpy float32 arithmetic
    val = torch.from_numpy(q["code"].copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    unit = (val / np.float32(448.0)).astype(np.float32)
    want_c2 = (unit * np.repeat(q["c1"], 256)[:len(unit)]).astype(np.float32) + np.float32(q["mean"])
    np.testing.assert_array_equal(c2hat, want_c2.astype(np.float32))
    # relative error of the reconstructed constants is at the 8-bit-float level
    rel = np.abs(c2hat.astype(np.float64) - q["c2"]) / q["c2"]
    assert rel.max() < 4e-2 and np.sqrt((rel ** 2).mean()) < 1e-2
    # weights: table lookup, one fp32 product, library bf16 cast
    tab = oracle.nf4_table()
    idx = _unpack(q["packed"])
    prod = (tab[idx] * np.repeat(want_c2, 64)).astype(np.float32)
    np.testing.assert_array_equal(bits.reshape(-1), _bf16_bits(prod))
    # end-to-end: dequantised weights stay within the NF4 + DQ + bf16 error of the source
    back = _bf16_f64(bits).reshape(W.shape)
    tol = np.repeat(q["c2"], 64).reshape(W.shape) * (0.1519036 + 0.04 + 2.0 ** -8)
    assert np.all(np.abs(back - W) <= tol)


def test_quantize_rejects_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.nf4_quantize(np.zeros((3, 21), np.float32))
    bad = np.zeros((2, 64), np.float32)
    bad[0, 3] = np.inf
    with pytest.raises(ValueError):
        oracle.nf4_quantize(bad)


# ----------------------------------------------------------------------------- forward / backward

def _rand_bf16(rng, shape, scale=1.0):
    return _bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


@pytest.fixture(scope="module")
def lin_case():
    rng = np.random.default_rng(6)
    M, h, o, r = 9, 24, 40, 5
    return dict(M=M, h=h, o=o, r=r, s=0.75, X=_rand_bf16(rng, (M, h)), W=_rand_bf16(rng, (h, o), 0.05),
                L1=_rand_bf16(rng, (h, r), 0.1), L2=_rand_bf16(rng, (r, o), 0.1), dY=_rand_bf16(rng, (M, o)))


def test_forward_against_library_matmul(oracle, lin_case):
    c = lin_case
    X, W, L1, L2 = (_bf16_f64(c[k]) for k in ("X", "W", "L1", "L2"))
    want = X @ W + c["s"] * ((X @ L1) @ L2)
    got = oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], c["s"])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # W is h x o and is NOT transposed; a transposed operand would fail here
    assert np.abs(got - (X @ W[:, ::-1] + c["s"] * ((X @ L1) @ L2))).max() > 1e-3
    rows = np.array([8, 0, 3], np.int64)
    np.testing.assert_array_equal(oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], c["s"], rows=rows), got[rows])
    cols = np.array([39, 1, 17, 0], np.int64)
    np.testing.assert_allclose(oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], c["s"], cols=cols), got[:, cols],
                               rtol=0, atol=1e-12)


def test_forward_special_cases(oracle, lin_case):
    c = lin_case
    X, W = _bf16_f64(c["X"]), _bf16_f64(c["W"])
    base = X @ W
    np.testing.assert_allclose(oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], 0.0), base, atol=1e-12)
    np.testing.assert_allclose(oracle.linear_fwd(c["X"], c["W"], None, None, 1.0), base, atol=1e-12)
    zero = np.zeros_like(c["L2"])
    np.testing.assert_allclose(oracle.linear_fwd(c["X"], c["W"], c["L1"], zero, 2.0), base, atol=1e-12)


def test_brute_force_tiny(oracle):
    # hand-checkable 2x2x2 case with r = 1, all values exactly representable in bf16
    X = _bf16_bits(np.array([[1, 2], [3, 4]], np.float32))
    W = _bf16_bits(np.array([[1, -1], [0.5, 2]], np.float32))
    L1 = _bf16_bits(np.array([[1], [1]], np.float32))
    L2 = _bf16_bits(np.array([[2, -2]], np.float32))
    Y = oracle.linear_fwd(X, W, L1, L2, 0.5)
    np.testing.assert_array_equal(Y, [[1 + 1 + 3, -1 + 4 - 3], [3 + 2 + 7, -3 + 8 - 7]])
    dY = _bf16_bits(np.array([[1, 0], [0, 1]], np.float32))
    dX = oracle.linear_bwd_dx(dY, W, L1, L2, 0.5)
    np.testing.assert_array_equal(dX, [[1 + 1, 0.5 + 1], [-1 - 1, 2 - 1]])
    dL1, dL2 = oracle.linear_bwd_dl(dY, X, L1, L2, 0.5)
    np.testing.assert_array_equal(dL1, [[0.5 * (1 * 2 + 3 * -2)], [0.5 * (2 * 2 + 4 * -2)]])
    np.testing.assert_array_equal(dL2, [[0.5 * 3, 0.5 * 7]])


def _energy(oracle, c, X=None, L1=None, L2=None):
    Y = oracle.linear_fwd(c["X"] if X is None else X, c["W"], c["L1"] if L1 is None else L1,
                          c["L2"] if L2 is None else L2, c["s"])
    return float((Y * _bf16_f64(c["dY"])).sum())


def test_backward_by_exact_central_differences(oracle):
    # E = sum(Y * dY) is linear in X, in L1 and in L2, so a central difference with a
    # bf16-representable step is exact up to fp64 rounding: small integers, step 1.
    rng = np.random.default_rng(7)
    M, h, o, r = 5, 12, 16, 3
    ints = lambda shape, k: _bf16_bits(rng.integers(-k, k + 1, shape).astype(np.float32))
    c = dict(M=M, h=h, o=o, r=r, s=0.25, X=ints((M, h), 6), W=ints((h, o), 4), L1=ints((h, r), 3),
             L2=ints((r, o), 3), dY=ints((M, o), 5))
    dX = oracle.linear_bwd_dx(c["dY"], c["W"], c["L1"], c["L2"], c["s"])
    dL1, dL2 = oracle.linear_bwd_dl(c["dY"], c["X"], c["L1"], c["L2"], c["s"])

    def bump(bits, i, j, d):
        a = _bf16_f64(bits).astype(np.float32).copy()
        a[i, j] += d
        return _bf16_bits(a)

    for (i, j) in [(0, 0), (4, 11), (2, 5), (3, 7)]:
        num = (_energy(oracle, c, X=bump(c["X"], i, j, 1)) - _energy(oracle, c, X=bump(c["X"], i, j, -1))) / 2
        assert abs(num - dX[i, j]) < 1e-9
    for (i, j) in [(0, 0), (11, 2), (6, 1)]:
        num = (_energy(oracle, c, L1=bump(c["L1"], i, j, 1)) - _energy(oracle, c, L1=bump(c["L1"], i, j, -1))) / 2
        assert abs(num - dL1[i, j]) < 1e-9
    for (i, j) in [(0, 0), (2, 15), (1, 8)]:
        num = (_energy(oracle, c, L2=bump(c["L2"], i, j, 1)) - _energy(oracle, c, L2=bump(c["L2"], i, j, -1))) / 2
        assert abs(num - dL2[i, j]) < 1e-9


def test_backward_against_library_matmul(oracle, lin_case):
    c = lin_case
    X, W, L1, L2, dY = (_bf16_f64(c[k]) for k in ("X", "W", "L1", "L2", "dY"))
    s = c["s"]
    want_dx = dY @ W.T + s * ((dY @ L2.T) @ L1.T)
    got_dx = oracle.linear_bwd_dx(c["dY"], c["W"], c["L1"], c["L2"], s)
    np.testing.assert_allclose(got_dx, want_dx, rtol=0, atol=1e-12)
    rows = np.array([2, 7], np.int64)
    np.testing.assert_array_equal(oracle.linear_bwd_dx(c["dY"], c["W"], c["L1"], c["L2"], s, rows=rows), got_dx[rows])
    cols = np.array([23, 0, 5], np.int64)
    np.testing.assert_allclose(oracle.linear_bwd_dx(c["dY"], c["W"], c["L1"], c["L2"], s, cols=cols),
                               got_dx[:, cols], rtol=0, atol=1e-12)
    dL1, dL2 = oracle.linear_bwd_dl(c["dY"], c["X"], c["L1"], c["L2"], s)
    np.testing.assert_allclose(dL1, s * (X.T @ (dY @ L2.T)), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dL2, s * ((X @ L1).T @ dY), rtol=0, atol=1e-12)
    # L2 = 0 kills dL1; L1 = 0 kills dL2
    z1, z2 = np.zeros_like(c["L1"]), np.zeros_like(c["L2"])
    assert np.all(oracle.linear_bwd_dl(c["dY"], c["X"], c["L1"], z2, s)[0] == 0)
    assert np.all(oracle.linear_bwd_dl(c["dY"], c["X"], z1, c["L2"], s)[1] == 0)


# ----------------------------------------------------------------------------- LoRA dropout

def test_dropout_reduces_to_known_cases(oracle, lin_case):
    """LoRA dropout (hyperparameter appendix) acts on the input of the adapter branch only.  All multipliers 1 is no
    dropout, bit for bit; all 0 removes the adapter; the frozen product never sees the mask; and the result equals
    the library matmul on the masked, rescaled input."""
    c = lin_case
    M, h = c["M"], c["h"]
    X, W, L1, L2, dY = (_bf16_f64(c[k]) for k in ("X", "W", "L1", "L2", "dY"))
    s = c["s"]
    ones, zeros = np.ones((M, h)), np.zeros((M, h))
    base = oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], s)
    np.testing.assert_array_equal(oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], s, D=ones), base)
    np.testing.assert_allclose(oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], s, D=zeros), X @ W, atol=1e-12)
    rng = np.random.default_rng(8)
    keep = rng.random((M, h)) >= 0.25
    D = oracle.dropout_multipliers(keep, 0.25)
    assert set(np.unique(D)) == {0.0, 1.0 / 0.75} and np.array_equal(D != 0, keep)
    Xd = X * D
    np.testing.assert_allclose(oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], s, D=D),
                               X @ W + s * ((Xd @ L1) @ L2), rtol=0, atol=1e-12)
    rows = np.array([5, 1], np.int64)
    np.testing.assert_array_equal(oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], s, rows=rows, D=D),
                                  oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], s, D=D)[rows])
    got_dx = oracle.linear_bwd_dx(c["dY"], c["W"], c["L1"], c["L2"], s, D=D)
    np.testing.assert_allclose(got_dx, dY @ W.T + s * D * ((dY @ L2.T) @ L1.T), rtol=0, atol=1e-12)
    np.testing.assert_array_equal(oracle.linear_bwd_dx(c["dY"], c["W"], c["L1"], c["L2"], s, rows=rows, D=D), got_dx[rows])
    dL1, dL2 = oracle.linear_bwd_dl(c["dY"], c["X"], c["L1"], c["L2"], s, D=D)
    np.testing.assert_allclose(dL1, s * (Xd.T @ (dY @ L2.T)), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dL2, s * ((Xd @ L1).T @ dY), rtol=0, atol=1e-12)
    # a dropped input element gets no gradient through the adapter, and gives none to its row of L1
    m, k = np.argwhere(~keep)[0]
    assert abs(got_dx[m, k] - (dY @ W.T)[m, k]) < 1e-12
    only = np.zeros((M, h)); only[:, 3] = 2.0                          # everything dropped but feature 3
    dL1_only, _ = oracle.linear_bwd_dl(c["dY"], c["X"], c["L1"], c["L2"], s, D=only)
    assert np.all(dL1_only[np.arange(h) != 3] == 0) and np.any(dL1_only[3] != 0)


def test_dropout_backward_by_exact_central_differences(oracle):
    """With a fixed mask E = sum(Y * dY) is still linear in X, L1 and L2: central differences with step 1 on small
    integers (multipliers 0 and 2, i.e. p = 1/2, keep every product exact) reproduce the three gradients."""
    rng = np.random.default_rng(9)
    M, h, o, r = 5, 12, 16, 3
    ints = lambda shape, k: _bf16_bits(rng.integers(-k, k + 1, shape).astype(np.float32))
    c = dict(s=0.25, X=ints((M, h), 6), W=ints((h, o), 4), L1=ints((h, r), 3), L2=ints((r, o), 3), dY=ints((M, o), 5))
    keep = rng.random((M, h)) >= 0.5
    keep[0, 0], keep[4, 11] = True, False
    D = oracle.dropout_multipliers(keep, 0.5)
    dX = oracle.linear_bwd_dx(c["dY"], c["W"], c["L1"], c["L2"], c["s"], D=D)
    dL1, dL2 = oracle.linear_bwd_dl(c["dY"], c["X"], c["L1"], c["L2"], c["s"], D=D)

    def energy(X=None, L1=None, L2=None):
        Y = oracle.linear_fwd(c["X"] if X is None else X, c["W"], c["L1"] if L1 is None else L1,
                              c["L2"] if L2 is None else L2, c["s"], D=D)
        return float((Y * _bf16_f64(c["dY"])).sum())

    def bump(bits, i, j, d):
        a = _bf16_f64(bits).astype(np.float32).copy()
        a[i, j] += d
        return _bf16_bits(a)

    for (i, j) in [(0, 0), (4, 11), (2, 5), (3, 7)]:                  # a kept and a dropped element among them
        num = (energy(X=bump(c["X"], i, j, 1)) - energy(X=bump(c["X"], i, j, -1))) / 2
        assert abs(num - dX[i, j]) < 1e-9
    for (i, j) in [(0, 0), (11, 2), (6, 1)]:
        num = (energy(L1=bump(c["L1"], i, j, 1)) - energy(L1=bump(c["L1"], i, j, -1))) / 2
        assert abs(num - dL1[i, j]) < 1e-9
    for (i, j) in [(0, 0), (2, 15), (1, 8)]:
        num = (energy(L2=bump(c["L2"], i, j, 1)) - energy(L2=bump(c["L2"], i, j, -1))) / 2
        assert abs(num - dL2[i, j]) < 1e-9


def test_dropout_keeps_the_expectation(oracle, lin_case):
    """Inverted dropout: averaged over many independent masks the adapter term returns to its no-dropout value
    (the 1/(1-p) rescaling), within the sampling error."""
    c = lin_case
    rng = np.random.default_rng(10)
    p, n = 0.1, 400
    base = oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], c["s"])
    acc = np.zeros_like(base)
    for _ in range(n):
        acc += oracle.linear_fwd(c["X"], c["W"], c["L1"], c["L2"], c["s"],
                                 D=oracle.dropout_multipliers(rng.random((c["M"], c["h"])) >= p, p))
    frozen = _bf16_f64(c["X"]) @ _bf16_f64(c["W"])
    adapter = base - frozen
    err = np.abs(acc / n - base).max()
    assert err < 0.1 * np.abs(adapter).max(), (err, np.abs(adapter).max())


# ----------------------------------------------------------------------------- other 4-bit data types

def test_codebooks_of_the_compared_data_types(oracle):
    """Section 4 compares NF4 with Int4, Float4 E2M1 and Float4 E3M0 under the same blockwise scheme.  E2M1's
    magnitudes are the published ones of the format (0, 0.5, 1, 1.5, 2, 3, 4, 6), E3M0 has an exponent only
    (powers of two), Int4 is Eq. 1 with the range [-7, 7]; every table is normalised to [-1, 1], ascending,
    antisymmetric, and NF4 through the table argument is the NF4 path."""
    e2m1 = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6]) / 6
    t = oracle.codebook4("fp4_e2m1").astype(np.float64)
    np.testing.assert_allclose(t[8:], e2m1, rtol=0, atol=3e-8)
    np.testing.assert_array_equal(t[:8], -t[:7:-1])
    t = oracle.codebook4("fp4_e3m0").astype(np.float64)
    np.testing.assert_array_equal(t[9:], 2.0 ** np.arange(-6, 1))
    assert t[7] == 0 and t[8] == 0 and np.array_equal(t[:8], -t[:7:-1])
    t = oracle.codebook4("int4").astype(np.float64)
    np.testing.assert_allclose(t[:15], np.arange(-7, 8) / 7, rtol=0, atol=3e-8)
    assert t[15] == 1.0
    np.testing.assert_array_equal(oracle.codebook4("nf4"), oracle.nf4_table())
    for k in oracle.KINDS:
        t = oracle.codebook4(k)
        assert t.dtype == np.float32 and np.all(np.diff(t) >= 0) and t[0] == -1 and t[15] == 1
    with pytest.raises(ValueError):
        oracle.codebook4(4)


def test_index4_is_nearest_value_bruteforce(oracle):
    """For any non-decreasing table the index points at the nearest value, the lower one on an exact tie; where a
    value occurs twice (the two zeros of the float types) either copy decodes the same."""
    rng = np.random.default_rng(12)
    tables = [oracle.codebook4(k) for k in oracle.KINDS]
    tables.append(np.sort(rng.uniform(-1, 1, 16)).astype(np.float32))
    for t in tables:
        t64 = t.astype(np.float64)
        xs = np.concatenate([rng.uniform(-1.05, 1.05, 400), t64, (t64[:-1] + t64[1:]) / 2]).astype(np.float32)
        for x in xs:
            d = np.abs(t64 - np.float64(x))
            got, want = oracle.index4(t, x), int(np.argmin(d))           # argmin returns the first minimum
            assert t64[got] == t64[want], (x, t)
            if np.all(np.diff(t64) > 0):
                assert got == want, (x, t)
    # Int4 is Eq. 1: round(7 x / absmax), away from the ties
    t = oracle.codebook4("int4")
    for x in rng.uniform(-1, 1, 500).astype(np.float32):
        if abs(7 * float(x) - np.floor(7 * float(x)) - 0.5) > 1e-3:
            assert oracle.index4(t, x) - 7 == int(np.round(7 * float(x)))


def test_quantize4_round_trip_and_ranking(oracle):
    """Through the table argument NF4 reproduces the NF4 path bit for bit; every data type's round-trip error stays
    within half its widest gap times the block's absmax; and on normally distributed weights NF4 has the smallest
    mean error of the four (Section 3: quantile quantisation is optimal for normal data; Section 4: NF4 > FP4 > Int4)."""
    rng = np.random.default_rng(13)
    W = rng.standard_normal((128, 1024)).astype(np.float32)
    q0 = oracle.nf4_quantize(W)
    q1 = oracle.nf4_quantize(W, table=oracle.codebook4("nf4"))
    for k in ("packed", "code", "c1"):
        np.testing.assert_array_equal(q0[k], q1[k])
    np.testing.assert_array_equal(oracle.nf4_dequant(q0), oracle.nf4_dequant(q1))
    err = {}
    for kind in oracle.KINDS:
        t = oracle.codebook4(kind)
        q = oracle.nf4_quantize(W, table=t)
        What, c2hat = oracle.nf4_dequant(q, return_c2hat=True)
        What = _bf16_f64(What)
        gap = np.diff(t.astype(np.float64)).max()
        c2 = np.repeat(q["c2"].astype(np.float64), 64).reshape(W.shape)
        c2h = np.repeat(c2hat.astype(np.float64), 64).reshape(W.shape)
        # nearest value within gap/2 of x = w/c2; then c2 is replaced by its 8-bit reconstruction and the product rounded to bf16
        bound = gap / 2 * c2 + np.abs(c2h - c2) + 2.0 ** -8 * np.abs(What) + 1e-6
        assert np.all(np.abs(What - W) <= bound), kind
        err[kind] = np.abs(What - W).mean()
    assert err["nf4"] < min(err["fp4_e2m1"], err["fp4_e3m0"], err["int4"]), err


# ----------------------------------------------------------------------------- without Double Quantization

def test_without_double_quantization(oracle):
    """Section 3: fp32 constants at blocksize 64 cost 32/64 = 0.5 bit per parameter, Double Quantization brings that
    to 0.127.  Without it the weights are nf4[idx] * c2 rounded to bf16 (checked against numpy's fp32 product and the
    library bf16 cast), the indices are those of the double-quantised tensor, and the reconstruction can only be
    closer: the double-quantised constants differ from c2 by at most half an 8-bit step of their run."""
    import torch
    rng = np.random.default_rng(14)
    W = (rng.standard_normal((96, 512)) * 0.02).astype(np.float32)
    q0 = oracle.nf4_quantize(W, dq_blocksize=0)
    q1 = oracle.nf4_quantize(W)
    assert q0["code"] is None and q0["c1"] is None and q0["dq_blocksize"] == 0
    np.testing.assert_array_equal(q0["packed"], q1["packed"])
    np.testing.assert_array_equal(q0["c2"], np.abs(W.reshape(-1, 64)).max(axis=1))
    bits = (4 * q0["packed"].size * 2 + 32 * q0["c2"].size) / W.size
    assert bits == 4.5
    idx = np.empty(W.size, np.uint8)
    idx[0::2], idx[1::2] = q0["packed"] & 15, q0["packed"] >> 4
    prod = oracle.nf4_table()[idx].reshape(-1, 64) * q0["c2"][:, None]          # numpy fp32 multiply
    want = torch.from_numpy(prod.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.nf4_dequant(q0)
    np.testing.assert_array_equal(got.reshape(-1, 64), want)
    e0 = np.abs(_bf16_f64(got) - W).mean()
    e1 = np.abs(_bf16_f64(oracle.nf4_dequant(q1)) - W).mean()
    assert e0 <= e1 * 1.001, (e0, e1)
    # another data type without Double Quantization
    t = oracle.codebook4("int4")
    q2 = oracle.nf4_quantize(W, dq_blocksize=0, table=t)
    idx[0::2], idx[1::2] = q2["packed"] & 15, q2["packed"] >> 4
    prod = t[idx].reshape(-1, 64) * q2["c2"][:, None]
    want = torch.from_numpy(prod.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(oracle.nf4_dequant(q2).reshape(-1, 64), want)


# ----------------------------------------------------------------------------- 8-bit integers (Eq. 1, Eq. 2)

def test_int8_is_equation_1_and_2(oracle):
    """Eq. 1 / Eq. 2 with numpy: q = rint(127 / absmax * x) per block (numpy's rint rounds ties to even), the range is
    [-127, 127] with absmax hitting +-127, zeros stay zero, the round trip is within half a step, the constants go
    through the same Double Quantization as the 4-bit types', and without it the reconstruction is q * absmax / 127."""
    import torch
    rng = np.random.default_rng(15)
    W = (rng.standard_normal((64, 512)) * 0.02).astype(np.float32)
    W.reshape(-1)[:64] = 0.0                                              # an all-zero block
    q = oracle.int8_quantize(W, dq_blocksize=0)
    Wb = W.reshape(-1, 64)
    c2 = np.abs(Wb).max(axis=1)
    np.testing.assert_array_equal(q["c2"], c2)
    with np.errstate(divide="ignore"):
        c = np.where(c2 > 0, np.float32(127) / c2, np.float32(0)).astype(np.float32)
    want = np.rint((c[:, None] * Wb).astype(np.float32)).clip(-127, 127).astype(np.int8)
    np.testing.assert_array_equal(q["q8"].reshape(-1, 64), want)
    assert q["q8"].min() == -127 and q["q8"].max() == 127 and np.all(q["q8"][:64] == 0)
    assert np.all(np.abs(q["q8"].reshape(-1, 64)).max(axis=1)[1:] == 127)
    got = _bf16_f64(oracle.int8_dequant(q)).reshape(-1, 64)
    step = (c2 / np.float32(127)).astype(np.float32)
    ref = torch.from_numpy((q["q8"].reshape(-1, 64).astype(np.float32) * step[:, None]).astype(np.float32))
    np.testing.assert_array_equal(oracle.int8_dequant(q).reshape(-1, 64),
                                  ref.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    assert np.all(np.abs(got - Wb) <= 0.5 * step[:, None].astype(np.float64) * (1 + 2.0 ** -20) + 2.0 ** -8 * np.abs(got) + 1e-12)  # half a step + half a bf16 ulp
    # with Double Quantization the constants are those of the NF4 path on the same tensor
    qd = oracle.int8_quantize(W)
    qn = oracle.nf4_quantize(W)
    for k in ("code", "c1", "c2"):
        np.testing.assert_array_equal(qd[k], qn[k])
    assert np.float32(qd["mean"]).view(np.uint32) == np.float32(qn["mean"]).view(np.uint32)
    np.testing.assert_array_equal(qd["q8"], q["q8"])
    e_dq = np.abs(_bf16_f64(oracle.int8_dequant(qd)) - W).mean()
    e_nf4 = np.abs(_bf16_f64(oracle.nf4_dequant(qn)) - W).mean()
    assert e_dq < 0.2 * e_nf4                                            # 8 bits against 4


def test_int8_dq_constants_are_those_of_double_dequant(oracle):
    """With Double Quantization the 8-bit-integer path rebuilds its constants with the same two fp32 steps as
    doubleDequant (Eq. 6): bit for bit the c2hat that nf4_dequant reports for the NF4 quantisation of the same tensor
    (itself pinned against numpy / torch pieces above), and again from numpy fp32 pieces here -- table value / 448
    times c1, rounded, plus mean, rounded.  The dequantised weights are then q * fl32(c2hat / 127) with the library
    bf16 cast."""
    import torch
    rng = np.random.default_rng(16)
    W = (rng.standard_normal((96, 512)) * 0.02).astype(np.float32)
    W[5] *= 40.0                                                          # a run of constants far from the mean
    qd = oracle.int8_quantize(W)
    qn = oracle.nf4_quantize(W)
    _, c2hat_nf4 = oracle.nf4_dequant(qn, return_c2hat=True)
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()   # library E4M3 decode
    unit = (lib / np.float32(448)).astype(np.float32)
    c1 = np.repeat(qd["c1"], 256)[:qd["code"].size]
    c2hat_np = ((unit[qd["code"]] * c1).astype(np.float32) + np.float32(qd["mean"])).astype(np.float32)
    np.testing.assert_array_equal(c2hat_np.view(np.uint32), c2hat_nf4.view(np.uint32))
    step = (c2hat_np / np.float32(127)).astype(np.float32)
    ref = torch.from_numpy((qd["q8"].reshape(-1, 64).astype(np.float32) * step[:, None]).astype(np.float32))
    np.testing.assert_array_equal(oracle.int8_dequant(qd).reshape(-1, 64),
                                  ref.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    # a planted mistake in the constants (one fused rounding instead of two) must show: the pin is not vacuous
    fused = (unit[qd["code"]].astype(np.float64) * c1.astype(np.float64) + np.float64(qd["mean"])).astype(np.float32)
    assert np.any(fused.view(np.uint32) != c2hat_np.view(np.uint32))


def test_int8_ties_and_clamp(oracle):
    """A block whose absmax is 127 has c = 1, so the codes are the inputs rounded: halves go to the even neighbour,
    and the sign is kept."""
    w = np.zeros((1, 64), np.float32)
    w[0, :9] = [127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, -126.5]
    q = oracle.int8_quantize(w, dq_blocksize=0)
    assert list(q["q8"][:9]) == [127, 0, 2, 2, 0, -2, -2, 126, -126]
    np.testing.assert_array_equal(_bf16_f64(oracle.int8_dequant(q))[0, :4], [127.0, 0.0, 2.0, 2.0])


# ----------------------------------------------------------------------------- k-bit NormalFloat, k = 2, 3 (Section 3)

def test_nfk_construction(oracle):
    """The general-k construction: k = 4 gives back the derivation that matches the printed table; for k = 2, 3 every
    value is the stated quantile (library normal quantile), there are 2^k distinct ascending values with one exact
    zero, one more positive than negative, ends at -1 and +1, and the 16-entry table is padded with +1."""
    from scipy.stats import norm
    d4 = oracle.nfk_derive(4)
    np.testing.assert_array_equal(d4, oracle.nf4_derive(1.0 - 0.5 * (1.0 / 32.0 + 1.0 / 30.0)))
    assert np.abs(d4 - oracle.nf4_table().astype(np.float64)).max() <= 2e-7
    for k in (2, 3):
        d = oracle.nfk_derive(k)
        n = 1 << k
        n_neg, n_pos = n // 2, n // 2 + 1
        p_max = 1.0 - 0.5 * (1.0 / (2 * n) + 1.0 / (2 * n - 2))
        top = norm.ppf(p_max)
        want = [-norm.ppf(0.5 + (p_max - 0.5) * i / (n_neg - 1)) / top for i in range(n_neg - 1, 0, -1)]
        want += [norm.ppf(0.5 + (p_max - 0.5) * i / (n_pos - 1)) / top for i in range(n_pos)]
        assert len(want) == n
        np.testing.assert_allclose(d[:n], want, rtol=0, atol=1e-12)
        assert np.all(np.diff(d[:n]) > 0) and d[0] == -1.0 and d[n - 1] == 1.0 and d[n_neg - 1] == 0.0
        assert (d[:n] < 0).sum() == n_neg - 1 and (d[:n] > 0).sum() == n_neg
        assert np.all(d[n:] == 1.0)
        tab = oracle.codebook4("nf3" if k == 3 else "nf2")
        np.testing.assert_array_equal(tab, d.astype(np.float32))
    # NF2 in closed form: {-1, 0, Q((1/2 + p_max) / 2) / Q(p_max), 1}
    p2 = 1.0 - 0.5 * (1.0 / 8 + 1.0 / 6)
    np.testing.assert_allclose(oracle.nfk_derive(2)[:4], [-1.0, 0.0, norm.ppf((0.5 + p2) / 2) / norm.ppf(p2), 1.0], atol=1e-12)


def test_nfk_error_ordering_and_codes(oracle):
    """On normal data fewer bits cost more error (NF2 > NF3 > NF4), a k-bit NormalFloat beats the k-bit integer grid of
    Eq. 1 (the paper's argument for quantile quantisation), and codes >= 2^k never occur."""
    rng = np.random.default_rng(16)
    W = (rng.standard_normal((128, 512)) * 0.02).astype(np.float32)
    err = {}
    for name, k in (("nf2", 2), ("nf3", 3), ("nf4", 4)):
        q = oracle.nf4_quantize(W, table=oracle.codebook4(name))
        codes = np.concatenate([q["packed"] & 15, q["packed"] >> 4])
        assert codes.max() == (1 << k) - 1 and codes.min() == 0
        err[name] = np.abs(_bf16_f64(oracle.nf4_dequant(q)) - W).mean()
    assert err["nf2"] > 1.5 * err["nf3"] > 1.5 * 1.5 * err["nf4"]
    int3 = np.array([j / 3.0 for j in range(-3, 4)] + [1.0] * 9, np.float32)      # Eq. 1 with the range [-3, 3]
    q = oracle.nf4_quantize(W, table=int3)
    assert err["nf3"] < np.abs(_bf16_f64(oracle.nf4_dequant(q)) - W).mean()
