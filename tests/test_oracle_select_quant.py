"""Pins for the oracle's key, top-k selection and range-based N-bit float.

Selection: brute force on tiny inputs, crafted ties, the exactly-k invariant.
Quantizer: Algorithm 1's stated properties (Sec. 3.2.1) and a hand-worked example
stored in tests/golden/quantizer_example.txt.
"""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_kv(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                out[k.strip()] = v.strip()
    return out


def f2u(x):
    return int(np.float32(x).view(np.uint32))


def u2f(u):
    return float(np.uint32(u).view(np.float32))


# ------------------------------------------------------------------ key -----
def round_to_f32(frac):
    """correctly rounded (nearest, ties to even) binary32 of an exact rational"""
    from fractions import Fraction
    c = np.float32(float(frac))
    cands = {float(c), float(np.nextafter(c, np.float32(-np.inf))), float(np.nextafter(c, np.float32(np.inf)))}
    best = None
    for x in cands:
        if not np.isfinite(x):
            continue
        d = abs(Fraction(x) - frac)
        even = (f2u(x) & 1) == 0
        if best is None or d < best[0] or (d == best[0] and even):
            best = (d, x)
    return np.float32(best[1])


def test_key_is_fused_square_sum_bit_pattern(ref):
    """key = bits( round( re*re (exact) + round(im*im) ) ): one product rounded, then one fused step"""
    from fractions import Fraction
    rng = np.random.default_rng(0)
    differs_from_unfused = 0
    for _ in range(3000):
        re, im = rng.standard_normal(2).astype(np.float32) * np.float32(10.0 ** rng.integers(-15, 10))
        p = round_to_f32(Fraction(float(im)) ** 2)
        want = round_to_f32(Fraction(float(re)) ** 2 + Fraction(float(p)))
        assert ref.key(re, im) == f2u(want)
        unfused = np.float32(np.float32(re * re) + np.float32(im * im))
        differs_from_unfused += int(f2u(unfused) != f2u(want))
    assert differs_from_unfused > 100          # the pin does tell a fused key from an unfused one
    assert ref.key(0.0, 0.0) == 0
    assert ref.key(-3.0, 4.0) == f2u(25.0)
    assert ref.key(1e-20, 0.0) == f2u(np.float32(1e-20) * np.float32(1e-20))   # subnormal result kept, not flushed
    assert 0 < ref.key(1e-20, 0.0) < 0x00800000


def test_key_order_equals_modulus_order(ref):
    rng = np.random.default_rng(1)
    v = rng.standard_normal((500, 2)).astype(np.float32)
    keys = np.array([ref.key(a, b) for a, b in v], dtype=np.uint32)
    mod = np.hypot(v[:, 0].astype(np.float64), v[:, 1].astype(np.float64))
    order_k = np.argsort(keys, kind="stable")
    # allow swaps only between moduli closer than binary32 rounding
    assert np.all(np.diff(mod[order_k]) > -1e-6)


# ---------------------------------------------------------------- k rule ----
@pytest.mark.parametrize("L,theta,k", [
    (1 << 16, 0.25, 8192), (1 << 16, 0.5, 16385), (1 << 20, 0.1, 52429), (1 << 20, 0.9, 471860),
    (1 << 20, 0.5, 262145), (64, 0.0, 0), (64, 1.0, 33), (64, 0.5, 17), (32, 0.3, 5), (1 << 22, 0.9, 1887438),
])
def test_kept_per_chunk_table(ref, L, theta, k):
    """k = floor(theta*B + 1/2) in double, B = L/2+1 (values computed by hand / exact rational arithmetic)."""
    assert ref.kept_per_chunk(L, theta) == k
    from fractions import Fraction
    B = L // 2 + 1
    exact = int(Fraction(float(np.float32(theta))) * B + Fraction(1, 2))
    assert min(max(exact, 0), B) == k


def test_kept_per_chunk_rejects(ref):
    for theta in (-0.1, 1.5, float("nan")):
        with pytest.raises(ref.OracleError):
            ref.kept_per_chunk(64, theta)


# -------------------------------------------------------------- selection ---
def brute_select(keys, k):
    """pick, k times, the largest remaining key; among equals the lowest index"""
    keys = [int(x) for x in keys]
    left = set(range(len(keys)))
    flags = np.zeros(len(keys), np.uint8)
    for _ in range(k):
        best = min(left, key=lambda j: (-keys[j], j))
        flags[best] = 1
        left.remove(best)
    return flags


def test_selection_brute_force_tiny(ref):
    rng = np.random.default_rng(2)
    for trial in range(200):
        B = int(rng.integers(1, 65))
        hi = int(rng.choice([2, 5, 1000, 2 ** 32 - 1]))       # small ranges force many ties
        keys = rng.integers(0, hi, size=B, dtype=np.uint64).astype(np.uint32)
        for k in {0, 1, B // 2, B - 1 if B > 1 else 0, B}:
            got = ref.select(keys, k)
            assert got.sum() == k
            assert np.array_equal(got, brute_select(keys, k))


def test_selection_ties_lowest_index(ref):
    keys = np.full(33, 7, np.uint32)                          # impulse input: all moduli equal
    for k in (0, 1, 5, 33):
        f = ref.select(keys, k)
        assert np.array_equal(np.flatnonzero(f), np.arange(k))
    keys = np.array([5, 9, 5, 9, 5, 1, 5], np.uint32)
    assert np.array_equal(np.flatnonzero(ref.select(keys, 4)), [0, 1, 2, 3])
    assert np.array_equal(np.flatnonzero(ref.select(keys, 3)), [0, 1, 3])
    assert np.array_equal(np.flatnonzero(ref.select(keys, 2)), [1, 3])


def test_selection_threshold_property(ref):
    rng = np.random.default_rng(3)
    keys = rng.integers(0, 2 ** 31, size=5000, dtype=np.uint64).astype(np.uint32)
    for k in (1, 10, 2500, 4999):
        f = ref.select(keys, k).astype(bool)
        assert f.sum() == k
        assert keys[f].min() >= keys[~f].max()


# -------------------------------------------------------------- quantizer ---
def test_default_mantissa_bits(ref):
    want = {3: 1, 4: 1, 5: 1, 6: 2, 7: 2, 8: 3, 9: 4, 10: 5, 11: 6, 12: 7, 13: 7, 14: 8, 15: 9, 16: 10, 32: 23}
    for N, m in want.items():
        assert ref.mantissa_bits(N) == m
    for N in (0, 1, 2, 17, 31, 33):
        assert ref.mantissa_bits(N) == -1


def test_hand_worked_example(ref):
    g = read_kv("quantizer_example.txt")
    N, m = int(g["bits"]), int(g["m"])
    pb = ref.pbase(int(g["vmax_bits"], 16), N, m)
    assert pb == int(g["pbase"])
    assert ref.dequantize(1, pb, N, m) == int(g["eps_bits"], 16)            # eps <-> code 0...01
    assert ref.quantize(int(g["value_bits"], 16), pb, N, m) == int(g["code"])
    assert ref.dequantize(int(g["code"]), pb, N, m) == int(g["back_bits"], 16)
    assert ref.quantize(int(g["value_bits"], 16) | 0x80000000, pb, N, m) == int(g["neg_code"])
    assert ref.quantize(int(g["vmax_bits"], 16), pb, N, m) == 2 ** (N - 1) - 1


@pytest.mark.parametrize("N", [3, 4, 6, 8, 10, 12, 16])
@pytest.mark.parametrize("vmax", [1.0, 0.37, 3.1e-5, 1e-38, 2.5e-44, 7e37])
def test_grid_properties(ref, N, vmax):
    m = ref.mantissa_bits(N)
    s = 23 - m
    Mmax = 2 ** (N - 1) - 1
    vb = f2u(vmax)
    pb = ref.pbase(vb, N, m)
    assert pb >= 1
    if (vb >> s) >= Mmax:
        assert ref.quantize(vb, pb, N, m) == Mmax          # largest survivor lands on the top code
    codes = np.arange(2 ** N)
    back = [ref.dequantize(int(c), pb, N, m) for c in codes]
    # exactly representable on its grid: Q(D(c)) = c, except -0 which is canonicalised to code 0
    for c, b in zip(codes, back):
        want = 0 if (c & Mmax) == 0 else c
        assert ref.quantize(b, pb, N, m) == want
    # magnitudes strictly increase with the magnitude code; code 0 is exactly zero
    mags = [u2f(b) for b in back[:Mmax + 1]]
    assert mags[0] == 0.0 and all(b > a for a, b in zip(mags[:-1], mags[1:]))
    # 0...01 is eps = pbase << (23-m)
    assert back[1] == pb << s
    # all-ones is the most negative representable number (Sec. 3.2.1)
    vals = [u2f(b) for b in back]
    assert min(vals) == vals[2 ** N - 1] == -mags[Mmax]
    # spacing doubles every 2^m codes, for normal numbers (Sec. 3.2.1, role of m)
    d = np.diff(np.array(mags[1:], dtype=np.float64))
    for i in range(len(d) - 2 ** m):
        if back[1 + i] >= 0x00800000:       # both ends normal
            assert d[i + 2 ** m] == 2 * d[i]


@pytest.mark.parametrize("N", [6, 8, 10])
def test_monotone_truncating_and_error_bound(ref, N):
    m = ref.mantissa_bits(N)
    Mmax = 2 ** (N - 1) - 1
    vmax = 0.8125
    pb = ref.pbase(f2u(vmax), N, m)
    eps = u2f(ref.dequantize(1, pb, N, m))
    rng = np.random.default_rng(N)
    pats = np.unique(np.concatenate([
        rng.integers(0, f2u(vmax) + 1, size=20000, dtype=np.uint64),
        np.array([ref.dequantize(c, pb, N, m) + d for c in range(1, Mmax + 1) for d in (-1, 0, 1)], dtype=np.uint64),
    ])).astype(np.uint32)
    pats = pats[pats <= f2u(vmax)]
    prev = -1
    for p in pats:                                 # ascending bit patterns = ascending non-negative floats
        v = u2f(p)
        c = ref.quantize(int(p), pb, N, m)
        assert c >= prev                           # monotone
        prev = c
        b = u2f(ref.dequantize(c, pb, N, m))
        assert b <= v                              # truncation toward zero
        if v >= eps:
            assert (v - b) < v * 2.0 ** (-m)       # inside the window: relative error < 2^-m
        else:
            assert c == 0
        # negative side mirrors
        cn = ref.quantize(int(p) | 0x80000000, pb, N, m)
        assert cn == (c | (1 << (N - 1)) if c else 0)


def test_clamp_above_max(ref):
    """Algorithm 1: a value above max is treated as max."""
    N, m = 8, 3
    pb = ref.pbase(f2u(1.0), N, m)
    for v in (1.5, 100.0, 3e38):
        assert ref.quantize(f2u(v), pb, N, m) == 127
        assert ref.quantize(f2u(-v), pb, N, m) == 255


def test_raw_mode(ref):
    for v in (0.0, -0.0, 1.25, -3e-41):
        assert ref.quantize(f2u(v), 0, 32, 23) == f2u(v)
        assert ref.dequantize(f2u(v), 0, 32, 23) == f2u(v)
    assert ref.pbase(f2u(1.0), 32, 23) == 0


def test_tiny_range_clamps_pbase(ref):
    N, m = 8, 3
    pb = ref.pbase(5, N, m)            # a subnormal range: pbase would be negative
    assert pb == 1
    assert ref.pbase(0, N, m) == 1
    assert ref.quantize(0, 1, N, m) == 0
