"""Pins for the quantizer options of Sec. 3.2.1: user-chosen m and a static range [-max, +max].

The paper's own procedure for eps (iterate on the most negative code until it meets the range) is implemented
separately from the codec's closed form and must land on the same pbase; the static mode is tied to the fitted
mode (already pinned) at the point where they coincide, and to Algorithm 1's clamp above max.
"""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads


def f2u(x):
    return int(np.float32(x).view(np.uint32))


def u2f(u):
    return float(np.uint32(u).view(np.float32))


def fields(ref, packed, L, c=0):
    pbase, vmax_bits, k, word3, _, _ = ref.record_fields(packed, L, c)
    return {"pbase": pbase, "vmax_bits": vmax_bits, "k": k}


@pytest.mark.parametrize("bits", [3, 4, 6, 8, 10, 12, 16])
def test_iterated_eps_lands_on_the_closed_form_pbase(ref, bits):
    rng = np.random.default_rng(bits)
    for m in range(1, bits):
        for vmax in list(10.0 ** rng.uniform(-30, 30, 6)) + [1.0, 0.5, 5.0, 1e-38]:
            eps = ref.tune_eps(vmax, bits, m)
            assert eps > 0
            assert f2u(eps) >> (23 - m) == ref.pbase(f2u(vmax), bits, m), (bits, m, vmax)
            if not np.isfinite(np.float32(vmax)):
                continue
            # the state the paper's tuning converges to: the most negative code decodes inside the range, and one
            # step of eps further up would leave it
            pb = f2u(eps) >> (23 - m)
            if (f2u(vmax) >> (23 - m)) - ((1 << (bits - 1)) - 2) < 1:
                assert pb == 1   # range narrower than the code space: eps bottoms out, the top codes go unused
                continue
            lowest = u2f(ref.dequantize((1 << bits) - 1, pb, bits, m))
            assert -vmax <= lowest < 0
            beyond = u2f(ref.dequantize((1 << bits) - 1, pb + 1, bits, m))
            assert beyond < -vmax


def test_static_range_equal_to_the_largest_survivor_is_the_fitted_mode(ref):
    L, n, theta, bits = 256, 256, 0.4, 8
    g = workloads.small_mixed(n, seed=3)
    spec = ref.rfft(g, L)
    fitted = ref.encode_spectrum(spec, n, L, theta, bits)
    vmax = u2f(fields(ref, fitted, L)["vmax_bits"])
    static = ref.encode_spectrum_q(spec, n, L, theta, bits, 0, vmax)
    assert np.array_equal(static, fitted)
    assert np.array_equal(ref.encode_spectrum_q(spec, n, L, theta, bits, 0, 0.0), fitted)  # 0 = fitted


def test_values_above_the_static_range_clamp_to_the_top_code(ref):
    # Algorithm 1: "if 32bit_float > max then 32bit_float = max"
    L, n, bits, m = 64, 64, 8, 3
    B = L // 2 + 1
    spec = np.zeros(2 * B, np.float32)
    spec[2 * 3] = 7.5      # far above the range
    spec[2 * 5 + 1] = -3.0
    spec[2 * 9] = 0.75     # inside
    pk = ref.encode_spectrum_q(spec, n, L, 1.0, bits, m, 1.0)
    f = fields(ref, pk, L)
    assert f["vmax_bits"] == f2u(1.0) and f["pbase"] == ref.pbase(f2u(1.0), bits, m)
    dec = ref.decode_spectrum_q(pk, n, L, 1.0, bits, m)
    top = u2f(ref.dequantize((1 << (bits - 1)) - 1, f["pbase"], bits, m))
    assert top == 1.0                               # max itself is on the grid for max = 1.0
    assert dec[2 * 3] == top and dec[2 * 5 + 1] == -top
    assert dec[2 * 9] == 0.75                       # exactly representable with 3 mantissa bits
    assert np.count_nonzero(dec) == 3


@pytest.mark.parametrize("bits,m", [(10, 1), (10, 5), (10, 9), (6, 4), (16, 3)])
def test_chosen_m_sets_the_relative_step(ref, bits, m):
    L, n = 512, 512
    g = workloads.small_mixed(n, seed=bits + m)
    spec = ref.rfft(g, L)
    pk = ref.encode_spectrum_q(spec, n, L, 1.0, bits, m, 0.0)
    assert ref.parse_header(pk)["m"] == m
    dec = ref.decode_spectrum_q(pk, n, L, 1.0, bits, m)
    kept = dec != 0
    err = np.abs(dec[kept].astype(np.float64) - spec[kept]) / np.abs(spec[kept])
    assert err.max() < 2.0 ** -m                    # truncation to m mantissa bits
    assert (np.abs(dec[kept]) <= np.abs(spec[kept])).all()
    if m < 9:
        assert err.max() > 2.0 ** -(m + 3)          # and not finer than that
    # decoding with another m is a header mismatch
    with pytest.raises(ref.OracleError):
        ref.decode_spectrum_q(pk, n, L, 1.0, bits, m + 1 if m + 1 < bits else m - 1)


def test_papers_experimental_setting(ref):
    # Sec. 4.2 "Algorithm Setup": N = 10 bits, range (-1, 1); round trip through the whole codec
    L, n = 1024, 3 * 1024 - 17
    g = workloads.small_mixed(n, seed=10)
    pk = ref.compress_q(g, L, 0.15, 10, 0, 1.0)
    out = ref.decompress_q(pk, n, L, 0.15, 10, 0)
    assert pk.size == ref.packed_bytes(n, L, 0.15, 10)
    assert np.isfinite(out).all() and np.linalg.norm(out - g) <= np.linalg.norm(g)
    for c in range(3):
        assert fields(ref, pk, L, c)["vmax_bits"] == f2u(1.0)


def test_option_errors(ref):
    spec = np.zeros(2 * 33, np.float32)
    for m in (-1, 8, 9):
        with pytest.raises(ref.OracleError):
            ref.encode_spectrum_q(spec, 64, 64, 0.5, 8, m, 0.0)
    for bad in (-1.0, float("inf"), float("nan")):
        with pytest.raises(ref.OracleError):
            ref.encode_spectrum_q(spec, 64, 64, 0.5, 8, 0, bad)
    assert ref.tune_eps(0.0, 8, 3) == 0.0 and ref.tune_eps(1.0, 8, 8) == 0.0
