"""Pins for the oracle's half-precision variant (Sec. 3.1.1, "Our approach": the gradients go to 16 bits for the
transform).  The variant is a definition — exact DFT, times 2^s, each component rounded once to binary16 — so the
pins are: the rounding against numpy's binary16 conversion (a library routine written by someone else), the
whole spectrum against numpy's float64 transform rounded by numpy, the size of the loss against the already
pinned binary32 path (what the paper calls negligible), exactness of the scale, and the header field.
"""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads


def test_rounding_is_binary16_nearest_even_and_saturates(ref):
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(4000) * 10.0 ** rng.uniform(-9, 4.8, 4000),     # subnormal range up to the top
        np.array([0.0, -0.0, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -14, 65504.0, 65519.9, 1.0 + 2.0 ** -11,
                  1.0 + 3 * 2.0 ** -11, 2049.0, 2051.0, -2049.0]),          # ties: to even, both ways
    ])
    vals = vals[np.abs(vals) < 65520.0]                  # numpy rounds to infinity from there on
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).astype(np.float64)
    got = np.array([ref.round_half(v) for v in vals])
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(want))
    for v in (65520.0, 7e4, 1e30, float("inf")):         # saturating, not to infinity
        assert ref.round_half(v) == 65504.0 and ref.round_half(-v) == -65504.0
    assert np.isnan(ref.round_half(float("nan")))


def test_spectrum_is_numpys_transform_rounded_by_numpy(ref):
    """the whole definition through two library routines: numpy's float64 FFT, times 2^s, numpy's conversion to
    binary16.  The two double-precision transforms differ in the last bits, which can flip a rounding that sits on
    a tie: at most a handful of components may differ, and then by one binary16 unit"""
    L, n, s = 2048, 3 * 2048 - 100, 9
    g = workloads.small_mixed(n, seed=12)
    got = ref.rfft_h(g, L, s).reshape(3, L + 2)
    for c in range(3):
        chunk = np.zeros(L)
        seg = g[c * L:(c + 1) * L]
        chunk[:seg.size] = seg
        X = np.fft.rfft(chunk) * 2.0 ** s
        want = np.empty(L + 2, np.float64)
        want[0::2] = X.real.astype(np.float16)
        want[1::2] = X.imag.astype(np.float16)
        want[1] = want[L + 1] = 0.0
        diff = np.flatnonzero(got[c] != want)
        assert diff.size <= 3
        unit = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want[diff]), 2.0 ** -14))) - 10)
        assert np.all(np.abs(got[c][diff] - want[diff]) <= unit)


@pytest.mark.parametrize("scale_log2", [0, 6, 12])
def test_loss_is_one_binary16_rounding(ref, scale_log2):
    """every component is within half a binary16 unit of the binary32 path's value (times 2^s), and the relative
    L2 loss of the whole spectrum is about 2^-11 / sqrt(3) per normal component"""
    L, n = 4096, 3 * 4096 - 17
    g = workloads.small_mixed(n, seed=8)
    full = ref.rfft(g, L).astype(np.float64) * 2.0 ** scale_log2
    half = ref.rfft_h(g, L, scale_log2).astype(np.float64)
    assert np.all(np.abs(half) <= 65504.0)
    quantum = np.maximum(2.0 ** -24, 2.0 ** (np.floor(np.log2(np.maximum(np.abs(full), 1e-300))) - 10))
    assert np.all(np.abs(half - full) <= 0.5 * quantum * (1 + 1e-6) + np.abs(full) * 2.0 ** -23)
    rel = np.linalg.norm(half - full) / np.linalg.norm(full)
    if scale_log2 >= 6:                                  # out of the subnormals: the textbook figure
        assert 1e-4 < rel < 4e-4
    else:
        assert rel < 3e-2                                # small tensors sit in binary16's subnormals without a scale


def test_scale_is_exact_and_undone(ref):
    L, n, theta, bits = 1024, 2 * 1024 + 5, 0.4, 32
    g = workloads.small_mixed(n, seed=2)
    s = 10
    a = ref.rfft_h(g, L, s)
    b = ref.rfft_h(g * np.float32(2.0 ** s), L, 0)       # scaling the input by a power of two is exact
    assert np.array_equal(a, b)
    pk = ref.compress_h(g, L, theta, bits, s)
    h = ref.parse_header(pk)
    assert h["scale_log2"] == s and h["domain"] == 0
    out = ref.decompress_h(pk, n, L, theta, bits, s)
    # the receiver is the exact inverse of what was kept: same as the binary32 receiver on the same values / 2^s
    plain = pk.copy()
    plain[48:52] = 0
    out2 = ref.decompress(plain, n, L, theta, bits) / np.float32(2.0 ** s)
    assert np.array_equal(out, out2)
    with pytest.raises(ref.OracleError):
        ref.decompress(pk, n, L, theta, bits)            # a scaled stream is not a plain stream
    with pytest.raises(ref.OracleError):
        ref.decompress_h(pk, n, L, theta, bits, s + 1)


def test_round_trip_error_is_the_dropped_energy_plus_a_binary16_rounding(ref):
    """at kept fraction 1 and raw codes the only loss is the rounding: about 3e-4 relative; at 0.5 kept the
    reconstruction error is that of the binary32 path to three digits"""
    L, n = 8192, 8192 * 2
    g = workloads.small_mixed(n, seed=5)
    s = 12
    nrm = np.linalg.norm(g.astype(np.float64))
    out = ref.decompress_h(ref.compress_h(g, L, 1.0, 32, s), n, L, 1.0, 32, s)
    assert 5e-5 < np.linalg.norm(out - g.astype(np.float64)) / nrm < 5e-4
    eh = np.linalg.norm(ref.decompress_h(ref.compress_h(g, L, 0.5, 32, s), n, L, 0.5, 32, s) - g.astype(np.float64)) / nrm
    ef = np.linalg.norm(ref.decompress(ref.compress(g, L, 0.5, 32), n, L, 0.5, 32) - g.astype(np.float64)) / nrm
    assert abs(eh - ef) < 2e-3 * ef
