"""Pins for the oracle's receiver-side accumulation (sum of the peers' spectra, one inverse transform).

The paper fixes only what is summed (Sec. 4, implementation: every worker gathers all peers' packed gradients;
Sec. 3.1: the receiver inverts the sender's steps); the arithmetic order is this build's reading, so the pins are
the already pinned single-peer functions, linearity of the transform, closed forms and a rounding-order witness.
"""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads


def _streams(ref, L, n, theta, bits, peers, seed=5):
    gs = [workloads.small_mixed(n, seed=seed + 17 * p) for p in range(peers)]
    return gs, [ref.compress(g, L, theta, bits) for g in gs]


def test_single_peer_is_decompress(ref):
    L, n = 256, 3 * 256 - 11
    _, (pk,) = _streams(ref, L, n, 0.4, 8, 1)
    a = ref.decompress_accumulate([pk], 1.0, n, L, 0.4, 8)
    b = ref.decompress(pk, n, L, 0.4, 8)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    sa = ref.decode_accumulate_spectrum([pk], n, L, 0.4, 8)
    sb = ref.decode_spectrum(pk, n, L, 0.4, 8)
    assert np.array_equal(sa, sb)  # 0 + x == x (and -0 never comes out of an 8-bit code)


def test_same_stream_twice_halved_is_exact(ref):
    L, n = 512, 2 * 512
    _, (pk,) = _streams(ref, L, n, 0.3, 10, 1)
    twice = ref.decode_accumulate_spectrum([pk, pk], n, L, 0.3, 10)
    once = ref.decode_spectrum(pk, n, L, 0.3, 10)
    assert np.array_equal(twice, 2.0 * once)  # doubling is exact in binary32
    a = ref.decompress_accumulate([pk, pk], 0.5, n, L, 0.3, 10)
    b = ref.decompress(pk, n, L, 0.3, 10)
    # the inverse transform is linear and 2x, 0.5x are exact: only the final roundings can differ by an ulp
    assert np.max(np.abs(a.astype(np.float64) - b)) <= 2e-7 * np.max(np.abs(b))


@pytest.mark.parametrize("peers,bits,theta", [(2, 8, 0.5), (3, 6, 0.25), (5, 16, 0.9), (4, 32, 1.0)])
def test_linearity_against_sum_of_reconstructions(ref, peers, bits, theta):
    L, n = 1024, 4 * 1024 - 100
    _, pks = _streams(ref, L, n, theta, bits, peers)
    scale = 1.0 / peers
    got = ref.decompress_accumulate(pks, scale, n, L, theta, bits).astype(np.float64)
    want = scale * sum(ref.decompress(pk, n, L, theta, bits).astype(np.float64) for pk in pks)
    assert np.linalg.norm(got - want) <= 1e-6 * np.linalg.norm(want)


def test_two_cosines_closed_form(ref):
    # peer A keeps only bin 3, peer B only bin 5 (raw fp32 codes): the sum is the two cosines added
    L = 64
    t = np.arange(L)
    xa = np.cos(2 * np.pi * 3 * t / L).astype(np.float32)
    xb = (0.25 * np.cos(2 * np.pi * 5 * t / L)).astype(np.float32)
    theta = 1.0 / (L // 2 + 1)  # k = 1
    assert ref.kept_per_chunk(L, theta) == 1
    pa, pb = ref.compress(xa, L, theta, 32), ref.compress(xb, L, theta, 32)
    out = ref.decompress_accumulate([pa, pb], 1.0, L, L, theta, 32)
    assert np.max(np.abs(out - (xa.astype(np.float64) + xb))) <= 1e-6


def test_sum_is_taken_in_list_order_in_binary32(ref):
    # 1e8 + (-1e8) + 1 is 1 from the left but (1 + 1e8) + (-1e8) is 0 in binary32
    L, n = 32, 32
    B = L // 2 + 1

    def stream(v):
        spec = np.zeros(2 * B, np.float32)
        spec[2 * 4] = v  # real part of bin 4
        return ref.encode_spectrum(spec, n, L, 1.0, 32)

    a, b, c = stream(1e8), stream(-1e8), stream(1.0)
    assert ref.decode_accumulate_spectrum([a, b, c], n, L, 1.0, 32)[2 * 4] == 1.0
    assert ref.decode_accumulate_spectrum([c, a, b], n, L, 1.0, 32)[2 * 4] == 0.0


def test_scale_is_one_binary32_multiplication_after_the_inverse(ref):
    L, n = 128, 128
    _, pks = _streams(ref, L, n, 0.5, 8, 3)
    one = ref.decompress_accumulate(pks, 1.0, n, L, 0.5, 8)
    third = ref.decompress_accumulate(pks, 1.0 / 3.0, n, L, 0.5, 8)
    assert np.array_equal(third, one * np.float32(1.0 / 3.0))


def test_errors(ref):
    L, n = 64, 64
    _, pks = _streams(ref, L, n, 0.5, 8, 2)
    with pytest.raises(ref.OracleError):
        ref.decompress_accumulate([], 1.0, n, L, 0.5, 8)
    bad = pks[1].copy()
    bad[8] ^= 0xFF  # n in the stream header
    with pytest.raises(ref.OracleError):
        ref.decompress_accumulate([pks[0], bad], 1.0, n, L, 0.5, 8)
    with pytest.raises(ref.OracleError):
        ref.decompress_accumulate([pks[0]], 1.0, n, L, 0.25, 8)  # other theta than the stream's
