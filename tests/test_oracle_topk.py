"""Pins for the oracle's time-domain Top-k (the sparsifier the paper compares its own against: Sec. 4, "Choice of
Algorithms"; the Sec. 3.1.1 figure that sets FFT Top-k beside direct Top-k).

Top-k has a plain definition (keep the k samples of largest magnitude, zero the rest), so the oracle is pinned to
that definition computed another way (a stable sort in numpy), to the closed form of its error, to what the paper
says about its compression ratio, and to the already pinned quantizer primitives.  The byte layout is this
build's; the layout tests re-read it field by field.
"""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads


def _topk_by_sort(chunk, k):
    """the definition, independently: indices of the k largest |x|, ties to the lowest index"""
    mag = np.abs(chunk.astype(np.float32)).view(np.uint32).astype(np.int64)
    order = np.lexsort((np.arange(chunk.size), -mag))
    keep = np.zeros(chunk.size, bool)
    keep[order[:k]] = True
    return keep


@pytest.mark.parametrize("L, n, theta", [(256, 1000, 0.25), (64, 64 * 5, 0.1), (2048, 5000, 0.5), (32, 45, 0.9)])
def test_32_bit_codes_are_plain_topk(ref, L, n, theta):
    """N = 32 keeps the survivors bit for bit: the reconstruction is the definition of Top-k, chunk by chunk"""
    g = workloads.small_mixed(n, seed=L)
    g[3] = -g[7]                                       # an exact tie in magnitude with opposite signs
    packed = ref.topk_compress(g, L, theta, 32)
    out = ref.topk_decompress(packed, n, L, theta, 32)
    k = ref.topk_kept_per_chunk(L, theta)
    assert k == int(np.floor(theta * L + 0.5))
    for c in range((n + L - 1) // L):
        chunk = np.zeros(L, np.float32)
        seg = g[c * L:(c + 1) * L]
        chunk[:seg.size] = seg
        keep = _topk_by_sort(chunk, k)
        want = np.where(keep, chunk, np.float32(0))[:seg.size]
        assert np.array_equal(out[c * L:c * L + seg.size].view(np.uint32), want.view(np.uint32)), c


def test_error_is_the_energy_of_the_dropped_tail(ref):
    """closed form: ||g - topk(g)||^2 is the sum of the L-k smallest squares, and no other k-sparse vector on the
    same support size does better"""
    L, theta = 1024, 0.2
    g = workloads.small_mixed(L, seed=3)
    out = ref.topk_decompress(ref.topk_compress(g, L, theta, 32), L, L, theta, 32)
    k = ref.topk_kept_per_chunk(L, theta)
    sq = np.sort(g.astype(np.float64) ** 2)
    err = np.sum((g.astype(np.float64) - out) ** 2)
    assert np.isclose(err, sq[:L - k].sum(), rtol=1e-12)
    rng = np.random.default_rng(0)
    for _ in range(20):                                # any other support of k samples loses at least as much
        other = np.zeros(L, bool)
        other[rng.choice(L, k, replace=False)] = True
        assert np.sum(np.where(other, 0.0, g.astype(np.float64)) ** 2) >= err * (1 - 1e-12)


def test_ratio_is_what_the_paper_quotes_for_topk(ref):
    """Sec. 4 prices Top-k at 1/(1 - theta_drop) with 32-bit values: at 85 % dropped the kept values alone are
    a 6.67x smaller payload.  The status bitmap (1 bit per sample, Sec. 3.2) comes on top."""
    L, n, kept = 1 << 14, 1 << 16, 0.15
    k = ref.topk_kept_per_chunk(L, kept)
    S = ref.topk_record_stride(L, k, 32)
    assert S == 16 + L // 8 + 4 * k + (-(16 + L // 8 + 4 * k)) % 16
    values_only = 4 * L / (4 * k)
    assert abs(values_only - 1 / (1 - 0.85)) < 0.01
    assert ref.topk_packed_bytes(n, L, kept, 32) == 64 + (n // L) * S


def test_all_and_nothing(ref):
    g = workloads.small_mixed(700, seed=9)
    out = ref.topk_decompress(ref.topk_compress(g, 256, 1.0, 32), 700, 256, 1.0, 32)
    assert np.array_equal(out.view(np.uint32), g.view(np.uint32))
    out = ref.topk_decompress(ref.topk_compress(g, 256, 0.0, 8), 700, 256, 0.0, 8)
    assert not out.any()


@pytest.mark.parametrize("bits", [3, 6, 8, 10, 13, 16])
def test_quantized_survivors_go_through_algorithm_1(ref, bits):
    """same support as N = 32; every survivor is Nbit_to_32bit(32bit_to_Nbit(x)) with eps from the chunk's largest
    survivor, i.e. within one code step of x (relative 2^-m) or flushed below eps"""
    L, n, theta = 512, 512 * 3 - 5, 0.3
    g = workloads.small_mixed(n, seed=bits)
    p32 = ref.topk_compress(g, L, theta, 32)
    pq = ref.topk_compress(g, L, theta, bits)
    m = ref.mantissa_bits(bits)
    out = ref.topk_decompress(pq, n, L, theta, bits)
    for c in range(3):
        pb, vmax, k, w3, bm, codes = ref.topk_record_fields(pq, L, c)
        _, vmax32, k32, _, bm32, _ = ref.topk_record_fields(p32, L, c)
        assert np.array_equal(bm, bm32) and k == k32 == bm.sum() and vmax == vmax32 and w3 == 0
        seg = np.zeros(L, np.float32)
        seg[:g[c * L:(c + 1) * L].size] = g[c * L:(c + 1) * L]
        kept_vals = seg[bm.astype(bool)]
        assert vmax == int(np.abs(kept_vals).view(np.uint32).max())
        assert pb == ref.pbase(vmax, bits, m)
        got = ref.unpack_codes(codes, k, bits)
        want = [ref.quantize(int(v), pb, bits, m) for v in kept_vals.view(np.uint32)]
        assert np.array_equal(got, np.array(want, np.uint32))
        rec = np.array([ref.dequantize(int(q), pb, bits, m) for q in got], np.uint32).view(np.float32)
        valid = min(L, n - c * L)
        full = np.zeros(L, np.float32)
        full[bm.astype(bool)] = rec
        assert np.array_equal(out[c * L:c * L + valid].view(np.uint32), full[:valid].view(np.uint32))
        eps = float(np.uint32(pb << (23 - m)).view(np.float32))
        big = np.abs(kept_vals) >= eps
        assert np.all(np.abs(rec[big] - kept_vals[big]) <= 2.0 ** (-m) * np.abs(kept_vals[big]))
        assert not rec[~big].any()


def test_header_marks_the_time_domain(ref):
    g = workloads.small_mixed(300, seed=1)
    pt = ref.topk_compress(g, 128, 0.5, 8)
    pf = ref.compress(g, 128, 0.5, 8)
    assert ref.parse_header(pt)["domain"] == 1 and ref.parse_header(pf)["domain"] == 0
    with pytest.raises(ref.OracleError):               # a frequency stream is not a time-domain stream
        ref.topk_decompress(pf, 300, 128, 0.5, 8)
    bad = pt.copy()
    bad[64 + 8] ^= 1                                   # record 0 claims another k
    with pytest.raises(ref.OracleError):
        ref.topk_decompress(bad, 300, 128, 0.5, 8)


def test_transform_pays_on_a_smooth_signal_and_not_on_noise(ref):
    """the shape of the paper's FFT-Top-k-against-Top-k figure: at the same kept fraction a signal with a trend is
    reconstructed better from its largest frequencies than from its largest samples; on white noise, whose
    spectrum is as flat as the signal itself, the transform buys nothing of that size"""
    L, theta = 4096, 0.1
    t = np.arange(L) / L
    rng = np.random.default_rng(11)
    smooth = (np.sin(2 * np.pi * 3 * t) + 0.5 * np.sin(2 * np.pi * 17 * t + 1.0) + 0.05 * rng.standard_normal(L))
    smooth = (1e-3 * smooth).astype(np.float32)
    noise = (1e-3 * rng.standard_normal(L)).astype(np.float32)

    def errs(g):
        f = ref.decompress(ref.compress(g, L, theta, 32), L, L, theta, 32)
        d = ref.topk_decompress(ref.topk_compress(g, L, theta, 32), L, L, theta, 32)
        nrm = np.linalg.norm(g.astype(np.float64))
        return np.linalg.norm(f - g.astype(np.float64)) / nrm, np.linalg.norm(d - g.astype(np.float64)) / nrm

    ef, et = errs(smooth)
    assert ef < 0.25 * et
    ef, et = errs(noise)
    assert 0.8 < ef / et < 1.25
