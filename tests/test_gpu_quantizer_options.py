"""GPU parity of the quantizer options (chosen m, static range) against the oracle: packed bytes and decoded
spectra bit for bit when fed the oracle's spectrum, reconstructions within 1e-5 relative L2."""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads
from tests.gpu_harness import Device, explain_end_to_end, rel_l2

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def dev():
    return Device()


CASES = [
    # n, L, theta, bits, m, range_max
    (3 * 256 - 7, 256, 0.4, 8, 0, 1.0),          # static range far above the data: low codes only
    (3 * 256 - 7, 256, 0.4, 8, 5, 0.0),          # chosen m, fitted range
    (5000, 4096, 0.37, 6, 1, 1e-3),              # range inside the data: clamping at work
    (40000, 16384, 0.15, 10, 0, 1.0),            # the paper's experimental setting (N = 10, range (-1, 1))
    (2 * 32768 + 77, 32768, 0.5, 10, 7, 3e-4),   # two-pass FFT sizes, clamping, chosen m
    (2 * 32768 + 77, 32768, 0.5, 16, 15, 0.0),   # widest mantissa
    (70000, 65536, 0.3, 32, 0, 1.0),             # raw codes: options have nothing to change but the header word
    (1 << 20, 1 << 20, 0.5, 8, 2, 5e-2),
]


@pytest.mark.parametrize("n,L,theta,bits,m,range_max", CASES)
def test_quantizer_options_parity(dev, ref, n, L, theta, bits, m, range_max):
    print(f"options n={n} L={L} theta={theta} bits={bits} m={m} range_max={range_max}", flush=True)
    g = workloads.small_mixed(n, seed=bits + m)
    spec_or = ref.rfft(g, L, nthreads=8)
    packed_or = ref.encode_spectrum_q(spec_or, n, L, theta, bits, m, range_max, nthreads=8)
    packed_gpu = dev.encode_q(spec_or, n, L, theta, bits, m, range_max)
    assert np.array_equal(packed_gpu, packed_or), f"{np.count_nonzero(packed_gpu != packed_or)} bytes differ"
    dec_or = ref.decode_spectrum_q(packed_or, n, L, theta, bits, m, nthreads=8)
    dec_gpu, st = dev.decode_q(packed_or, n, L, theta, bits, m)
    assert st == 0 and np.array_equal(dec_gpu.view(np.uint32), dec_or.view(np.uint32))
    out_gpu, st = dev.decompress_q(packed_or, n, L, theta, bits, m)
    out_or = ref.decompress_q(packed_or, n, L, theta, bits, m, nthreads=8)
    assert st == 0 and rel_l2(out_gpu, out_or) <= TOL
    # whole sender: header and ranges are the oracle's, the rest is explainable by binary32 rounding of the FFT
    e2e = dev.compress_q(g, L, theta, bits, m, range_max)
    assert np.array_equal(e2e[:64], packed_or[:64])
    if bits != 32:
        explain_end_to_end(ref, e2e, packed_or, spec_or, n, L, theta, bits, m)


def test_static_range_is_written_to_every_record(dev, ref):
    n, L, theta, bits = 5 * 4096, 4096, 0.25, 8
    g = workloads.small_mixed(n, seed=1)
    pk = dev.compress_q(g, L, theta, bits, 0, 0.5)
    one = int(np.float32(0.5).view(np.uint32))
    for c in range(5):
        pbase, vmax_bits, k, _, _, _ = ref.record_fields(pk, L, c)
        assert vmax_bits == one and pbase == ref.pbase(one, bits, ref.mantissa_bits(bits))


def test_receiver_with_another_m_reports_the_mismatch(dev, ref):
    n, L, theta, bits = 4096, 4096, 0.5, 8
    g = workloads.small_mixed(n, seed=2)
    pk = dev.compress_q(g, L, theta, bits, 5, 0.0)
    _, st = dev.decompress_q(pk, n, L, theta, bits, 3)
    assert st == 6
    out, st = dev.decompress_q(pk, n, L, theta, bits, 5)
    assert st == 0 and np.isfinite(out).all()
