"""GPU parity of the receiver-side accumulation (several peers' streams, one inverse transform) against the oracle.

The summed spectrum is compared bit for bit (both sides add the peers in list order in binary32, from zero); the
reconstruction within 1e-5 relative L2.
"""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads
from tests.gpu_harness import Device, rel_l2

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def dev():
    return Device()


def peer_streams(ref, n, L, theta, bits, peers, seed=0, threads=8):
    gs = [workloads.small_mixed(n, seed=seed + 101 * p) * np.float32(1.0 + 0.5 * p) for p in range(peers)]
    return gs, [ref.compress(g, L, theta, bits, nthreads=threads) for g in gs]


CASES = [
    # n, L, theta, bits, peers
    (3 * 256 - 7, 256, 0.4, 8, 1),
    (3 * 256 - 7, 256, 0.4, 8, 3),
    (5000, 4096, 0.37, 6, 2),              # two tiles per chunk, ragged tail
    (40000, 16384, 0.6, 16, 5),            # largest single-workgroup FFT, two 16-byte pieces per lane
    (2 * 32768 + 77, 32768, 0.5, 8, 4),    # two-pass FFT, paired spectrum order
    (2 * 32768 + 77, 32768, 0.3, 12, 3),
    (2 * 32768 + 77, 32768, 1.0, 32, 2),   # everything kept, raw codes
    (70000, 65536, 0.0, 8, 2),             # nothing kept
    (1 << 20, 1 << 18, 0.5, 8, 8),
    (300000, 1 << 20, 0.25, 10, 2),        # one ragged 2^20 chunk
    (1 << 22, 1 << 22, 0.1, 8, 3),         # longest chunk
]


@pytest.mark.parametrize("n,L,theta,bits,peers", CASES)
def test_accumulate_parity(dev, ref, n, L, theta, bits, peers):
    print(f"accumulate n={n} L={L} theta={theta} bits={bits} peers={peers}", flush=True)
    _, pks = peer_streams(ref, n, L, theta, bits, peers, seed=bits)
    spec_gpu, st = dev.decode_accumulate(pks, n, L, theta, bits)
    spec_or = ref.decode_accumulate_spectrum(pks, n, L, theta, bits, nthreads=8)
    assert st == 0
    assert np.array_equal(spec_gpu.view(np.uint32), spec_or.view(np.uint32))
    scale = 1.0 / peers
    out_gpu, st = dev.decompress_accumulate(pks, scale, n, L, theta, bits)
    out_or = ref.decompress_accumulate(pks, scale, n, L, theta, bits, nthreads=8)
    assert st == 0 and np.isfinite(out_gpu).all()
    if out_or.any():
        assert rel_l2(out_gpu, out_or) <= TOL
    else:
        assert not out_gpu.any()


def test_single_peer_equals_decompress(dev, ref):
    n, L, theta, bits = 2 * 65536 + 5, 65536, 0.5, 8
    _, (pk,) = peer_streams(ref, n, L, theta, bits, 1)
    a, st = dev.decompress_accumulate([pk], 1.0, n, L, theta, bits)
    b = dev.decompress(pk, n, L, theta, bits)
    assert st == 0 and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_sum_order_is_the_list_order(dev, ref):
    L, n = 32, 32
    B = L // 2 + 1

    def stream(v):
        spec = np.zeros(2 * B, np.float32)
        spec[2 * 4] = v
        return ref.encode_spectrum(spec, n, L, 1.0, 32)

    a, b, c = stream(1e8), stream(-1e8), stream(1.0)
    assert dev.decode_accumulate([a, b, c], n, L, 1.0, 32)[0][2 * 4] == 1.0
    assert dev.decode_accumulate([c, a, b], n, L, 1.0, 32)[0][2 * 4] == 0.0


def test_maximum_number_of_peers(dev, ref):
    n, L, theta, bits = 9000, 8192, 0.2, 8
    _, pks = peer_streams(ref, n, L, theta, bits, 32)
    spec_gpu, st = dev.decode_accumulate(pks, n, L, theta, bits)
    assert st == 0
    assert np.array_equal(spec_gpu.view(np.uint32),
                          ref.decode_accumulate_spectrum(pks, n, L, theta, bits, nthreads=8).view(np.uint32))


def test_one_bad_peer_raises_the_status(dev, ref):
    n, L, theta, bits = 3 * 4096, 4096, 0.5, 8
    _, pks = peer_streams(ref, n, L, theta, bits, 3)
    bad = pks[1].copy()
    bad[64 + 16] ^= 0x01   # first bitmap byte of the first record: the count no longer matches k
    out, st = dev.decompress_accumulate([pks[0], bad, pks[2]], 1.0, n, L, theta, bits)
    assert st == 6 and np.isfinite(out).all()
    bad = pks[2].copy()
    bad[16] ^= 0x01        # chunk length in the stream header
    _, st = dev.decompress_accumulate([pks[0], pks[1], bad], 1.0, n, L, theta, bits)
    assert st == 6
