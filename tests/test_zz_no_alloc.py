"""fftsp_compress_static, the sender that allocates nothing and brings its own scratch array, against
fftsp_compress on the same inputs: the packed bytes must be identical (integer, byte and index work: bit-exact).
Two calls in a row share the array, the second with a smaller input, so whatever the first call left behind
must not leak into the second.  A size beyond the array is refused on the host."""
import numpy as np
import pytest

from tests.gpu_harness import Device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return Device()


def both(dev, g, L, theta, bits):
    t, f = dev.torch, dev.f
    n = g.size
    gd = dev.to_dev(g)
    nb = f.packed_bytes(n, L, theta, bits)
    want = t.full((nb,), 0xEE, dtype=t.uint8, device=dev.dev)
    f.compress(gd, L, theta, bits, want, dev.ws_for(n, L, bits))
    got = t.full((nb + 256,), 0xEE, dtype=t.uint8, device=dev.dev)
    f.compress_static(gd, L, theta, bits, got[:nb])
    dev.sync()
    got = got.cpu().numpy()
    assert (got[nb:] == 0xEE).all()
    return got[:nb], want.cpu().numpy()


def test_static_scratch_matches_workspace_sender_twice(dev):
    rng = np.random.default_rng(20250711)
    # first call: two-pass transform, 15 full chunks and a ragged one; second call: smaller, single-workgroup chunks
    g1 = (rng.laplace(size=15 * (1 << 16) + 12345) * 1e-3).astype(np.float32)
    got, want = both(dev, g1, 1 << 16, 0.5, 8)
    assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} bytes differ (first call)"
    g2 = (rng.standard_normal(5 * (1 << 12) + 77) * 1e-4).astype(np.float32)
    got, want = both(dev, g2, 1 << 12, 0.25, 6)
    assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} bytes differ (second, smaller call)"
    # and once more the first shape, after the small one
    got, want = both(dev, g1, 1 << 16, 0.5, 8)
    assert np.array_equal(got, want)


def test_static_scratch_refuses_what_does_not_fit(dev):
    f = dev.f
    n, L = 1 << 22, 1 << 20
    assert f.workspace_bytes(n, L, 8) > f.STATIC_SCRATCH_BYTES
    gd = dev.empty(n, dev.torch.float32)
    packed = dev.empty(f.packed_bytes(n, L, 0.5, 8), dev.torch.uint8)
    with pytest.raises(f.FftspError) as e:
        f.compress_static(gd, L, 0.5, 8, packed)
    assert e.value.code == f.EWORKSPACE
