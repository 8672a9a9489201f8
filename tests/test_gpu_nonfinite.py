"""Non-finite gradients (NaN of either sign, infinities) must leave the sender memory-safe.

include/fftsp.h promises nothing about the values such a call packs, only that it stays inside its
buffers.  A NaN that carries a sign bit used to give a rank key outside the 31-bit key space; the key
is now masked, so selection on such bins is ordinary integer work and exactly k bins survive.  Checked
here: the bytes behind the packed stream are untouched, every record still has its own header and a
bitmap with exactly k set bits, and a decompress of the stream stays in bounds as well.
"""
import numpy as np
import pytest

from tests.gpu_harness import Device

pytestmark = pytest.mark.gpu

GUARD = 4096


@pytest.fixture(scope="module")
def dev():
    return Device()


def poisoned(rng, n, kind):
    g = rng.standard_normal(n).astype(np.float32) * 1e-3
    u = g.view(np.uint32)
    idx = rng.choice(n, size=max(1, n // 50), replace=False)
    if kind == "pos_nan":
        u[idx] = 0x7FC00000
    elif kind == "neg_nan":
        u[idx] = 0xFFC00000
    elif kind == "inf":
        u[idx[::2]] = 0x7F800000
        u[idx[1::2]] = 0xFF800000
    elif kind == "mixed":
        u[idx[0::3]] = 0xFFC00001
        u[idx[1::3]] = 0x7F800000
        u[idx[2::3]] = 0x7FFFFFFF
    elif kind == "all_neg_nan":
        u[:] = 0xFFC00000
    return g


def check_stream(dev, packed, nb, n, L, theta, bits):
    f = dev.f
    host = packed.cpu().numpy()
    assert (host[nb:] == 0xEE).all(), "bytes behind the packed stream were written"
    C = (n + L - 1) // L
    k = f.kept_per_chunk(L, theta)
    B = L // 2 + 1
    W = (B + 31) // 32
    S = (nb - 64) // C
    for c in range(C):
        rec = host[64 + c * S: 64 + (c + 1) * S].view(np.uint32)
        assert rec[2] == k and rec[3] == 0, f"record {c}: header overwritten"
        bitmap = rec[4:4 + W]
        assert int(np.unpackbits(bitmap.view(np.uint8)).sum()) == k, f"record {c}: survivors != k"


@pytest.mark.parametrize("L", [1 << 10, 1 << 15, 1 << 20])
@pytest.mark.parametrize("kind", ["pos_nan", "neg_nan", "inf", "mixed", "all_neg_nan"])
def test_sender_stays_in_bounds(dev, L, kind):
    t, f = dev.torch, dev.f
    rng = np.random.default_rng(1234 + L % 1000)
    n = 2 * L + L // 3
    theta, bits = 0.5, 8
    g = poisoned(rng, n, kind)
    nb = f.packed_bytes(n, L, theta, bits)
    packed = t.full((nb + GUARD,), 0xEE, dtype=t.uint8, device=dev.dev)
    ws = dev.ws_for(n, L, bits)
    f.compress(dev.to_dev(g), L, theta, bits, packed[:nb], ws)
    dev.sync()
    check_stream(dev, packed, nb, n, L, theta, bits)
    out = t.full((n + GUARD,), 7.0, dtype=t.float32, device=dev.dev)
    f.decompress(packed[:nb], nb, out[:n], L, theta, bits, ws)
    assert f.device_status(ws) == 0
    assert (out[n:] == 7.0).all().item()


@pytest.mark.parametrize("kind", ["neg_nan", "mixed", "all_neg_nan"])
def test_encode_of_a_nonfinite_spectrum(dev, kind):
    t, f = dev.torch, dev.f
    L, theta, bits = 1 << 12, 0.3, 6
    n = 3 * L
    rng = np.random.default_rng(99)
    spec = poisoned(rng, 3 * (L + 2), kind)
    nb = f.packed_bytes(n, L, theta, bits)
    packed = t.full((nb + GUARD,), 0xEE, dtype=t.uint8, device=dev.dev)
    f.encode_spectrum(dev.to_dev(spec), n, L, theta, bits, packed[:nb], dev.ws_for(n, L, bits))
    dev.sync()
    check_stream(dev, packed, nb, n, L, theta, bits)


def test_per_tensor_and_half_variants_stay_in_bounds(dev):
    t, f = dev.torch, dev.f
    rng = np.random.default_rng(5)
    offs = [0, 100, 1124, 70000, 70000 + (1 << 15)]
    n = offs[-1]
    g = poisoned(rng, n, "mixed")
    theta, bits = 0.3, 6
    nb = f.packed_bytes_segments(offs, theta, bits)
    packed = t.full((nb + GUARD,), 0xEE, dtype=t.uint8, device=dev.dev)
    ws = dev.workspace(f.workspace_bytes_segments(offs, bits))
    f.compress_segments(dev.to_dev(g), offs, theta, bits, packed[:nb], ws)
    dev.sync()
    assert (packed[nb:] == 0xEE).all().item()
    L = 1 << 15
    n = 2 * L + 17
    g = poisoned(rng, n, "neg_nan")
    nb = f.packed_bytes(n, L, 0.5, 8)
    packed = t.full((nb + GUARD,), 0xEE, dtype=t.uint8, device=dev.dev)
    f.compress_h(dev.to_dev(g), L, 0.5, 8, 10, packed[:nb], dev.ws_for(n, L, 8))
    dev.sync()
    check_stream(dev, packed, nb, n, L, 0.5, 8)
