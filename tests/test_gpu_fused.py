"""The fused, cache-resident two-pass transforms (csrc/fused.hip) against the oracle and against the per-pass kernels.

Calls whose two-pass intermediate is at least 96 MiB (about 25 million samples) take the fused kernels; the small
parity cases never do, so the cases here are sized for them: chunk lengths 2^15 .. 2^20, several turns per XCD, a ragged last chunk, a last
turn that is only partly filled.  Parity with the oracle is the same contract as everywhere (tests/test_gpu_parity.py:
spectra and reconstructions within 1e-5, bytes identical on the oracle's spectrum); on top of it the fused sender
must produce the very bytes of the per-pass kernels it replaces, and the fused receiver
the same samples up to the rounding of a few fused multiply-adds (the compiler contracts the same expressions
differently in the two kernels: 1e-6 relative L2, ten times inside the parity bound), also when a hand-over wait
expires and the stand-by kernels redo the transform (then bit for bit: they are the per-pass kernels).
"""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads
from tests.gpu_harness import Device, rel_l2
from tests.test_gpu_parity import full_parity

pytestmark = pytest.mark.gpu

GAVE_UP_WORD = 1  # u32 index inside the workspace's control block


@pytest.fixture(scope="module")
def dev():
    return Device()


def round_trip(dev, g, L, theta, bits):
    """(packed bytes, reconstruction, give-up word after compress, after decompress)"""
    t, f = dev.torch, dev.f
    n = g.size
    gd = dev.to_dev(g)
    nb = f.packed_bytes(n, L, theta, bits)
    ws = dev.ws_for(n, L, bits)
    packed = t.full((nb,), 0xEE, dtype=t.uint8, device=dev.dev)
    f.compress(gd, L, theta, bits, packed, ws)
    dev.sync()
    gave_c = int(ws[4 * GAVE_UP_WORD:4 * GAVE_UP_WORD + 4].view(t.int32).item())
    out = t.full((n + 64,), 7.0, dtype=t.float32, device=dev.dev)
    f.decompress(packed, nb, out[:n], L, theta, bits, ws)
    assert f.device_status(ws) == 0
    gave_d = int(ws[4 * GAVE_UP_WORD:4 * GAVE_UP_WORD + 4].view(t.int32).item())
    assert (out[n:] == 7.0).all().item()
    return packed.cpu().numpy(), out[:n].cpu().numpy(), gave_c, gave_d


CASES = [
    # (log2 L, chunks, samples missing from the last chunk); at least 96 MiB of intermediate each
    (15, 769, 1234),   # 32 chunks per turn: 25 turns, the last one holds a single chunk
    (16, 390, 5),
    (17, 200, 99),
    (18, 100, 70000),
    (20, 25, 4321),    # one chunk per turn; XCD 0 takes four turns
    (20, 35, 0),       # five turns on some XCDs: every turn buffer is reused
]


@pytest.mark.parametrize("logL,C,tail", CASES)
def test_fused_transforms_match_the_oracle(dev, ref, monkeypatch, logL, C, tail):
    monkeypatch.setenv("FFTSP_FUSED", "1")
    L = 1 << logL
    g = workloads.small_mixed(C * L - tail, seed=logL)
    full_parity(dev, ref, g, L, 0.5, 8, end_to_end=True)


@pytest.mark.parametrize("logL,C,tail", CASES)
def test_fused_agrees_with_per_pass_kernels(dev, monkeypatch, logL, C, tail):
    L = 1 << logL
    g = workloads.small_mixed(C * L - tail, seed=100 + logL)
    monkeypatch.setenv("FFTSP_FUSED", "0")
    want_p, want_r, gc, gd = round_trip(dev, g, L, 0.3, 8)
    assert gc != 1 and gd != 1                     # the word is not even written on this path
    monkeypatch.setenv("FFTSP_FUSED", "1")
    got_p, got_r, gc, gd = round_trip(dev, g, L, 0.3, 8)
    assert gc == 0 and gd == 0, "the fused kernels gave up on an idle GPU"
    assert np.array_equal(got_p, want_p), "packed bytes differ"
    assert rel_l2(got_r, want_r) <= 1e-6


def test_expired_wait_hands_over_to_the_stand_by_kernels(dev, monkeypatch):
    """A spin limit of zero makes the first hand-over wait that is not already satisfied expire: every workgroup
    leaves, the give-up word is set, and the per-pass kernels behind the fused one produce the result."""
    L, C = 1 << 17, 200
    g = workloads.small_mixed(C * L - 99, seed=7)
    monkeypatch.setenv("FFTSP_FUSED", "0")
    want_p, want_r, _, _ = round_trip(dev, g, L, 0.5, 8)
    monkeypatch.setenv("FFTSP_FUSED", "1")
    monkeypatch.setenv("FFTSP_FUSED_SPIN", "0")
    got_p, got_r, gc, gd = round_trip(dev, g, L, 0.5, 8)
    assert gc == 1 and gd == 1
    assert np.array_equal(got_p, want_p)
    assert np.array_equal(got_r.view(np.uint32), want_r.view(np.uint32))
