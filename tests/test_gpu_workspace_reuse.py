"""One workspace, one stream, many calls with different shapes back to back and no synchronisation in between:
nothing a call leaves behind (histograms, candidate lists, prefixes, status) may leak into the next one."""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads
from tests.gpu_harness import Device, rel_l2

pytestmark = pytest.mark.gpu

CALLS = [
    # n, L, theta, bits
    (2 * 65536 + 5, 65536, 0.5, 8),
    (5000, 4096, 0.37, 6),
    (3 * 32768, 32768, 0.9, 16),
    (2 * 65536 + 5, 65536, 0.1, 8),      # same shape as the first, other theta
    (100, 64, 1.0, 32),
    (1 << 20, 1 << 18, 0.25, 10),
    (3 * 32768, 32768, 0.0, 8),
    (70000, 1 << 20, 0.5, 8),
]


def test_back_to_back_calls_share_one_workspace(ref):
    d = Device()
    f, torch = d.f, d.torch
    wsb = max(f.workspace_bytes(n, L, b) for n, L, _, b in CALLS)
    ws = d.workspace(wsb)                                         # poisoned once, then reused as it is left
    gs = [workloads.small_mixed(n, seed=i) for i, (n, _, _, _) in enumerate(CALLS)]
    specs = [ref.rfft(g, L, nthreads=8) for g, (_, L, _, _) in zip(gs, CALLS)]
    want = [ref.encode_spectrum(s, n, L, t, b, nthreads=8) for s, (n, L, t, b) in zip(specs, CALLS)]
    sd = [d.to_dev(s) for s in specs]
    packed = [torch.full((w.size,), 0xEE, dtype=torch.uint8, device=d.dev) for w in want]
    out = [torch.full((n,), float("nan"), dtype=torch.float32, device=d.dev) for n, _, _, _ in CALLS]
    # all encodes and decodes queued without a host wait
    for i, (n, L, t, b) in enumerate(CALLS):
        f.encode_spectrum(sd[i], n, L, t, b, packed[i], ws)
        f.decompress(packed[i], packed[i].numel(), out[i], L, t, b, ws)
    assert f.device_status(ws) == 0
    for i, (n, L, t, b) in enumerate(CALLS):
        assert np.array_equal(packed[i].cpu().numpy(), want[i]), f"call {i}"
        exp = ref.decompress(want[i], n, L, t, b, nthreads=8)
        got = out[i].cpu().numpy()
        assert np.isfinite(got).all()
        if exp.any():
            assert rel_l2(got, exp) <= 1e-5, f"call {i}"
        else:
            assert not got.any()
    # and the whole sender twice over the dirty workspace gives the same bytes
    n, L, t, b = CALLS[0]
    gd = d.to_dev(gs[0])
    a1 = torch.empty_like(packed[0]); a2 = torch.empty_like(packed[0])
    f.compress(gd, L, t, b, a1, ws)
    f.compress(d.to_dev(gs[5]), CALLS[5][1], CALLS[5][2], CALLS[5][3], packed[5], ws)
    f.compress(gd, L, t, b, a2, ws)
    assert f.device_status(ws) == 0
    assert torch.equal(a1, a2)
