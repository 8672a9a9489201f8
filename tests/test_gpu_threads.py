"""Two host threads use the library at once, each on a stream and workspace of its own.

The uniform entry points share nothing but constants; the per-tensor entry points share the device's side streams and
enqueue under a lock.  Either way every call must give the bytes the same call gives alone."""
import threading

import numpy as np
import pytest

from paper_1811_08596_amd import workloads
from tests.gpu_harness import Device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return Device()


def test_two_threads_on_their_own_streams(dev):
    torch, f = dev.torch, dev.f
    L, theta, bits = 1 << 15, 0.4, 8
    n = 9 * L - 11
    w = workloads.config2()
    offs = [int(v) for v in w.seg_offsets]
    ns = offs[-1]
    nb = f.packed_bytes(n, L, theta, bits)
    nbs = f.packed_bytes_segments(offs, w.theta, w.bits)

    class Job:
        def __init__(self, seed):
            self.stream = torch.cuda.Stream()
            self.g = dev.to_dev(workloads.small_mixed(n, seed=seed))
            self.sg = dev.to_dev(w.grad * np.float32(1.0 + 0.5 * seed))
            self.ws = dev.ws_for(n, L, bits)
            self.sws = dev.workspace(f.workspace_bytes_segments(offs, w.bits))
            self.packed = torch.zeros(nb, dtype=torch.uint8, device=dev.dev)
            self.out = torch.zeros(n, dtype=torch.float32, device=dev.dev)
            self.spacked = torch.zeros(nbs, dtype=torch.uint8, device=dev.dev)
            self.sout = torch.zeros(ns, dtype=torch.float32, device=dev.dev)
            self.error = None

        def step(self):
            s = self.stream
            f.compress(self.g, L, theta, bits, self.packed, self.ws, s)
            f.decompress(self.packed, nb, self.out, L, theta, bits, self.ws, s)
            f.compress_segments(self.sg, offs, w.theta, w.bits, self.spacked, self.sws, s)
            f.decompress_segments(self.spacked, nbs, self.sout, offs, w.theta, w.bits, self.sws, s)

        def results(self):
            return [t.clone() for t in (self.packed, self.out.view(torch.int32), self.spacked, self.sout.view(torch.int32))]

        def clear(self):
            self.packed.fill_(0xEE)
            self.spacked.fill_(0xEE)
            self.out.fill_(float("nan"))
            self.sout.fill_(float("nan"))

    jobs = [Job(1), Job(2)]
    want = []
    for j in jobs:                                   # each alone first
        j.step()
        torch.cuda.synchronize()
        want.append(j.results())
        j.clear()
    torch.cuda.synchronize()

    def run(j):
        try:
            for _ in range(25):
                j.step()
            j.stream.synchronize()
        except Exception as e:                      # reported by the main thread
            j.error = e

    threads = [threading.Thread(target=run, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a worker thread is stuck"
    torch.cuda.synchronize()
    for j, w_ in zip(jobs, want):
        assert j.error is None, j.error
        assert f.device_status(j.ws) == 0 and f.device_status(j.sws) == 0
        for got, exp in zip(j.results(), w_):
            assert torch.equal(got, exp)
