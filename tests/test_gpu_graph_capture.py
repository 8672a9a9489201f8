"""The library's calls enqueue kernels only (no allocation, no memset, no host synchronisation, from the first call
on: the twiddle tables are constants in the code object), so a caller can record them into a HIP graph.  A graph is replayed several times with eager work and
synchronisations in between, and every replay is checked against the eager result."""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads
from tests.gpu_harness import Device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return Device()


def test_per_tensor_round_trip_replays_from_a_graph(dev):
    torch, f = dev.torch, dev.f
    w = workloads.config2()                                # ResNet-20-shaped: 22 tensors
    offs = [int(v) for v in w.seg_offsets]
    theta, bits = w.theta, w.bits
    n = offs[-1]
    nb = f.packed_bytes_segments(offs, theta, bits)
    ws = dev.workspace(f.workspace_bytes_segments(offs, bits))
    g = dev.to_dev(w.grad)
    packed = torch.zeros(nb, dtype=torch.uint8, device=dev.dev)
    out = torch.zeros(n, dtype=torch.float32, device=dev.dev)

    def step():
        f.compress_segments(g, offs, theta, bits, packed, ws)
        f.decompress_segments(packed, nb, out, offs, theta, bits, ws)

    step()                                                 # the per-tensor path creates its side streams on first use
    torch.cuda.synchronize()
    want_packed, want_out = packed.clone(), out.clone()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    for replay in range(4):
        # new input each time, eager result first, then the graph on the same buffers
        g.copy_(dev.to_dev(w.grad * np.float32(rng.uniform(0.5, 2.0))))
        step()
        torch.cuda.synchronize()
        want_packed.copy_(packed)
        want_out.copy_(out)
        packed.fill_(0xEE)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert f.device_status(ws) == 0
        assert torch.equal(packed, want_packed), replay
        assert torch.equal(out.view(torch.int32), want_out.view(torch.int32)), replay


def test_per_tensor_call_beside_an_open_capture(dev):
    """While one stream's capture holds the library's side streams, a per-tensor call on another stream must
    neither be recorded into that capture nor fail: it runs on its own stream alone and gives the same bytes."""
    torch, f = dev.torch, dev.f
    w = workloads.config2()
    offs = [int(v) for v in w.seg_offsets]
    theta, bits = w.theta, w.bits
    n = offs[-1]
    nb = f.packed_bytes_segments(offs, theta, bits)
    wsb = f.workspace_bytes_segments(offs, bits)
    ws_a, ws_b = dev.workspace(wsb), dev.workspace(wsb)
    g = dev.to_dev(w.grad)
    g_b = dev.to_dev(w.grad * np.float32(1.5))
    packed_a = torch.zeros(nb, dtype=torch.uint8, device=dev.dev)
    packed_b = torch.full((nb,), 0xEE, dtype=torch.uint8, device=dev.dev)
    want_b = torch.zeros(nb, dtype=torch.uint8, device=dev.dev)
    out_b = torch.full((n,), float("nan"), dtype=torch.float32, device=dev.dev)
    want_out_b = torch.zeros(n, dtype=torch.float32, device=dev.dev)
    f.compress_segments(g_b, offs, theta, bits, want_b, ws_b)       # eager reference, side streams exist from here on
    f.decompress_segments(want_b, nb, want_out_b, offs, theta, bits, ws_b)
    f.compress_segments(g, offs, theta, bits, packed_a, ws_a)
    torch.cuda.synchronize()
    want_a = packed_a.clone()
    graph = torch.cuda.CUDAGraph()
    side, other = torch.cuda.Stream(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side, capture_error_mode="thread_local"):
            f.compress_segments(g, offs, theta, bits, packed_a, ws_a)
            # the capture is still open and owns the side streams: this call must stay out of it
            f.compress_segments(g_b, offs, theta, bits, packed_b, ws_b, other)
            f.decompress_segments(packed_b, nb, out_b, offs, theta, bits, ws_b, other)
    torch.cuda.synchronize()
    assert f.device_status(ws_b) == 0
    assert torch.equal(packed_b, want_b), "the eager call beside the capture gave other bytes"
    assert torch.equal(out_b.view(torch.int32), want_out_b.view(torch.int32))
    packed_a.fill_(0xEE)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(packed_a, want_a)


def test_uniform_round_trip_replays_from_a_graph(dev, ref):
    """the uniform-chunk path at a two-pass chunk length (fused histogram, persistent kernels) from a graph"""
    torch, f = dev.torch, dev.f
    L, theta, bits = 1 << 15, 0.4, 8
    n = 14 * L - 5
    nb = f.packed_bytes(n, L, theta, bits)
    ws = dev.ws_for(n, L, bits)
    g0 = workloads.small_mixed(n, seed=8)
    g = dev.to_dev(g0)
    packed = torch.zeros(nb, dtype=torch.uint8, device=dev.dev)
    out = torch.zeros(n, dtype=torch.float32, device=dev.dev)

    def step():
        f.compress(g, L, theta, bits, packed, ws)
        f.decompress(packed, nb, out, L, theta, bits, ws)

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for replay in range(4):
        g.copy_(dev.to_dev(g0 * np.float32(rng.uniform(0.5, 2.0))))
        step()
        torch.cuda.synchronize()
        want_packed, want_out = packed.clone(), out.clone()
        packed.fill_(0xEE)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert f.device_status(ws) == 0
        assert torch.equal(packed, want_packed), replay
        assert torch.equal(out.view(torch.int32), want_out.view(torch.int32)), replay
    # and the eager result is the one the oracle explains: receiver on the oracle's bytes within the bound
    por = ref.compress(g.cpu().numpy(), L, theta, bits, nthreads=8)
    back, st = dev.decompress(por, n, L, theta, bits, want_status=True)
    assert st == 0
    want = ref.decompress(por, n, L, theta, bits, nthreads=8)
    assert np.linalg.norm(back - want) <= 1e-5 * np.linalg.norm(want)


FIRST_CALL_SCRIPT = r"""
import sys
import numpy as np
import torch
sys.path.insert(0, sys.argv[1])
from paper_1811_08596_amd import fftsp, workloads
fftsp.load()
dev = torch.device("cuda:0")
L, theta, bits = 1 << 15, 0.4, 8
n = 14 * L - 5
nb = fftsp.packed_bytes(n, L, theta, bits)
ws = torch.full((fftsp.workspace_bytes(n, L, bits),), 0xFF, dtype=torch.uint8, device=dev)
g0 = workloads.small_mixed(n, seed=8)
g = torch.from_numpy(g0).to(dev)
packed = torch.zeros(nb, dtype=torch.uint8, device=dev)
out = torch.zeros(n, dtype=torch.float32, device=dev)
offs = [0, 100, 1124, 70000, 70000 + (1 << 15), 200000]
sn = offs[-1]
sg0 = workloads.small_mixed(sn, seed=9)
sg = torch.from_numpy(sg0).to(dev)
snb = fftsp.packed_bytes_segments(offs, 0.5, 8)
sws = torch.full((fftsp.workspace_bytes_segments(offs, 8),), 0xFF, dtype=torch.uint8, device=dev)
spacked = torch.zeros(snb, dtype=torch.uint8, device=dev)
sout = torch.zeros(sn, dtype=torch.float32, device=dev)
torch.cuda.synchronize()
graph = torch.cuda.CUDAGraph()
side = torch.cuda.Stream()
side.wait_stream(torch.cuda.current_stream())
with torch.cuda.stream(side):
    with torch.cuda.graph(graph, stream=side):
        # the first calls into the library in this process
        fftsp.compress(g, L, theta, bits, packed, ws, side)
        fftsp.decompress(packed, nb, out, L, theta, bits, ws, side)
        # also the first per-tensor calls: no side stream exists yet, so they stay on the capturing stream
        fftsp.compress_segments(sg, offs, 0.5, 8, spacked, sws, side)
        fftsp.decompress_segments(spacked, snb, sout, offs, 0.5, 8, sws, side)
torch.cuda.synchronize()
for replay in range(3):
    g.copy_(torch.from_numpy(g0 * np.float32(1.0 + 0.25 * replay)).to(dev))
    sg.copy_(torch.from_numpy(sg0 * np.float32(1.0 + 0.5 * replay)).to(dev))
    packed.fill_(0xEE)
    out.fill_(float("nan"))
    spacked.fill_(0xEE)
    sout.fill_(float("nan"))
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    got_p, got_o, got_sp, got_so = packed.clone(), out.clone(), spacked.clone(), sout.clone()
    fftsp.compress(g, L, theta, bits, packed, ws)
    fftsp.decompress(packed, nb, out, L, theta, bits, ws)
    fftsp.compress_segments(sg, offs, 0.5, 8, spacked, sws)
    fftsp.decompress_segments(spacked, snb, sout, offs, 0.5, 8, sws)
    torch.cuda.synchronize()
    assert fftsp.device_status(ws) == 0 and fftsp.device_status(sws) == 0
    assert torch.equal(got_p, packed), replay
    assert torch.equal(got_o.view(torch.int32), out.view(torch.int32)), replay
    assert torch.equal(got_sp, spacked), replay
    assert torch.equal(got_so.view(torch.int32), sout.view(torch.int32)), replay
print("FIRST_CALL_CAPTURE_OK")
"""


def test_first_library_call_of_a_process_may_sit_inside_a_capture(tmp_path):
    """A fresh process records its very first compress + decompress into a graph (nothing is allocated, copied or
    filled on first use), replays it on new inputs and compares each replay with eager calls."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    script = tmp_path / "first_call.py"
    script.write_text(FIRST_CALL_SCRIPT)
    r = subprocess.run([sys.executable, str(script), root], capture_output=True, text=True, timeout=170)
    assert r.returncode == 0 and "FIRST_CALL_CAPTURE_OK" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
