"""CPU-only checks of the C-ABI library: it loads, exports every symbol include/fftsp.h declares,
its host arithmetic agrees with the oracle's, and argument errors are reported before any launch.
No compute entry point is given valid device pointers here (there is no GPU in this tier)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1811_08596_amd import fftsp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fftsp.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return fftsp.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fftsp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fftsp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = declared_symbols()
    assert len(names) >= 17
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(fftsp.SIGNATURES) == names


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(ImportError):
        fftsp.load(str(tmp_path / "nope.so"))


def test_host_arithmetic_matches_oracle(lib, ref):
    for L in (32, 64, 1 << 10, 1 << 16, 1 << 20, 1 << 22):
        for theta in (0.0, 0.1, 0.25, 0.3, 0.5, 0.7, 0.9, 1.0, 0.123456):
            assert fftsp.kept_per_chunk(L, theta) == ref.kept_per_chunk(L, theta)
            for bits in (3, 6, 8, 10, 16, 32):
                for n in (1, L - 1, L, L + 1, 5 * L + 3):
                    assert fftsp.packed_bytes(n, L, theta, bits) == ref.packed_bytes(n, L, theta, bits)
    for bits in range(0, 40):
        assert fftsp.mantissa_bits(bits) == ref.mantissa_bits(bits)
    offs = [0, 10, 74, 174, 431, 1431, 70000]
    assert fftsp.packed_bytes_segments(offs, 0.3, 6) == ref.packed_bytes_segments(np.array(offs), 0.3, 6)
    assert fftsp.workspace_bytes_segments(offs, 6) >= fftsp.workspace_bytes(1 << 17, 1 << 17, 6)


def test_headline_sizes(lib):
    n = 62378344
    assert fftsp.packed_bytes(n, 1 << 20, 0.5, 8) == 64 + 60 * (-(-(16 + 4 * 16385 + 4 * (2 * 262145 * 8 // 32 + 1)) // 16) * 16)
    assert 0 < fftsp.workspace_bytes(n, 1 << 20, 8) <= 550 * 1000 * 1000   # 2.2 x the gradient


def test_argument_errors_come_back_before_any_launch(lib):
    a = 4096  # a fake, aligned, non-null "device" address: must never be dereferenced on these paths
    call = lambda **kw: lib.fftsp_compress(kw.get("g", a), kw.get("n", 100), kw.get("L", 64), kw.get("theta", 0.5),
                                           kw.get("bits", 8), kw.get("p", a), kw.get("cap", 1 << 20),
                                           kw.get("ws", a), kw.get("wsb", 1 << 30), None)
    assert call(n=0) == fftsp.EINVAL
    assert call(g=None) == fftsp.EINVAL
    assert call(p=None) == fftsp.EINVAL
    assert call(ws=None) == fftsp.EINVAL
    assert call(g=a + 4) == fftsp.EINVAL                      # misaligned
    assert call(L=48) == fftsp.EUNSUPPORTED
    assert call(L=16) == fftsp.EUNSUPPORTED
    assert call(L=1 << 23) == fftsp.EUNSUPPORTED
    assert call(theta=-0.01) == fftsp.EINVAL
    assert call(theta=1.01) == fftsp.EINVAL
    assert call(theta=float("nan")) == fftsp.EINVAL
    for bits in (0, 2, 17, 31, 33):
        assert call(bits=bits) == fftsp.EINVAL
    assert call(cap=fftsp.packed_bytes(100, 64, 0.5, 8) - 1) == fftsp.ENOSPC
    assert call(wsb=fftsp.workspace_bytes(100, 64, 8) - 1) == fftsp.EWORKSPACE
    # decompress: short stream
    rc = lib.fftsp_decompress(a, fftsp.packed_bytes(100, 64, 0.5, 8) - 1, a, 100, 64, 0.5, 8, a, 1 << 30, None)
    assert rc == fftsp.EFORMAT
    assert fftsp.packed_bytes(0, 64, 0.5, 8) == 0 and fftsp.workspace_bytes(10, 63, 8) == 0
    # quantizer options
    def cq(m, r, bits=8):
        q = fftsp.Quantizer(m, r)
        return lib.fftsp_compress_q(a, 100, 64, 0.5, bits, a, 1 << 20, a, 1 << 30, C.byref(q), None)
    assert cq(8, 0.0) == fftsp.EINVAL and cq(-1, 0.0) == fftsp.EINVAL          # m must be 1..bits-1 (0 = default)
    assert cq(0, -1.0) == fftsp.EINVAL and cq(0, float("inf")) == fftsp.EINVAL and cq(0, float("nan")) == fftsp.EINVAL
    # several peers: list checks
    peers = (C.c_void_p * 2)(a, a)
    nb, wsb = fftsp.packed_bytes(100, 64, 0.5, 8), fftsp.workspace_bytes_accumulate(100, 64, 8, 2)
    assert wsb > fftsp.workspace_bytes(100, 64, 8)
    acc = lambda **kw: lib.fftsp_decompress_accumulate(kw.get("lst", peers), kw.get("np", 2), kw.get("nb", nb),
                                                       kw.get("scale", 0.5), a, 100, 64, 0.5, 8, a,
                                                       kw.get("wsb", wsb), None)
    assert acc(np=0) == fftsp.EINVAL
    assert acc(lst=None) == fftsp.EINVAL
    assert acc(np=33, lst=(C.c_void_p * 33)(*([a] * 33))) == fftsp.EUNSUPPORTED
    assert acc(lst=(C.c_void_p * 2)(a, None)) == fftsp.EINVAL
    assert acc(lst=(C.c_void_p * 2)(a, a + 8)) == fftsp.EINVAL
    assert acc(scale=float("nan")) == fftsp.EINVAL
    assert acc(nb=nb - 1) == fftsp.EFORMAT
    assert acc(wsb=wsb - 1) == fftsp.EWORKSPACE
    assert fftsp.workspace_bytes_accumulate(100, 64, 8, 0) == 0 and fftsp.workspace_bytes_accumulate(100, 64, 8, 33) == 0
    # segments
    arr = (C.c_size_t * 3)(0, 10, 10)
    assert lib.fftsp_compress_segments(a, arr, 2, 0.5, 8, a, 1 << 20, a, 1 << 30, None) == fftsp.EINVAL
    arr = (C.c_size_t * 2)(0, (1 << 22) + 1)
    assert lib.fftsp_compress_segments(a, arr, 1, 0.5, 8, a, 1 << 30, a, 1 << 30, None) == fftsp.EUNSUPPORTED
    assert lib.fftsp_strerror(fftsp.EFORMAT).decode().startswith("packed stream")


def test_topk_host_arithmetic_and_argument_errors(lib, ref):
    for L in (32, 1 << 10, 1 << 16, 1 << 21):
        for theta in (0.0, 0.15, 0.5, 1.0, 0.123456):
            assert fftsp.topk_kept_per_chunk(L, theta) == ref.topk_kept_per_chunk(L, theta)
            for bits in (3, 8, 10, 32):
                for n in (1, L - 1, L, L + 1, 5 * L + 3):
                    assert fftsp.topk_packed_bytes(n, L, theta, bits) == ref.topk_packed_bytes(n, L, theta, bits)
    # the time-domain workspace holds no spectrum and no FFT intermediate
    n, L = 1 << 22, 1 << 20
    assert 0 < fftsp.topk_workspace_bytes(n, L, 8) < 8.5 * n      # candidate list (8 bytes per sample) and little else
    a = 4096
    call = lambda **kw: lib.fftsp_topk_compress(kw.get("g", a), kw.get("n", 100), kw.get("L", 64), kw.get("theta", 0.5),
                                                kw.get("bits", 8), kw.get("p", a), kw.get("cap", 1 << 20),
                                                kw.get("ws", a), kw.get("wsb", 1 << 30), None)
    assert call(n=0) == fftsp.EINVAL
    assert call(g=None) == fftsp.EINVAL
    assert call(g=a + 4) == fftsp.EINVAL
    assert call(L=48) == fftsp.EUNSUPPORTED
    assert call(L=1 << 22) == fftsp.EUNSUPPORTED              # one chunk's selection state is sized for 2^21 samples
    assert call(theta=1.5) == fftsp.EINVAL
    assert call(bits=2) == fftsp.EINVAL
    assert call(cap=10) == fftsp.ENOSPC
    assert call(wsb=10) == fftsp.EWORKSPACE
    dec = lambda **kw: lib.fftsp_topk_decompress(kw.get("p", a), kw.get("pb", 1 << 20), kw.get("g", a), kw.get("n", 100),
                                                 kw.get("L", 64), 0.5, kw.get("bits", 8), kw.get("ws", a),
                                                 kw.get("wsb", 1 << 30), None)
    assert dec(pb=10) == fftsp.EFORMAT
    assert dec(g=None) == fftsp.EINVAL
    assert dec(L=1 << 22) == fftsp.EUNSUPPORTED
    assert dec(wsb=10) == fftsp.EWORKSPACE


def test_half_variant_argument_errors(lib):
    a = 4096
    call = lambda **kw: lib.fftsp_compress_h(kw.get("g", a), kw.get("n", 1 << 16), kw.get("L", 1 << 15),
                                             kw.get("theta", 0.5), kw.get("bits", 8), kw.get("s", 8), kw.get("p", a),
                                             kw.get("cap", 1 << 30), kw.get("ws", a), kw.get("wsb", 1 << 30), None)
    assert call(L=1 << 14) == fftsp.EUNSUPPORTED              # single-workgroup chunk lengths have no stored intermediate
    assert call(L=1 << 23) == fftsp.EUNSUPPORTED
    assert call(s=25) == fftsp.EINVAL
    assert call(s=-25) == fftsp.EINVAL
    assert call(g=None) == fftsp.EINVAL
    assert call(g=a + 8) == fftsp.EINVAL
    assert call(theta=-0.1) == fftsp.EINVAL
    assert call(bits=17) == fftsp.EINVAL
    assert call(cap=100) == fftsp.ENOSPC
    assert call(wsb=100) == fftsp.EWORKSPACE
    dec = lambda **kw: lib.fftsp_decompress_h(kw.get("p", a), kw.get("pb", 1 << 30), kw.get("g", a), kw.get("n", 1 << 16),
                                              kw.get("L", 1 << 15), 0.5, 8, kw.get("s", 8), kw.get("ws", a),
                                              kw.get("wsb", 1 << 30), None)
    assert dec(L=1 << 14) == fftsp.EUNSUPPORTED
    assert dec(s=30) == fftsp.EINVAL
    assert dec(pb=100) == fftsp.EFORMAT
    assert dec(wsb=100) == fftsp.EWORKSPACE
    assert dec(g=None) == fftsp.EINVAL


def test_bench_refuses_more_than_one_gpu():
    """one GPU per box: the bench says so instead of starting a multi-rank run"""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "single-GPU" in r.stderr and not r.stdout.strip()


def test_product_does_not_import_the_oracle():
    """The GPU package and its C sources must not use oracle/ (and vice versa)."""
    pkg = os.path.join(ROOT, "paper_1811_08596_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                for needle in ("import oracle", "from oracle", "fftsp_ref", "libfftsp_ref"):
                    assert needle not in text, (f, needle)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            for needle in ("paper_1811_08596_amd", "libfftsp.so", "csrc", "hip_runtime"):
                assert needle not in text, (f, needle)
