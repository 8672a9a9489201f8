"""Helpers for the GPU parity tests: torch is used only to own device memory and a stream.
Every compute call goes through the C ABI (paper_1811_08596_amd.fftsp)."""
from __future__ import annotations

import numpy as np


class Device:
    def __init__(self):
        import torch
        from paper_1811_08596_amd import fftsp
        if not torch.cuda.is_available():
            raise RuntimeError("GPU tests need a GPU")
        self.torch = torch
        self.f = fftsp
        fftsp.load()
        self.dev = torch.device("cuda:0")

    # -- memory --
    def to_dev(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)

    def empty(self, n, dtype):
        return self.torch.empty(int(n), dtype=dtype, device=self.dev)

    def workspace(self, nbytes):
        """workspace poisoned with 0xFF so that a read of something the call did not write shows up"""
        return self.torch.full((int(nbytes),), 0xFF, dtype=self.torch.uint8, device=self.dev)

    def ws_for(self, n, L, bits=32):
        nb = self.f.workspace_bytes(n, L, bits)
        assert nb > 0
        return self.workspace(nb)

    def sync(self):
        self.torch.cuda.synchronize()

    # -- stage calls, numpy in / numpy out --
    def rfft(self, g, L):
        n = g.size
        C = (n + L - 1) // L
        gd = self.to_dev(g.astype(np.float32))
        spec = self.torch.full((C * (L + 2),), float("nan"), dtype=self.torch.float32, device=self.dev)
        self.f.rfft(gd, L, spec, self.ws_for(n, L))
        self.sync()
        return spec.cpu().numpy()

    def irfft(self, spec, n, L):
        sd = self.to_dev(np.asarray(spec, np.float32))
        out = self.torch.full((n,), float("nan"), dtype=self.torch.float32, device=self.dev)
        self.f.irfft(sd, n, L, out, self.ws_for(n, L))
        self.sync()
        return out.cpu().numpy()

    def encode(self, spec, n, L, theta, bits):
        sd = self.to_dev(np.asarray(spec, np.float32))
        nb = self.f.packed_bytes(n, L, theta, bits)
        assert nb > 0
        packed = self.torch.full((nb,), 0xEE, dtype=self.torch.uint8, device=self.dev)
        self.f.encode_spectrum(sd, n, L, theta, bits, packed, self.ws_for(n, L, bits))
        self.sync()
        return packed.cpu().numpy()

    def decode(self, packed, n, L, theta, bits, want_status=False):
        pd = self.to_dev(np.asarray(packed, np.uint8))
        C = (n + L - 1) // L
        spec = self.torch.full((C * (L + 2),), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.ws_for(n, L, bits)
        self.f.decode_spectrum(pd, pd.numel(), n, L, theta, bits, spec, ws)
        st = self.f.device_status(ws)
        out = spec.cpu().numpy()
        return (out, st) if want_status else out

    def compress(self, g, L, theta, bits):
        n = g.size
        gd = self.to_dev(g.astype(np.float32))
        nb = self.f.packed_bytes(n, L, theta, bits)
        packed = self.torch.full((nb,), 0xEE, dtype=self.torch.uint8, device=self.dev)
        self.f.compress(gd, L, theta, bits, packed, self.ws_for(n, L, bits))
        self.sync()
        return packed.cpu().numpy()

    def decompress(self, packed, n, L, theta, bits, want_status=False):
        pd = self.to_dev(np.asarray(packed, np.uint8))
        out = self.torch.full((n,), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.ws_for(n, L, bits)
        self.f.decompress(pd, pd.numel(), out, L, theta, bits, ws)
        st = self.f.device_status(ws)
        res = out.cpu().numpy()
        return (res, st) if want_status else res

    def encode_q(self, spec, n, L, theta, bits, m=0, range_max=0.0):
        sd = self.to_dev(np.asarray(spec, np.float32))
        nb = self.f.packed_bytes(n, L, theta, bits)
        packed = self.torch.full((nb,), 0xEE, dtype=self.torch.uint8, device=self.dev)
        self.f.encode_spectrum_q(sd, n, L, theta, bits, packed, self.ws_for(n, L, bits), m, range_max)
        self.sync()
        return packed.cpu().numpy()

    def decode_q(self, packed, n, L, theta, bits, m=0):
        pd = self.to_dev(np.asarray(packed, np.uint8))
        C = (n + L - 1) // L
        spec = self.torch.full((C * (L + 2),), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.ws_for(n, L, bits)
        self.f.decode_spectrum_q(pd, pd.numel(), n, L, theta, bits, spec, ws, m)
        return spec.cpu().numpy(), self.f.device_status(ws)

    def compress_q(self, g, L, theta, bits, m=0, range_max=0.0):
        n = g.size
        gd = self.to_dev(g.astype(np.float32))
        nb = self.f.packed_bytes(n, L, theta, bits)
        packed = self.torch.full((nb,), 0xEE, dtype=self.torch.uint8, device=self.dev)
        self.f.compress_q(gd, L, theta, bits, packed, self.ws_for(n, L, bits), m, range_max)
        self.sync()
        return packed.cpu().numpy()

    def decompress_q(self, packed, n, L, theta, bits, m=0):
        pd = self.to_dev(np.asarray(packed, np.uint8))
        out = self.torch.full((n,), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.ws_for(n, L, bits)
        self.f.decompress_q(pd, pd.numel(), out, L, theta, bits, ws, m)
        return out.cpu().numpy(), self.f.device_status(ws)

    def decode_accumulate(self, packed_list, n, L, theta, bits):
        pds = [self.to_dev(np.asarray(p, np.uint8)) for p in packed_list]
        C = (n + L - 1) // L
        spec = self.torch.full((C * (L + 2),), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.workspace(self.f.workspace_bytes_accumulate(n, L, bits, len(pds)))
        self.f.decode_accumulate_spectrum(pds, pds[0].numel(), n, L, theta, bits, spec, ws)
        st = self.f.device_status(ws)
        return spec.cpu().numpy(), st

    def decompress_accumulate(self, packed_list, scale, n, L, theta, bits):
        pds = [self.to_dev(np.asarray(p, np.uint8)) for p in packed_list]
        out = self.torch.full((n,), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.workspace(self.f.workspace_bytes_accumulate(n, L, bits, len(pds)))
        self.f.decompress_accumulate(pds, pds[0].numel(), scale, out, L, theta, bits, ws)
        st = self.f.device_status(ws)
        return out.cpu().numpy(), st

    def compress_h(self, g, L, theta, bits, scale_log2):
        n = g.size
        gd = self.to_dev(g.astype(np.float32))
        nb = self.f.packed_bytes(n, L, theta, bits)
        packed = self.torch.full((nb,), 0xEE, dtype=self.torch.uint8, device=self.dev)
        self.f.compress_h(gd, L, theta, bits, scale_log2, packed, self.ws_for(n, L, bits))
        self.sync()
        return packed.cpu().numpy()

    def decompress_h(self, packed, n, L, theta, bits, scale_log2, pad=0):
        pd = self.to_dev(np.asarray(packed, np.uint8))
        out = self.torch.full((n + pad,), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.ws_for(n, L, bits)
        self.f.decompress_h(pd, pd.numel(), out[:n], L, theta, bits, scale_log2, ws)
        st = self.f.device_status(ws)
        res = out.cpu().numpy()
        return res[:n], st, res[n:]

    def topk_compress(self, g, L, theta, bits):
        n = g.size
        gd = self.to_dev(g.astype(np.float32))
        nb = self.f.topk_packed_bytes(n, L, theta, bits)
        assert nb > 0
        packed = self.torch.full((nb,), 0xEE, dtype=self.torch.uint8, device=self.dev)
        self.f.topk_compress(gd, L, theta, bits, packed, self.workspace(self.f.topk_workspace_bytes(n, L, bits)))
        self.sync()
        return packed.cpu().numpy()

    def topk_decompress(self, packed, n, L, theta, bits, pad=0):
        """returns (reconstruction, status, tail): `pad` extra floats behind the output must come back untouched"""
        pd = self.to_dev(np.asarray(packed, np.uint8))
        out = self.torch.full((n + pad,), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.workspace(self.f.topk_workspace_bytes(n, L, bits))
        self.f.topk_decompress(pd, pd.numel(), out[:n], L, theta, bits, ws)
        st = self.f.device_status(ws)
        res = out.cpu().numpy()
        return res[:n], st, res[n:]

    def compress_segments(self, g, offs, theta, bits):
        gd = self.to_dev(g.astype(np.float32))
        nb = self.f.packed_bytes_segments(offs, theta, bits)
        packed = self.torch.full((nb,), 0xEE, dtype=self.torch.uint8, device=self.dev)
        ws = self.workspace(self.f.workspace_bytes_segments(offs, bits))
        self.f.compress_segments(gd, offs, theta, bits, packed, ws)
        self.sync()
        return packed.cpu().numpy()

    def decompress_segments(self, packed, offs, theta, bits):
        pd = self.to_dev(np.asarray(packed, np.uint8))
        out = self.torch.full((int(offs[-1]),), float("nan"), dtype=self.torch.float32, device=self.dev)
        ws = self.workspace(self.f.workspace_bytes_segments(offs, bits))
        self.f.decompress_segments(pd, pd.numel(), out, offs, theta, bits, ws)
        st = self.f.device_status(ws)
        return out.cpu().numpy(), st


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def per_chunk_rel_l2(a, b, C):
    a = np.asarray(a).reshape(C, -1)
    b = np.asarray(b).reshape(C, -1)
    return max(rel_l2(a[c], b[c]) for c in range(C))


def fft_component_tolerance(L, rms_bin):
    """How far one component of a binary32 transform of length L may sit from the exact value: a radix-2^k FFT in
    binary32 has relative L2 error sigma = 2^-24 * sqrt(log2 L) (2.7e-7 at L = 2^20; 2.3e-7 was measured), spread
    evenly over the bins, so a bin is off by sigma * rms_bin in the root mean square; eight times that is the bound
    used for single components (a tail that a million bins do not reach)."""
    return 8.0 * 2.0 ** -24 * np.sqrt(np.log2(L)) * rms_bin


def explain_end_to_end(ref, packed_gpu, packed_or, spec_or, n, L, theta, bits, m=0):
    """End-to-end streams come from two different spectra (binary32 FFT on the GPU, double FFT rounded once in
    the oracle), so they may differ, but only in ways rounding explains.  With d = fft_component_tolerance:
      - a bin may be kept by one side only if its oracle key is within 4*sqrt(2*tau)*d + 4*d^2 of the oracle's
        threshold key tau (a key re^2 + im^2 near tau moves by at most 2*sqrt(2*tau)*d + 2*d^2 when both components
        move by d, and the threshold itself moves as much); where tau is of the order of the mean key this is the
        1e-5 * tau of the survey's rule;
      - a bin kept by both may differ by at most one quantization level (plus one more if eps moved by one), plus d
        where the codes are finer than the transforms agree.
    Returns (selection mismatches, code mismatches)."""
    C = (n + L - 1) // L
    B = L // 2 + 1
    Xo = np.asarray(spec_or).reshape(C, L + 2).view(np.complex64)
    Sg = ref.decode_spectrum_q(packed_gpu, n, L, theta, bits, m).reshape(C, L + 2).view(np.complex64)
    So = ref.decode_spectrum_q(packed_or, n, L, theta, bits, m).reshape(C, L + 2).view(np.complex64)
    m = m if m and bits != 32 else ref.mantissa_bits(bits)
    sel_mis = code_mis = 0
    for c in range(C):
        _, _, k, _, bg, _ = ref.record_fields(packed_gpu, L, c)
        _, _, _, _, bo, _ = ref.record_fields(packed_or, L, c)
        assert bg.sum() == k == bo.sum()
        rms = np.sqrt(np.mean(np.abs(Xo[c]).astype(np.float64) ** 2))
        d = fft_component_tolerance(L, rms)
        diff = np.flatnonzero(bg != bo)
        if diff.size:
            re, im = Xo[c].real.astype(np.float32), Xo[c].imag.astype(np.float32)
            keyf = (re.astype(np.float64) ** 2 + im.astype(np.float64) ** 2)
            tau = keyf[bo.astype(bool)].min()
            window = 4.0 * np.sqrt(2.0 * tau) * d + 4.0 * d * d
            assert np.all(np.abs(keyf[diff] - tau) <= window), "selection differs away from the threshold"
            sel_mis += diff.size
        both = np.flatnonzero(bg & bo)
        a = Sg[c][both].view(np.float32).astype(np.float64)
        b = So[c][both].view(np.float32).astype(np.float64)
        if bits == 32:
            xo = Xo[c][both].view(np.float32).astype(np.float64)
            assert np.all(np.abs(a - xo) <= d)
            continue
        step = 2.0 ** (-m) * np.maximum(np.abs(a), np.abs(b))
        pbg = ref.record_fields(packed_gpu, L, c)[0]
        eps = float(np.uint32(max(pbg, 1) << (23 - m)).view(np.float32))
        bad = np.abs(a - b) > 2.05 * step + 2.05 * eps + d
        assert not bad.any(), "codes differ by more than rounding explains"
        code_mis += int((a != b).sum())
    return sel_mis, code_mis
