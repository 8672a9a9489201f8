"""ctypes front end of the CPU oracle (oracle/fftsp_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  It imports nothing from the GPU package and the
GPU package imports nothing from here.  Arrays are numpy, host memory.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fftsp_ref.c")
_LIB = os.path.join(_HERE, "libfftsp_ref.so")

OK, EINVAL, ENOSPC, EFORMAT = 0, 1, 2, 6


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, no SIMD intrinsics, no FFT library)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        fp = C.POINTER(C.c_float)
        u8p = C.POINTER(C.c_uint8)
        u32p = C.POINTER(C.c_uint32)
        szp = C.POINTER(C.c_size_t)
        sig = {
            "fftsp_ref_rfft": (C.c_int, [fp, C.c_size_t, C.c_uint32, fp, C.c_int]),
            "fftsp_ref_irfft": (C.c_int, [fp, C.c_size_t, C.c_uint32, fp, C.c_int]),
            "fftsp_ref_key": (C.c_uint32, [C.c_float, C.c_float]),
            "fftsp_ref_kept_per_chunk": (C.c_int, [C.c_uint32, C.c_float, u32p]),
            "fftsp_ref_select": (C.c_int, [u32p, C.c_uint32, C.c_uint32, u8p]),
            "fftsp_ref_mantissa_bits": (C.c_int, [C.c_int]),
            "fftsp_ref_pbase": (C.c_uint32, [C.c_uint32, C.c_int, C.c_int]),
            "fftsp_ref_quantize": (C.c_uint32, [C.c_uint32, C.c_uint32, C.c_int, C.c_int]),
            "fftsp_ref_dequantize": (C.c_uint32, [C.c_uint32, C.c_uint32, C.c_int, C.c_int]),
            "fftsp_ref_pack_dense": (C.c_size_t, [fp, C.c_size_t, u8p, u32p, fp]),
            "fftsp_ref_record_stride": (C.c_size_t, [C.c_uint32, C.c_uint32, C.c_int]),
            "fftsp_ref_packed_bytes": (C.c_size_t, [C.c_size_t, C.c_uint32, C.c_float, C.c_int]),
            "fftsp_ref_encode_spectrum": (C.c_int, [fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, u8p, C.c_size_t, C.c_int]),
            "fftsp_ref_decode_spectrum": (C.c_int, [u8p, C.c_size_t, C.c_size_t, C.c_uint32, C.c_float, C.c_int, fp, C.c_int]),
            "fftsp_ref_compress": (C.c_int, [fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, u8p, C.c_size_t, C.c_int]),
            "fftsp_ref_decompress": (C.c_int, [u8p, C.c_size_t, fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int]),
            "fftsp_ref_encode_spectrum_q": (C.c_int, [fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int, C.c_float, u8p, C.c_size_t, C.c_int]),
            "fftsp_ref_decode_spectrum_q": (C.c_int, [u8p, C.c_size_t, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int, fp, C.c_int]),
            "fftsp_ref_compress_q": (C.c_int, [fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int, C.c_float, u8p, C.c_size_t, C.c_int]),
            "fftsp_ref_decompress_q": (C.c_int, [u8p, C.c_size_t, fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int, C.c_int]),
            "fftsp_ref_tune_eps": (C.c_float, [C.c_float, C.c_int, C.c_int]),
            "fftsp_ref_decode_accumulate_spectrum": (C.c_int, [C.POINTER(u8p), C.c_int, C.c_size_t, C.c_size_t, C.c_uint32, C.c_float, C.c_int, fp, C.c_int]),
            "fftsp_ref_decompress_accumulate": (C.c_int, [C.POINTER(u8p), C.c_int, C.c_size_t, C.c_float, fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int]),
            "fftsp_ref_segment_length": (C.c_uint32, [C.c_size_t]),
            "fftsp_ref_packed_bytes_segments": (C.c_size_t, [szp, C.c_int, C.c_float, C.c_int]),
            "fftsp_ref_compress_segments": (C.c_int, [fp, szp, C.c_int, C.c_float, C.c_int, u8p, C.c_size_t, C.c_int]),
            "fftsp_ref_decompress_segments": (C.c_int, [u8p, C.c_size_t, fp, szp, C.c_int, C.c_float, C.c_int, C.c_int]),
            "fftsp_ref_topk_kept_per_chunk": (C.c_int, [C.c_uint32, C.c_float, u32p]),
            "fftsp_ref_topk_record_stride": (C.c_size_t, [C.c_uint32, C.c_uint32, C.c_int]),
            "fftsp_ref_topk_packed_bytes": (C.c_size_t, [C.c_size_t, C.c_uint32, C.c_float, C.c_int]),
            "fftsp_ref_topk_compress": (C.c_int, [fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, u8p, C.c_size_t, C.c_int]),
            "fftsp_ref_topk_decompress": (C.c_int, [u8p, C.c_size_t, fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int]),
            "fftsp_ref_round_half": (C.c_float, [C.c_double]),
            "fftsp_ref_rfft_h": (C.c_int, [fp, C.c_size_t, C.c_uint32, C.c_int, fp, C.c_int]),
            "fftsp_ref_compress_h": (C.c_int, [fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int, u8p, C.c_size_t, C.c_int]),
            "fftsp_ref_decompress_h": (C.c_int, [u8p, C.c_size_t, fp, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int, C.c_int]),
            "fftsp_ref_max_threads": (C.c_int, []),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"{where}: oracle status {code}")
        self.code = code


def _chk(code, where):
    if code != OK:
        raise OracleError(code, where)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint8))


def _offs(seg_offsets):
    a = np.ascontiguousarray(seg_offsets, dtype=np.uintp)
    return a, a.ctypes.data_as(C.POINTER(C.c_size_t))


def max_threads() -> int:
    return lib().fftsp_ref_max_threads()


def n_chunks(n, L):
    if L < 2 or (L & (L - 1)):
        raise OracleError(EINVAL, "chunk length must be a power of two >= 2")
    return (n + L - 1) // L


def rfft(g, L, nthreads=1):
    """(C, L/2+1) complex64 view of the oracle's spectrum (double FFT rounded once)."""
    g, gp = _f32(g)
    Cn = n_chunks(g.size, L)
    spec = np.empty(Cn * (L + 2), dtype=np.float32)
    _chk(lib().fftsp_ref_rfft(gp, g.size, L, spec.ctypes.data_as(C.POINTER(C.c_float)), nthreads), "rfft")
    return spec


def irfft(spec, n, L, nthreads=1):
    spec, sp = _f32(spec)
    out = np.empty(n, dtype=np.float32)
    _chk(lib().fftsp_ref_irfft(sp, n, L, out.ctypes.data_as(C.POINTER(C.c_float)), nthreads), "irfft")
    return out


def key(re, im) -> int:
    return lib().fftsp_ref_key(np.float32(re), np.float32(im))


def kept_per_chunk(L, theta) -> int:
    k = C.c_uint32()
    _chk(lib().fftsp_ref_kept_per_chunk(L, np.float32(theta), C.byref(k)), "kept_per_chunk")
    return k.value


def select(keys, k):
    keys = np.ascontiguousarray(keys, dtype=np.uint32)
    flags = np.zeros(keys.size, dtype=np.uint8)
    _chk(lib().fftsp_ref_select(keys.ctypes.data_as(C.POINTER(C.c_uint32)), keys.size, k,
                                flags.ctypes.data_as(C.POINTER(C.c_uint8))), "select")
    return flags


def mantissa_bits(bits) -> int:
    return lib().fftsp_ref_mantissa_bits(bits)


def pbase(vmax_bits, bits, m) -> int:
    return lib().fftsp_ref_pbase(int(vmax_bits), bits, m)


def quantize(fbits, pb, bits, m) -> int:
    return lib().fftsp_ref_quantize(int(fbits), int(pb), bits, m)


def dequantize(code, pb, bits, m) -> int:
    return lib().fftsp_ref_dequantize(int(code), int(pb), bits, m)


def pack_dense(sparse):
    """Sec. 3.2's three steps on a float vector: (status, inclusive location, dense)."""
    sparse, sp = _f32(sparse)
    status = np.zeros(sparse.size, dtype=np.uint8)
    loc = np.zeros(sparse.size, dtype=np.uint32)
    dense = np.zeros(sparse.size, dtype=np.float32)
    cnt = lib().fftsp_ref_pack_dense(sp, sparse.size, status.ctypes.data_as(C.POINTER(C.c_uint8)),
                                     loc.ctypes.data_as(C.POINTER(C.c_uint32)),
                                     dense.ctypes.data_as(C.POINTER(C.c_float)))
    return status, loc, dense[:cnt]


def record_stride(L, k, bits) -> int:
    return lib().fftsp_ref_record_stride(L, k, bits)


def packed_bytes(n, L, theta, bits) -> int:
    return lib().fftsp_ref_packed_bytes(n, L, np.float32(theta), bits)


def encode_spectrum(spec, n, L, theta, bits, nthreads=1):
    spec, sp = _f32(spec)
    nb = packed_bytes(n, L, theta, bits)
    if nb == 0:
        raise OracleError(EINVAL, "encode_spectrum")
    out = np.empty(nb, dtype=np.uint8)
    _chk(lib().fftsp_ref_encode_spectrum(sp, n, L, np.float32(theta), bits,
                                         out.ctypes.data_as(C.POINTER(C.c_uint8)), nb, nthreads), "encode_spectrum")
    return out


def decode_spectrum(packed, n, L, theta, bits, nthreads=1):
    packed, pp = _u8(packed)
    spec = np.empty(n_chunks(n, L) * (L + 2), dtype=np.float32)
    _chk(lib().fftsp_ref_decode_spectrum(pp, packed.size, n, L, np.float32(theta), bits,
                                         spec.ctypes.data_as(C.POINTER(C.c_float)), nthreads), "decode_spectrum")
    return spec


def compress(g, L, theta, bits, nthreads=1):
    g, gp = _f32(g)
    nb = packed_bytes(g.size, L, theta, bits)
    if nb == 0:
        raise OracleError(EINVAL, "compress")
    out = np.empty(nb, dtype=np.uint8)
    _chk(lib().fftsp_ref_compress(gp, g.size, L, np.float32(theta), bits,
                                  out.ctypes.data_as(C.POINTER(C.c_uint8)), nb, nthreads), "compress")
    return out


def decompress(packed, n, L, theta, bits, nthreads=1):
    packed, pp = _u8(packed)
    out = np.empty(n, dtype=np.float32)
    _chk(lib().fftsp_ref_decompress(pp, packed.size, out.ctypes.data_as(C.POINTER(C.c_float)), n, L,
                                    np.float32(theta), bits, nthreads), "decompress")
    return out


# ---- quantizer options of Sec. 3.2.1: m (0 = default for the width), static range [-range_max, range_max] (0 = fitted)
def encode_spectrum_q(spec, n, L, theta, bits, m=0, range_max=0.0, nthreads=1):
    spec, sp = _f32(spec)
    nb = packed_bytes(n, L, theta, bits)
    if nb == 0:
        raise OracleError(EINVAL, "encode_spectrum_q")
    out = np.empty(nb, dtype=np.uint8)
    _chk(lib().fftsp_ref_encode_spectrum_q(sp, n, L, np.float32(theta), bits, m, np.float32(range_max),
                                           out.ctypes.data_as(C.POINTER(C.c_uint8)), nb, nthreads), "encode_spectrum_q")
    return out


def decode_spectrum_q(packed, n, L, theta, bits, m=0, nthreads=1):
    packed, pp = _u8(packed)
    spec = np.empty(n_chunks(n, L) * (L + 2), dtype=np.float32)
    _chk(lib().fftsp_ref_decode_spectrum_q(pp, packed.size, n, L, np.float32(theta), bits, m,
                                           spec.ctypes.data_as(C.POINTER(C.c_float)), nthreads), "decode_spectrum_q")
    return spec


def compress_q(g, L, theta, bits, m=0, range_max=0.0, nthreads=1):
    g, gp = _f32(g)
    nb = packed_bytes(g.size, L, theta, bits)
    if nb == 0:
        raise OracleError(EINVAL, "compress_q")
    out = np.empty(nb, dtype=np.uint8)
    _chk(lib().fftsp_ref_compress_q(gp, g.size, L, np.float32(theta), bits, m, np.float32(range_max),
                                    out.ctypes.data_as(C.POINTER(C.c_uint8)), nb, nthreads), "compress_q")
    return out


def decompress_q(packed, n, L, theta, bits, m=0, nthreads=1):
    packed, pp = _u8(packed)
    out = np.empty(n, dtype=np.float32)
    _chk(lib().fftsp_ref_decompress_q(pp, packed.size, out.ctypes.data_as(C.POINTER(C.c_float)), n, L,
                                      np.float32(theta), bits, m, nthreads), "decompress_q")
    return out


def tune_eps(range_max, bits, m) -> float:
    """The paper's iterative choice of eps for a static range (bisection on the most negative code)."""
    return float(lib().fftsp_ref_tune_eps(np.float32(range_max), bits, m))


def _peer_list(packed_list):
    """ctypes array of byte pointers for a list of equally long packed streams (kept alive by the caller)."""
    arrs = [np.ascontiguousarray(p, dtype=np.uint8) for p in packed_list]
    if not arrs or any(a.size != arrs[0].size for a in arrs):
        raise OracleError(EINVAL, "peer streams must be non-empty and equally long")
    u8p = C.POINTER(C.c_uint8)
    ptrs = (u8p * len(arrs))(*[a.ctypes.data_as(u8p) for a in arrs])
    return arrs, ptrs


def decode_accumulate_spectrum(packed_list, n, L, theta, bits, nthreads=1):
    """Bin-wise binary32 sum, in list order, of the peers' decoded spectra (receiver under an allgather)."""
    arrs, ptrs = _peer_list(packed_list)
    spec = np.empty(n_chunks(n, L) * (L + 2), dtype=np.float32)
    _chk(lib().fftsp_ref_decode_accumulate_spectrum(ptrs, len(arrs), arrs[0].size, n, L, np.float32(theta), bits,
                                                    spec.ctypes.data_as(C.POINTER(C.c_float)), nthreads),
         "decode_accumulate_spectrum")
    return spec


def decompress_accumulate(packed_list, scale, n, L, theta, bits, nthreads=1):
    """scale * iFFT(sum of the peers' decoded spectra): one inverse transform for all peers."""
    arrs, ptrs = _peer_list(packed_list)
    out = np.empty(n, dtype=np.float32)
    _chk(lib().fftsp_ref_decompress_accumulate(ptrs, len(arrs), arrs[0].size, np.float32(scale),
                                               out.ctypes.data_as(C.POINTER(C.c_float)), n, L, np.float32(theta), bits,
                                               nthreads), "decompress_accumulate")
    return out


def segment_length(size) -> int:
    return lib().fftsp_ref_segment_length(size)


def packed_bytes_segments(seg_offsets, theta, bits) -> int:
    a, ap = _offs(seg_offsets)
    return lib().fftsp_ref_packed_bytes_segments(ap, a.size - 1, np.float32(theta), bits)


def compress_segments(g, seg_offsets, theta, bits, nthreads=1):
    g, gp = _f32(g)
    a, ap = _offs(seg_offsets)
    nb = packed_bytes_segments(a, theta, bits)
    if nb == 0:
        raise OracleError(EINVAL, "compress_segments")
    out = np.empty(nb, dtype=np.uint8)
    _chk(lib().fftsp_ref_compress_segments(gp, ap, a.size - 1, np.float32(theta), bits,
                                           out.ctypes.data_as(C.POINTER(C.c_uint8)), nb, nthreads), "compress_segments")
    return out


def decompress_segments(packed, seg_offsets, theta, bits, nthreads=1):
    packed, pp = _u8(packed)
    a, ap = _offs(seg_offsets)
    out = np.zeros(int(a[-1]), dtype=np.float32)
    _chk(lib().fftsp_ref_decompress_segments(pp, packed.size, out.ctypes.data_as(C.POINTER(C.c_float)), ap,
                                             a.size - 1, np.float32(theta), bits, nthreads), "decompress_segments")
    return out


# ---- half-precision variant (Sec. 3.1.1, "Our approach"): spectrum scaled by 2^scale_log2, rounded once to binary16
def round_half(v) -> float:
    return float(lib().fftsp_ref_round_half(float(v)))


def rfft_h(g, L, scale_log2=0, nthreads=1):
    g, gp = _f32(g)
    spec = np.empty(n_chunks(g.size, L) * (L + 2), dtype=np.float32)
    _chk(lib().fftsp_ref_rfft_h(gp, g.size, L, scale_log2, spec.ctypes.data_as(C.POINTER(C.c_float)), nthreads), "rfft_h")
    return spec


def compress_h(g, L, theta, bits, scale_log2=0, nthreads=1):
    g, gp = _f32(g)
    nb = packed_bytes(g.size, L, theta, bits)
    if nb == 0:
        raise OracleError(EINVAL, "compress_h")
    out = np.empty(nb, dtype=np.uint8)
    _chk(lib().fftsp_ref_compress_h(gp, g.size, L, np.float32(theta), bits, scale_log2,
                                    out.ctypes.data_as(C.POINTER(C.c_uint8)), nb, nthreads), "compress_h")
    return out


def decompress_h(packed, n, L, theta, bits, scale_log2=0, nthreads=1):
    packed, pp = _u8(packed)
    out = np.empty(n, dtype=np.float32)
    _chk(lib().fftsp_ref_decompress_h(pp, packed.size, out.ctypes.data_as(C.POINTER(C.c_float)), n, L,
                                      np.float32(theta), bits, scale_log2, nthreads), "decompress_h")
    return out


# ---- time-domain Top-k (Sec. 4, "Choice of Algorithms"): same selector, quantizer and packing, no transform ----
def topk_kept_per_chunk(L, theta) -> int:
    k = C.c_uint32(0)
    _chk(lib().fftsp_ref_topk_kept_per_chunk(L, np.float32(theta), C.byref(k)), "topk_kept_per_chunk")
    return int(k.value)


def topk_record_stride(L, k, bits) -> int:
    return int(lib().fftsp_ref_topk_record_stride(L, k, bits))


def topk_packed_bytes(n, L, theta, bits) -> int:
    return int(lib().fftsp_ref_topk_packed_bytes(n, L, np.float32(theta), bits))


def topk_compress(g, L, theta, bits, nthreads=1):
    g, gp = _f32(g)
    nb = topk_packed_bytes(g.size, L, theta, bits)
    if nb == 0:
        raise OracleError(EINVAL, "topk_compress")
    out = np.empty(nb, dtype=np.uint8)
    _chk(lib().fftsp_ref_topk_compress(gp, g.size, L, np.float32(theta), bits,
                                       out.ctypes.data_as(C.POINTER(C.c_uint8)), nb, nthreads), "topk_compress")
    return out


def topk_decompress(packed, n, L, theta, bits, nthreads=1):
    packed, pp = _u8(packed)
    out = np.empty(n, dtype=np.float32)
    _chk(lib().fftsp_ref_topk_decompress(pp, packed.size, out.ctypes.data_as(C.POINTER(C.c_float)), n, L,
                                         np.float32(theta), bits, nthreads), "topk_decompress")
    return out


def topk_record_fields(packed, L, c=0):
    """pbase, vmax_bits, k, word3, bitmap bits (L,) and code bytes of record c of a time-domain stream."""
    h = parse_header(packed)
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    W = (L + 31) // 32
    rec = p[64 + c * h["S"]: 64 + (c + 1) * h["S"]]
    hdr = rec[:16].view("<u4")
    bitmap = np.unpackbits(rec[16:16 + 4 * W], bitorder="little")[:L]
    return int(hdr[0]), int(hdr[1]), int(hdr[2]), int(hdr[3]), bitmap, rec[16 + 4 * W:]


# ---- helpers that only parse the documented byte layout (used by tests) ----
def parse_header(packed):
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    u32 = lambda o: int(p[o:o + 4].view("<u4")[0])
    return dict(magic=bytes(p[0:4]), version=u32(4), n=int(p[8:16].view("<u8")[0]), L=u32(16), C=u32(20),
                bits=u32(24), m=u32(28), k=u32(32), S=u32(36), theta=float(p[40:44].view("<f4")[0]),
                domain=u32(44), scale_log2=int(p[48:52].view("<i4")[0]))


def record_fields(packed, L, c=0):
    """pbase, vmax_bits, k, word3, bitmap bits (B,) and code words of record c (uniform chunking)."""
    h = parse_header(packed)
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    B = L // 2 + 1
    W = (B + 31) // 32
    rec = p[64 + c * h["S"]: 64 + (c + 1) * h["S"]]
    hdr = rec[:16].view("<u4")
    bitmap = np.unpackbits(rec[16:16 + 4 * W], bitorder="little")[:B]
    codes = rec[16 + 4 * W:]
    return int(hdr[0]), int(hdr[1]), int(hdr[2]), int(hdr[3]), bitmap, codes


def unpack_codes(code_bytes, count, bits):
    """first `count` N-bit codes of an LSB-first stream"""
    allbits = np.unpackbits(np.ascontiguousarray(code_bytes, dtype=np.uint8), bitorder="little")
    allbits = allbits[:count * bits].reshape(count, bits).astype(np.uint64)
    return (allbits << np.arange(bits, dtype=np.uint64)).sum(axis=1).astype(np.uint32)
