"""Thin ctypes binding over libfftsp.so (include/fftsp.h): argument marshalling only.

Every step of the codec runs in the HIP kernels behind the C ABI; torch is used
for device memory and streams.  There is no CPU fallback: if the shared library
is missing or fails to load, importing callers get an ImportError.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfftsp.so")

OK, EINVAL, ENOSPC, EWORKSPACE, EUNSUPPORTED, EHIP, EFORMAT = range(7)

# name -> (restype, argtypes); every symbol include/fftsp.h declares
_szp = C.POINTER(C.c_size_t)
class Quantizer(C.Structure):
    """fftsp_quantizer: mantissa_bits (0 = default for the width), range_max (0 = fitted per chunk)."""
    _fields_ = [("mantissa_bits", C.c_int), ("range_max", C.c_float)]


_qp = C.POINTER(Quantizer)

SIGNATURES = {
    "fftsp_kept_per_chunk": (C.c_int, [C.c_uint32, C.c_float, C.POINTER(C.c_uint32)]),
    "fftsp_mantissa_bits": (C.c_int, [C.c_int]),
    "fftsp_packed_bytes": (C.c_size_t, [C.c_size_t, C.c_uint32, C.c_float, C.c_int]),
    "fftsp_workspace_bytes": (C.c_size_t, [C.c_size_t, C.c_uint32, C.c_int]),
    "fftsp_compress": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_void_p, C.c_size_t,
                                 C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_decompress": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int,
                                   C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_compress_static": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_void_p,
                                        C.c_size_t, C.c_void_p]),
    "fftsp_compress_h": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_int, C.c_void_p,
                                   C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_decompress_h": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int,
                                     C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_topk_kept_per_chunk": (C.c_int, [C.c_uint32, C.c_float, C.POINTER(C.c_uint32)]),
    "fftsp_topk_packed_bytes": (C.c_size_t, [C.c_size_t, C.c_uint32, C.c_float, C.c_int]),
    "fftsp_topk_workspace_bytes": (C.c_size_t, [C.c_size_t, C.c_uint32, C.c_int]),
    "fftsp_topk_compress": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_void_p, C.c_size_t,
                                      C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_topk_decompress": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_uint32, C.c_float,
                                        C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_compress_q": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_void_p, C.c_size_t,
                                   C.c_void_p, C.c_size_t, _qp, C.c_void_p]),
    "fftsp_decompress_q": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int,
                                     C.c_void_p, C.c_size_t, _qp, C.c_void_p]),
    "fftsp_encode_spectrum_q": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_void_p,
                                          C.c_size_t, C.c_void_p, C.c_size_t, _qp, C.c_void_p]),
    "fftsp_decode_spectrum_q": (C.c_int, [C.c_void_p, C.c_size_t, C.c_size_t, C.c_uint32, C.c_float, C.c_int,
                                          C.c_void_p, C.c_void_p, C.c_size_t, _qp, C.c_void_p]),
    "fftsp_workspace_bytes_accumulate": (C.c_size_t, [C.c_size_t, C.c_uint32, C.c_int, C.c_int]),
    "fftsp_decompress_accumulate": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_size_t, C.c_float, C.c_void_p,
                                              C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_void_p, C.c_size_t,
                                              C.c_void_p]),
    "fftsp_decode_accumulate_spectrum": (C.c_int, [C.POINTER(C.c_void_p), C.c_int, C.c_size_t, C.c_size_t, C.c_uint32,
                                                   C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t,
                                                   C.c_void_p]),
    "fftsp_rfft": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_irfft": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_encode_spectrum": (C.c_int, [C.c_void_p, C.c_size_t, C.c_uint32, C.c_float, C.c_int, C.c_void_p,
                                        C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_decode_spectrum": (C.c_int, [C.c_void_p, C.c_size_t, C.c_size_t, C.c_uint32, C.c_float, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_packed_bytes_segments": (C.c_size_t, [_szp, C.c_int, C.c_float, C.c_int]),
    "fftsp_workspace_bytes_segments": (C.c_size_t, [_szp, C.c_int, C.c_int]),
    "fftsp_compress_segments": (C.c_int, [C.c_void_p, _szp, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_size_t,
                                          C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_decompress_segments": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, _szp, C.c_int, C.c_float, C.c_int,
                                            C.c_void_p, C.c_size_t, C.c_void_p]),
    "fftsp_device_status": (C.c_int, [C.c_void_p, C.POINTER(C.c_int)]),
    "fftsp_profile_enable": (C.c_int, [C.c_int]),
    "fftsp_profile_report": (C.c_size_t, [C.c_char_p, C.c_size_t]),
    "fftsp_strerror": (C.c_char_p, [C.c_int]),
    "fftsp_version": (C.c_char_p, []),
}

_lib = None


def load(path: Optional[str] = None):
    """dlopen the C-ABI library and attach prototypes; raises ImportError if it is not built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise ImportError(f"{p} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    try:
        lib = C.CDLL(p)
    except OSError as e:
        raise ImportError(f"cannot load {p}: {e}") from e
    for name, (res, args) in SIGNATURES.items():
        f = getattr(lib, name)
        f.restype, f.argtypes = res, args
    if path is None:
        _lib = lib
    return lib


class FftspError(RuntimeError):
    def __init__(self, code: int, where: str):
        msg = load().fftsp_strerror(code).decode()
        super().__init__(f"{where}: {msg} (status {code})")
        self.code = code


def _check(code: int, where: str):
    if code != OK:
        raise FftspError(code, where)


def _stream(stream=None) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _offsets(seg_offsets: Sequence[int]):
    arr = (C.c_size_t * len(seg_offsets))(*[int(v) for v in seg_offsets])
    return arr, len(seg_offsets) - 1


# ---- host arithmetic ----
def kept_per_chunk(chunk_len: int, theta: float) -> int:
    k = C.c_uint32()
    _check(load().fftsp_kept_per_chunk(chunk_len, theta, C.byref(k)), "fftsp_kept_per_chunk")
    return k.value


def mantissa_bits(bits: int) -> int:
    return load().fftsp_mantissa_bits(bits)


def packed_bytes(n: int, chunk_len: int, theta: float, bits: int) -> int:
    return load().fftsp_packed_bytes(n, chunk_len, theta, bits)


def workspace_bytes(n: int, chunk_len: int, bits: int) -> int:
    return load().fftsp_workspace_bytes(n, chunk_len, bits)


def packed_bytes_segments(seg_offsets, theta: float, bits: int) -> int:
    arr, nseg = _offsets(seg_offsets)
    return load().fftsp_packed_bytes_segments(arr, nseg, theta, bits)


def workspace_bytes_segments(seg_offsets, bits: int) -> int:
    arr, nseg = _offsets(seg_offsets)
    return load().fftsp_workspace_bytes_segments(arr, nseg, bits)


# ---- device entry points: tensors are torch CUDA tensors, contiguous ----
def _ptr(t) -> int:
    assert t.is_cuda and t.is_contiguous(), "device entry points take contiguous CUDA tensors"
    return t.data_ptr()


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def compress(grad, chunk_len: int, theta: float, bits: int, packed, workspace, stream=None):
    _check(load().fftsp_compress(_ptr(grad), grad.numel(), chunk_len, theta, bits, _ptr(packed), _nbytes(packed),
                                 _ptr(workspace), _nbytes(workspace), _stream(stream)), "fftsp_compress")


STATIC_SCRATCH_BYTES = 16 << 20  # FFTSP_STATIC_SCRATCH_BYTES


def compress_static(grad, chunk_len: int, theta: float, bits: int, packed, stream=None):
    """fftsp_compress on the library's own fixed scratch array: no workspace argument, no allocation."""
    _check(load().fftsp_compress_static(_ptr(grad), grad.numel(), chunk_len, theta, bits, _ptr(packed),
                                        _nbytes(packed), _stream(stream)), "fftsp_compress_static")


def decompress(packed, packed_nbytes: int, grad_out, chunk_len: int, theta: float, bits: int, workspace, stream=None):
    _check(load().fftsp_decompress(_ptr(packed), packed_nbytes, _ptr(grad_out), grad_out.numel(), chunk_len, theta,
                                   bits, _ptr(workspace), _nbytes(workspace), _stream(stream)), "fftsp_decompress")


def compress_h(grad, chunk_len: int, theta: float, bits: int, scale_log2: int, packed, workspace, stream=None):
    _check(load().fftsp_compress_h(_ptr(grad), grad.numel(), chunk_len, theta, bits, scale_log2, _ptr(packed),
                                   _nbytes(packed), _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_compress_h")


def decompress_h(packed, packed_nbytes: int, grad_out, chunk_len: int, theta: float, bits: int, scale_log2: int,
                 workspace, stream=None):
    _check(load().fftsp_decompress_h(_ptr(packed), packed_nbytes, _ptr(grad_out), grad_out.numel(), chunk_len, theta,
                                     bits, scale_log2, _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_decompress_h")


def topk_kept_per_chunk(chunk_len: int, theta: float) -> int:
    k = C.c_uint32()
    _check(load().fftsp_topk_kept_per_chunk(chunk_len, theta, C.byref(k)), "fftsp_topk_kept_per_chunk")
    return k.value


def topk_packed_bytes(n: int, chunk_len: int, theta: float, bits: int) -> int:
    return load().fftsp_topk_packed_bytes(n, chunk_len, theta, bits)


def topk_workspace_bytes(n: int, chunk_len: int, bits: int) -> int:
    return load().fftsp_topk_workspace_bytes(n, chunk_len, bits)


def topk_compress(grad, chunk_len: int, theta: float, bits: int, packed, workspace, stream=None):
    _check(load().fftsp_topk_compress(_ptr(grad), grad.numel(), chunk_len, theta, bits, _ptr(packed), _nbytes(packed),
                                      _ptr(workspace), _nbytes(workspace), _stream(stream)), "fftsp_topk_compress")


def topk_decompress(packed, packed_nbytes: int, grad_out, chunk_len: int, theta: float, bits: int, workspace,
                    stream=None):
    _check(load().fftsp_topk_decompress(_ptr(packed), packed_nbytes, _ptr(grad_out), grad_out.numel(), chunk_len,
                                        theta, bits, _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_topk_decompress")


def compress_q(grad, chunk_len: int, theta: float, bits: int, packed, workspace, mantissa_bits=0, range_max=0.0,
               stream=None):
    q = Quantizer(mantissa_bits, range_max)  # kept alive until the call returns
    _check(load().fftsp_compress_q(_ptr(grad), grad.numel(), chunk_len, theta, bits, _ptr(packed), _nbytes(packed),
                                   _ptr(workspace), _nbytes(workspace), C.byref(q),
                                   _stream(stream)), "fftsp_compress_q")


def decompress_q(packed, packed_nbytes: int, grad_out, chunk_len: int, theta: float, bits: int, workspace,
                 mantissa_bits=0, stream=None):
    q = Quantizer(mantissa_bits, 0.0)  # kept alive until the call returns
    _check(load().fftsp_decompress_q(_ptr(packed), packed_nbytes, _ptr(grad_out), grad_out.numel(), chunk_len, theta,
                                     bits, _ptr(workspace), _nbytes(workspace),
                                     C.byref(q), _stream(stream)), "fftsp_decompress_q")


def encode_spectrum_q(spec, n: int, chunk_len: int, theta: float, bits: int, packed, workspace, mantissa_bits=0,
                      range_max=0.0, stream=None):
    q = Quantizer(mantissa_bits, range_max)  # kept alive until the call returns
    _check(load().fftsp_encode_spectrum_q(_ptr(spec), n, chunk_len, theta, bits, _ptr(packed), _nbytes(packed),
                                          _ptr(workspace), _nbytes(workspace),
                                          C.byref(q), _stream(stream)),
           "fftsp_encode_spectrum_q")


def decode_spectrum_q(packed, packed_nbytes: int, n: int, chunk_len: int, theta: float, bits: int, spec, workspace,
                      mantissa_bits=0, stream=None):
    q = Quantizer(mantissa_bits, 0.0)  # kept alive until the call returns
    _check(load().fftsp_decode_spectrum_q(_ptr(packed), packed_nbytes, n, chunk_len, theta, bits, _ptr(spec),
                                          _ptr(workspace), _nbytes(workspace),
                                          C.byref(q), _stream(stream)),
           "fftsp_decode_spectrum_q")


def workspace_bytes_accumulate(n: int, chunk_len: int, bits: int, npeers: int) -> int:
    return load().fftsp_workspace_bytes_accumulate(n, chunk_len, bits, npeers)


def _peer_array(packed_list):
    return (C.c_void_p * len(packed_list))(*[_ptr(p) for p in packed_list])


def decompress_accumulate(packed_list, packed_nbytes: int, scale: float, grad_out, chunk_len: int, theta: float,
                          bits: int, workspace, stream=None):
    """grad_out = scale * iFFT(sum of the peers' decoded spectra); packed_list: equally long device buffers."""
    _check(load().fftsp_decompress_accumulate(_peer_array(packed_list), len(packed_list), packed_nbytes, scale,
                                              _ptr(grad_out), grad_out.numel(), chunk_len, theta, bits,
                                              _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_decompress_accumulate")


def decode_accumulate_spectrum(packed_list, packed_nbytes: int, n: int, chunk_len: int, theta: float, bits: int, spec,
                               workspace, stream=None):
    _check(load().fftsp_decode_accumulate_spectrum(_peer_array(packed_list), len(packed_list), packed_nbytes, n,
                                                   chunk_len, theta, bits, _ptr(spec), _ptr(workspace),
                                                   _nbytes(workspace), _stream(stream)),
           "fftsp_decode_accumulate_spectrum")


def rfft(grad, chunk_len: int, spec, workspace, stream=None):
    _check(load().fftsp_rfft(_ptr(grad), grad.numel(), chunk_len, _ptr(spec), _ptr(workspace), _nbytes(workspace),
                             _stream(stream)), "fftsp_rfft")


def irfft(spec, n: int, chunk_len: int, grad_out, workspace, stream=None):
    _check(load().fftsp_irfft(_ptr(spec), n, chunk_len, _ptr(grad_out), _ptr(workspace), _nbytes(workspace),
                              _stream(stream)), "fftsp_irfft")


def encode_spectrum(spec, n: int, chunk_len: int, theta: float, bits: int, packed, workspace, stream=None):
    _check(load().fftsp_encode_spectrum(_ptr(spec), n, chunk_len, theta, bits, _ptr(packed), _nbytes(packed),
                                        _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_encode_spectrum")


def decode_spectrum(packed, packed_nbytes: int, n: int, chunk_len: int, theta: float, bits: int, spec, workspace,
                    stream=None):
    _check(load().fftsp_decode_spectrum(_ptr(packed), packed_nbytes, n, chunk_len, theta, bits, _ptr(spec),
                                        _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_decode_spectrum")


def compress_segments(grad, seg_offsets, theta: float, bits: int, packed, workspace, stream=None):
    arr, nseg = _offsets(seg_offsets)
    _check(load().fftsp_compress_segments(_ptr(grad), arr, nseg, theta, bits, _ptr(packed), _nbytes(packed),
                                          _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_compress_segments")


def decompress_segments(packed, packed_nbytes: int, grad_out, seg_offsets, theta: float, bits: int, workspace,
                        stream=None):
    arr, nseg = _offsets(seg_offsets)
    _check(load().fftsp_decompress_segments(_ptr(packed), packed_nbytes, _ptr(grad_out), arr, nseg, theta, bits,
                                            _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "fftsp_decompress_segments")


def device_status(workspace) -> int:
    st = C.c_int()
    _check(load().fftsp_device_status(_ptr(workspace), C.byref(st)), "fftsp_device_status")
    return st.value


def profile_enable(on: bool) -> None:
    _check(load().fftsp_profile_enable(1 if on else 0), "fftsp_profile_enable")


def profile_report() -> dict:
    """{kernel name: (calls, total milliseconds)} of the launches since profile_enable(True)"""
    need = load().fftsp_profile_report(None, 0)
    buf = C.create_string_buffer(need + 64)
    load().fftsp_profile_report(buf, len(buf))
    out = {}
    for line in buf.value.decode().splitlines():
        name, calls, ms = line.split()
        out[name] = (int(calls), float(ms))
    return out


def version() -> str:
    return load().fftsp_version().decode()
