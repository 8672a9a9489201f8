"""When does compressing pay?  Host arithmetic of arXiv 1811.08596, Sec. 3.3 (Eq. 1-4).

For a message of M bytes, compressing costs  M * (2/T_m + 1/T_f + 1/T_p + 1/T_s)  (Eq. 1: precision conversions,
FFT, packing, top-k selection, each as a throughput in bytes of gradient per second), decompressing the same again,
and the wire time drops from M / T_comm to M / (k * T_comm) for an overall compression ratio k (Eq. 2, 3).
Compression is a net win iff twice the codec cost is below the wire time saved, i.e. (Eq. 4)

    k  >  1 / (1 - 2 * T_comm * (2/T_m + 1/T_f + 1/T_p + 1/T_s)),

and never if the denominator is not positive: then the codec alone takes longer than sending the raw message.
All throughputs in the same unit (here GB/s of fp32 gradient).
"""
from __future__ import annotations

import math


def codec_seconds_per_byte(T_m: float, T_f: float, T_p: float, T_s: float) -> float:
    """Eq. 1 divided by M: seconds of one direction of the codec per byte of gradient."""
    return 2.0 / T_m + 1.0 / T_f + 1.0 / T_p + 1.0 / T_s


def min_useful_ratio(T_comm: float, T_m: float, T_f: float, T_p: float, T_s: float) -> float:
    """Eq. 4: smallest compression ratio that pays on a link of throughput T_comm; math.inf if none does."""
    return min_useful_ratio_measured(T_comm, 1.0 / codec_seconds_per_byte(T_m, T_f, T_p, T_s),
                                     1.0 / codec_seconds_per_byte(T_m, T_f, T_p, T_s))


def min_useful_ratio_measured(T_comm: float, T_compress: float, T_decompress: float) -> float:
    """Eq. 4 with the two codec directions measured as wholes (the paper's 2 * cost_comp is their sum)."""
    slack = 1.0 - T_comm * (1.0 / T_compress + 1.0 / T_decompress)
    return 1.0 / slack if slack > 0.0 else math.inf


def break_even_link(T_compress: float, T_decompress: float) -> float:
    """Link throughput at and above which no ratio pays (the denominator of Eq. 4 reaches zero)."""
    return 1.0 / (1.0 / T_compress + 1.0 / T_decompress)
