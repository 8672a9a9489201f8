"""MI355X-native FFT-sparsifying gradient codec (arXiv 1811.08596, Sec. 3).

`fftsp` is the thin ctypes binding over the C-ABI library built from csrc/;
`workloads` holds the seeded synthetic gradients.  Nothing is loaded at import.
"""
__all__ = ["fftsp", "workloads"]
