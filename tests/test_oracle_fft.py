"""Pins for the oracle's forward / inverse real FFT (Sec. 3.1.1 DFT sum).

None of these call back into the oracle for the expected value: they use a naive
O(L^2) DFT written here, closed forms, Parseval's identity and numpy's FFT.
"""
import numpy as np
import pytest

from paper_1811_08596_amd import workloads


def naive_rdft(x, L):
    """X_j = sum_t x_t exp(-2 pi i j t / L), j = 0..L/2, straight from the definition."""
    x = np.asarray(x, dtype=np.float64)
    xp = np.zeros(L)
    xp[:x.size] = x
    j = np.arange(L // 2 + 1)[:, None]
    t = np.arange(L)[None, :]
    return (np.exp(-2j * np.pi * j * t / L) * xp[None, :]).sum(axis=1)


def naive_irdft(X, L):
    """x_t = (1/L) sum_{j<L} Xfull_j exp(+2 pi i j t / L) with the Hermitian extension."""
    X = np.asarray(X, dtype=np.complex128)
    full = np.zeros(L, dtype=np.complex128)
    full[:L // 2 + 1] = X
    full[0] = full[0].real
    full[L // 2] = full[L // 2].real
    for j in range(1, L // 2):
        full[L - j] = np.conj(full[j])
    t = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    return ((np.exp(2j * np.pi * j * t / L) * full[None, :]).sum(axis=1) / L).real


def as_complex(spec, L):
    return np.asarray(spec).reshape(-1, L + 2).view(np.complex64)


@pytest.mark.parametrize("L", [2, 4, 8, 16, 32, 64, 128, 256])
def test_forward_matches_naive_dft(ref, L):
    rng = np.random.default_rng(L)
    g = rng.standard_normal(L).astype(np.float32)
    got = as_complex(ref.rfft(g, L), L)[0]
    want = naive_rdft(g, L)
    assert np.abs(got - want).max() <= 2e-7 * np.abs(want).max()
    assert got[0].imag == 0 and got[-1].imag == 0


@pytest.mark.parametrize("n,L", [(5, 8), (100, 64), (129, 128), (300, 256), (257, 256)])
def test_forward_chunks_and_zero_padded_tail(ref, n, L):
    g = workloads.small_mixed(n, seed=n)
    got = as_complex(ref.rfft(g, L), L)
    C = (n + L - 1) // L
    assert got.shape == (C, L // 2 + 1)
    for c in range(C):
        want = naive_rdft(g[c * L:(c + 1) * L], L)
        assert np.abs(got[c] - want).max() <= 2e-7 * max(np.abs(want).max(), 1e-30)


@pytest.mark.parametrize("L", [2, 8, 64, 256])
def test_inverse_matches_naive_inverse(ref, L):
    rng = np.random.default_rng(100 + L)
    X = (rng.standard_normal(L // 2 + 1) + 1j * rng.standard_normal(L // 2 + 1)).astype(np.complex64)
    spec = X.view(np.float32).copy()
    got = ref.irfft(spec, L, L)
    want = naive_irdft(X, L)          # ignores imag of bins 0 and L/2, as the oracle must
    assert np.abs(got - want).max() <= 2e-7 * np.abs(want).max()


def test_inverse_writes_only_first_n(ref):
    L, n = 64, 100
    X = np.zeros((2, L // 2 + 1), dtype=np.complex64)
    X[:, 3] = 1 + 2j
    out = ref.irfft(X.view(np.float32).ravel(), n, L)
    assert out.size == n
    want = naive_irdft(X[0], L)
    assert np.allclose(out[:L], want, atol=1e-7)
    assert np.allclose(out[L:], want[:n - L], atol=1e-7)


@pytest.mark.parametrize("L", [8, 64, 1024])
def test_closed_forms(ref, L):
    B = L // 2 + 1
    # impulse at 0 -> every bin is exactly 1
    d = np.zeros(L, np.float32)
    d[0] = 1
    X = as_complex(ref.rfft(d, L), L)[0]
    assert np.all(X == 1 + 0j)
    # impulse at 1 -> exp(-2 pi i j / L): catches a wrong sign of the exponent
    d = np.zeros(L, np.float32)
    d[1] = 1
    X = as_complex(ref.rfft(d, L), L)[0]
    j = np.arange(B)
    assert np.abs(X - np.exp(-2j * np.pi * j / L)).max() < 1e-7
    assert X[1].imag < 0
    # constant -> only DC = L*c
    X = as_complex(ref.rfft(np.full(L, 0.5, np.float32), L), L)[0]
    assert X[0] == L * 0.5 and np.abs(X[1:]).max() < 1e-6 * L
    # cosine at bin j0 -> L/2 there, zero elsewhere;  sine -> -i L/2
    j0 = 3 if L > 8 else 1
    t = np.arange(L)
    X = as_complex(ref.rfft(np.cos(2 * np.pi * j0 * t / L).astype(np.float32), L), L)[0]
    assert abs(X[j0] - L / 2) < 1e-5 * L and np.abs(np.delete(X, j0)).max() < 1e-5 * L
    X = as_complex(ref.rfft(np.sin(2 * np.pi * j0 * t / L).astype(np.float32), L), L)[0]
    assert abs(X[j0] - (-0.5j * L)) < 1e-5 * L
    # alternating +-1 -> only Nyquist = L
    X = as_complex(ref.rfft(((-1.0) ** t).astype(np.float32), L), L)[0]
    assert X[-1] == L and np.abs(X[:-1]).max() < 1e-6 * L


def test_linearity_and_parseval(ref):
    L = 512
    rng = np.random.default_rng(5)
    a = rng.standard_normal(L).astype(np.float32)
    b = rng.standard_normal(L).astype(np.float32)
    A, Bq = as_complex(ref.rfft(a, L), L)[0], as_complex(ref.rfft(b, L), L)[0]
    S = as_complex(ref.rfft((2 * a + b).astype(np.float32), L), L)[0]
    assert np.abs(S - (2 * A + Bq)).max() < 5e-6 * np.abs(S).max()
    # Parseval for the half spectrum
    e_time = float((a.astype(np.float64) ** 2).sum())
    p = np.abs(A.astype(np.complex128)) ** 2
    e_freq = (p[0] + 2 * p[1:-1].sum() + p[-1]) / L
    assert abs(e_time - e_freq) < 1e-6 * e_time


@pytest.mark.parametrize("L", [256, 4096, 1 << 16])
def test_matches_numpy_fft_in_float64(ref, L):
    """Library special case (a cross-check, not the definition)."""
    g = workloads.small_mixed(3 * L - 17, seed=L)
    got = as_complex(ref.rfft(g, L), L).astype(np.complex128)
    x = np.zeros(3 * L)
    x[:g.size] = g
    want = np.fft.rfft(x.reshape(3, L), axis=1)
    # the oracle rounds each component once to binary32
    assert np.abs(got - want).max() <= 1.2e-7 * np.abs(want).max()
    back = ref.irfft(want.astype(np.complex64).view(np.float32).ravel(), g.size, L)
    assert np.linalg.norm(back - g) <= 2e-7 * np.linalg.norm(g)


def test_round_trip_identity(ref):
    """iFFT(FFT(g)) = g (spec invariant), through the spectrum rounded to binary32."""
    for L in (32, 1024, 1 << 14):
        g = workloads.small_mixed(2 * L + 11, seed=3)
        back = ref.irfft(ref.rfft(g, L), g.size, L)
        assert np.linalg.norm(back.astype(np.float64) - g) <= 1e-6 * np.linalg.norm(g)


def test_bad_arguments(ref):
    g = np.ones(8, np.float32)
    for L in (0, 1, 3, 12):
        with pytest.raises(ref.OracleError):
            ref.rfft(g, L)
