"""Host-side PCA entry point (no GPU needed): the library's eigen-solver
against the oracle's eigen-decomposition (numpy's LAPACK routine)."""
import numpy as np
import pytest

import paper_2508_15881_amd as tp
from paper_2508_15881_amd import workloads as wl
from oracle import tpla_oracle as orc


@pytest.mark.parametrize("d,g", [(8, 2), (64, 2), (128, 4), (96, 3)])
def test_pca_basis_matches_oracle(d, g):
    F = wl.draw_anisotropic_latents(d, 5 * d, d).astype(np.float64)
    s, G = orc.latent_moments(F)
    U, eig, frac = tp.tpla_pca_basis(d, g, F.shape[0], s, G)
    U_ref, lam = orc.pca_U(F)
    assert np.all(np.diff(eig) <= 0)                                   # descending
    assert np.max(np.abs(eig - lam)) <= 1e-12 * lam[0]
    U64 = U.astype(np.float64)
    assert np.max(np.abs(U64.T @ U64 - np.eye(d))) <= 1e-6            # orthonormal to float rounding
    # eigenvectors are unique up to sign (the spectrum is simple): columns line up
    assert np.min(np.abs(np.sum(U64 * U_ref, axis=0))) >= 1.0 - 1e-6
    # stated sign convention: the largest component of every column is positive
    assert np.all(U64[np.argmax(np.abs(U64), axis=0), np.arange(d)] > 0)
    assert np.allclose(frac, orc.variance_fractions(lam, g), rtol=1e-12)
    assert abs(frac.sum() - 1.0) <= 1e-12


def test_pca_basis_full_width_and_repeated_eigenvalues():
    # the width of the benchmark configurations, in well under a second ...
    import time
    d = 512
    F = wl.draw_anisotropic_latents(3, 4 * d, d).astype(np.float64)
    s, G = orc.latent_moments(F)
    t0 = time.perf_counter()
    U, eig, frac = tp.tpla_pca_basis(d, 2, F.shape[0], s, G)
    dt = time.perf_counter() - t0
    _, lam = orc.pca_U(F)
    assert np.max(np.abs(eig - lam)) <= 1e-12 * lam[0]
    U64 = U.astype(np.float64)
    assert np.max(np.abs(U64.T @ U64 - np.eye(d))) <= 1e-5
    cov = np.cov(F.T, bias=True)
    assert np.max(np.abs(U64.T @ cov @ U64 - np.diag(eig))) <= 1e-5 * lam[0]
    assert dt < 5.0
    # ... and a spectrum with repeated values: the eigenvectors are no longer unique, the
    # decomposition still is one (orthonormal U, U^T C U diagonal, the right values)
    rng = np.random.default_rng(8)
    q, _ = np.linalg.qr(rng.standard_normal((48, 48)))
    vals = np.repeat([5.0, 2.0, 2.0, 0.5], 12)
    C = (q * vals) @ q.T
    n = 1000
    U, eig, frac = tp.tpla_pca_basis(48, 4, n, np.zeros(48), C * n)
    assert np.allclose(eig, np.sort(vals)[::-1], atol=1e-12)
    U64 = U.astype(np.float64)
    assert np.max(np.abs(U64.T @ U64 - np.eye(48))) <= 1e-6
    assert np.max(np.abs(U64.T @ C @ U64 - np.diag(eig))) <= 1e-5
    assert np.allclose(frac, [60 / 114, 24 / 114, 24 / 114, 6 / 114])


def test_pca_basis_diagonal_input_is_a_sorting_permutation():
    # a diagonal covariance needs no rotation: U is the permutation that sorts the variances
    var = np.array([0.5, 4.0, 1.0, 9.0])
    n = 10
    U, eig, frac = tp.tpla_pca_basis(4, 2, n, np.zeros(4), np.diag(var) * n)
    assert np.array_equal(eig, [9.0, 4.0, 1.0, 0.5])
    assert np.array_equal(U, np.eye(4, dtype=np.float32)[:, [3, 1, 2, 0]])
    assert np.allclose(frac, [13.0 / 14.5, 1.5 / 14.5])


def test_pca_basis_rejects_bad_arguments():
    z, Z = np.zeros(4), np.eye(4)
    for d, g, n in ((4, 3, 10), (4, 2, 0), (4, 9, 10)):
        with pytest.raises(tp.TplaError) as e:
            tp.tpla_pca_basis(d, g, n, z, Z)
        assert e.value.code == -2
    lib = tp.load_library()
    assert lib.tpla_pca_basis(0, 1, 10, z.ctypes.data, Z.ctypes.data, z.ctypes.data, z.ctypes.data, z.ctypes.data) == -2
    assert lib.tpla_pca_basis(4, 2, 10, None, Z.ctypes.data, z.ctypes.data, z.ctypes.data, z.ctypes.data) == -1
