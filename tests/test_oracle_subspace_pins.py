"""Pins for the oracle's Cholesky-based subspace iteration (Alg. 1 steps 6-13,
App. E): one iteration against LAPACK's Cholesky and solver, the orthonormality
identity of App. E (with and without the ridge), convergence to the leading
eigenspace at the rate the power method fixes, a diagonal closed form, and the
paper's claim that T = 5 reproduces the attention output of the full
eigendecomposition on low-rank Keys.  CPU only."""
import numpy as np
import pytest

import oracle
from rk_inputs import HeadSpec, make_keys, make_normal
from rk_inputs import stream
from rk_inputs.generator import TAG_A, TAG_Q, TAG_V

D = 128


def spd_with_spectrum(lam, seed):
    """Q diag(lam) Q^T with a seeded random orthogonal Q."""
    Q, _ = np.linalg.qr(stream(104, seed, 0, 0, TAG_A).standard_normal((lam.size, lam.size)))
    return (Q * lam) @ Q.T, Q


def v0(d, k, seed):
    return stream(104, seed, 1, 0, TAG_A).standard_normal((d, k))


def projector(V):
    Q, _ = np.linalg.qr(V)
    return Q @ Q.T


def test_one_iteration_matches_lapack():
    lam = np.linspace(5.0, 0.5, 48)
    Cq, _ = spd_with_spectrum(lam, 1)
    V0 = v0(48, 12, 1)
    got = oracle.subspace_iter(Cq, V0, T=1, eps=1e-3)
    W = Cq @ V0
    G = W.T @ W
    L = np.linalg.cholesky(G + 1e-3 * np.trace(G) / 12 * np.eye(12))
    want = np.linalg.solve(L, W.T).T                  # W L^{-T}
    assert np.abs(got - want).max() <= 1e-11 * np.abs(want).max()
    # a transposed factor (W L^{-1}) is a different matrix: the pin can tell them apart
    wrong = W @ np.linalg.inv(L)
    assert np.abs(got - wrong).max() > 1e-3


def test_orthonormal_columns_without_ridge():
    lam = np.linspace(3.0, 1.0, 64)
    Cq, _ = spd_with_spectrum(lam, 2)
    V = oracle.subspace_iter(Cq, v0(64, 16, 2), T=3, eps=0.0)
    assert np.abs(V.T @ V - np.eye(16)).max() <= 1e-11


def test_ridge_identity():
    """With the ridge, V^T V = L^{-1} G L^{-T} = I - rho L^{-1} L^{-T} (L from LAPACK):
    columns are slightly short, by exactly this amount."""
    lam = np.geomspace(100.0, 0.01, 64)
    Cq, _ = spd_with_spectrum(lam, 3)
    V0 = v0(64, 20, 3)
    eps = 1e-4
    V4 = oracle.subspace_iter(Cq, V0, T=4, eps=eps)
    V5 = oracle.subspace_iter(Cq, V0, T=5, eps=eps)
    W = Cq @ V4
    G = W.T @ W
    rho = eps * np.trace(G) / 20
    Li = np.linalg.inv(np.linalg.cholesky(G + rho * np.eye(20)))
    want = np.eye(20) - rho * Li @ Li.T
    assert np.abs(V5.T @ V5 - want).max() <= 1e-9
    assert np.abs(V5.T @ V5 - np.eye(20)).max() > 1e-6       # and the shortfall is really there


@pytest.mark.parametrize("gamma", [0.1, 0.3])
def test_converges_to_leading_eigenspace_at_power_rate(gamma):
    """Top-k eigenvalues in [1, 2], the rest <= gamma: the distance of span(V) to the
    leading eigenspace shrinks at least like gamma^T (power method)."""
    k, d = 10, 40
    lam = np.concatenate([np.linspace(2.0, 1.0, k), np.linspace(gamma, 0.01, d - k)])
    Cq, Q = spd_with_spectrum(lam, 4)
    P = Q[:, :k] @ Q[:, :k].T
    V0 = v0(d, k, 4)
    dist = [np.linalg.norm(projector(oracle.subspace_iter(Cq, V0, T=T, eps=1e-12)) - P, 2) for T in (1, 2, 3, 5, 8)]
    assert all(b < a for a, b in zip(dist, dist[1:]))
    # tan(theta_T) <= gamma^T tan(theta_0); tan(theta_0) of a Gaussian start is modest (< 50 here)
    assert dist[3] <= 50 * gamma ** 5 and dist[4] <= 50 * gamma ** 8


def test_diagonal_closed_form():
    """Cq diagonal with distinct entries and V0 whose top-k block is the identity (zeros
    below): every iterate stays in span(e_top), so V = +-e columns exactly (eps = 0)."""
    d, k = 24, 5
    rng = stream(104, 5, 0, 0, TAG_A)
    diag = rng.permutation(np.arange(1.0, d + 1))
    top = np.argsort(-diag)[:k]
    V0 = np.zeros((d, k))
    V0[top, np.arange(k)] = [2.0, -3.0, 0.5, 1.0, 7.0]
    V = oracle.subspace_iter(np.diag(diag), V0, T=5, eps=0.0)
    want = np.zeros((d, k))
    want[top, np.arange(k)] = np.sign([2.0, -3.0, 0.5, 1.0, 7.0])
    assert np.abs(V - want).max() <= 1e-12


def test_rank_deficient_without_ridge_is_reported():
    A = stream(104, 6, 0, 0, TAG_A).standard_normal((3, 16))
    Cq = A.T @ A                                    # rank 3
    with pytest.raises(RuntimeError):
        oracle.subspace_iter(Cq, v0(16, 8, 6), T=3, eps=0.0)
    V = oracle.subspace_iter(Cq, v0(16, 8, 6), T=3, eps=1e-6)   # the ridge makes it go through
    assert np.isfinite(V).all()


def test_t5_reproduces_full_eigendecomposition_attention():
    """Sec. 3.2 / App. ablation: T = 5 matches the full eigendecomposition.  On low-rank + outlier
    Keys (16 dominant directions, k = 32) both solvers keep the dominant subspace, so the attention
    outputs agree to the level of the discarded noise."""
    L, k = 600, 32
    K = make_keys(HeadSpec(L=L, mean_shift=1.0), "f32", 104, 0, 0, 7).astype(np.float64)
    V = make_normal((L, D), "f32", 104, 0, 0, 7, TAG_V).astype(np.float64)
    q = make_normal((D,), "f32", 104, 0, 0, 7, TAG_Q).astype(np.float64)
    fe = oracle.fit(K, k)
    fs = oracle.fit_subspace(K, v0(D, k, 7), T=5, eps=1e-6)
    oe = oracle.decode_head(q, oracle.compress(K, fe["Rr"]), V, fe["Rr"], fe["dmu"])
    os_ = oracle.decode_head(q, oracle.compress(K, fs["Rr"]), V, fs["Rr"], fs["dmu"])
    full = oracle.full_attn_head(q, K, V)
    err_e, err_s = np.abs(oe - full).max(), np.abs(os_ - full).max()
    assert np.abs(oe - os_).max() <= 2e-2, (np.abs(oe - os_).max(), err_e, err_s)
    # the dominant 16-dimensional subspace (the rank of the generator's signal part) is captured
    lam, U = np.linalg.eigh(fe["Cq"])
    assert lam[-16] > 100 * lam[-17]
    Ptop = U[:, -16:] @ U[:, -16:].T
    Vs = fs["Rr"]
    Ps = projector(Vs)
    assert np.linalg.norm(Ptop - Ps @ Ptop, 2) <= 1e-6
