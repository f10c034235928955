"""Pins for the oracle's query-window weights (Alg. 1 step 4, Sec. 3.2 "Query-Weighted
PCA"): sigma_j = ||(Q_W)_{:,j}||_2, checked against numpy's norm, closed forms, and the
effect the paper motivates it with (channels with large query magnitude are kept
preferentially).  CPU only."""
import numpy as np

import oracle
from rk_inputs import make_normal, stream
from rk_inputs.generator import TAG_A, TAG_Q

D = 128


def test_matches_numpy_norm_and_gqa_pooling():
    Qw = np.stack([make_normal((32, D), "f32", 105, 0, 0, g, TAG_Q) for g in range(7)]).astype(np.float64)
    got = oracle.sigma_window(Qw)                              # [G, W, d]: pooled over the group
    assert np.abs(got - np.linalg.norm(Qw.reshape(-1, D), axis=0)).max() <= 1e-12
    one = oracle.sigma_window(Qw[0])                           # G = 1: the paper's formula as printed
    assert np.abs(one - np.sqrt((Qw[0] ** 2).sum(axis=0))).max() <= 1e-12
    # pooling = root of the sum of the per-head squares
    per_head = np.stack([oracle.sigma_window(Qw[g]) for g in range(7)])
    assert np.abs(got - np.sqrt((per_head ** 2).sum(axis=0))).max() <= 1e-12


def test_closed_forms():
    Qw = np.zeros((32, D))
    Qw[5, 3] = -4.0
    Qw[9, 3] = 3.0
    Qw[:, 7] = 0.5
    s = oracle.sigma_window(Qw)
    assert s[3] == 5.0 and abs(s[7] - 0.5 * np.sqrt(32)) <= 1e-15 and s[0] == 0.0
    assert np.abs(oracle.sigma_window(-2.0 * Qw) - 2.0 * s).max() <= 1e-15     # |.|-homogeneous


def test_query_aware_fit_prefers_channels_the_queries_use():
    """Keys with equal variance on two groups of 8 coordinates; queries that only use the second
    group.  Plain PCA cannot tell the groups apart; with sigma from the query window the kept
    subspace is the second group (Sec. 3.2: weight each Key channel by the query magnitude)."""
    rng = stream(105, 1, 0, 0, TAG_A)
    K = np.zeros((400, D))
    K[:, :16] = rng.standard_normal((400, 16))
    K[:, 16:] = 0.01 * rng.standard_normal((400, D - 16))
    Qw = np.zeros((32, D))
    Qw[:, 8:16] = rng.standard_normal((32, 8)) * 3.0
    Qw[:, :8] = rng.standard_normal((32, 8)) * 0.1
    Qw[:, 16:] = rng.standard_normal((32, D - 16)) * 0.1
    sigma = oracle.sigma_window(Qw)
    f = oracle.fit(K, 8, sigma=sigma)
    P = f["Rr"] @ f["Rr"].T
    assert np.trace(P[8:16, 8:16]) >= 7.99 and np.trace(P[:8, :8]) <= 0.01
    f0 = oracle.fit(K, 8)                                       # query-agnostic: a mix of both groups
    P0 = f0["Rr"] @ f0["Rr"].T
    assert 1.0 <= np.trace(P0[8:16, 8:16]) <= 7.0
