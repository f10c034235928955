"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- identities the paper states (Eq. 1-4, Alg. 1-2), closed
forms, LAPACK on special cases, and brute force on tiny heads.  CPU only."""
import itertools
import os

import numpy as np
import pytest

import oracle
from rk_inputs import HeadSpec, make_keys, make_normal, bf16_round
from rk_inputs import stream
from rk_inputs.generator import TAG_A, TAG_B, TAG_Q, TAG_V, TAG_SIGMA

D = 128


def keys(L=512, seed_h=0, **kw):
    return make_keys(HeadSpec(L=L, **kw), "f32", 101, 0, 0, seed_h).astype(np.float64)


def exact_low_rank(L, rho, h, outliers=2, offset=0.0):
    """fp64 product of seeded factors: exactly rank rho (the fp32 generator
    rounds the product, which leaves it low-rank only to 1e-7)."""
    A = stream(101, 0, 0, h, TAG_A).standard_normal((L, rho))
    Bm = stream(101, 0, 0, h, TAG_B).standard_normal((rho, D))
    Bm[:, :outliers] *= 10.0
    return A @ Bm + offset


def normal(shape, tag, h=0):
    return make_normal(shape, "f32", 101, 0, 0, h, tag).astype(np.float64)


@pytest.fixture(scope="module")
def head():
    K = keys(L=512, mean_shift=3.0)
    V = normal((512, D), TAG_V)
    q = normal((D,), TAG_Q)
    return K, V, q


# ---- P1: R^T R = R R^T = I (Sec. 3.1 "Rotation Matrix") --------------------
def test_p1_orthogonality(head):
    K, _, _ = head
    f = oracle.fit(K, 32)
    R = f["R"]
    assert np.abs(R.T @ R - np.eye(D)).max() <= 1e-12
    assert np.abs(R @ R.T - np.eye(D)).max() <= 1e-12


# ---- P2: r = d reproduces exact full attention (Eq. 1), delta_mu = 0 --------
def test_p2_full_rank_is_lossless(head):
    K, V, q = head
    f = oracle.fit(K, D)
    Kt = oracle.compress(K, f["Rr"])
    out = oracle.decode_head(q, Kt, V, f["Rr"], f["dmu"])
    ref = oracle.full_attn_head(q, K, V)
    assert np.abs(out - ref).max() <= 1e-12
    assert np.abs(f["dmu"]).max() <= 1e-12 * max(1.0, np.abs(f["mu"]).max())
    # and the reference attention itself against a direct numpy softmax
    s = (K @ q) / np.sqrt(D)
    p = np.exp(s - s.max()); p /= p.sum()
    assert np.abs(ref - p @ V).max() <= 1e-12


# ---- P3: rotated-truncated scores = q P_r K^T, residual = q (I-P_r) K^T (Eq. 2-3)
def test_p3_projector_identities(head):
    K, _, q = head
    for r in (8, 32, 64):
        f = oracle.fit(K, r)
        Rr = f["Rr"]
        Kt = oracle.compress(K, Rr)                 # unrounded
        qt = q @ Rr                                  # numpy route
        P = Rr @ Rr.T
        scores = Kt @ qt
        assert np.abs(scores - K @ (P @ q)).max() <= 1e-10 * np.abs(K @ q).max()
        resid = K @ q - scores
        assert np.abs(resid - K @ ((np.eye(D) - P) @ q)).max() <= 1e-10 * np.abs(K @ q).max()
        assert np.abs(Rr.T @ Rr - np.eye(r)).max() <= 1e-12     # R_k^T R_k = I_k


# ---- P4: eigenvalue ordering, PSD, trace, eigen-equation ---------------------
def test_p4_spectrum(head):
    K, _, _ = head
    sigma = np.abs(normal((D,), TAG_SIGMA)) + 0.1
    f = oracle.fit(K, 32, sigma=sigma)
    lam, R, Cq = f["lam"], f["R"], f["Cq"]
    assert np.all(np.diff(lam) <= 0)
    assert lam.min() >= -1e-10 * lam[0]
    assert abs(lam.sum() - np.trace(Cq)) <= 1e-10 * np.trace(Cq)
    assert np.abs(Cq @ R - R * lam[None, :]).max() <= 1e-11 * lam[0]
    assert np.array_equal(f["keep_idx"], np.arange(32))
    assert np.array_equal(f["mask"], (np.arange(D) < 32).astype(np.uint8))


# ---- P5: LAPACK cross-check; covariance against numpy.cov --------------------
def test_p5_lapack_and_cov(head):
    K, _, _ = head
    mu, Cm = oracle.mean_scatter(K)
    assert np.abs(mu - K.mean(axis=0)).max() <= 1e-12
    ref = np.cov(K, rowvar=False) * (K.shape[0] - 1)
    assert np.abs(Cm - ref).max() <= 1e-10 * np.abs(ref).max()
    # uncentered flag = literal K^T K
    _, C0 = oracle.mean_scatter(K, center=False)
    assert np.abs(C0 - K.T @ K).max() <= 1e-10 * np.abs(C0).max()
    # eigenvalues of the generator's (nearly degenerate bulk) covariance
    R, lam, _ = oracle.jacobi_eigh(Cm)
    w = np.linalg.eigvalsh(Cm)[::-1]
    assert np.abs(lam - w).max() <= 1e-12 * w[0]
    # eigenvectors on a well-separated spectrum: |R^T U| = I
    rng = np.random.default_rng(5)
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    A = (Q * np.linspace(1.0, 200.0, D)[None, :]) @ Q.T
    R, lam, _ = oracle.jacobi_eigh(A)
    w, U = np.linalg.eigh(A)
    U = U[:, ::-1]
    assert np.abs(lam - w[::-1]).max() <= 1e-11
    assert np.abs(np.abs(R.T @ U) - np.eye(D)).max() <= 1e-9
    # sign canonicalisation: largest-magnitude entry of each column positive
    assert np.all(R[np.abs(R).argmax(axis=0), np.arange(D)] > 0)


# ---- P6: Eckart-Young closed form --------------------------------------------
def test_p6_eckart_young(head):
    K, _, _ = head
    for r in (4, 18, 32, 100):
        f = oracle.fit(K, r)
        Kc = K - f["mu"][None, :]
        P = f["Rr"] @ f["Rr"].T
        err = np.linalg.norm(Kc - Kc @ P, "fro") ** 2
        tail = f["lam"][r:].sum()
        assert abs(err - tail) <= 1e-9 * f["lam"].sum()


# ---- P7: with every token on the sparse path the bias is a constant shift ----
def test_p7_bias_is_constant_shift(head):
    K, V, q = head
    f = oracle.fit(K, 32)
    assert np.abs(f["dmu"]).max() > 1e-3          # the bias is really there
    Kt = oracle.compress(K, f["Rr"], rounding="bf16")
    a, lse_a = oracle.decode_head(q, Kt, V, f["Rr"], f["dmu"], return_lse=True)
    b, lse_b = oracle.decode_head(q, Kt, V, f["Rr"], None, return_lse=True)
    assert np.abs(a - b).max() <= 1e-12
    # ... but the max score moves by exactly q.dmu / sqrt(d)
    assert abs((lse_a[0] - lse_b[0]) - (q @ f["dmu"]) / np.sqrt(D)) <= 1e-10
    # delta_mu = (I - P) mu, and R_k^T delta_mu = 0
    P = f["Rr"] @ f["Rr"].T
    assert np.abs(f["dmu"] - (np.eye(D) - P) @ f["mu"]).max() <= 1e-12 * np.abs(f["mu"]).max()
    assert np.abs(f["Rr"].T @ f["dmu"]).max() <= 1e-12 * np.abs(f["mu"]).max()


# ---- P8: exactly low-rank Keys: pruning at r >= rank is lossless -------------
@pytest.mark.parametrize("center", [True, False])
def test_p8_low_rank_exact(center):
    rho = 6
    K = exact_low_rank(300, rho, 1)
    V = normal((300, D), TAG_V, 1)
    q = normal((D,), TAG_Q, 1)
    f = oracle.fit(K, rho, center=center)
    Kt = oracle.compress(K, f["Rr"])
    out = oracle.decode_head(q, Kt, V, f["Rr"], f["dmu"])
    ref = oracle.full_attn_head(q, K, V)
    assert np.abs(out - ref).max() <= 1e-9
    assert np.abs(f["dmu"]).max() <= 1e-9 * np.abs(K).max()


def test_p8_offset_pins_bias_value():
    """K = A Bm + 1 c^T with a centered fit: (I-P)K_n = (I-P)c = delta_mu for
    every n, so the biased scores q~.K~_n + q.dmu equal q.K_n exactly."""
    rho = 6
    K = exact_low_rank(300, rho, 2, outliers=0, offset=2.5)
    q = normal((D,), TAG_Q, 2)
    f = oracle.fit(K, rho, center=True)
    assert np.abs(f["dmu"]).max() > 0.1
    Kt = oracle.compress(K, f["Rr"])
    V = np.eye(300, D)                      # V = identity rows: output = softmax weights
    out, lse = oracle.decode_head(q, Kt, V, f["Rr"], f["dmu"], return_lse=True)
    s = (K @ q) / np.sqrt(D)
    assert abs(lse[0] - s.max()) <= 1e-9     # max of the biased scores = max of exact scores
    p = np.exp(s - s.max()); p /= p.sum()
    assert np.abs(out - p[:D]).max() <= 1e-10
    # without the bias the max differs by q.dmu/sqrt(d)
    _, lse0 = oracle.decode_head(q, Kt, V, f["Rr"], None, return_lse=True)
    assert abs(lse0[0] - s.max()) > 1e-3


# ---- P9: diagonal covariance: R is a signed permutation, kept set = argsort --
def test_p9_diagonal_covariance():
    rng = np.random.default_rng(9)
    N = 400
    M = np.concatenate([np.ones((N, 1)), rng.standard_normal((N, D))], axis=1)
    Q, _ = np.linalg.qr(M)
    Q = Q[:, 1:]                                    # orthonormal columns, each orthogonal to 1
    s = rng.permutation(np.linspace(1.0, 50.0, D))
    K = Q * s[None, :]
    sigma = rng.permutation(np.linspace(0.5, 3.0, D))
    for sg in (None, sigma):
        w = s ** 2 if sg is None else (sg * s) ** 2
        f = oracle.fit(K, 20, sigma=sg)
        Rabs = np.abs(f["R"])
        assert np.abs(Rabs.sum(axis=0) - 1).max() <= 1e-8 and np.abs(Rabs.max(axis=0) - 1).max() <= 1e-8
        kept_channels = np.sort(Rabs[:, :20].argmax(axis=0))
        assert np.array_equal(kept_channels, np.sort(np.argsort(-w)[:20]))
        assert np.abs(f["lam"] - np.sort(w)[::-1]).max() <= 1e-9 * w.max()


# ---- P10: brute force on tiny heads; 2x2 closed form --------------------------
def _captured(Cq, F):
    return np.trace(F.T @ Cq @ F)


@pytest.mark.parametrize("d,r", [(4, 1), (4, 2), (8, 3)])
def test_p10_brute_force_tiny(d, r):
    rng = np.random.default_rng(100 + d + r)
    K = rng.standard_normal((40, d)) @ np.diag(rng.uniform(0.2, 3.0, d)) @ rng.standard_normal((d, d))
    f = oracle.fit(K, r)
    best = _captured(f["Cq"], f["Rr"])
    for sub in itertools.combinations(range(d), r):
        assert best >= _captured(f["Cq"], np.eye(d)[:, list(sub)]) - 1e-10
    for _ in range(20000):
        F, _ = np.linalg.qr(rng.standard_normal((d, r)))
        assert best >= _captured(f["Cq"], F) - 1e-10
    assert abs(best - f["lam"][:r].sum()) <= 1e-10 * f["lam"].sum()


def test_p10_two_by_two_closed_form():
    a, b, c = 3.0, 1.25, -0.5
    R, lam, _ = oracle.jacobi_eigh(np.array([[a, b], [b, c]]))
    disc = np.sqrt((a - c) ** 2 / 4 + b * b)
    assert np.allclose(lam, [(a + c) / 2 + disc, (a + c) / 2 - disc], rtol=0, atol=1e-14)
    v = np.array([b, lam[0] - a]); v /= np.linalg.norm(v)
    assert abs(abs(R[:, 0] @ v) - 1) <= 1e-14


# ---- P11: split into chunks + online-softmax merge = one-pass softmax (App. C.3)
def test_p11_split_merge(head):
    K, V, q = head
    f = oracle.fit(K, 32)
    Kt = oracle.compress(K, f["Rr"], rounding="bf16")
    whole = oracle.decode_head(q, Kt, V, f["Rr"], f["dmu"])
    bounds = [0, 7, 64, 200, 201, 512]
    parts = [oracle.decode_head(q, Kt[a:b], V[a:b], f["Rr"], f["dmu"], return_lse=True)
             for a, b in zip(bounds[:-1], bounds[1:])]
    M = max(l[0] for _, l in parts)
    den = sum(l[1] * np.exp(l[0] - M) for _, l in parts)
    num = sum(o * l[1] * np.exp(l[0] - M) for o, l in parts)
    assert np.abs(num / den - whole).max() <= 1e-12
    # empty cache -> zeros
    z = oracle.decode_head(q, Kt[:0], V[:0], f["Rr"], f["dmu"])
    assert np.array_equal(z, np.zeros(D))


# ---- P12: Eq. 4 both routes ---------------------------------------------------
def test_p12_reweighting_routes(head):
    K, _, _ = head
    sigma = np.abs(normal((D,), TAG_SIGMA, 3)) + 0.05
    mu, Cm = oracle.mean_scatter(K)
    Cq = oracle.weight(Cm, sigma)
    route_a = np.diag(sigma) @ Cm @ np.diag(sigma)
    route_b = np.outer(sigma, sigma) * Cm
    Kq = (K - K.mean(axis=0)[None, :]) * sigma[None, :]
    route_c = Kq.T @ Kq
    for ref in (route_a, route_b, route_c):
        assert np.abs(Cq - ref).max() <= 1e-10 * np.abs(ref).max()
    assert np.array_equal(oracle.weight(Cm, None), Cm)


# ---- selection semantics -------------------------------------------------------
def test_select_any_order_and_ties():
    lam = np.array([3.0, 7.0, 3.0, -1.0, 7.0, 0.5])
    mask, keep = oracle.select(lam, 3)
    assert keep.tolist() == [1, 4, 0]               # ties -> lower column first
    assert mask.tolist() == [1, 1, 0, 0, 1, 0]
    rng = np.random.default_rng(3)
    lam = rng.standard_normal(D)
    lam[10] = lam[90]
    for r in (1, 32, 127, 128):
        mask, keep = oracle.select(lam, r)
        ref = np.argsort(-lam, kind="stable")[:r]
        assert np.array_equal(keep, ref)
        assert mask.sum() == r and np.all(mask[ref] == 1)


def test_gather_and_token_list(head):
    K, _, _ = head
    f = oracle.fit(K, 16)
    keep = np.array([5, 0, 9], np.int32)
    assert np.array_equal(oracle.gather_rotation(f["R"], keep), f["R"][:, keep])
    tok = np.array([3, 1, 400, 7], np.int32)
    assert np.array_equal(oracle.compress(K, f["Rr"], tok=tok), oracle.compress(K[tok], f["Rr"]))
    mu_t, C_t = oracle.mean_scatter(K, tok=tok)
    mu_g, C_g = oracle.mean_scatter(K[tok])
    assert np.array_equal(mu_t, mu_g) and np.array_equal(C_t, C_g)
    # compress against a numpy matmul
    assert np.abs(oracle.compress(K, f["Rr"]) - K @ f["Rr"]).max() <= 1e-11 * np.abs(K).max()


# ---- storage rounding -----------------------------------------------------------
def test_bf16_rounding_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "bf16_rounding.txt")
    n = 0
    for line in open(path):
        line = line.split("#")[0].split()
        if len(line) != 2:
            continue
        x, want = float.fromhex(line[0]), float.fromhex(line[1])
        assert oracle.round_bf16(np.array([x]))[0] == want, line
        n += 1
    assert n >= 12


def test_bf16_rounding_vs_bit_trick():
    """On fp32-exact inputs the oracle's frexp/nearbyint rounding must agree
    with the generator's independent integer bit manipulation."""
    rng = np.random.default_rng(11)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    got = oracle.round_bf16(x.astype(np.float64))
    assert np.array_equal(got, bf16_round(x).astype(np.float64))
    Kt = oracle.compress(x[:256].reshape(2, 128).astype(np.float64), np.eye(128), rounding="bf16")
    assert np.array_equal(Kt, bf16_round(x[:256]).reshape(2, 128).astype(np.float64))


# ---- batched drivers = the single-head functions, GQA head mapping --------------
def test_batched_drivers_match_single_head():
    B, Hq, Hkv, L, r = 2, 6, 2, 96, 16
    rng = np.random.default_rng(21)
    K = np.stack([keys(L=L, seed_h=10 + u) for u in range(B * Hkv)])
    V = rng.standard_normal((B, Hkv, L, D))
    q = rng.standard_normal((B, Hq, D))
    lens = np.array([96, 50], np.int32)
    fb = oracle.fit_batch(K, r, lens=np.repeat(lens, Hkv))
    for u in range(B * Hkv):
        f = oracle.fit(K[u, :lens[u // Hkv]], r)
        for k in ("mu", "C", "R", "lam", "mask", "keep_idx", "Rr", "dmu"):
            assert np.array_equal(fb[k][u], f[k]), k
    Kt = oracle.compress_batch(K, fb["Rr"], rounding="bf16", lens=np.repeat(lens, Hkv))
    Kt4 = Kt.reshape(B, Hkv, L, r)
    out = oracle.decode_batch(q, Kt4, V, fb["Rr"].reshape(B, Hkv, D, r), fb["dmu"].reshape(B, Hkv, D), lens=lens)
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            u = b * Hkv + h // G
            ref = oracle.decode_head(q[b, h], Kt[u, :lens[b]], V[b, h // G, :lens[b]], fb["Rr"][u], fb["dmu"][u])
            assert np.array_equal(out[b, h], ref)


def test_planted_mistakes_are_caught(head):
    """Sanity of the pins themselves: typical slips (transposed rotation, wrong
    softmax scale, missing centering) move the results far beyond tolerance."""
    K, V, q = head
    f = oracle.fit(K, 32)
    Kt = oracle.compress(K, f["Rr"])
    good = oracle.decode_head(q, Kt, V, f["Rr"], f["dmu"])
    wrong_scale = oracle.decode_head(q, Kt, V, f["Rr"], f["dmu"], scale=1 / np.sqrt(32))
    assert np.abs(good - wrong_scale).max() > 1e-3
    f0 = oracle.fit(K, 32, center=False)
    assert np.abs(f0["C"] - f["C"]).max() > 1e-3 * np.abs(f["C"]).max()
