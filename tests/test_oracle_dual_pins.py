"""Pins for the oracle's dual-path decode (Alg. 2 steps 1-6: rotated visual
segment with the mean-correction bias, unrotated prompt/text segment, one softmax
over the concatenation).  Checked against plain full attention in the cases where
the two must agree exactly, against a numpy softmax written out here, and against
the single-path oracle where the dual path degenerates to it.  CPU only."""
import numpy as np
import pytest

import oracle
from rk_inputs import make_normal
from rk_inputs import stream
from rk_inputs.generator import TAG_A, TAG_B, TAG_Q, TAG_V

D = 128


def normal(shape, tag, h=0):
    return make_normal(shape, "f32", 103, 0, 0, h, tag).astype(np.float64)


def low_rank_offset(L, rho, h, offset):
    A = stream(103, 0, 0, h, TAG_A).standard_normal((L, rho))
    Bm = stream(103, 0, 0, h, TAG_B).standard_normal((rho, D))
    return A @ Bm + offset


def softmax_attn(scores, V):
    p = np.exp(scores - scores.max())
    p /= p.sum()
    return p @ V


@pytest.fixture(scope="module")
def case():
    """Visual Keys that are exactly rank 6 plus a constant offset, fitted with r = 6
    and centering: the biased rotated scores then equal the exact q.K_n (Sec. 3.2
    mean residual), so the dual path must equal full attention over [K_vis; K_pt]."""
    N, M, rho = 300, 37, 6
    K = low_rank_offset(N, rho, 3, offset=2.5)
    V = normal((N, D), TAG_V, 3)
    Kpt = 1.5 * normal((M, D), TAG_A, 4)            # unrelated full-rank text Keys
    Vpt = normal((M, D), TAG_V, 4)
    q = normal((D,), TAG_Q, 3)
    f = oracle.fit(K, rho, center=True)
    Kt = oracle.compress(K, f["Rr"])
    return dict(K=K, V=V, Kpt=Kpt, Vpt=Vpt, q=q, f=f, Kt=Kt)


def test_dual_equals_full_attention_over_concatenation(case):
    c = case
    out = oracle.decode_dual_head(c["q"], c["Kt"], c["V"], c["Kpt"], c["Vpt"], c["f"]["Rr"], c["f"]["dmu"])
    ref = oracle.full_attn_head(c["q"], np.vstack([c["K"], c["Kpt"]]), np.vstack([c["V"], c["Vpt"]]))
    assert np.abs(out - ref).max() <= 1e-9
    # the same thing from a numpy softmax over exact scores, independent of the oracle's C code
    s = np.concatenate([c["K"] @ c["q"], c["Kpt"] @ c["q"]]) / np.sqrt(D)
    assert np.abs(out - softmax_attn(s, np.vstack([c["V"], c["Vpt"]]))).max() <= 1e-9


def test_bias_now_matters(case):
    """In the dual path the bias shifts only the visual scores, so leaving it out
    (or putting it on the text scores instead) changes the output."""
    c = case
    assert np.abs(c["f"]["dmu"]).max() > 0.1
    ref = oracle.full_attn_head(c["q"], np.vstack([c["K"], c["Kpt"]]), np.vstack([c["V"], c["Vpt"]]))
    nob = oracle.decode_dual_head(c["q"], c["Kt"], c["V"], c["Kpt"], c["Vpt"], c["f"]["Rr"], None)
    assert np.abs(nob - ref).max() > 1e-3
    # numpy model of "no bias": visual scores miss q.dmu/sqrt(d)
    b = c["q"] @ c["f"]["dmu"]
    s = np.concatenate([c["K"] @ c["q"] - b, c["Kpt"] @ c["q"]]) / np.sqrt(D)
    assert np.abs(nob - softmax_attn(s, np.vstack([c["V"], c["Vpt"]]))).max() <= 1e-9


def test_segment_mass_split(case):
    """With V = indicator of the segment, the output is the softmax mass of each segment."""
    c = case
    N, M = c["K"].shape[0], c["Kpt"].shape[0]
    Vv = np.zeros((N, D)); Vv[:, 0] = 1.0
    Vt = np.zeros((M, D)); Vt[:, 1] = 1.0
    out = oracle.decode_dual_head(c["q"], c["Kt"], Vv, c["Kpt"], Vt, c["f"]["Rr"], c["f"]["dmu"])
    s = np.concatenate([c["K"] @ c["q"], c["Kpt"] @ c["q"]]) / np.sqrt(D)
    p = np.exp(s - s.max()); p /= p.sum()
    assert abs(out[0] - p[:N].sum()) <= 1e-12 and abs(out[1] - p[N:].sum()) <= 1e-12
    assert abs(out[0] + out[1] - 1.0) <= 1e-12 and np.abs(out[2:]).max() == 0.0


def test_degenerate_segments(case):
    c = case
    f = c["f"]
    empty_k, empty_v = np.zeros((0, D)), np.zeros((0, D))
    # M = 0: the single-path decode (whose own pins are elsewhere)
    a = oracle.decode_dual_head(c["q"], c["Kt"], c["V"], empty_k, empty_v, f["Rr"], f["dmu"])
    b = oracle.decode_head(c["q"], c["Kt"], c["V"], f["Rr"], f["dmu"])
    assert np.abs(a - b).max() <= 1e-13
    # N = 0: plain full attention over the text segment, bias irrelevant
    a = oracle.decode_dual_head(c["q"], np.zeros((0, 6)), empty_v, c["Kpt"], c["Vpt"], f["Rr"], f["dmu"])
    b = oracle.full_attn_head(c["q"], c["Kpt"], c["Vpt"])
    assert np.abs(a - b).max() <= 1e-13
    # both empty: zeros
    a = oracle.decode_dual_head(c["q"], np.zeros((0, 6)), empty_v, empty_k, empty_v, f["Rr"], f["dmu"])
    assert np.abs(a).max() == 0.0


def test_lossy_case_against_numpy():
    """Generic (lossy) case: full-rank visual Keys, r = 32; numpy restatement of Alg. 2."""
    N, M, r = 200, 50, 32
    K = normal((N, D), TAG_A, 7) + 2.0
    V, Kpt, Vpt = normal((N, D), TAG_V, 7), normal((M, D), TAG_B, 7), normal((M, D), TAG_V, 8)
    q = normal((D,), TAG_Q, 7)
    f = oracle.fit(K, r, center=True)
    Kt = oracle.compress(K, f["Rr"])
    out = oracle.decode_dual_head(q, Kt, V, Kpt, Vpt, f["Rr"], f["dmu"], scale=0.11)
    s = np.concatenate([Kt @ (q @ f["Rr"]) + q @ f["dmu"], Kpt @ q]) * 0.11
    assert np.abs(out - softmax_attn(s, np.vstack([V, Vpt]))).max() <= 1e-12
    # swapping the segments' roles in the call must not give the same answer (argument order pin)
    wrong = oracle.decode_dual_head(q, Kt, V, Vpt, Kpt, f["Rr"], f["dmu"], scale=0.11)
    assert np.abs(out - wrong).max() > 1e-3


def test_dual_batch_matches_heads():
    B, Hq, Hkv, cap, cap_t, r = 2, 4, 2, 40, 9, 16
    rng = stream(103, 1, 0, 0, TAG_A)
    q = rng.standard_normal((B, Hq, D))
    Kt = rng.standard_normal((B, Hkv, cap, r))
    V = rng.standard_normal((B, Hkv, cap, D))
    Kpt = rng.standard_normal((B, Hkv, cap_t, D))
    Vpt = rng.standard_normal((B, Hkv, cap_t, D))
    Rr = rng.standard_normal((B, Hkv, D, r)) / np.sqrt(D)
    dmu = rng.standard_normal((B, Hkv, D))
    lens, lens_t = np.array([40, 17], np.int32), np.array([0, 9], np.int32)
    out = oracle.decode_dual_batch(q, Kt, V, Kpt, Vpt, Rr, dmu, lens, lens_t)
    for b in range(B):
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            ref = oracle.decode_dual_head(q[b, h], Kt[b, hk, :lens[b]], V[b, hk, :lens[b]], Kpt[b, hk, :lens_t[b]],
                                          Vpt[b, hk, :lens_t[b]], Rr[b, hk], dmu[b, hk])
            assert np.abs(out[b, h] - ref).max() <= 1e-13
