"""GPU parity of the smaller follow-on rows: the query-window channel weights
(Alg. 1 step 4) through rk_query_sigma, and two comparison workloads that run
through the unchanged kernels -- the dense cache (r = d, the paper's full-channel
baseline under a common launcher) and a magnitude-based original-basis channel mask
(a head-wise mask with R = I, the kind of pruner the paper compares against)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_19218_amd as rk
from rk_inputs import make_normal, stream
from rk_inputs.generator import TAG_A, TAG_Q

from gpu_util import D, DEV, Pipeline, to_dev, to_host
from test_gpu_parity import TOL_F32, check_out, layer, oracle_decode, rel_max, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


def query_history(B, Hq, T, dtype, cid):
    return np.stack([np.stack([make_normal((T, D), dtype, cid, 0, b, h, TAG_Q) for h in range(Hq)])
                     for b in range(B)])


@pytest.mark.parametrize("dtype,B,Hq,Hkv,T,W", [
    ("f32", 1, 2, 2, 32, 32),        # G = 1: the formula as the paper prints it
    ("bf16", 2, 14, 2, 32, 32),      # G = 7, the paper's W
    ("bf16", 1, 8, 4, 100, 32),      # window = last 32 rows of a longer query history (strided view)
    ("bf16", 1, 4, 1, 5, 5),         # odd window
])
def test_query_sigma_parity(ctx, dtype, B, Hq, Hkv, T, W):
    Q = query_history(B, Hq, T, dtype, 51)
    Qd = to_dev(Q, dtype)
    win = Qd[:, :, T - W:, :]                       # a view: strides of the full history
    sigma = torch.zeros(B, Hkv, D, device=DEV, dtype=torch.float32)
    rk.rk_query_sigma(ctx, rk.Layout(B, Hq, Hkv, 32, rk.RK_BF16 if dtype == "bf16" else rk.RK_F32, 32, 0), win, W,
                      sigma)
    torch.cuda.synchronize()
    got = to_host(sigma)
    G = Hq // Hkv
    for b in range(B):
        for hk in range(Hkv):
            want = oracle.sigma_window(Q[b, hk * G:(hk + 1) * G, T - W:].astype(np.float64))
            assert rel_max(got[b, hk], want) <= TOL_F32


def test_query_aware_fit_on_device(ctx):
    """sigma computed on the device steers the fit as Sec. 3.2 intends: Keys with equal variance on
    coordinates 0-7 and 8-15, queries that use only 8-15 -> the kept subspace is 8-15."""
    B, Hq, Hkv, L, r, dtype = 1, 2, 1, 400, 8, "f32"
    rng = stream(52, 0, 0, 0, TAG_A)
    K = np.zeros((B, Hkv, L, D), np.float32)
    K[..., :16] = rng.standard_normal((B, Hkv, L, 16))
    K[..., 16:] = 0.01 * rng.standard_normal((B, Hkv, L, D - 16))
    Qw = 0.1 * rng.standard_normal((B, Hq, 32, D)).astype(np.float32)
    Qw[..., 8:16] = 3.0 * rng.standard_normal((B, Hq, 32, 8))
    sigma = torch.zeros(B, Hkv, D, device=DEV, dtype=torch.float32)
    p = Pipeline(ctx, B, Hq, Hkv, r, dtype, L)
    rk.rk_query_sigma(ctx, p.layout(), to_dev(Qw, dtype), 32, sigma)
    p.fit(to_dev(K, dtype), L, sigma=sigma)
    Rr = to_host(p.Rr)[0, 0]
    P = Rr @ Rr.T
    assert np.trace(P[8:16, 8:16]) >= 7.99 and np.trace(P[:8, :8]) <= 0.01
    p.fit(to_dev(K, dtype), L)                       # query-agnostic: cannot prefer either group
    Rr0 = to_host(p.Rr)[0, 0]
    assert 1.0 <= np.trace((Rr0 @ Rr0.T)[8:16, 8:16]) <= 7.0


def test_dense_cache_is_exact_attention(ctx):
    """r = d: the rotation is a change of basis and nothing is pruned (Eq. 1 with P = I); the only
    loss is the bf16 rounding of the rotated Keys."""
    dtype, B, Hq, Hkv, L = "bf16", 1, 8, 2, 700
    data = layer(B, Hq, Hkv, L, dtype, 53, mean_shift=1.0)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, D, dtype)
    got = p.decode(to_dev(data["q"], dtype))
    check_out(got, oracle_decode(p, data["q"], [L]), dtype)
    G = Hq // Hkv
    for h in range(Hq):
        full = oracle.full_attn_head(data["q"][0, h], data["K"][0, h // G], data["V"][0, h // G])
        assert np.abs(got[0, h] - full).max() <= 3e-2


def test_original_basis_magnitude_mask(ctx):
    """A head-wise mask in the ORIGINAL basis: R = I, keep the r channels with the largest Key
    energy.  rk_gather_rotation turns (R, keep_idx) into a column selection, rk_compress then copies
    the kept channels bit for bit, and decode attends over them."""
    dtype, B, Hq, Hkv, L, r = "bf16", 2, 8, 2, 500, 32
    data = layer(B, Hq, Hkv, L, dtype, 54)
    K = data["K"].astype(np.float64)
    energy = (K ** 2).sum(axis=2)                                   # [B, Hkv, d]
    keep = np.argsort(-energy, axis=-1, kind="stable")[..., :r].astype(np.int32)
    p = Pipeline(ctx, B, Hq, Hkv, r, dtype, L + 8)
    eye = torch.eye(D, device=DEV, dtype=torch.float32).expand(B, Hkv, D, D).contiguous()
    rk.rk_gather_rotation(ctx, p.layout(), eye, torch.from_numpy(keep).to(DEV), p.Rr)
    p.dmu.zero_()
    Kd, Vd = to_dev(data["K"], dtype), to_dev(data["V"], dtype)
    p.compress(Kd, L, V_dev=Vd)
    Kt, _ = p.unpacked()
    for b in range(B):
        for h in range(Hkv):
            assert np.array_equal(Kt[b, h, :L], K[b, h][:, keep[b, h]])
    got = p.decode(to_dev(data["q"], dtype), use_bias=False)
    check_out(got, oracle_decode(p, data["q"], [L] * B, use_bias=False), dtype)
