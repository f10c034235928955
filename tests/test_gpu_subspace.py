"""GPU-vs-oracle parity of the Cholesky-based subspace iteration (Alg. 1 steps
6-13) through rk_fit_subspace.  Staged protocol as for the eigensolver: the
oracle's iteration is fed the GPU's own scatter matrix (fp32, itself checked
against the oracle in test_gpu_parity.py), so the comparison isolates the
solver.  Both sides run it in fp64 from the same start basis, so R_r agrees to
fp32 output rounding; tolerance 1e-4 relative to max|y| as for every fp32 result."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_19218_amd as rk
from rk_inputs import make_normal
from rk_inputs.generator import TAG_A, TAG_SIGMA

from gpu_util import D, DEV, Pipeline, to_dev, to_host
from test_gpu_parity import TOL_F32, check_out, check_packed, layer, oracle_decode, rel_max

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


def start_basis(B, Hkv, k, cid):
    return np.stack([np.stack([make_normal((D, k), "f32", cid, 0, b, h, TAG_A) for h in range(Hkv)])
                     for b in range(B)])


def fit_subspace(ctx, p, K_dev, n_tokens, V0, T=5, eps=1e-6, sigma=None, center=True, n_dev=None):
    lay = p.layout()
    ws = torch.empty(rk.rk_fit_workspace_size(lay, n_tokens), device=DEV, dtype=torch.uint8)
    status = torch.full((p.B, p.Hkv), -1, device=DEV, dtype=torch.int32)
    rk.rk_fit_subspace(ctx, lay, rk.Rows(K_dev, n_tokens, n_tokens_dev=n_dev), sigma,
                       rk.RK_FIT_CENTER if center else 0, to_dev(V0, "f32"), T, eps, p.Rr, p.mu, p.dmu, ws,
                       cov=p.cov, status=status)
    torch.cuda.synchronize()
    return status.cpu().numpy()


CASES = [
    # id, dtype, B, Hkv, L, lengths, k, T, eps, sigma, center
    ("f32_k32", "f32", 1, 2, 512, None, 32, 5, 1e-6, False, True),
    ("bf16_k64", "bf16", 2, 2, 1300, [1300, 777], 64, 5, 1e-6, False, True),
    ("bf16_k16_sigma", "bf16", 1, 2, 600, None, 16, 5, 1e-6, True, True),
    ("bf16_k96_uncentered", "bf16", 1, 2, 600, None, 96, 5, 1e-6, False, False),
    ("bf16_k104_max", "bf16", 1, 1, 400, None, 104, 3, 1e-5, False, True),
    ("bf16_k37_odd", "bf16", 1, 2, 400, None, 37, 5, 1e-6, True, True),
    # k = 72 leaves no padding columns in the basis's LDS rows, k = 80 gives a thread an odd number of columns
    ("bf16_k72_unpadded", "bf16", 1, 2, 500, None, 72, 5, 1e-6, True, True),
    ("bf16_k80", "bf16", 2, 1, 700, [700, 333], 80, 5, 1e-6, False, True),
    ("bf16_k8_T1", "bf16", 1, 1, 300, None, 8, 1, 0.0, False, True),
    ("bf16_k1", "bf16", 1, 1, 300, None, 1, 4, 1e-6, False, True),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_subspace_parity(ctx, case):
    _, dtype, B, Hkv, L, lengths, k, T, eps, with_sigma, center = case
    data = layer(B, Hkv, Hkv, L, dtype, 41, lengths=lengths, mean_shift=1.0)
    p = Pipeline(ctx, B, Hkv, Hkv, k, dtype, L + 8)
    V0 = start_basis(B, Hkv, k, 42)
    sigma_h = None
    if with_sigma:
        sigma_h = np.abs(np.stack([np.stack([make_normal((D,), "f32", 43, 0, b, h, TAG_SIGMA) for h in range(Hkv)])
                                   for b in range(B)])) + 0.25
    n_dev = None if lengths is None else torch.tensor(lengths, device=DEV, dtype=torch.int32)
    st = fit_subspace(ctx, p, to_dev(data["K"], dtype), L, V0, T, eps,
                      sigma=None if sigma_h is None else to_dev(sigma_h, "f32"), center=center, n_dev=n_dev)
    assert not st.any()
    cov, mu, Rr, dmu = to_host(p.cov), to_host(p.mu), to_host(p.Rr), to_host(p.dmu)
    for b in range(B):
        for h in range(Hkv):
            Cq = oracle.weight(cov[b, h], None if sigma_h is None else sigma_h[b, h].astype(np.float64))
            want = oracle.subspace_iter(Cq, V0[b, h].astype(np.float64), T, eps)
            assert rel_max(Rr[b, h], want) <= TOL_F32, (b, h, rel_max(Rr[b, h], want))
            want_dmu = oracle.delta_mu(mu[b, h], want)
            assert np.abs(dmu[b, h] - want_dmu).max() <= TOL_F32 * max(np.abs(mu[b, h]).max(), 1e-30)


def test_zero_keys_report_the_failed_pivot(ctx):
    """All-zero Keys: C_q = 0, the Gram matrix is 0 and, without a ridge, the first pivot is
    not positive.  The oracle reports iteration 0; the kernel must report the same code."""
    B, Hkv, L, k = 1, 2, 64, 16
    p = Pipeline(ctx, B, Hkv, Hkv, k, "bf16", 64)
    V0 = start_basis(B, Hkv, k, 44)
    st = fit_subspace(ctx, p, to_dev(np.zeros((B, Hkv, L, D), np.float32), "bf16"), L, V0, T=5, eps=0.0)
    with pytest.raises(RuntimeError, match="iteration 0"):
        oracle.subspace_iter(np.zeros((D, D)), V0[0, 0].astype(np.float64), 5, 0.0)
    assert st.tolist() == [[1, 1]]


def test_subspace_route_end_to_end(ctx):
    """fit (subspace) -> compress -> decode against the oracle fed the same R_r, and the paper's
    claim that T = 5 is as accurate as the full eigendecomposition (both GPU routes against exact
    attention from the oracle)."""
    dtype, B, Hq, Hkv, L, k = "bf16", 2, 8, 2, 900, 32
    lengths = [900, 500]
    data = layer(B, Hq, Hkv, L, dtype, 45, lengths=lengths, mean_shift=1.0)
    Kd, Vd = to_dev(data["K"], dtype), to_dev(data["V"], dtype)
    n_dev = torch.tensor(lengths, device=DEV, dtype=torch.int32)
    q = to_dev(data["q"], dtype)

    p = Pipeline(ctx, B, Hq, Hkv, k, dtype, L + 8)
    assert not fit_subspace(ctx, p, Kd, L, start_basis(B, Hkv, k, 46), n_dev=n_dev).any()
    p.compress(Kd, L, V_dev=Vd, n_dev=n_dev)
    Kt, _ = p.unpacked()
    Rr = to_host(p.Rr)
    for b in range(B):
        for h in range(Hkv):
            check_packed(Kt[b, h, :lengths[b]], data["K"][b, h, :lengths[b]].astype(np.float64), Rr[b, h], dtype)
    out_sub = p.decode(q).copy()
    check_out(out_sub, oracle_decode(p, data["q"], lengths), dtype)

    pe = Pipeline(ctx, B, Hq, Hkv, k, dtype, L + 8)
    pe.fit(Kd, L, n_dev=n_dev)
    pe.compress(Kd, L, V_dev=Vd, n_dev=n_dev)
    out_eig = pe.decode(q).copy()
    # Both routes keep the 16 dominant directions and differ in which noise directions fill the
    # other 16 columns, so they differ from each other by about as much as each differs from exact
    # attention: the claim to check is that the subspace route loses no more than the eigen route.
    G = Hq // Hkv
    err_sub = err_eig = 0.0
    for b in range(B):
        for h in range(Hq):
            n = lengths[b]
            full = oracle.full_attn_head(data["q"][b, h], data["K"][b, h // G, :n], data["V"][b, h // G, :n])
            err_sub = max(err_sub, np.abs(out_sub[b, h] - full).max())
            err_eig = max(err_eig, np.abs(out_eig[b, h] - full).max())
    assert err_sub <= 1.5 * err_eig + 2e-2, (err_sub, err_eig)
