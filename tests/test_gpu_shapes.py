"""GPU parity at the shapes of the joint token+channel pruning workload (ragged
batch of 16, kept-token lists, MHA) and of the long prefill + frozen-R decode loop
(L = 32768, r = 48, layer-varying Key rank, appended tokens), scaled in head count so
that the oracle side finishes in seconds; per-(b, h) work is at the real size."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_19218_amd as rk
from rk_inputs import CONFIGS, ragged_lengths, token_keep_lists

from gpu_util import D, DEV, Pipeline, to_dev, to_host
from test_gpu_parity import TOL_F32, check_out, check_packed, layer, oracle_decode, rel_max

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


def test_ragged_batch16_token_lists(ctx):
    """Batch 16, lengths uniform in [1024, 8192] (the workload's [1024, 32768] scaled by 4), 64 text
    rows always kept and half of the visual rows kept by a seeded list, r = 64, 4 MHA heads."""
    B, H, r, dtype = 16, 4, 64, "bf16"
    lengths = ragged_lengths(4, B, 1024, 8192)
    L = int(lengths.max())
    data = layer(B, H, H, L, dtype, 4, lengths=lengths)
    tok_idx, tok_off = token_keep_lists(4, lengths, n_text=64, keep_frac=0.5)
    n_keep = np.diff(tok_off).astype(int)
    Kd, Vd = to_dev(data["K"], dtype), to_dev(data["V"], dtype)
    ti, to = torch.from_numpy(tok_idx).to(DEV), torch.from_numpy(tok_off).to(DEV)
    p = Pipeline(ctx, B, H, H, r, dtype, int(n_keep.max()))
    p.fit(Kd, int(n_keep.max()), tok_idx=ti, tok_off=to)
    p.compress(Kd, int(n_keep.max()), V_dev=Vd, tok_idx=ti, tok_off=to)
    assert p.seq_len.cpu().tolist() == n_keep.tolist()
    cov, mu, Rr, lam, mask = to_host(p.cov), to_host(p.mu), to_host(p.Rr), to_host(p.lam), to_host(p.mask)
    Kt, Vc = p.unpacked()
    order = np.argsort(lengths)
    for b, h in ((int(order[0]), 0), (int(order[-1]), 3), (int(order[B // 2]), 1)):     # shortest, longest, median
        rows = tok_idx[tok_off[b]:tok_off[b + 1]]
        mu_o, C_o = oracle.mean_scatter(data["K"][b, h], tok=rows)
        assert rel_max(cov[b, h], C_o) <= TOL_F32 and rel_max(mu[b, h], mu_o) <= TOL_F32
        m_o, _ = oracle.select(lam[b, h], r)
        assert np.array_equal(mask[b, h], m_o)
        check_packed(Kt[b, h, :rows.size], data["K"][b, h][rows].astype(np.float64), Rr[b, h], dtype)
        assert np.array_equal(Vc[b, h, :rows.size], data["V"][b, h][rows].astype(np.float64))
    got = p.decode(to_dev(data["q"], dtype))
    check_out(got, oracle_decode(p, data["q"], n_keep), dtype)


@pytest.mark.parametrize("layer_id", [0, 31])
def test_long_prefill_then_appends(ctx, layer_id):
    """One layer of the 32-layer workload (Key rank 8 at layer 0, 32 at layer 31), L = 32768, r = 48,
    4 of the 32 heads; then 6 appended tokens with the frozen rotation, decode checked after the
    first and the last."""
    cfg = CONFIGS["C5"]
    B, H, L, r, dtype = 1, 4, cfg["L"], cfg["keep"], "bf16"
    data = layer(B, H, H, L, dtype, 5, rho=cfg["rho_by_layer"](layer_id))
    p = Pipeline(ctx, B, H, H, r, dtype, L + 32)
    Kd, Vd = to_dev(data["K"], dtype), to_dev(data["V"], dtype)
    p.fit(Kd, L)
    p.compress(Kd, L, V_dev=Vd)
    lam, mask, Rr = to_host(p.lam), to_host(p.mask), to_host(p.Rr)
    for h in range(H):
        m_o, _ = oracle.select(lam[0, h], r)
        assert np.array_equal(mask[0, h], m_o)
    _, C_o = oracle.mean_scatter(data["K"][0, 1])
    assert rel_max(to_host(p.cov)[0, 1], C_o) <= TOL_F32
    n = L
    for step in range(6):
        new = layer(B, H, H, 1, dtype, 5000 + 10 * layer_id + step)
        p.append(to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype))
        n += 1
        if step in (0, 5):
            assert p.seq_len.cpu().tolist() == [n]
            Kt, Vc = p.unpacked()
            sel = np.r_[0:16, L - 16:n]
            for h in (0, 3):
                Kall = np.concatenate([data["K"][0, h], np.zeros((n - L, D), np.float32)])
                # appended rows are checked against their own inputs below; prefill rows here
                check_packed(Kt[0, h][sel[sel < L]], Kall[sel[sel < L]].astype(np.float64), Rr[0, h], dtype)
            check_packed(Kt[0, 2, n - 1:n], new["k_new"][0, 2][None].astype(np.float64), Rr[0, 2], dtype)
            assert np.array_equal(Vc[0, 2, n - 1], new["v_new"][0, 2].astype(np.float64))
            got = p.decode(to_dev(new["q"], dtype))
            check_out(got, oracle_decode(p, new["q"], [n]), dtype)
