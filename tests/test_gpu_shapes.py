"""GPU parity at the stated sizes of the two largest workloads.

Joint token+channel pruning (Fig. 3(a)): batch 16, per-sequence lengths uniform in
[1024, 32768] (unscaled), a seeded kept-token list that retains half of the visual
rows, r = 64, MHA.  Long prefill + frozen-R decode loop (Sec. 3.2 Step (1): R is
fitted once and reused): L = 32768, r = 48, layer-varying Key rank, 128 appended
tokens through the two-call and through the fused entry points.

Only the HEAD COUNT is reduced (2 resp. 4 of the 32 heads): heads are independent
grid units that share no state, so per-(batch item, head) work, the ragged split
plan, the token gathers and the tile crossings are all at the real size, and the
oracle side still finishes in seconds.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_19218_amd as rk
from rk_inputs import CONFIGS, ragged_lengths, token_keep_lists

from gpu_util import D, DEV, Pipeline, bf16_ulp, to_dev, to_host, torch_dtype
from test_gpu_parity import KT_ABS, TOL_F32, check_out, check_packed, layer, oracle_decode, rel_max

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


def test_ragged_batch16_token_lists_full_lengths(ctx):
    """Batch 16, lengths uniform in [1024, 32768], 64 text rows always kept and half of the visual
    rows kept by a seeded list, r = 64, 2 of the 32 MHA heads.  Covariance, mean, mask, packed Keys
    and Values on the shortest, median and longest sequence; EVERY decode output."""
    c4 = CONFIGS["C4"]
    B, H, r, dtype = c4["batch"], 2, c4["keep"], c4["dtype"]
    lo, hi = c4["ragged"]
    lengths = ragged_lengths(c4["id"], B, lo, hi)
    assert lengths.min() >= lo and lengths.max() <= hi and lengths.max() > hi // 2
    L = int(lengths.max())
    data = layer(B, H, H, L, dtype, c4["id"], lengths=lengths)
    tok_idx, tok_off = token_keep_lists(c4["id"], lengths, n_text=c4["n_text"], keep_frac=c4["token_keep"])
    n_keep = np.diff(tok_off).astype(int)
    n_max = int(n_keep.max())
    Kd, Vd = to_dev(data["K"], dtype), to_dev(data["V"], dtype)
    ti, to = torch.from_numpy(tok_idx).to(DEV), torch.from_numpy(tok_off).to(DEV)
    p = Pipeline(ctx, B, H, H, r, dtype, n_max)
    p.fit(Kd, n_max, tok_idx=ti, tok_off=to)
    p.compress(Kd, n_max, V_dev=Vd, tok_idx=ti, tok_off=to)
    assert p.seq_len.cpu().tolist() == n_keep.tolist()
    # the plan that the timed configuration uses: more than one split, ragged shares
    n_splits, _ = rk.rk_decode_plan(ctx, p.layout())
    assert n_splits >= 2
    cov, mu, Rr, lam, mask = to_host(p.cov), to_host(p.mu), to_host(p.Rr), to_host(p.lam), to_host(p.mask)
    keep = to_host(p.keep_idx)
    Kt, Vc = p.unpacked()
    order = np.argsort(lengths)
    for b, h in ((int(order[0]), 0), (int(order[-1]), 1), (int(order[B // 2]), 1)):     # shortest, longest, median
        rows = tok_idx[tok_off[b]:tok_off[b + 1]]
        mu_o, C_o = oracle.mean_scatter(data["K"][b, h], tok=rows)
        assert rel_max(cov[b, h], C_o) <= TOL_F32 and rel_max(mu[b, h], mu_o) <= TOL_F32
        m_o, k_o = oracle.select(lam[b, h], r)
        assert np.array_equal(mask[b, h], m_o) and np.array_equal(keep[b, h], k_o)
        check_packed(Kt[b, h, :rows.size], data["K"][b, h][rows].astype(np.float64), Rr[b, h], dtype)
        assert np.array_equal(Vc[b, h, :rows.size], data["V"][b, h][rows].astype(np.float64))
        assert not Kt[b, h, rows.size:].any() and not Vc[b, h, rows.size:].any()
    q = to_dev(data["q"], dtype)
    got = p.decode(q)
    check_out(got, oracle_decode(p, data["q"], n_keep), dtype)
    assert np.array_equal(got, p.decode(q))


# appended-token counts at which the decode output is compared with the oracle: every 16th, both sides
# of every 16- and 32-token block edge of the tiled caches that the loop crosses, the first token (it
# opens a new 128-token tile: 32768 is a multiple of 128) and the last two
C5_CHECK_STEPS = sorted({1, 2, 127, 128} | {s for s in range(16, 129, 16)} | {s + 1 for s in range(16, 128, 16)})


class NewTokens:
    """The 128 appended tokens of one layer, generated up front (device copies made per step)."""

    def __init__(self, B, H, dtype, base, steps):
        self.dtype = dtype
        self.rows = [layer(B, H, H, 1, dtype, base + s) for s in range(steps)]

    def dev(self, s):
        n = self.rows[s]
        return to_dev(n["k_new"], self.dtype), to_dev(n["v_new"], self.dtype), to_dev(n["q"], self.dtype)


def new_row_on_host(p, n):
    """Row n of both caches (every batch item and head) as fp64: unpacked on the device, one row copied."""
    td = torch_dtype(p.dtype)
    k_rows = torch.zeros(p.B, p.Hkv, p.cap, p.r, device=DEV, dtype=td)
    v_rows = torch.zeros(p.B, p.Hkv, p.cap, D, device=DEV, dtype=td)
    rk.rk_unpack_cache(p.ctx, p.layout(), p.Kp, p.Vc, k_rows, v_rows)
    torch.cuda.synchronize()
    return to_host(k_rows[:, :, n].contiguous()), to_host(v_rows[:, :, n].contiguous())


@pytest.mark.parametrize("layer_id", [0, 31])
def test_long_prefill_then_128_appends(ctx, layer_id):
    """One layer of the 32-layer workload (Key rank 8 at layer 0, 32 at layer 31), L = 32768, r = 48, 4 of
    the 32 heads.  128 decode steps twice from the same prefill state: rk_append + rk_decode_attn, and
    the fused rk_append_decode_attn.  The length and the appended row are checked at EVERY step of both
    loops, the decode output against the oracle at C5_CHECK_STEPS, and the two loops against each other
    at every step."""
    cfg = CONFIGS["C5"]
    B, H, L, r, dtype, steps = 1, 4, cfg["L"], cfg["keep"], cfg["dtype"], cfg["decode_steps"]
    assert steps == 128 and L % 128 == 0
    data = layer(B, H, H, L, dtype, cfg["id"], rho=cfg["rho_by_layer"](layer_id))
    cap = L + steps
    two = Pipeline(ctx, B, H, H, r, dtype, cap)
    Kd, Vd = to_dev(data["K"], dtype), to_dev(data["V"], dtype)
    two.fit(Kd, L)
    two.compress(Kd, L, V_dev=Vd)
    lam, mask, Rr = to_host(two.lam), to_host(two.mask), to_host(two.Rr)
    for h in range(H):
        m_o, _ = oracle.select(lam[0, h], r)
        assert np.array_equal(mask[0, h], m_o)
    _, C_o = oracle.mean_scatter(data["K"][0, 1])
    assert rel_max(to_host(two.cov)[0, 1], C_o) <= TOL_F32
    Kt0, _ = two.unpacked()
    sel = np.r_[0:16, L // 2:L // 2 + 16, L - 16:L]
    for h in (0, 3):
        check_packed(Kt0[0, h][sel], data["K"][0, h][sel].astype(np.float64), Rr[0, h], dtype)
    del Kt0
    # the fused loop starts from a copy of the same prefill state (same frozen rotation)
    fused = Pipeline(ctx, B, H, H, r, dtype, cap)
    for name in ("Rr", "dmu", "Kp", "Vc", "seq_len"):
        getattr(fused, name).copy_(getattr(two, name))
    fused.max_seq_len = two.max_seq_len
    new = NewTokens(B, H, dtype, 5000 + 1000 * layer_id, steps)

    for s in range(1, steps + 1):
        n = L + s
        kn, vn, q = new.dev(s - 1)
        row = new.rows[s - 1]
        two.append(kn, vn)
        got_two = two.decode(q).copy()
        got_fused = fused.append_decode(kn, vn, q).copy()
        assert two.seq_len.cpu().tolist() == [n] and fused.seq_len.cpu().tolist() == [n], s
        k2, v2 = new_row_on_host(two, n - 1)
        kf, vf = new_row_on_host(fused, n - 1)
        for h in range(H):
            want_k = row["k_new"][0, h][None].astype(np.float64)
            check_packed(k2[0, h][None], want_k, Rr[0, h], dtype)
            check_packed(kf[0, h][None], want_k, Rr[0, h], dtype)
            # the two entry points agree up to one storage ulp plus twice the fp32 accumulation bound
            # (an entry that nearly cancels is small against the row norm, not against its own ulp)
            slack = bf16_ulp(k2[0, h]) + 2 * KT_ABS * np.linalg.norm(want_k)
            assert np.all(np.abs(kf[0, h] - k2[0, h]) <= slack), s
            assert np.array_equal(v2[0, h], row["v_new"][0, h].astype(np.float64)), s
            assert np.array_equal(vf[0, h], row["v_new"][0, h].astype(np.float64)), s
        check_out(got_fused, got_two, dtype)
        if s in C5_CHECK_STEPS:
            check_out(got_two, oracle_decode(two, row["q"], [n]), dtype)
            check_out(got_fused, oracle_decode(fused, row["q"], [n]), dtype)
    # the prefill rows are untouched by 128 appends (sampled) and the caches are full
    Kt1, _ = two.unpacked()
    for h in (0, 3):
        check_packed(Kt1[0, h][sel], data["K"][0, h][sel].astype(np.float64), Rr[0, h], dtype)
    with pytest.raises(rk.RotateKError) as e:
        two.append(kn, vn)
    assert e.value.status == rk.RK_ERR_CAPACITY
