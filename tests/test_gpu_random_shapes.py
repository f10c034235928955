"""Seeded random shapes through the whole GPU path (fit -> compress -> decode, one fused decode
step, dual-path decode with a ragged text segment), each compared with the oracle: batch size,
head grouping, cache length, ragged lengths (empty sequences included), keep r anywhere in 1..128,
storage type and split count are drawn per seed, so that corners no hand-written case names
(r = 93 with 15 query heads per KV head and 5 splits, ...) are visited too."""
import numpy as np
import pytest
import torch

import paper_2605_19218_amd as rk

from gpu_util import DEV, to_dev, to_host
from test_gpu_dual import TextSeg, decode_dual, oracle_dual
from test_gpu_parity import check_out, check_packed, layer, oracle_decode, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


def draw(seed, wide=False):
    """wide: many (batch item, KV head) units and short caches, so that each XCD serves several units, a
    compute unit several work-groups in turn, and the folded merge its two- and three-split forms."""
    g = np.random.Generator(np.random.Philox(key=9000 + seed))
    B = int(g.integers(4, 13)) if wide else int(g.integers(1, 4))
    Hkv = int(g.choice([8, 16, 32])) if wide else int(g.choice([1, 2, 4]))
    G = int(g.choice([1, 1, 2, 4])) if wide else int(g.choice([1, 2, 4, 7, 8, 15, 16, 20]))
    L = int(g.choice([97, 160, 300, 700])) if wide else int(g.choice([1, 31, 33, 127, 129, 500, 1023, 1500, 2100]))
    lengths = [int(g.integers(0, L + 1)) for _ in range(B)]
    lengths[int(g.integers(0, B))] = L                       # one sequence is full
    r = int(g.integers(1, 129))
    dtype = "f32" if seed % 5 == 4 else "bf16"
    splits = int(g.choice([0, 0, 1, 3, 5]))
    cap_t = int(g.choice([8, 70, 200]))
    lens_t = [int(g.integers(0, cap_t - 2)) for _ in range(B)]
    return B, Hkv, G, L, lengths, r, dtype, splits, cap_t, lens_t


@pytest.mark.parametrize("seed", list(range(16)) + [100 + i for i in range(6)])
def test_random_shape(ctx, seed):
    B, Hkv, G, L, lengths, r, dtype, splits, cap_t, lens_t = draw(seed, wide=seed >= 100)
    Hq = Hkv * G
    data = layer(B, Hq, Hkv, L, dtype, 70 + seed, lengths=lengths, mean_shift=1.0)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, lengths=lengths, cap=L + 3)
    p.max_seq_len = max(lengths)
    Rr = to_host(p.Rr)
    Kt, Vc = p.unpacked()
    for b in range(B):
        n = lengths[b]
        check_packed(Kt[b, 0, :n], data["K"][b, 0, :n].astype(np.float64), Rr[b, 0], dtype)
        assert np.array_equal(Vc[b, -1, :n], data["V"][b, -1, :n].astype(np.float64))
    rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, splits)
    try:
        q = to_dev(data["q"], dtype)
        check_out(p.decode(q), oracle_decode(p, data["q"], lengths), dtype)
        # dual path over a ragged text segment
        tdata = layer(B, Hq, Hkv, cap_t, dtype, 700 + seed, lengths=lens_t)
        seg = TextSeg(B, Hkv, cap_t, dtype, lens_t)
        seg.fill(tdata["K"], tdata["V"])
        check_out(decode_dual(ctx, p, q, seg.arg()), oracle_dual(p, data["q"], lengths, seg, lens_t), dtype)
        # one fused step (falls back to the two calls where the shape has no fused form)
        new = layer(B, Hq, Hkv, 1, dtype, 7000 + seed)
        got = p.append_decode(to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype), to_dev(new["q"], dtype))
        lens1 = [n + 1 for n in lengths]
        assert p.seq_len.cpu().tolist() == lens1
        check_out(got, oracle_decode(p, new["q"], lens1), dtype)
    finally:
        rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, 0)
