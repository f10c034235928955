"""GPU parity of the fused decode step (frozen-R append inside the decode launches)
against the oracle's append followed by its decode, and against the unfused calls."""
import numpy as np
import pytest
import torch

import paper_2605_19218_amd as rk

from gpu_util import DEV, Pipeline, bf16_ulp, to_dev, to_host
from test_gpu_dual import TextSeg, decode_dual, oracle_dual
from test_gpu_parity import KT_ABS, check_out, check_packed, layer, oracle_decode, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


def clone_state(ctx, p):
    """A second pipeline holding copies of p's caches and fit results."""
    c = Pipeline(ctx, p.B, p.Hq, p.Hkv, p.r, p.dtype, p.cap)
    for name in ("Rr", "dmu", "Kp", "Vc", "seq_len"):
        getattr(c, name).copy_(getattr(p, name))
    c.max_seq_len = p.max_seq_len
    return c


# name, dtype, B, Hq, Hkv, L, lengths, r, steps, splits (0 = planned), generic
FUSED_CASES = [
    ("gqa2_r48", "bf16", 2, 8, 4, 500, [500, 250], 48, 6, 0, False),
    ("gqa7_r64_splits", "bf16", 2, 28, 4, 2500, [2500, 1100], 64, 4, 0, False),
    ("gqa7_r64_s5", "bf16", 2, 14, 2, 1500, [1500, 3], 64, 3, 5, False),
    ("mha_r16", "bf16", 2, 4, 4, 300, [300, 17], 16, 3, 0, False),
    ("gqa15_r128", "bf16", 1, 15, 1, 700, [700], 128, 3, 0, False),
    ("gqa4_r80", "bf16", 2, 8, 2, 640, [640, 127], 80, 4, 3, False),
    ("gqa4_r56_padded", "bf16", 2, 8, 2, 640, [640, 127], 56, 4, 3, False),          # r padded to 64 in the cache
    ("gqa7_r37_padded", "bf16", 1, 7, 1, 900, [900], 37, 3, 0, False),
    ("tile_edge", "bf16", 3, 4, 2, 256, [128, 256, 127], 32, 3, 0, False),       # new rows open a new tile
    ("from_empty", "bf16", 3, 4, 2, 40, [0, 1, 40], 32, 3, 0, False),
    ("g16_two_launch", "bf16", 1, 16, 1, 300, [300], 32, 3, 0, False),           # no free column: unfused launches
    ("generic_bf16", "bf16", 2, 4, 2, 300, [300, 100], 24, 3, 0, True),
    ("f32", "f32", 2, 4, 2, 200, [200, 50], 32, 3, 0, False),
]


@pytest.mark.parametrize("case", FUSED_CASES, ids=[c[0] for c in FUSED_CASES])
def test_append_decode_fused(ctx, case):
    _, dtype, B, Hq, Hkv, L, lengths, r, steps, splits, generic = case
    data = layer(B, Hq, Hkv, L, dtype, 61, lengths=lengths)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, lengths=lengths, cap=L + steps)
    p.max_seq_len = max(lengths)
    ref = clone_state(ctx, p)
    Rr = to_host(p.Rr)
    lens = list(lengths)
    rk.rk_set_option(ctx, rk.RK_OPT_FORCE_GENERIC, int(generic))
    rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, splits)
    try:
        for step in range(steps):
            new = layer(B, Hq, Hkv, 1, dtype, 6100 + step)
            kn, vn, q = to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype), to_dev(new["q"], dtype)
            got = p.append_decode(kn, vn, q)
            ref.append(kn, vn)
            got_ref = ref.decode(q)
            Kt, Vc = p.unpacked()
            Kt_ref, _ = ref.unpacked()
            for b in range(B):
                for h in range(Hkv):
                    row = Kt[b, h, lens[b]:lens[b] + 1]
                    check_packed(row, new["k_new"][b, h][None].astype(np.float64), Rr[b, h], dtype)
                    assert np.array_equal(Vc[b, h, lens[b]], new["v_new"][b, h].astype(np.float64))
                    # the same row as rk_append's: one storage ulp plus twice the fp32 accumulation bound
                    # (an entry that nearly cancels is small against the row norm, not against its own ulp)
                    ref_row = Kt_ref[b, h, lens[b]:lens[b] + 1]
                    tol = bf16_ulp(ref_row) if dtype == "bf16" else 1e-5 * np.abs(ref_row).max()
                    tol = tol + 2 * KT_ABS * np.linalg.norm(new["k_new"][b, h].astype(np.float64))
                    assert np.all(np.abs(row - ref_row) <= tol)
                    # the prefill rows are untouched
                    assert np.array_equal(Kt[b, h, :lengths[b]], Kt_ref[b, h, :lengths[b]])
            lens = [x + 1 for x in lens]
            assert p.seq_len.cpu().tolist() == lens
            check_out(got, oracle_decode(p, new["q"], lens), dtype)
            check_out(got, got_ref, dtype)
    finally:
        rk.rk_set_option(ctx, rk.RK_OPT_FORCE_GENERIC, 0)
        rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, 0)


def test_fused_full_size_gqa_16k(ctx):
    """The benchmark configuration (B=8, 28 query / 4 KV heads, L=16384, r=64, bf16), the launch
    configuration of bench.py's token loop: two fused steps, every output compared with the oracle."""
    B, Hq, Hkv, L, r, dtype = 8, 28, 4, 16384, 64, "bf16"
    data = layer(B, Hq, Hkv, L, dtype, 3)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, cap=L + 32)
    p.max_seq_len = L
    Rr = to_host(p.Rr)
    for step in range(2):
        new = layer(B, Hq, Hkv, 1, dtype, 6600 + step)
        got = p.append_decode(to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype), to_dev(new["q"], dtype))
        assert p.seq_len.cpu().tolist() == [L + step + 1] * B
        Kt, Vc = p.unpacked()
        for (b, h) in ((0, 0), (7, 3), (3, 1)):
            check_packed(Kt[b, h, L + step:L + step + 1], new["k_new"][b, h][None].astype(np.float64), Rr[b, h], dtype)
            assert np.array_equal(Vc[b, h, L + step], new["v_new"][b, h].astype(np.float64))
        check_out(got, oracle_decode(p, new["q"], [L + step + 1] * B), dtype)


@pytest.mark.parametrize("shape", [(2, 28, 4, 2500, [2500, 1100], 64), (8, 8, 8, 1200, [1200, 0, 5, 700, 1200, 64, 333, 1], 48),
                                   (4, 12, 6, 4096, [4096, 4096, 2048, 4000], 96)])
def test_fused_append_folded_against_two_launches(ctx, shape):
    """The fused append with the split-K merge folded into its launch (the length bumped by the last
    work-group of a batch item) against the same steps with the separate merge launch: same lengths,
    bit-equal stored rows, outputs within the output tolerance of each other and of the oracle, and
    bit-equal outputs when the folded form is repeated from the same state.  The unit counts (8, 64, 24
    head groups) all deal evenly over the 8 XCDs, and every shape plans at least two splits."""
    B, Hq, Hkv, L, lengths, r = shape
    dtype = "bf16"
    data = layer(B, Hq, Hkv, L, dtype, 64, lengths=lengths)
    a = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, lengths=lengths, cap=L + 4)
    a.max_seq_len = max(lengths)
    n_splits, _ = rk.rk_decode_plan(ctx, a.layout())
    assert n_splits >= 2
    two, again = clone_state(ctx, a), clone_state(ctx, a)
    lens = list(lengths)
    for step in range(3):
        new = layer(B, Hq, Hkv, 1, dtype, 6400 + step)
        kn, vn, q = to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype), to_dev(new["q"], dtype)
        got = a.append_decode(kn, vn, q).copy()
        rep = again.append_decode(kn, vn, q).copy()
        rk.rk_set_option(ctx, rk.RK_OPT_FUSE_MERGE, 0)
        try:
            ref = two.append_decode(kn, vn, q).copy()
        finally:
            rk.rk_set_option(ctx, rk.RK_OPT_FUSE_MERGE, 1)
        lens = [x + 1 for x in lens]
        assert a.seq_len.cpu().tolist() == lens and two.seq_len.cpu().tolist() == lens
        assert np.array_equal(got, rep)
        check_out(got, ref, dtype)
        check_out(got, oracle_decode(a, new["q"], lens), dtype)
        assert torch.equal(a.Kp, two.Kp) and torch.equal(a.Vc, two.Vc)


def test_fused_new_token_matters(ctx):
    """Vacuity guard: a new Key aligned with the query must change the output visibly,
    i.e. the appended row really takes part in the softmax of its own step."""
    B, Hq, Hkv, L, r, dtype = 1, 4, 2, 400, 64, "bf16"
    data = layer(B, Hq, Hkv, L, dtype, 62)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, cap=L + 2)
    p.max_seq_len = L
    new = layer(B, Hq, Hkv, 1, dtype, 6200)
    q = new["q"]
    before = p.decode(to_dev(q, dtype)).copy()
    k_new = (4.0 * q[:, ::Hq // Hkv]).astype(np.float32)          # [B,Hkv,d]: along the group's first query
    v_new = np.full_like(new["v_new"], 1.5)
    got = p.append_decode(to_dev(k_new, dtype), to_dev(v_new, dtype), to_dev(q, dtype))
    assert np.abs(got - before).max() > 1.0
    check_out(got, oracle_decode(p, q, [L + 1]), dtype)


def test_fused_device_guard_and_capacity(ctx):
    """A sequence already at capacity keeps its rows and length and attends over what it has;
    the host bound refuses a call that cannot fit."""
    B, Hq, Hkv, r, dtype, cap = 2, 4, 2, 32, "bf16", 64
    data = layer(B, Hq, Hkv, cap, dtype, 63, lengths=[64, 10])
    p = run_prefill(ctx, data, B, Hq, Hkv, cap, r, dtype, lengths=[64, 10], cap=cap)
    assert p.cap == cap
    before = p.unpacked()[0].copy()
    p.max_seq_len = 10                      # host bound of the short sequence only
    new = layer(B, Hq, Hkv, 1, dtype, 6300)
    got = p.append_decode(to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype), to_dev(new["q"], dtype))
    assert p.seq_len.cpu().tolist() == [64, 11]
    after = p.unpacked()[0]
    assert np.array_equal(after[0], before[0])
    check_out(got, oracle_decode(p, new["q"], [64, 11]), dtype)
    p.max_seq_len = cap
    with pytest.raises(rk.RotateKError) as e:
        p.append_decode(to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype), to_dev(new["q"], dtype))
    assert e.value.status == rk.RK_ERR_CAPACITY
    assert p.seq_len.cpu().tolist() == [64, 11]


# ---------------------------------------------------------------------------
# the fused text append (new tokens stay full-width, the paper's decode loop)


def fused_dual(ctx, p, kn, vn, q_dev, text):
    lay = p.layout()
    ws = torch.empty(rk.rk_decode_workspace_size(ctx, lay), device=DEV, dtype=torch.uint8)
    rk.rk_append_text_decode_attn_dual(ctx, lay, kn, vn, q_dev, p.Kp, p.Vc, p.Rr, p.dmu, text, 0.0, p.out, ws)
    torch.cuda.synchronize()
    return to_host(p.out).copy()


# name, dtype, B, Hq, Hkv, L, lengths, r, text lengths, generic, row stride
TEXT_FUSED_CASES = [
    ("gqa2_bf16", "bf16", 2, 8, 4, 500, [500, 250], 48, [3, 0], False, 128),
    ("gqa7_splits", "bf16", 2, 28, 4, 2500, [2500, 1100], 64, [64, 5], False, 128),
    ("mha32_heads", "bf16", 1, 32, 32, 700, [700], 64, [10], False, 128),           # 1024 pieces: the copy loops
    ("empty_visual", "bf16", 2, 4, 2, 130, [0, 130], 32, [0, 7], False, 160),        # split 0 empty, padded rows
    ("generic_f32", "f32", 2, 4, 2, 300, [300, 20], 24, [5, 1], False, 128),
    ("generic_bf16", "bf16", 2, 4, 2, 300, [300, 20], 24, [5, 1], True, 128),
]


@pytest.mark.parametrize("fold", [1, 0], ids=["merge_folded", "merge_launch"])
@pytest.mark.parametrize("case", TEXT_FUSED_CASES, ids=[c[0] for c in TEXT_FUSED_CASES])
def test_append_text_decode_fused(ctx, case, fold):
    """`fold`: with the split-K merge folded into the split launch where the shape allows it (the text length
    is then bumped by the batch item's last work-group), and with the separate merge launch."""
    _, dtype, B, Hq, Hkv, L, lengths, r, lens_t, generic, stride = case
    steps, cap_t = 5, max(lens_t) + 5
    data = layer(B, Hq, Hkv, L, dtype, 64, lengths=lengths, mean_shift=1.5)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, lengths=lengths)
    tdata = layer(B, Hq, Hkv, cap_t, dtype, 65, lengths=lens_t)
    seg = TextSeg(B, Hkv, cap_t, dtype, lens_t, row_stride=stride)
    seg.fill(tdata["K"], tdata["V"])
    ref = TextSeg(B, Hkv, cap_t, dtype, lens_t, row_stride=stride)
    ref.fill(tdata["K"], tdata["V"])
    lens_t = list(lens_t)
    rk.rk_set_option(ctx, rk.RK_OPT_FORCE_GENERIC, int(generic))
    rk.rk_set_option(ctx, rk.RK_OPT_FUSE_MERGE, fold)
    try:
        for step in range(steps):
            new = layer(B, Hq, Hkv, 1, dtype, 6400 + step)
            kn, vn, q = to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype), to_dev(new["q"], dtype)
            got = fused_dual(ctx, p, kn, vn, q, seg.arg())
            rk.rk_append_text(ctx, p.layout(), ref.arg(), kn, vn)
            Kh, Vh = seg.host()
            for b in range(B):
                assert np.array_equal(Kh[b, :, lens_t[b]], new["k_new"][b].astype(np.float64))
                assert np.array_equal(Vh[b, :, lens_t[b]], new["v_new"][b].astype(np.float64))
            lens_t = [x + 1 for x in lens_t]
            seg.max_len += 1
            ref.max_len += 1
            assert seg.len.cpu().tolist() == lens_t
            check_out(got, oracle_dual(p, new["q"], lengths, seg, lens_t), dtype)
            # the two separate calls: same rows in the segment, same result up to the fp32 summation order
            # (the plain dual call may run its text attention in slices next to the visual splits)
            check_out(got, decode_dual(ctx, p, q, ref.arg()), dtype)
            assert torch.equal(seg.k, ref.k) and torch.equal(seg.v, ref.v)
    finally:
        rk.rk_set_option(ctx, rk.RK_OPT_FORCE_GENERIC, 0)
        rk.rk_set_option(ctx, rk.RK_OPT_FUSE_MERGE, 1)
    assert seg.max_len == cap_t
    with pytest.raises(rk.RotateKError) as e:
        fused_dual(ctx, p, kn, vn, q, seg.arg())
    assert e.value.status == rk.RK_ERR_CAPACITY
    # understated host bound: the full sequence is left alone on the device
    full = [b for b in range(B) if lens_t[b] == cap_t]
    before = seg.host()[0].copy()
    seg.max_len = cap_t - 1
    got = fused_dual(ctx, p, kn, vn, q, seg.arg())
    now = seg.len.cpu().tolist()
    for b in range(B):
        assert now[b] == (lens_t[b] if b in full else lens_t[b] + 1)
    for b in full:
        assert np.array_equal(seg.host()[0][b], before[b])
    seg.max_len = cap_t
    check_out(got, oracle_dual(p, new["q"], lengths, seg, now), dtype)
