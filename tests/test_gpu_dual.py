"""GPU-vs-oracle parity of the dual-path decode (Alg. 2 steps 1-6: rotated visual
segment + unrotated prompt/text segment under one softmax) and of the full-width
text append, through the C ABI binding.  Same tolerances as the single-path tests:
fp32 outputs 1e-4 relative to max|y|, bf16 outputs 2e-2 absolute; copied rows
bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_19218_amd as rk
from rk_inputs import bf16_round

from gpu_util import D, DEV, to_dev, to_host, torch_dtype
from test_gpu_parity import check_out, layer, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


class TextSeg:
    """Device buffers of a text segment [B, H_kv, cap_t, d] (optionally with padded row stride)."""

    def __init__(self, B, Hkv, cap_t, dtype, lens, row_stride=D):
        self.dtype, self.cap = dtype, cap_t
        td = torch_dtype(dtype)
        self.k = torch.zeros(B, Hkv, cap_t, row_stride, device=DEV, dtype=td)
        self.v = torch.zeros(B, Hkv, cap_t, row_stride, device=DEV, dtype=td)
        self.len = torch.tensor(lens, device=DEV, dtype=torch.int32)
        self.max_len = int(max(lens)) if len(lens) else 0

    def fill(self, K_pt, V_pt):
        self.k[..., :D] = to_dev(K_pt, self.dtype)
        self.v[..., :D] = to_dev(V_pt, self.dtype)

    def arg(self, with_len=True):
        return rk.Text(self.k, self.v, self.max_len, self.len if with_len else None, capacity=self.cap)

    def host(self):
        return to_host(self.k[..., :D]), to_host(self.v[..., :D])


def decode_dual(ctx, p, q_dev, text, use_bias=True, scale=0.0):
    lay = p.layout()
    ws = torch.empty(rk.rk_decode_workspace_size(ctx, lay), device=DEV, dtype=torch.uint8)
    rk.rk_decode_attn_dual(ctx, lay, q_dev, p.Kp, p.Vc, p.Rr, p.dmu if use_bias else None, text, scale, p.out, ws)
    torch.cuda.synchronize()
    return to_host(p.out).copy()


def oracle_dual(p, q, lens, seg, lens_t, use_bias=True, scale=0.0):
    Kt, V = p.unpacked()
    Kpt, Vpt = seg.host()
    return oracle.decode_dual_batch(q.astype(np.float64), Kt, V, Kpt, Vpt, to_host(p.Rr),
                                    to_host(p.dmu) if use_bias else None, lens=np.asarray(lens, np.int32),
                                    lens_t=np.asarray(lens_t, np.int32), scale=scale)


DUAL_CASES = [
    # id, dtype, B, Hq, Hkv, L, lengths, r, text lengths, cap_t, generic, splits, row stride
    ("f32_tiny", "f32", 1, 2, 2, 512, None, 32, [20], 32, False, 0, D),
    ("llava_2880_plus_64", "bf16", 1, 32, 32, 2880, None, 64, [64], 64, False, 0, D),
    ("gqa7_ragged_text", "bf16", 2, 14, 2, 1000, [1000, 333], 64, [64, 5], 80, False, 0, D),
    ("gqa7_generic", "bf16", 2, 14, 2, 1000, [1000, 333], 64, [64, 5], 80, True, 0, D),
    ("text_spans_chunks", "bf16", 1, 8, 2, 700, None, 32, [300], 320, False, 0, D),
    ("padded_rows", "bf16", 2, 4, 2, 300, None, 48, [17, 129], 136, False, 0, D + 8),
    # long segments: the 512-thread form of the text kernel (bf16, more than 128 rows), several passes, a batch
    # whose KV-head count (6) is padded to 8 in the block map; fp32 keeps the 128-thread form at any length
    ("wide_text_ragged", "bf16", 3, 14, 2, 600, [600, 100, 0], 64, [700, 1, 513], 704, False, 0, D),
    ("f32_long_text", "f32", 1, 2, 1, 200, None, 16, [200], 200, False, 0, D),
    ("one_split", "bf16", 2, 14, 2, 120, [120, 64], 64, [9, 9], 16, False, 1, D),
    ("empty_segments", "bf16", 4, 4, 2, 130, [0, 0, 130, 77], 32, [0, 12, 0, 3], 16, False, 0, D),
    ("r37_odd_f32rows", "f32", 1, 4, 2, 300, None, 37, [40], 40, False, 0, D),
]


@pytest.mark.parametrize("case", DUAL_CASES, ids=[c[0] for c in DUAL_CASES])
def test_dual_decode_parity(ctx, case):
    _, dtype, B, Hq, Hkv, L, lengths, r, lens_t, cap_t, generic, splits, stride = case
    data = layer(B, Hq, Hkv, L, dtype, 31, lengths=lengths, mean_shift=1.5)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, lengths=lengths)
    lens = lengths or [L] * B
    tdata = layer(B, Hq, Hkv, cap_t, dtype, 32, lengths=lens_t, mean_shift=0.5)
    seg = TextSeg(B, Hkv, cap_t, dtype, lens_t, row_stride=stride)
    seg.fill(tdata["K"], tdata["V"])
    rk.rk_set_option(ctx, rk.RK_OPT_FORCE_GENERIC, int(generic))
    rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, splits)
    try:
        q = to_dev(data["q"], dtype)
        got = decode_dual(ctx, p, q, seg.arg())
        got_nobias = decode_dual(ctx, p, q, seg.arg(), use_bias=False)
        again = decode_dual(ctx, p, q, seg.arg())
        single = p.decode(q).copy()
        # the same call with the separate merge launch (where the merge is folded into the split launch)
        rk.rk_set_option(ctx, rk.RK_OPT_FUSE_MERGE, 0)
        two_launch = decode_dual(ctx, p, q, seg.arg())
    finally:
        rk.rk_set_option(ctx, rk.RK_OPT_FUSE_MERGE, 1)
        rk.rk_set_option(ctx, rk.RK_OPT_FORCE_GENERIC, 0)
        rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, 0)
    want = oracle_dual(p, data["q"], lens, seg, lens_t)
    want_nobias = oracle_dual(p, data["q"], lens, seg, lens_t, use_bias=False)
    check_out(got, want, dtype)
    check_out(got_nobias, want_nobias, dtype)
    check_out(two_launch, want, dtype)
    assert np.array_equal(got, again)
    for b in range(B):
        if lens[b] == 0 and lens_t[b] == 0:
            assert not got[b].any()
        if lens_t[b] == 0:                       # no text rows: exactly the single-path result
            assert np.array_equal(got[b], single[b])


def test_bias_changes_the_dual_result(ctx):
    """Guards the test above against vacuity: on these inputs the bias moves the
    result by far more than the tolerance, in the oracle and on the GPU alike."""
    dtype, B, Hq, Hkv, L, r = "bf16", 1, 8, 2, 600, 16
    data = layer(B, Hq, Hkv, L, dtype, 33)
    # a constant offset on every channel is invisible to the centered covariance, so most of
    # it lands in delta_mu (Sec. 3.2, mean residual) and the bias q . delta_mu is large
    data["K"] = bf16_round(data["K"] + 2.0)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype)
    assert np.abs(to_host(p.dmu)).max() > 1.0
    tdata = layer(B, Hq, Hkv, 64, dtype, 34)
    seg = TextSeg(B, Hkv, 64, dtype, [64])
    seg.fill(tdata["K"], tdata["V"])
    q = to_dev(data["q"], dtype)
    got, got_nb = decode_dual(ctx, p, q, seg.arg()), decode_dual(ctx, p, q, seg.arg(), use_bias=False)
    want, want_nb = oracle_dual(p, data["q"], [L], seg, [64]), oracle_dual(p, data["q"], [L], seg, [64], use_bias=False)
    assert np.abs(want - want_nb).max() > 0.1
    check_out(got, want, dtype)
    check_out(got_nb, want_nb, dtype)


def test_dual_null_len_and_scale(ctx):
    dtype, B, Hq, Hkv, L, r = "bf16", 2, 4, 2, 400, 32
    data = layer(B, Hq, Hkv, L, dtype, 35, mean_shift=1.0)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype)
    tdata = layer(B, Hq, Hkv, 24, dtype, 36)
    seg = TextSeg(B, Hkv, 24, dtype, [24, 24])
    seg.fill(tdata["K"], tdata["V"])
    got = decode_dual(ctx, p, to_dev(data["q"], dtype), seg.arg(with_len=False), scale=0.05)
    check_out(got, oracle_dual(p, data["q"], [L, L], seg, [24, 24], scale=0.05), dtype)


def test_text_append_then_dual_decode(ctx):
    """The paper's decode loop: tokens after prefill stay full-width in the text segment."""
    dtype, B, Hq, Hkv, L, r, cap_t = "bf16", 2, 8, 4, 500, 48, 10
    lengths = [500, 250]
    data = layer(B, Hq, Hkv, L, dtype, 37, lengths=lengths, mean_shift=1.5)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, lengths=lengths)
    lens_t = [3, 0]
    tdata = layer(B, Hq, Hkv, cap_t, dtype, 38, lengths=lens_t)
    seg = TextSeg(B, Hkv, cap_t, dtype, lens_t)
    seg.fill(tdata["K"], tdata["V"])
    for step in range(7):
        new = layer(B, Hq, Hkv, 1, dtype, 3700 + step)
        kn, vn = to_dev(new["k_new"], dtype), to_dev(new["v_new"], dtype)
        rk.rk_append_text(ctx, p.layout(), seg.arg(), kn, vn)
        torch.cuda.synchronize()
        Kh, Vh = seg.host()
        for b in range(B):
            assert np.array_equal(Kh[b, :, lens_t[b]], new["k_new"][b].astype(np.float64))
            assert np.array_equal(Vh[b, :, lens_t[b]], new["v_new"][b].astype(np.float64))
        lens_t = [x + 1 for x in lens_t]
        seg.max_len += 1
        assert seg.len.cpu().tolist() == lens_t
        got = decode_dual(ctx, p, to_dev(new["q"], dtype), seg.arg())
        check_out(got, oracle_dual(p, new["q"], lengths, seg, lens_t), dtype)
    assert seg.max_len == cap_t
    # host check refuses at capacity; on the device a full sequence is left alone when the bound is understated
    with pytest.raises(rk.RotateKError) as e:
        rk.rk_append_text(ctx, p.layout(), seg.arg(), kn, vn)
    assert e.value.status == rk.RK_ERR_CAPACITY
    before = seg.host()[0].copy()
    seg.max_len = 7
    rk.rk_append_text(ctx, p.layout(), seg.arg(), kn, vn)
    torch.cuda.synchronize()
    assert seg.len.cpu().tolist() == [10, 8]
    assert np.array_equal(seg.host()[0][0], before[0])
