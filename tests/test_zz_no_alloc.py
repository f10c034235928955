"""rk_decode_attn_static (the entry point for callers that cannot allocate: the split-K partials live in
a scratch array built into the library) against rk_decode_attn on the same inputs, through the C ABI:
two calls in a row on one context, the second with a smaller input, then the oracle."""
import numpy as np
import pytest
import torch

import paper_2605_19218_amd as rk

from gpu_util import DEV, to_dev, to_host
from test_gpu_parity import check_out, layer, oracle_decode, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


def decode_static(ctx, p, q_dev):
    out = torch.zeros_like(p.out)
    rk.rk_decode_attn_static(ctx, p.layout(), q_dev, p.Kp, p.Vc, p.Rr, p.dmu, 0.0, out)
    torch.cuda.synchronize()
    return to_host(out)


def test_static_scratch_matches_workspace_call(ctx):
    dtype = "bf16"
    # first call: GQA 7, ragged, several splits; second call: a smaller batch, shorter cache, other r
    shapes = [(2, 14, 2, 5000, [5000, 1234], 64), (1, 8, 2, 700, [700], 48)]
    for i, (B, Hq, Hkv, L, lengths, r) in enumerate(shapes):
        data = layer(B, Hq, Hkv, L, dtype, 91 + i, lengths=lengths, mean_shift=1.5)
        p = run_prefill(ctx, data, B, Hq, Hkv, L, r, dtype, lengths=lengths)
        n_splits, _ = rk.rk_decode_plan(ctx, p.layout())
        assert rk.rk_decode_workspace_size(ctx, p.layout()) <= rk.RK_STATIC_SCRATCH_BYTES
        if i == 0:
            assert n_splits > 1                          # the scratch array really carries partials
        q = to_dev(data["q"], dtype)
        got = decode_static(ctx, p, q)
        want = p.decode(q)                               # rk_decode_attn with a caller workspace
        assert np.array_equal(got, want)                 # same kernels, same merge order: identical
        check_out(got, oracle_decode(p, data["q"], lengths), dtype)
    # a single-split plan goes through the same entry point (nothing is staged then)
    B, Hq, Hkv, L, r = 1, 4, 2, 200, 32
    data = layer(B, Hq, Hkv, L, "f32", 93)
    p = run_prefill(ctx, data, B, Hq, Hkv, L, r, "f32")
    q = to_dev(data["q"], "f32")
    assert np.array_equal(decode_static(ctx, p, q), p.decode(q))


def test_static_scratch_refuses_oversized_shape(ctx):
    """A shape whose partials exceed the built-in array is refused on the host; nothing runs."""
    lay = rk.Layout(4096, 64, 64, 64, rk.RK_BF16, 1 << 16, 1 << 16,
                    seq_len=torch.zeros(4096, device=DEV, dtype=torch.int32))
    assert rk.rk_decode_workspace_size(ctx, lay) > rk.RK_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, device=DEV, dtype=torch.bfloat16)
    with pytest.raises(rk.RotateKError) as e:
        rk.rk_decode_attn_static(ctx, lay, dummy, dummy, dummy, dummy.float(), None, 0.0, dummy)
    assert e.value.status == rk.RK_ERR_WORKSPACE
    assert "scratch" in str(e.value)
