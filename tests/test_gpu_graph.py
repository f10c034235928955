"""The per-token serving loop (rk_append + rk_decode_attn for every layer, or the fused
rk_append_decode_attn) captured once into a
HIP graph and replayed: the entry points allocate nothing, clear nothing with memsets and take the
caller's stream, so the caller's capture sees only kernel launches.  Every replay is checked
bit for bit against the same calls made eagerly on a second, identically prefilled set of caches,
with eager work and synchronisations between the replays; the last step is also checked against
the oracle."""
import numpy as np
import pytest
import torch

import paper_2605_19218_amd as rk

from gpu_util import D, DEV, Pipeline, to_dev, to_host
from test_gpu_parity import check_out, layer, oracle_decode, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = rk.rk_create(0)
    yield c
    rk.rk_destroy(c)


@pytest.mark.parametrize("fused", [False, True], ids=["two_calls", "fused_call"])
def test_decode_loop_under_graph_replay(ctx, fused):
    dtype, B, Hq, Hkv, L, r, NLAY, NSTEP = "bf16", 2, 8, 2, 700, 64, 3, 5
    lengths = [700, 350]
    cap = L + NSTEP + 1
    datas = [layer(B, Hq, Hkv, L, dtype, 60 + i, lengths=lengths, mean_shift=1.0) for i in range(NLAY)]
    eager = [run_prefill(ctx, d, B, Hq, Hkv, L, r, dtype, lengths=lengths, cap=cap) for d in datas]
    graph = [run_prefill(ctx, d, B, Hq, Hkv, L, r, dtype, lengths=lengths, cap=cap) for d in datas]
    steps = [[layer(B, Hq, Hkv, 1, dtype, 6000 + 10 * s + i) for i in range(NLAY)] for s in range(NSTEP)]
    td = torch.bfloat16
    kbuf = [torch.zeros(B, Hkv, D, device=DEV, dtype=td) for _ in range(NLAY)]
    vbuf = [torch.zeros(B, Hkv, D, device=DEV, dtype=td) for _ in range(NLAY)]
    qbuf = [torch.zeros(B, Hq, D, device=DEV, dtype=td) for _ in range(NLAY)]

    def one_step(pipes, stream=None):
        for i, p in enumerate(pipes):
            # the host bound covers every replay: L + NSTEP tokens at most
            lay = rk.Layout(B, Hq, Hkv, r, rk.RK_BF16, p.cap, L + NSTEP, seq_len=p.seq_len)
            before = rk.Layout(B, Hq, Hkv, r, rk.RK_BF16, p.cap, L + NSTEP - 1, seq_len=p.seq_len)
            if fused:
                rk.rk_append_decode_attn(ctx, before, kbuf[i], vbuf[i], qbuf[i], p.Rr, p.dmu, p.Kp, p.Vc, p.seq_len,
                                         0.0, p.out, ws[i], stream=stream)
                continue
            rk.rk_append(ctx, before, kbuf[i], vbuf[i], p.Rr, p.Kp, p.Vc, p.seq_len, stream=stream)
            rk.rk_decode_attn(ctx, lay, qbuf[i], p.Kp, p.Vc, p.Rr, p.dmu, 0.0, p.out, ws[i], stream=stream)

    lay0 = rk.Layout(B, Hq, Hkv, r, rk.RK_BF16, eager[0].cap, L + NSTEP, seq_len=eager[0].seq_len)
    ws = [torch.empty(rk.rk_decode_workspace_size(ctx, lay0), device=DEV, dtype=torch.uint8) for _ in range(NLAY)]

    def load_inputs(s):
        for i in range(NLAY):
            kbuf[i].copy_(to_dev(steps[s][i]["k_new"], dtype))
            vbuf[i].copy_(to_dev(steps[s][i]["v_new"], dtype))
            qbuf[i].copy_(to_dev(steps[s][i]["q"], dtype))

    # eager reference, step by step
    ref = []
    for s in range(NSTEP):
        load_inputs(s)
        one_step(eager)
        torch.cuda.synchronize()
        ref.append([to_host(p.out).copy() for p in eager])

    # capture one step on a side stream (all kernels have run once above, so nothing is set up lazily
    # inside the capture), then replay it NSTEP times
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    load_inputs(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        one_step(graph, stream=torch.cuda.current_stream())
    # the capture itself does not execute: the graph caches still hold the prefill state
    assert graph[0].seq_len.cpu().tolist() == lengths
    for s in range(NSTEP):
        load_inputs(s)                       # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i, p in enumerate(graph):
            assert np.array_equal(to_host(p.out), ref[s][i]), (s, i)
        assert graph[0].seq_len.cpu().tolist() == [n + s + 1 for n in lengths]
    for i, p in enumerate(graph):
        p.max_seq_len = L + NSTEP
        want = oracle_decode(p, steps[-1][i]["q"], [n + NSTEP for n in lengths])
        check_out(to_host(p.out), want, dtype)


def test_dual_fused_loop_under_graph_replay(ctx):
    """The paper's own decode loop (new tokens stay full-width in the text segment) through
    rk_append_text_decode_attn_dual: one captured step replayed, every replay bit for bit equal to
    the eager calls, text lengths advancing on the device, the last step checked against the oracle."""
    from test_gpu_dual import TextSeg, oracle_dual
    dtype, B, Hq, Hkv, L, r, NLAY, NSTEP, M0 = "bf16", 2, 8, 2, 700, 64, 2, 4, 5
    lengths, lens_t = [700, 350], [M0, 0]
    cap_t = M0 + NSTEP + 1
    datas = [layer(B, Hq, Hkv, L, dtype, 80 + i, lengths=lengths, mean_shift=1.0) for i in range(NLAY)]
    tdata = [layer(B, Hq, Hkv, cap_t, dtype, 85 + i, lengths=lens_t) for i in range(NLAY)]
    steps = [[layer(B, Hq, Hkv, 1, dtype, 8000 + 10 * s + i) for i in range(NLAY)] for s in range(NSTEP)]
    td = torch.bfloat16
    kbuf = [torch.zeros(B, Hkv, D, device=DEV, dtype=td) for _ in range(NLAY)]
    vbuf = [torch.zeros(B, Hkv, D, device=DEV, dtype=td) for _ in range(NLAY)]
    qbuf = [torch.zeros(B, Hq, D, device=DEV, dtype=td) for _ in range(NLAY)]

    def make_side():
        pipes = [run_prefill(ctx, d, B, Hq, Hkv, L, r, dtype, lengths=lengths) for d in datas]
        segs = []
        for i in range(NLAY):
            seg = TextSeg(B, Hkv, cap_t, dtype, lens_t)
            seg.fill(tdata[i]["K"], tdata[i]["V"])
            seg.max_len = cap_t - 1               # host bound before the append, good for every replay
            segs.append(seg)
        return pipes, segs
    eager, graph = make_side(), make_side()
    lay0 = eager[0][0].layout()
    ws = [torch.empty(rk.rk_decode_workspace_size(ctx, lay0), device=DEV, dtype=torch.uint8) for _ in range(NLAY)]

    def one_step(side, stream=None):
        for i, (p, seg) in enumerate(zip(*side)):
            rk.rk_append_text_decode_attn_dual(ctx, p.layout(), kbuf[i], vbuf[i], qbuf[i], p.Kp, p.Vc, p.Rr, p.dmu,
                                               seg.arg(), 0.0, p.out, ws[i], stream=stream)

    def load_inputs(s):
        for i in range(NLAY):
            kbuf[i].copy_(to_dev(steps[s][i]["k_new"], dtype))
            vbuf[i].copy_(to_dev(steps[s][i]["v_new"], dtype))
            qbuf[i].copy_(to_dev(steps[s][i]["q"], dtype))

    ref = []
    for s in range(NSTEP):
        load_inputs(s)
        one_step(eager)
        torch.cuda.synchronize()
        ref.append([to_host(p.out).copy() for p in eager[0]])
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    load_inputs(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        one_step(graph, stream=torch.cuda.current_stream())
    assert graph[1][0].len.cpu().tolist() == lens_t
    for s in range(NSTEP):
        load_inputs(s)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i, p in enumerate(graph[0]):
            assert np.array_equal(to_host(p.out), ref[s][i]), (s, i)
        assert graph[1][0].len.cpu().tolist() == [n + s + 1 for n in lens_t]
    final_t = [n + NSTEP for n in lens_t]
    for i, (p, seg) in enumerate(zip(*graph)):
        assert torch.equal(seg.k, eager[1][i].k) and torch.equal(seg.v, eager[1][i].v)
        want = oracle_dual(p, steps[-1][i]["q"], lengths, seg, final_t)
        check_out(to_host(p.out), want, dtype)
