#!/usr/bin/env python3
"""Benchmark of the RotateK hot path on one MI355X.

Headline workload ("C3"): one GQA attention layer, bf16, batch 8, 28 query heads over 4 KV
heads, head dim 128, 16384 cached tokens, r = 64 kept Key channels.  One step = one pass of
the whole path over one layer: fit (covariance, eigensolve, mask), compress (rotate + pack
16384 Keys), append one token, one decode-attention step.  Steps rotate over a ring of
distinct layers (several GB in total) so that every step streams its cache from HBM rather
than from the 256 MB last-level cache.  Inputs are seeded synthetic tensors already resident
in HBM.

Prints ONE JSON line.
  value      decode-attention achieved HBM bandwidth INSIDE the step: algorithmic bytes
             B*H_kv*L*(r+d)*2 / HIP-event time of the rk_decode_attn call in a second,
             instrumented pass of K steps (the event in front of the call costs the device
             5-6 idle microseconds, which this figure includes; ms_per_step comes from the
             first pass, which records nothing between its calls).
  roofline   the decode kernel itself: the same bytes / launch duration, HIP events around N
             back-to-back launches on the launch stream (what rocprofv3 --kernel-trace
             reports per launch), against the 8 TB/s datasheet peak and against the
             streaming-read rate measured in the same run (`stream_ceiling`).
  workloads  the other named configurations (LLaVA-shaped MHA layer; ragged batch of 16 with
             kept-token lists; one layer of the 32-layer L = 32768 workload with its decode loop),
             each stage timed back to back with its algorithmic bytes.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
D = 128


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--layers", type=int, default=8, help="distinct layer caches in the ring")
    ap.add_argument("--keep", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the decode sweep, dual path, token loops and solvers")
    ap.add_argument("--no-workloads", action="store_true", help="skip the other named configurations")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy a few times, so that a rocprofv3 --pmc run of this "
                         "command records FETCH_SIZE / WRITE_SIZE of a kernel with known traffic")
    return ap.parse_args()


def committed_traffic(kernel_tag):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc (FETCH_SIZE +
    WRITE_SIZE, calibrated against a plain copy); read from the committed summary, None if absent."""
    path = os.path.join(ROOT, "profiles", "pmc_hbm_traffic_C3.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch[%s]:" % kernel_tag):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (every unit of state is per "
              "(batch item, KV head), so more GPUs would each take a share of heads with no exchange)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_19218_amd as rk
    from rk_inputs import CONFIGS, f32_to_bf16_bits, make_layer, ragged_lengths, token_keep_lists

    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU fallback)"
    dev = "cuda:0"
    f32 = dict(device=dev, dtype=torch.float32)
    ctx = rk.rk_create(0)

    def to_bf16(x):
        bits = f32_to_bf16_bits(np.ascontiguousarray(x, dtype=np.float32)).view(np.int16)
        return torch.from_numpy(bits).to(dev).view(torch.bfloat16)

    def timed(fn, n, warm=3):
        """Mean microseconds per call of fn(i): HIP events on the launch stream around n back-to-back calls."""
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(warm + i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    def rate(nbytes, us):
        gbps = nbytes / (us * 1e-6) / 1e9
        return dict(us=us, GBps=gbps, frac_of_peak=gbps / HBM_PEAK_GBPS, algorithmic_bytes=int(nbytes))

    class LayerState:
        """Fit outputs and caches of one layer."""

        def __init__(self, B, Hq, Hkv, r, cap):
            kb, vb = rk.rk_cache_bytes(rk.Layout(B, Hq, Hkv, r, rk.RK_BF16, cap, cap))
            self.R = torch.empty(B, Hkv, D, D, **f32)
            self.lam = torch.empty(B, Hkv, D, **f32)
            self.mask = torch.empty(B, Hkv, D, device=dev, dtype=torch.uint8)
            self.keep = torch.empty(B, Hkv, r, device=dev, dtype=torch.int32)
            self.Rr = torch.empty(B, Hkv, D, r, **f32)
            self.mu = torch.empty(B, Hkv, D, **f32)
            self.dmu = torch.empty(B, Hkv, D, **f32)
            self.Kp = torch.zeros(kb, device=dev, dtype=torch.uint8)            # fragment-major caches
            self.Vc = torch.zeros(vb, device=dev, dtype=torch.uint8)
            self.seq_len = torch.zeros(B, device=dev, dtype=torch.int32)
            self.out = torch.empty(B, Hq, D, device=dev, dtype=torch.bfloat16)

        def fit_out(self):
            return rk.FitOut(self.R, self.lam, self.mask, self.keep, self.Rr, self.mu, self.dmu)

    # ======================================================================================
    # C3: the headline workload
    # ======================================================================================
    cfg = dict(CONFIGS["C3"])
    B, Hq, Hkv, L = cfg["batch"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["L"]
    r_main = args.keep
    cap = L + 64                                                # multiple of 32
    NL = args.layers

    t_gen = time.time()
    with ThreadPoolExecutor(max_workers=min(NL, 8)) as ex:
        host_layers = list(ex.map(lambda l: make_layer(cfg, layer=l), range(NL)))
    layers = []
    for hl in host_layers:
        layers.append(dict(K=to_bf16(hl["K"]), V=to_bf16(hl["V"]),          # [B,Hkv,L,D] prefill Keys / Values
                           q=to_bf16(hl["q"]), k_new=to_bf16(hl["k_new"]), v_new=to_bf16(hl["v_new"])))
    t_gen = time.time() - t_gen

    def alloc_state(r):
        return [LayerState(B, Hq, Hkv, r, cap) for _ in range(NL)]

    def layouts(r, st):
        fit_l = rk.Layout(B, Hq, Hkv, r, rk.RK_BF16, cap, L, seq_len=st.seq_len)
        dec_l = rk.Layout(B, Hq, Hkv, r, rk.RK_BF16, cap, L + 1, seq_len=st.seq_len)
        return fit_l, dec_l

    lay0 = rk.Layout(B, Hq, Hkv, 128, rk.RK_BF16, cap, L + 1)
    fit_ws = torch.empty(rk.rk_fit_workspace_size(lay0, L), device=dev, dtype=torch.uint8)
    dec_ws = torch.empty(rk.rk_decode_workspace_size(ctx, lay0) * 2, device=dev, dtype=torch.uint8)

    def do_fit(r, st, ly):
        rk.rk_fit_rotation(ctx, layouts(r, st)[0], rk.Rows(ly["K"], L), None, rk.RK_FIT_CENTER, st.fit_out(), fit_ws)

    def do_compress(r, st, ly, values=True):
        rk.rk_compress(ctx, layouts(r, st)[0], rk.Rows(ly["K"], L), st.Rr, st.Kp,
                       values=rk.Rows(ly["V"], L) if values else None, v_cache=st.Vc if values else None,
                       seq_len_out=st.seq_len)

    def do_append(r, st, ly):
        rk.rk_append(ctx, layouts(r, st)[0], ly["k_new"], ly["v_new"], st.Rr, st.Kp, st.Vc, st.seq_len)

    def do_decode(r, st, ly):
        rk.rk_decode_attn(ctx, layouts(r, st)[1], ly["q"], st.Kp, st.Vc, st.Rr, st.dmu, 0.0, st.out, dec_ws)

    STAGES = [("fit", do_fit), ("compress", do_compress), ("append", do_append), ("decode", do_decode)]
    state = alloc_state(r_main)

    def step(i, events=None):
        st, ly = state[i % NL], layers[i % NL]
        for s, (name, fn) in enumerate(STAGES):
            if events is not None:
                events[s].record()
            fn(r_main, st, ly)
        if events is not None:
            events[len(STAGES)].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # The timed region: K steps and nothing else.  An event recorded between two calls drains the device and the
    # kernel behind it starts 5-6 us later (rocprofv3 shows that idle gap after every record and none between
    # kernels of consecutive calls), so the per-stage events run in a second pass of K steps of their own.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(STAGES) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for i in range(args.steps):
        step(args.warmup + args.steps + i, evs[i])
    torch.cuda.synchronize()

    stage_us = {}
    for s, (name, _) in enumerate(STAGES):
        ts = sorted(e[s].elapsed_time(e[s + 1]) * 1e3 for e in evs)
        stage_us[name] = dict(mean=float(np.mean(ts)), median=float(ts[len(ts) // 2]),
                              p10=float(ts[len(ts) // 10]), p90=float(ts[(len(ts) * 9) // 10]))
    assert torch.isfinite(state[0].out.float()).all(), "decode output is not finite"

    def decode_bytes(r, Lc, B_=B, Hkv_=Hkv):
        return B_ * Hkv_ * Lc * (r + D) * 2

    dec_us = stage_us["decode"]["mean"]
    dec_gbps = decode_bytes(r_main, L + 1) / (dec_us * 1e-6) / 1e9
    n_splits, tps = rk.rk_decode_plan(ctx, layouts(r_main, state[0])[1])

    # ---- the streaming-read rate this device sustains, measured in this run ---------------------
    # (a) launches of exactly the decode's size, each on a different 201 MB region of a 3.2 GB buffer;
    # (b) one launch over the whole buffer.  Plain coalesced 16-byte streaming loads, no arithmetic.
    region = decode_bytes(r_main, L) // 4096 * 4096
    scratch = torch.empty(region * 16, device=dev, dtype=torch.uint8).random_(0, 255)
    us_a = timed(lambda i: rk.rk_stream_read(ctx, scratch[(i % 16) * region:], region), 64, warm=16)
    us_b = timed(lambda i: rk.rk_stream_read(ctx, scratch), 8, warm=2)
    ceiling = dict(per_launch_of_decode_size=rate(region, us_a), large_buffer=rate(scratch.numel(), us_b),
                   note="rk_stream_read: plain 16-byte streaming loads over a buffer, nothing kept; the first entry "
                        "reads %d bytes per launch (the decode's algorithmic bytes), back to back over 16 regions" % region)
    ceil_gbps = ceiling["per_launch_of_decode_size"]["GBps"]
    del scratch

    # ---- kernel-level figures, back to back over the ring ------------------------------------------
    def reset_lengths(r, stt):
        for i in range(NL):
            do_compress(r, stt[i], layers[i])

    def decode_b2b(r, stt):
        reset_lengths(r, stt)
        us = timed(lambda i: do_decode(r, stt[i % NL], layers[i % NL]), args.steps, warm=args.warmup)
        d = rate(decode_bytes(r, L), us)
        d["frac_of_stream_ceiling"] = d["GBps"] / ceil_gbps
        return d

    sweep = {str(r_main): decode_b2b(r_main, state)}
    main_b2b = sweep[str(r_main)]
    # compress: Alg. 1 step 14 moves K in and K~ out; the Value re-tiling is a cost of this build's cache layout
    k_only = timed(lambda i: do_compress(r_main, state[i % NL], layers[i % NL], values=False), args.steps, warm=4)
    k_and_v = timed(lambda i: do_compress(r_main, state[i % NL], layers[i % NL]), args.steps, warm=4)
    comp_bytes = B * Hkv * L * (D + r_main) * 2
    compress = dict(kernel=rate(comp_bytes, k_only), call_with_value_retiling=rate(comp_bytes, k_and_v),
                    layout_overhead_v_retile=dict(us=k_and_v - k_only, bytes_moved=int(B * Hkv * L * 2 * D * 2),
                                                  note="read V + write the tiled V: not part of Alg. 1 step 14, the price "
                                                       "of the fragment-major Value cache that the decode kernel streams"))
    fit_b2b_us = timed(lambda i: do_fit(r_main, state[i % NL], layers[i % NL]), 8, warm=2)

    if not args.no_sweep:
        for r in sorted(set(cfg["keep_sweep"]) | {128}):
            if r == r_main:
                continue
            stt = alloc_state(r)
            for i in range(NL):
                do_fit(r, stt[i], layers[i])
            sweep[str(r)] = decode_b2b(r, stt)
            del stt
            torch.cuda.empty_cache()
        sweep = dict(sorted(sweep.items(), key=lambda kv: int(kv[0])))

    # ---- dual-path decode (Alg. 2 steps 4-5): the same cache plus a full-width text segment ----------
    dual = None
    if not args.no_sweep:
        reset_lengths(r_main, state)
        by_len = {}
        for M in (64, 1024):                               # a prompt-sized segment, and a long generated answer
            tl = make_layer(dict(cfg, id=cfg["id"] + 500, L=M), 0)
            text = rk.Text(to_bf16(tl["K"]), to_bf16(tl["V"]), M,
                           torch.full((B,), M, device=dev, dtype=torch.int32), capacity=M)

            def do_dual(i):
                st, ly = state[i % NL], layers[i % NL]
                rk.rk_decode_attn_dual(ctx, layouts(r_main, st)[1], ly["q"], st.Kp, st.Vc, st.Rr, st.dmu, text, 0.0,
                                       st.out, dec_ws)
            by_len[M] = rate(decode_bytes(r_main, L) + B * Hkv * M * 2 * D * 2, timed(do_dual, args.steps, warm=args.warmup))
            del text
        dual = dict(text_tokens=64, us_per_step=by_len[64]["us"], GBps=by_len[64]["GBps"],
                    single_path_us=main_b2b["us"], text_tokens_1024_us_per_step=by_len[1024]["us"])

    # ---- the per-token serving loop (append + decode on every layer of the ring), eager and as a HIP graph ----
    loop = None
    if not args.no_sweep:
        NTOK = 16                                              # tokens generated per measurement (cap = L + 64)
        bound = L + 2 * NTOK + 2                               # host bound that covers warm-up, eager and replayed tokens

        def token_step(stream=None, fused=False):
            for i in range(NL):
                st, ly = state[i], layers[i]
                al = rk.Layout(B, Hq, Hkv, r_main, rk.RK_BF16, cap, bound - 1, seq_len=st.seq_len)
                dl = rk.Layout(B, Hq, Hkv, r_main, rk.RK_BF16, cap, bound, seq_len=st.seq_len)
                if fused:
                    rk.rk_append_decode_attn(ctx, al, ly["k_new"], ly["v_new"], ly["q"], st.Rr, st.dmu, st.Kp,
                                             st.Vc, st.seq_len, 0.0, st.out, dec_ws, stream=stream)
                    continue
                rk.rk_append(ctx, al, ly["k_new"], ly["v_new"], st.Rr, st.Kp, st.Vc, st.seq_len, stream=stream)
                rk.rk_decode_attn(ctx, dl, ly["q"], st.Kp, st.Vc, st.Rr, st.dmu, 0.0, st.out, dec_ws, stream=stream)

        def time_loop(fused):
            reset_lengths(r_main, state)
            token_step(fused=fused)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(NTOK):
                token_step(fused=fused)
            torch.cuda.synchronize()
            eager = (time.perf_counter() - t0) * 1e6 / (NTOK * NL)
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            with torch.cuda.graph(g, stream=side):
                token_step(stream=torch.cuda.current_stream(), fused=fused)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(NTOK - 1):
                g.replay()
            torch.cuda.synchronize()
            graph = (time.perf_counter() - t0) * 1e6 / ((NTOK - 1) * NL)
            assert int(state[0].seq_len[0]) == L + 2 * NTOK, "token loop lost count"
            del g
            return eager, graph
        eager_us, graph_us = time_loop(False)
        fused_eager_us, fused_graph_us = time_loop(True)
        loop = dict(layers=NL, tokens=NTOK, eager_us_per_layer=eager_us, graph_us_per_layer=graph_us,
                    fused_eager_us_per_layer=fused_eager_us, fused_graph_us_per_layer=fused_graph_us,
                    note="wall clock per layer of one generated token, host launch overhead included: "
                         "rk_append + rk_decode_attn against rk_append_decode_attn; "
                         "graph = one captured token step over the %d layers, replayed" % NL)

        # the paper's own decode loop: new tokens stay full-width in the text segment (Alg. 2 input K_pt)
        M0, CAP_T = 64, 128
        tl = make_layer(dict(cfg, id=cfg["id"] + 500, L=CAP_T), 0)
        texts = [rk.Text(to_bf16(tl["K"]), to_bf16(tl["V"]), CAP_T - 1,
                         torch.full((B,), M0, device=dev, dtype=torch.int32), capacity=CAP_T) for _ in range(NL)]
        reset_lengths(r_main, state)

        def text_step(fused):
            for i in range(NL):
                st, ly = state[i], layers[i]
                dl = layouts(r_main, st)[1]
                if fused:
                    rk.rk_append_text_decode_attn_dual(ctx, dl, ly["k_new"], ly["v_new"], ly["q"], st.Kp, st.Vc,
                                                       st.Rr, st.dmu, texts[i], 0.0, st.out, dec_ws)
                    continue
                rk.rk_append_text(ctx, dl, texts[i], ly["k_new"], ly["v_new"])
                texts[i].max_len += 1                              # host bound after the append
                rk.rk_decode_attn_dual(ctx, dl, ly["q"], st.Kp, st.Vc, st.Rr, st.dmu, texts[i], 0.0, st.out, dec_ws)
                texts[i].max_len -= 1
        res = {}
        for fused in (False, True):
            for t in texts:
                t.len.fill_(M0)
            text_step(fused)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(NTOK):
                text_step(fused)
            torch.cuda.synchronize()
            res[fused] = (time.perf_counter() - t0) * 1e6 / (NTOK * NL)
            assert int(texts[0].len[0]) == M0 + NTOK + 1, "text loop lost count"
        loop["dual_eager_us_per_layer"] = res[False]
        loop["dual_fused_eager_us_per_layer"] = res[True]
        loop["dual_note"] = ("rk_append_text + rk_decode_attn_dual against rk_append_text_decode_attn_dual, "
                             "text segment growing from %d rows" % M0)
        del texts

    # ---- the paper's default solver (Alg. 1 steps 6-13) against the full eigendecomposition ----
    solvers = None
    if not args.no_sweep:
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg["id"] * 7919 + 5)
        sub_status = torch.zeros(B, Hkv, device=dev, dtype=torch.int32)

        def fit_sub_us(k):
            v0 = torch.randn(B, Hkv, D, k, device=dev, dtype=torch.float32, generator=gen)
            Rr = torch.empty(B, Hkv, D, k, **f32)
            lay = rk.Layout(B, Hq, Hkv, k, rk.RK_BF16, cap, L)

            def call(i):
                st, ly = state[i % NL], layers[i % NL]
                rk.rk_fit_subspace(ctx, lay, rk.Rows(ly["K"], L), None, rk.RK_FIT_CENTER, v0, 5, 1e-6, Rr, st.mu,
                                   st.dmu, fit_ws, status=sub_status)
            us = timed(call, args.steps, warm=max(args.warmup, 1))
            assert not sub_status.any().item(), "subspace iteration met a non-positive pivot"
            return us
        solvers = dict(full_eigendecomposition_fit_us=stage_us["fit"]["mean"],
                       subspace_T5_fit_us=fit_sub_us(r_main), subspace_T5_k96_fit_us=fit_sub_us(96),
                       note="fit = covariance + solver; both in one rk_fit_* call, %d matrices of 128x128" % (B * Hkv))
        # the same two solvers with one matrix per compute unit: all NL layers of the ring in ONE call
        # (B * NL sequences of 1024 tokens each, so the covariance part stays small): a prefill that
        # defers the fit to its end can batch layers like this, and one launch then keeps the whole
        # chip busy instead of B * H_kv = 32 of its 256 compute units
        UB, LB = B * NL, 1024
        Kb = torch.stack([ly["K"][:, :, :LB] for ly in layers]).reshape(UB, Hkv, LB, D).contiguous()
        lb = rk.Layout(UB, Hq, Hkv, r_main, rk.RK_BF16, LB, LB)
        wsb = torch.empty(rk.rk_fit_workspace_size(lb, LB), device=dev, dtype=torch.uint8)
        ob = LayerState(UB, Hq, Hkv, r_main, LB)
        v0b = torch.randn(UB, Hkv, D, r_main, device=dev, dtype=torch.float32, generator=gen)
        stb = torch.zeros(UB, Hkv, device=dev, dtype=torch.int32)

        def fit_eig_batched(i):
            rk.rk_fit_rotation(ctx, lb, rk.Rows(Kb, LB), None, rk.RK_FIT_CENTER, ob.fit_out(), wsb)

        def fit_sub_batched(i):
            rk.rk_fit_subspace(ctx, lb, rk.Rows(Kb, LB), None, rk.RK_FIT_CENTER, v0b, 5, 1e-6, ob.Rr, ob.mu,
                               ob.dmu, wsb, status=stb)
        for name, fn in (("full_eigendecomposition", fit_eig_batched), ("subspace_T5", fit_sub_batched)):
            us = timed(fn, 4, warm=1)
            solvers[name + "_batched"] = dict(matrices=UB * Hkv, tokens_per_matrix=LB, fit_us=us,
                                              matrices_per_s=UB * Hkv / (us * 1e-6))
        assert not stb.any().item(), "subspace iteration met a non-positive pivot (batched)"
        del Kb, ob, wsb, v0b
        for i in range(NL):                                  # leave the ring as the eigen route made it
            do_fit(r_main, state[i], layers[i])
            do_compress(r_main, state[i], layers[i])

    # ======================================================================================
    # the other named configurations: device-generated inputs of the same recipe (low-rank + noise +
    # two outlier channels x10, N(0,1) Values and queries), every stage timed back to back
    # ======================================================================================
    workloads = None
    if not args.no_workloads:
        gen = torch.Generator(device=dev)
        gen.manual_seed(20260519)

        def synth_keys(Bw, Hw, Lw, rho):
            A = torch.randn(Bw, Hw, Lw, rho, generator=gen, **f32)
            Bm = torch.randn(Bw, Hw, rho, D, generator=gen, **f32)
            K = torch.matmul(A, Bm)
            del A
            K.add_(torch.randn(Bw, Hw, Lw, D, generator=gen, **f32), alpha=0.1)
            scale = torch.ones(Bw, Hw, 1, D, **f32)
            ch = torch.rand(Bw, Hw, D, generator=gen, device=dev).argsort(dim=-1)[..., :2]       # two distinct channels per head
            scale.scatter_(3, ch.unsqueeze(2), 10.0)
            return K.mul_(scale).to(torch.bfloat16)

        def synth_normal(*shape):
            return torch.randn(*shape, generator=gen, **f32).to(torch.bfloat16)

        def run_workload(name, Bw, Hqw, Hkvw, Lw, r, rho, n_layers, lengths=None, n_text=0, keep_frac=1.0,
                         decode_steps=0, reps=8, text_rows=0):
            """fit, compress and decode of one configuration over a ring of n_layers layers."""
            out = dict(batch=Bw, n_q_heads=Hqw, n_kv_heads=Hkvw, L=Lw, keep=r, ring_layers=n_layers)
            tok_idx = tok_off = None
            n_rows = np.full(Bw, Lw, np.int64)
            if lengths is not None:
                ti, to = token_keep_lists(CONFIGS["C4"]["id"], lengths, n_text=n_text, keep_frac=keep_frac)
                n_rows = np.diff(to)
                tok_idx, tok_off = torch.from_numpy(ti).to(dev), torch.from_numpy(to).to(dev)
                out["lengths"] = [int(x) for x in lengths]
                out["kept_tokens"] = [int(x) for x in n_rows]
            n_max = int(n_rows.max())
            capw = (n_max + decode_steps + 31) // 32 * 32
            ring = []
            for _ in range(n_layers):
                Kw = torch.cat([synth_keys(1, Hkvw, Lw, rho) for _ in range(Bw)])      # per batch item: bounds the fp32 temporaries
                Vw = torch.cat([synth_normal(1, Hkvw, Lw, D) for _ in range(Bw)])
                ring.append(dict(K=Kw, V=Vw, q=synth_normal(Bw, Hqw, D), k_new=synth_normal(Bw, Hkvw, D),
                                 v_new=synth_normal(Bw, Hkvw, D), st=LayerState(Bw, Hqw, Hkvw, r, capw)))
            layf = lambda ly, m: rk.Layout(Bw, Hqw, Hkvw, r, rk.RK_BF16, capw, m, seq_len=ly["st"].seq_len)
            rows = lambda t: rk.Rows(t, n_max, tok_idx=tok_idx, tok_off=tok_off)
            wsf = torch.empty(rk.rk_fit_workspace_size(layf(ring[0], n_max), n_max), device=dev, dtype=torch.uint8)
            wsd = torch.empty(rk.rk_decode_workspace_size(ctx, layf(ring[0], capw)), device=dev, dtype=torch.uint8)

            def fit(i):
                ly = ring[i % n_layers]
                rk.rk_fit_rotation(ctx, layf(ly, n_max), rows(ly["K"]), None, rk.RK_FIT_CENTER, ly["st"].fit_out(), wsf)

            def compress(i, values=True):
                ly = ring[i % n_layers]
                rk.rk_compress(ctx, layf(ly, n_max), rows(ly["K"]), ly["st"].Rr, ly["st"].Kp,
                               values=rows(ly["V"]) if values else None, v_cache=ly["st"].Vc if values else None,
                               seq_len_out=ly["st"].seq_len)

            def decode(i):
                ly = ring[i % n_layers]
                rk.rk_decode_attn(ctx, layf(ly, n_max), ly["q"], ly["st"].Kp, ly["st"].Vc, ly["st"].Rr, ly["st"].dmu,
                                  0.0, ly["st"].out, wsd)
            tokens = int(n_rows.sum())
            out["fit"] = dict(us=timed(fit, reps, warm=2), covariance_bytes=int(tokens * Hkvw * D * 2),
                              note="covariance over %d rows per KV head on average + eigensolve of %d matrices"
                                   % (tokens // Bw, Bw * Hkvw))
            out["compress_kernel"] = rate(tokens * Hkvw * (D + r) * 2, timed(lambda i: compress(i, False), reps, warm=2))
            out["compress_call_with_value_retiling"] = rate(tokens * Hkvw * (D + r) * 2, timed(compress, reps, warm=2))
            for i in range(n_layers):
                fit(i)
                compress(i)
            torch.cuda.synchronize()
            out["decode"] = rate(tokens * Hkvw * (r + D) * 2, timed(decode, 4 * reps, warm=n_layers))
            out["decode"]["frac_of_stream_ceiling"] = out["decode"]["GBps"] / ceil_gbps
            out["decode_plan"] = dict(zip(("n_splits", "tokens_per_split"), rk.rk_decode_plan(ctx, layf(ring[0], n_max))))
            assert torch.isfinite(ring[0]["st"].out.float()).all(), name
            if text_rows:
                # Alg. 2 in full: the same rotated cache plus a full-width text segment of text_rows rows per KV head
                text = rk.Text(synth_normal(Bw, Hkvw, text_rows, D), synth_normal(Bw, Hkvw, text_rows, D), text_rows,
                               torch.full((Bw,), text_rows, device=dev, dtype=torch.int32), capacity=text_rows)

                def decode_dual(i):
                    ly = ring[i % n_layers]
                    rk.rk_decode_attn_dual(ctx, layf(ly, n_max), ly["q"], ly["st"].Kp, ly["st"].Vc, ly["st"].Rr,
                                           ly["st"].dmu, text, 0.0, ly["st"].out, wsd)
                out["decode_dual"] = rate(tokens * Hkvw * (r + D) * 2 + Bw * Hkvw * text_rows * 2 * D * 2,
                                          timed(decode_dual, 4 * reps, warm=n_layers))
                out["decode_dual"]["text_rows"] = text_rows
                assert torch.isfinite(ring[0]["st"].out.float()).all(), name
                del text
            if decode_steps:
                # the decode loop with the frozen rotation: every step appends one token to every layer of the ring
                def loop_us(fused):
                    for i in range(n_layers):
                        compress(i)                                   # lengths back to n_max
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for s in range(decode_steps):
                        for ly in ring:
                            al, dl = layf(ly, n_max + s), layf(ly, n_max + s + 1)
                            st = ly["st"]
                            if fused:
                                rk.rk_append_decode_attn(ctx, al, ly["k_new"], ly["v_new"], ly["q"], st.Rr, st.dmu, st.Kp,
                                                         st.Vc, st.seq_len, 0.0, st.out, wsd)
                            else:
                                rk.rk_append(ctx, al, ly["k_new"], ly["v_new"], st.Rr, st.Kp, st.Vc, st.seq_len)
                                rk.rk_decode_attn(ctx, dl, ly["q"], st.Kp, st.Vc, st.Rr, st.dmu, 0.0, st.out, wsd)
                    torch.cuda.synchronize()
                    us = (time.perf_counter() - t0) * 1e6 / (decode_steps * n_layers)
                    assert ring[0]["st"].seq_len.cpu().tolist() == [n_max + decode_steps] * Bw, "decode loop lost count"
                    return us
                mean_tokens = tokens + Bw * (decode_steps + 1) / 2
                out["decode_loop"] = dict(steps=decode_steps,
                                          append_then_decode=rate(mean_tokens * Hkvw * (r + D) * 2, loop_us(False)),
                                          fused_append_decode=rate(mean_tokens * Hkvw * (r + D) * 2, loop_us(True)),
                                          note="wall clock per layer and generated token, host launch overhead included")
            del ring, wsf, wsd
            torch.cuda.empty_cache()
            return out

        c2, c4, c5 = CONFIGS["C2"], CONFIGS["C4"], CONFIGS["C5"]
        workloads = {}
        workloads["C2"] = run_workload("C2", c2["batch"], c2["n_q_heads"], c2["n_kv_heads"], c2["L"], c2["keep"], 16, 8, reps=16)
        # the same layer as the paper splits it: 2880 image tokens in the rotated cache, 64 prompt tokens full-width
        workloads["C2_dual"] = run_workload("C2_dual", c2["batch"], c2["n_q_heads"], c2["n_kv_heads"], c2["L"] - 64, c2["keep"],
                                            16, 8, reps=16, text_rows=64)
        workloads["C2"]["note"] = "LLaVA-NeXT-7B-shaped layer: one decode step is 36 MB, a launch-latency regime"
        lengths = ragged_lengths(c4["id"], c4["batch"], *c4["ragged"])
        workloads["C4"] = run_workload("C4", c4["batch"], c4["n_q_heads"], c4["n_kv_heads"], int(lengths.max()), c4["keep"], 16, 1,
                                       lengths=lengths, n_text=c4["n_text"], keep_frac=c4["token_keep"], reps=4)
        workloads["C4"]["note"] = ("joint token + channel pruning: ragged batch of 16, a seeded list keeps half of the visual rows; "
                                   "bytes are computed from the kept-token counts; one layer is 1.6 GB of cache")
        workloads["C5"] = run_workload("C5", c5["batch"], c5["n_q_heads"], c5["n_kv_heads"], c5["L"], c5["keep"],
                                       c5["rho_by_layer"](15), 4, decode_steps=c5["decode_steps"], reps=8)
        workloads["C5"]["note"] = ("one layer (of 32) of the long prefill: fit + compress at r = 48, then 128 decode steps with the "
                                   "frozen rotation over a ring of 4 such layers; a whole model multiplies every figure by 32")

    if args.calibration_copy:
        src = torch.empty(1 << 30, device=dev, dtype=torch.uint8).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the CPU oracle on the same workload (bounded sample) -------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from paper_2605_19218_amd.torch_harness import to_host
        st, ly, hl = state[0], layers[0], host_layers[0]
        do_compress(r_main, st, ly)
        k_rows = torch.empty(B, Hkv, cap, r_main, device=dev, dtype=torch.bfloat16)
        rk.rk_unpack_cache(ctx, layouts(r_main, st)[0], st.Kp, None, k_rows, None)
        torch.cuda.synchronize()
        Kt = to_host(k_rows[:, :, :L])
        Vh = to_host(ly["V"])
        Rr, dmu = to_host(st.Rr), to_host(st.dmu)
        qh = hl["q"].astype(np.float64)
        t = time.perf_counter()
        o = oracle.decode_batch(qh, Kt, Vh, Rr, dmu)
        t_dec = time.perf_counter() - t
        assert np.isfinite(o).all()
        # sanity only (exact parity is the tests' job): the GPU's decode of the same L tokens
        do_decode(r_main, st, ly)
        torch.cuda.synchronize()
        assert np.abs(to_host(st.out) - o).max() <= 2e-2, "GPU decode and oracle disagree"
        Kh = hl["K"].reshape(B * Hkv, L, D).astype(np.float64)  # all 32 KV heads
        t = time.perf_counter()
        f = oracle.fit_batch(Kh, r_main)
        t_fit = time.perf_counter() - t
        t = time.perf_counter()
        oracle.compress_batch(Kh, f["Rr"], rounding="bf16")
        t_cmp = time.perf_counter() - t
        cpu = dict(value=decode_bytes(r_main, L) / t_dec / 1e9, unit="GB/s", cores=oracle.num_threads(),
                   kind="oracle",
                   sample=("one whole step of the workload, no sampling: fp64 oracle decode step (%d query heads, "
                           "L=%d): %.3f s; fit of all %d KV heads: %.3f s; compress of all %d heads: %.3f s; "
                           "value = decode bytes / decode time")
                   % (B * Hq, L, t_dec, B * Hkv, t_fit, B * Hkv, t_cmp))

    fused = n_splits >= 2 and (B * Hkv) % 8 == 0
    res = {
        "metric": "decode_attn_hbm_GBps", "value": dec_gbps, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (seeded low-rank + outlier Keys, N(0,1) Values and queries)",
        "config": {"workload": "C3: GQA layer bf16, B=8, 28 q heads / 4 KV heads, d=128, L=16384, r=%d; step = "
                               "fit + compress + append + decode over a ring of %d layers" % (r_main, NL),
                   "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "L": L, "keep": r_main,
                   "ring_layers": NL, "decode_splits": n_splits, "tokens_per_split": tps},
        "us_per_decode_step": dec_us,
        "value_note": "HIP-event time of the rk_decode_attn call inside an instrumented step: it includes the 5-6 us the "
                      "device idles after the event recorded in front of the call; the kernel itself takes the same time "
                      "there as back to back (roofline.duration_us; profiles/kernel_trace_step_C3.md)",
        "stages_us": stage_us,
        "roofline": {"bound": "hbm", "achieved": main_b2b["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": main_b2b["frac_of_peak"], "traffic": committed_traffic("decode_split_mfma<64>"),
                     "kernel": ("decode_split_mfma<64> with the split-K merge folded in (one launch per rk_decode_attn call)"
                                if fused else "decode_split_mfma<64> + decode_merge (one rk_decode_attn call)"),
                     "duration_us": main_b2b["us"],
                     "measured": "HIP events on the launch stream around %d back-to-back launches over the ring" % args.steps,
                     "algorithmic_bytes": decode_bytes(r_main, L),
                     "stream_ceiling_GBps": ceil_gbps, "frac_of_stream_ceiling": main_b2b["frac_of_stream_ceiling"],
                     "in_step": {"us": dec_us, "GBps": dec_gbps, "frac": dec_gbps / HBM_PEAK_GBPS,
                                 "frac_of_stream_ceiling": dec_gbps / ceil_gbps}},
        "stream_ceiling": ceiling,
        "compress_GBps": compress["kernel"]["GBps"],
        "roofline_compress": {"bound": "hbm", "achieved": compress["kernel"]["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": compress["kernel"]["frac_of_peak"],
                              "frac_of_stream_ceiling": compress["kernel"]["GBps"] / ceil_gbps,
                              "algorithmic_bytes": comp_bytes, "kernel": "compress_mfma<64> (K read + K~ written)",
                              "duration_us": compress["kernel"]["us"],
                              "call_with_value_retiling": compress["call_with_value_retiling"],
                              "layout_overhead_v_retile": compress["layout_overhead_v_retile"]},
        "fit_us_back_to_back": fit_b2b_us,
        "decode_only_sweep": sweep,
        "dual_path_decode": dual,
        "fit_solvers": solvers,
        "token_loop": loop,
        "workloads": workloads,
        "cpu_baseline": cpu,
        "setup_s": t_gen,
    }
    print(json.dumps(res))
    rk.rk_destroy(ctx)


if __name__ == "__main__":
    main()
