#!/usr/bin/env python3
"""Benchmark of the binary-codebook linear layer on one MI355X.

Workload (BASELINE.json: "btc_gemv effective weight GB/s + us/call (13B shapes,
0.8-bit); GEMM TFLOP/s"): the seven linear projections of a LLaMA-2-13B decoder
layer (4 x 5120x5120, 2 x 13824x5120, 1 x 5120x13824) stored at v=10, K=256
(8-bit indices, 0.8 bit/weight), Zipf(1.1) indices, batch-1 fp16 activations.

One STEP = one decoder layer = 7 btc_gemv calls.  Consecutive steps walk
through `--layers` distinct copies of the packed weights (40 copies = 1.27 GB,
five times the 256 MB last-level cache), so every call streams its indices from
HBM ("cold").  value = algorithmic bytes of a step / time of a step.  All
inputs are resident in HBM before the timed region.  The launches of one
sweep over all copies are captured once in a HIP graph (the calls still go
through the C ABI, which only enqueues kernels) so that Python's per-call
overhead is not what is timed; --mode stream times plain per-call launches.

Also reported: prefill btc_gemm TFLOP/s on the same shapes (M = --gemm-m and
512), decode timings of the 7B shapes at batch 1/4/16 and of a 70B-shaped
layer at 1.11/0.9/0.7 bit, a roofline object for the GEMV, and the CPU oracle
timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes of one step (7 calls) measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a
# 256 MiB copy (profiles/gemv_13b_hbm_traffic.md): 37.1 MB fetched + 5.5 MB written.
HBM_TRAFFIC_PER_STEP = 45.2e6

SHAPES_13B = [(5120, 5120, 4), (13824, 5120, 2), (5120, 13824, 1)]   # (out, in, count per layer)
V, K = 10, 256


def gemv_bytes(s, batch, y_bytes=2):
    """Algorithmic bytes of one call: index stream + alpha, mu + x + y + codebook."""
    return s.out * s.words_per_row * 4 + s.out * 8 + batch * s.in_ * 2 + batch * s.out * y_bytes + (1 << s.b) * 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--layers", type=int, default=40, help="distinct weight copies walked by consecutive steps")
    ap.add_argument("--mode", choices=["graph", "stream"], default="graph")
    ap.add_argument("--gemm-m", type=int, default=2048)
    ap.add_argument("--gemm-iters", type=int, default=10)
    ap.add_argument("--no-gemm", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-transform", action="store_true", help="skip the btc_transform timings")
    ap.add_argument("--no-other", action="store_true", help="skip the 7B (batch 1/4/16) and 70B decode sweeps")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three 256 MiB device-to-device copies (reference for FETCH_SIZE/WRITE_SIZE) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); nothing here uses a second GPU", file=sys.stderr)
        sys.exit(2)

    import torch
    import btc_synth as S
    import paper_2506_12040_amd as B

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.copy_calibration:
        a = torch.full((256 << 20,), 1, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": 256 << 20, "copies": 3}))
        return
    B.lib()  # raises if the HIP library was not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # ---- one seeded layer per shape, packed on the GPU through btc_pack
    t_setup = time.time()
    protos = []
    for (out, n_in, count) in SHAPES_13B:
        layer, x = S.make_case(0, out, n_in, V, K, 1, dist="zipf")
        s = B.btc_shape_init(out, n_in, V, K)
        idx_d = torch.from_numpy(layer.idx).to(dev)
        packed = torch.empty(out * s.words_per_row, dtype=torch.int32, device=dev)
        ws = torch.zeros(64, dtype=torch.uint8, device=dev)
        B.btc_pack(s, idx_d, packed, ws)
        cb = np.zeros(1 << s.b, dtype=np.uint32)
        cb[:K] = layer.codebook
        protos.append(dict(s=s, layer=layer, count=count, packed=packed.view(out, s.words_per_row),
                           codebook=torch.from_numpy(cb.view(np.int32)).to(dev),
                           alpha=torch.from_numpy(layer.alpha).to(dev), mu=torch.from_numpy(layer.mu).to(dev),
                           x=torch.from_numpy(x.view(np.int16)).to(dev), x_host=x))
        del idx_d
    # distinct copies: copy c of a matrix is the prototype with its rows rotated by a copy-specific offset
    calls_per_layer = []
    for L in range(args.layers):
        calls = []
        for p in protos:
            for r in range(p["count"]):
                shift = (L * 7 + r * 3 + 1) * 37 % p["s"].out
                calls.append(dict(p=p, packed=torch.roll(p["packed"], shifts=shift, dims=0).contiguous(),
                                  y=torch.empty(p["s"].out, dtype=torch.float16, device=dev)))
        calls_per_layer.append(calls)
    ws = torch.zeros(max(B.btc_workspace_bytes(p["s"], 1, False) for p in protos), dtype=torch.uint8, device=dev)
    n_calls = len(calls_per_layer[0])
    step_bytes = sum(gemv_bytes(c["p"]["s"], 1) for c in calls_per_layer[0])
    total_weight_bytes = step_bytes * args.layers
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    def run_layer(L):
        for c in calls_per_layer[L]:
            p = c["p"]
            B.btc_gemv(p["s"], c["packed"], p["codebook"], p["alpha"], p["mu"], p["x"], 1, c["y"], B.BTC_F16, ws)

    # ---- warmup
    for i in range(max(args.warmup, 1)):
        run_layer(i % args.layers)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` layers
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.mode == "graph":
        full_sweeps, rest = divmod(args.steps, args.layers)
        g_full = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_full):
            for L in range(args.layers):
                run_layer(L)
        g_rest = None
        if rest:
            g_rest = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_rest):
                for L in range(rest):
                    run_layer(L)
        g_full.replay()
        torch.cuda.synchronize()
        start.record()
        for _ in range(full_sweeps):
            g_full.replay()
        if g_rest is not None:
            g_rest.replay()
        stop.record()
    else:
        torch.cuda.synchronize()
        start.record()
        for i in range(args.steps):
            run_layer(i % args.layers)
        stop.record()
    torch.cuda.synchronize()
    ms_total = start.elapsed_time(stop)
    ms_per_step = ms_total / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    us_per_call = ms_per_step * 1e3 / n_calls
    fp16_equiv = sum(2 * c["p"]["s"].out * c["p"]["s"].in_ for c in calls_per_layer[0]) / (ms_per_step * 1e-3) / 1e9

    # per-shape timing (cold, rotating through the copies), events on the launch stream
    per_shape = {}
    for si, p in enumerate(protos):
        mats = [c for calls in calls_per_layer for c in calls if c["p"] is p]
        reps = max(1, 200 // len(mats))
        gs = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gs):
            for c in mats:
                B.btc_gemv(p["s"], c["packed"], p["codebook"], p["alpha"], p["mu"], p["x"], 1, c["y"], B.BTC_F16, ws)
        gs.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            gs.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * len(mats))
        by = gemv_bytes(p["s"], 1)
        per_shape[f"{p['s'].out}x{p['s'].in_}"] = dict(us_per_call=round(us, 3), bytes=by,
                                                        eff_GBps=round(by / us / 1e3, 1),
                                                        frac_hbm=round(by / us / 1e3 / HBM_PEAK_GBS, 4))

    # ---- the other decode configurations of the benchmark spec (timing only; random index words of the
    # right shape, >= 1 GiB of distinct copies per shape so that every call streams from HBM)
    other = None
    if not args.no_other:
        other = {}

        def time_gemv(out_, in_, v_, K_, batch, reps_target=120):
            s2 = B.btc_shape_init(out_, in_, v_, K_)
            nbytes = out_ * s2.words_per_row * 4
            ncopies = int(min(64, max(8, -(-(1 << 30) // nbytes))))
            proto = torch.randint(0, 2**31 - 1, (out_, s2.words_per_row), dtype=torch.int32, device=dev)
            copies = [torch.roll(proto, shifts=(i * 37 + 1) % out_, dims=0).contiguous() for i in range(ncopies)]
            cb2 = torch.randint(0, 1 << v_, (1 << s2.b,), dtype=torch.int32, device=dev)
            al2 = torch.rand(out_, device=dev) * 0.02
            mu2 = torch.rand(out_, device=dev) * 0.002
            x2 = torch.randn(batch, in_, device=dev).half()
            y2 = torch.empty(batch, out_, dtype=torch.float16, device=dev)
            ws2 = torch.zeros(B.btc_workspace_bytes(s2, batch, False), dtype=torch.uint8, device=dev)
            for c in copies:
                B.btc_gemv(s2, c, cb2, al2, mu2, x2, batch, y2, B.BTC_F16, ws2)
            torch.cuda.synchronize()
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                for c in copies:
                    B.btc_gemv(s2, c, cb2, al2, mu2, x2, batch, y2, B.BTC_F16, ws2)
            g2.replay()
            torch.cuda.synchronize()
            reps = max(1, reps_target // ncopies)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                g2.replay()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (reps * ncopies)
            by = gemv_bytes(s2, batch)
            del copies, proto
            return dict(us_per_call=round(us, 2), eff_GBps=round(by / us / 1e3, 1),
                        frac_hbm=round(by / us / 1e3 / HBM_PEAK_GBS, 4))

        seven = {}
        for (o, i) in [(4096, 4096), (11008, 4096), (4096, 11008)]:
            seven[f"{o}x{i}"] = {f"batch{b}": time_gemv(o, i, 10, 512, b) for b in (1, 4, 16)}
        other["llama2-7b v=10 K=512 (0.9 bit)"] = seven
        for (v_, K_, tag) in [(9, 1024, "1.11 bit"), (10, 512, "0.9 bit"), (10, 128, "0.7 bit")]:
            per, layer_us, layer_bytes = {}, 0.0, 0
            for (o, i, cnt) in [(8192, 8192, 2), (1024, 8192, 2), (28672, 8192, 2), (8192, 28672, 1)]:
                r = time_gemv(o, i, v_, K_, 1, reps_target=60)
                per[f"{o}x{i}"] = r
                layer_us += cnt * r["us_per_call"]
                layer_bytes += cnt * gemv_bytes(B.btc_shape_init(o, i, v_, K_), 1)
            other[f"llama2-70b v={v_} K={K_} ({tag})"] = dict(
                per_shape=per, layer_us=round(layer_us, 1), layer_eff_GBps=round(layer_bytes / layer_us / 1e3, 1),
                layer_frac_hbm=round(layer_bytes / layer_us / 1e3 / HBM_PEAK_GBS, 4))
        # independent projections (q, k, v of one layer) on three streams, one graph per stream
        p0 = protos[0]
        mats = [c for calls in calls_per_layer for c in calls if c["p"] is p0][:120]
        streams = [torch.cuda.Stream() for _ in range(3)]
        graphs = []
        wss = [torch.zeros_like(ws) for _ in streams]
        for si, stq in enumerate(streams):
            gq = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gq, stream=stq):
                for c in mats[si::3]:
                    B.btc_gemv(p0["s"], c["packed"], p0["codebook"], p0["alpha"], p0["mu"], p0["x"], 1, c["y"],
                               B.BTC_F16, wss[si])
            graphs.append(gq)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            for gq, stq in zip(graphs, streams):
                with torch.cuda.stream(stq):
                    gq.replay()
        torch.cuda.synchronize()
        other["three_streams_5120x5120"] = dict(
            us_per_call=round((time.perf_counter() - t0) * 1e6 / (10 * len(mats)), 2),
            note="independent calls (as q, k, v of one layer) replayed from one graph per stream; host-timed")

        # The paper's own latency comparison: its MLP layer 8192 x 28672 against the dense fp16
        # product of the stock PyTorch build, for M = batch x sequence length (Section 5.3).  Here: torch's
        # fp16/bf16 matmul on this GPU (a library call, timed the same way: cold, rotating copies).
        def time_dense(out_, in_, M, dt):
            ncopies = 3                                    # 3 x 470 MB: more than the last-level cache holds
            Ws = [torch.randn(out_, in_, device=dev, dtype=dt) for _ in range(ncopies)]
            xd = torch.randn(M, in_, device=dev, dtype=dt)
            for w in Ws:
                torch.matmul(xd, w.t())
            torch.cuda.synchronize()
            reps = 8 if M <= 16 else 2
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                for w in Ws:
                    torch.matmul(xd, w.t())
            e1.record()
            torch.cuda.synchronize()
            del Ws
            return e0.elapsed_time(e1) * 1e3 / (reps * ncopies)

        def time_gemm(out_, in_, v_, K_, M):
            s2 = B.btc_shape_init(out_, in_, v_, K_)
            pk = torch.randint(0, 2**31 - 1, (out_, s2.words_per_row), dtype=torch.int32, device=dev)
            cb2 = torch.randint(0, 1 << v_, (1 << s2.b,), dtype=torch.int32, device=dev)
            al2 = torch.rand(out_, device=dev) * 0.02
            mu2 = torch.rand(out_, device=dev) * 0.002
            X2 = torch.randn(M, in_, device=dev).bfloat16()
            Y2 = torch.empty(M, out_, dtype=torch.bfloat16, device=dev)
            ws2 = torch.zeros(B.btc_workspace_bytes(s2, M, True), dtype=torch.uint8, device=dev)
            f = lambda: B.btc_gemm(s2, pk, cb2, al2, mu2, X2, B.BTC_BF16, M, Y2, B.BTC_BF16, ws2)
            f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(4):
                f()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / 4

        mlp = {}
        o_, i_ = 8192, 28672
        for M in (1, 16):
            dense_us = time_dense(o_, i_, M, torch.float16)
            row = {"torch_fp16_us": round(dense_us, 1)}
            for (v_, K_, tag) in [(10, 512, "0.9 bit"), (10, 256, "0.8 bit"), (10, 128, "0.7 bit")]:
                us = time_gemv(o_, i_, v_, K_, M, reps_target=40)["us_per_call"]
                row[tag] = dict(us=us, speedup_over_fp16=round(dense_us / us, 2))
            mlp[f"M{M}"] = row
        for M in (32, 64, 96, 128, 256, 512, 2048):        # btc_gemm, bf16 activations
            dense_us = time_dense(o_, i_, M, torch.bfloat16)
            us = time_gemm(o_, i_, 10, 256, M)
            mlp[f"M{M}"] = {"torch_bf16_us": round(dense_us, 1),
                            "0.8 bit": dict(us=round(us, 1), speedup_over_bf16=round(dense_us / us, 2),
                                            tflops=round(2.0 * M * o_ * i_ / us / 1e6, 1))}
        other["mlp_8192x28672_vs_dense_torch"] = mlp

    # ---- prefill GEMM on the same shapes (btc_gemm = one contraction kernel per call, plus a second pass when the call is split along k)
    gemm = None
    if not args.no_gemm:
        gemm = {}
        for M in sorted({args.gemm_m, 512}, reverse=True):
            per, tot_flop, tot_ms = {}, 0.0, 0.0
            for p in protos:
                s = p["s"]
                rng = np.random.Generator(np.random.PCG64(0))
                Xb = S.draw_x(rng, M, s.in_, "bf16")
                X = torch.from_numpy(Xb.view(np.int16)).to(dev)
                Y = torch.empty(M * s.out, dtype=torch.float32, device=dev)
                wsg = torch.zeros(B.btc_workspace_bytes(s, M, True), dtype=torch.uint8, device=dev)
                call = lambda: B.btc_gemm(s, p["packed"], p["codebook"], p["alpha"], p["mu"], X, B.BTC_BF16, M, Y,
                                          B.BTC_F32, wsg)
                call()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(args.gemm_iters):
                    call()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / args.gemm_iters
                flop = 2.0 * M * s.out * s.in_
                per[f"{s.out}x{s.in_}"] = dict(ms=round(ms, 4), tflops=round(flop / ms / 1e9, 1))
                tot_flop += flop * p["count"]
                tot_ms += ms * p["count"]
                del X, Y
            tf = tot_flop / tot_ms / 1e9
            gemm[f"M{M}"] = dict(M=M, x_dtype="bf16", y_dtype="f32", per_shape=per, layer_tflops=round(tf, 1),
                                 frac_mfma_peak=round(tf / MFMA_BF16_PEAK_TFLOPS, 4))

    # ---- the online activation transform in front of the layer (btc_transform), on the two input widths of
    # the 13B layer: decode rows from a captured graph of 20 launches, prefill rows event-timed
    transform = None
    if not args.no_transform:
        transform = {}
        for (n1, n2) in [(64, 80), (108, 128)]:
            n = n1 * n2
            bits, P1, P2 = S.draw_transform(0, n1, n2)
            bits_d = torch.from_numpy(bits.view(np.int32)).to(dev)
            P1_d, P2_d = torch.from_numpy(P1).to(dev), torch.from_numpy(P2).to(dev)
            row = {}
            for (M, kind) in [(1, "f16"), (16, "f16"), (2048, "bf16")]:
                tdt, bdt = (torch.float16, B.BTC_F16) if kind == "f16" else (torch.bfloat16, B.BTC_BF16)
                X = torch.from_numpy(S.draw_x(np.random.Generator(np.random.PCG64(1)), M, n, kind).view(np.int16)).to(dev)
                Y = torch.empty(M * n, dtype=tdt, device=dev)
                call = lambda: B.btc_transform(X, bdt, M, n1, n2, bits_d, P1_d, P2_d, Y, bdt)
                call()
                torch.cuda.synchronize()
                reps = 20 if M <= 16 else 5
                if M <= 16:
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        for _ in range(reps):
                            call()
                    run = g.replay
                else:
                    def run():
                        for _ in range(reps):
                            call()
                run()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(5):
                    run()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / (5 * reps)
                flop = 2.0 * M * n * (n1 + n2)
                nbytes = 2.0 * M * n * 2 + 4.0 * (n1 * n1 + n2 * n2) + n / 8
                row[f"M{M}"] = dict(us=round(us, 2), tflops=round(flop / us / 1e6, 2),
                                    GBps=round(nbytes / us / 1e3, 1), frac_hbm=round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                                    engine="fp32 vector ALU" if M <= 16 else "bf16 matrix cores, 2-part operands (16-bit output)")
            transform[f"n={n} ({n1}x{n2})"] = row
        # one decoder layer at decode with its four transforms in place (the inputs of q/k/v, of o, of gate/up
        # and of down), cold weights, one graph over all layer copies: what the transform adds to the headline step
        tr = {}
        for (n1, n2) in [(64, 80), (108, 128)]:
            bits, P1, P2 = S.draw_transform(0, n1, n2)
            tr[n1 * n2] = (n1, n2, torch.from_numpy(bits.view(np.int32)).to(dev), torch.from_numpy(P1).to(dev),
                           torch.from_numpy(P2).to(dev), torch.empty(n1 * n2, dtype=torch.float16, device=dev))

        def run_layer_t(L):
            for ci, c in enumerate(calls_per_layer[L]):
                p = c["p"]
                n1, n2, bd, p1d, p2d, xt = tr[p["s"].in_]
                if ci in (0, 3, 4, 6):
                    B.btc_transform(p["x"], B.BTC_F16, 1, n1, n2, bd, p1d, p2d, xt, B.BTC_F16)
                B.btc_gemv(p["s"], c["packed"], p["codebook"], p["alpha"], p["mu"], xt, 1, c["y"], B.BTC_F16, ws)

        run_layer_t(0)
        torch.cuda.synchronize()
        gt = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gt):
            for L in range(args.layers):
                run_layer_t(L)
        gt.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            gt.replay()
        e1.record()
        torch.cuda.synchronize()
        transform["decoder_layer_decode_with_4_transforms_us"] = round(e0.elapsed_time(e1) * 1e3 / (5 * args.layers), 2)
        transform["decoder_layer_decode_without_us"] = round(ms_per_step * 1e3, 2)

    # ---- E-step of the codebook clustering (btc_assign): the length-10 vectors of a 5120 x 5120 and of a
    # 13824 x 5120 sign matrix against 256 centroids; a setting with long vectors (no pattern table)
    assign = None
    if not args.no_transform:
        assign = {}
        for (tag, N, v_, K_) in [("5120x5120 v=10 K=256", 5120 * 512, 10, 256), ("13824x5120 v=10 K=256", 13824 * 512, 10, 256),
                                 ("4096x4096 v=16 K=4096", 4096 * 256, 16, 4096)]:
            g = torch.Generator(device=dev)
            g.manual_seed(0)
            vec = torch.randint(0, 2 ** v_, (N,), dtype=torch.int32, device=dev, generator=g)
            cbk = torch.randint(0, 2 ** v_, (K_,), dtype=torch.int32, device=dev, generator=g)
            zz = torch.empty(N, dtype=torch.int32, device=dev)
            dd = torch.empty(N, dtype=torch.int32, device=dev)
            call = lambda: B.btc_assign(vec, N, v_, cbk, K_, zz, dd)
            call()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                call()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 5
            table = v_ <= 12 and N >= (64 << v_)
            row = dict(us=round(us, 1), vectors_per_s=round(N / us * 1e6, -6), GBps=round(12.0 * N / us / 1e3, 1))
            if table:
                row.update(route="pattern table in LDS", frac_hbm=round(12.0 * N / us / 1e3 / HBM_PEAK_GBS, 4))
            else:   # xor, bit count, shift-or, minimum per (vector, centroid) pair on 256 x 64 lanes at 2.4 GHz
                row.update(route="all pairs", lane_ops_per_s=round(4.0 * N * K_ / us * 1e6, -9),
                           frac_alu=round(4.0 * N * K_ / us * 1e6 / 39.3e12, 4))
            # the M-step on the assignment just computed (the call waits for the stream: host round trip included)
            wsu = torch.zeros(B.btc_update_workspace_bytes(v_, K_), dtype=torch.uint8, device=dev)
            cb2 = cbk.clone()
            upd = lambda: B.btc_update(vec, zz, N, v_, cb2, K_, wsu)
            upd()
            t0 = time.perf_counter()
            for _ in range(5):
                upd()
            row["update_us"] = round((time.perf_counter() - t0) / 5 * 1e6, 1)
            assign[tag] = row
            del vec, zz, dd

    # ---- CPU oracle on the host cores, bounded sample of the same workload
    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.build()
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        for p in protos:
            p["packed_h"] = oracle.pack(p["layer"].idx, p["layer"].K)
        t0 = time.time()
        done_bytes, reps, cpu_s = 0, 0, 0.0
        while time.time() - t0 < 10.0:
            t1 = time.time()
            for p in protos:
                lay = p["layer"]
                oracle.linear(p["packed_h"], lay.codebook, lay.alpha, lay.mu, p["x_host"], lay.n_in, lay.v, lay.K)
                done_bytes += gemv_bytes(p["s"], 1)
            reps += 1
            cpu_s = time.time() - t1
        cpu_elapsed = time.time() - t0
        cpu = dict(value=round(done_bytes / cpu_elapsed / 1e9, 4), unit="GB/s", cores=threads, kind="oracle",
                   sample=f"{reps} pass(es) over one matrix of each 13B shape (unpack + materialise fp64 + multiply), "
                          f"{cpu_elapsed:.1f} s; last pass {cpu_s:.2f} s")

    out = {
        "metric": "btc_gemv effective weight GB/s (13B shapes, 0.8-bit, batch 1, cold)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 in / f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "llama2-13b decoder-layer projections (4x5120x5120, 2x13824x5120, 1x5120x13824), "
                               "v=10 K=256 (0.8 bit), Zipf(1.1) indices, batch-1 GEMV, "
                               f"{args.layers} distinct weight copies ({total_weight_bytes / 1e9:.2f} GB) walked cold",
                   "step": "one decoder layer = 7 btc_gemv calls", "launch": args.mode},
        "us_per_call": round(us_per_call, 3),
        "fp16_equivalent_GBps": round(fp16_equiv, 1),
        "per_shape": per_shape,
        "gemm": gemm,
        "other_decode_configs": other,
        "roofline": {"bound": "hbm", "achieved": round(value, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(value / HBM_PEAK_GBS, 4), "traffic": HBM_TRAFFIC_PER_STEP,
                     "note": "algorithmic bytes of the 7 calls of a step / event-timed duration of a step; "
                             "traffic = HBM bytes per step (fetched + written) from the rocprofv3 counter runs "
                             "summarised in profiles/gemv_13b_hbm_traffic.md, algorithmic bytes per step "
                             f"{step_bytes}"},
        "roofline_gemm": None if gemm is None else {
            "bound": "mfma", "achieved": gemm[f"M{args.gemm_m}"]["layer_tflops"], "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": gemm[f"M{args.gemm_m}"]["frac_mfma_peak"], "traffic": None,
            "note": f"2*M*out*in flop of the 7 projections at M={args.gemm_m} / event-timed btc_gemm calls "
                    "(whole calls)"},
        "transform": transform,
        "assign": assign,
        "cpu_baseline": cpu,
        "setup_s": round(t_setup, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
