#!/usr/bin/env python3
"""Benchmark of the binary-codebook linear layer on one MI355X.

Headline workload (BASELINE.json: "btc_gemv effective weight GB/s + us/call (13B shapes,
0.8-bit); GEMM TFLOP/s"): the seven linear projections of a LLaMA-2-13B decoder
layer (4 x 5120x5120, 2 x 13824x5120, 1 x 5120x13824) stored at v=10, K=256
(8-bit indices, 0.8 bit/weight), Zipf(1.1) indices, batch-1 fp16 activations.

One STEP = one decoder layer = 7 btc_gemv calls.  Consecutive steps walk
through `--layers` distinct copies of the packed weights (40 copies = 1.27 GB,
five times the 256 MB last-level cache), so every call streams its indices from
HBM ("cold").  value = algorithmic bytes of a step / time of a step.  All
inputs are resident in HBM before the timed region.  The launches of the K timed
steps are captured once in a HIP graph (the calls still go through the C ABI, which
only enqueues kernels) so that Python's per-call overhead is not what is timed;
--mode stream times plain per-call launches.  The K-step region is timed `--repeats`
times in a row (5 by default) and the mean is reported, every repeat listed.

Every sweep takes its layers from the seeded recipe of btc_synth.config_cases (packed on the
GPU by btc_pack).  For each decode shape the line carries: cold time (a graph over distinct
copies worth >= 1 GiB, i.e. streamed from HBM), warm time (one buffer, which the caches hold;
may exceed the HBM peak), the time of a single event-bracketed launch, and the in-kernel
time of the rocprofv3 summary under profiles/ when that file lists the shape.  Fractions are
given against the published peaks (8 TB/s, 2.5 PFLOP/s bf16) and against what plain
read / matrix-core loops reach on this machine (6.4 TB/s, 2.2 PFLOP/s).

Also reported: prefill btc_gemm TFLOP/s (config 3: M = 2048 and 512), the transform, the
clustering kernels, roofline objects (13B step, 70B-shaped layer, prefill), and the CPU oracle
timed on the host cores (all cores and one thread; unpack, materialise, multiply separately).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
# what a plain 16-byte-per-lane read of 2 GiB and a plain bf16 matrix-core loop reach on this machine
HBM_MEASURED_GBS = 6400.0
MFMA_BF16_MEASURED_TFLOPS = 2200.0
PROFILE_FIGURES = os.path.join(ROOT, "profiles", "gemv_13b_hbm_traffic.md")
PROFILE_KERNEL_US = os.path.join(ROOT, "profiles", "gemv_gemm_13b_kernel_trace.md")

SHAPES_13B_COUNT = {(5120, 5120): 4, (13824, 5120): 2, (5120, 13824): 1}
COUNT_70B = {(8192, 8192): 2, (1024, 8192): 2, (28672, 8192): 2, (8192, 28672): 1}


def gemv_bytes(s, batch, y_bytes=2):
    """Algorithmic bytes of one call: index stream + alpha, mu + x + y + codebook."""
    return s.out * s.words_per_row * 4 + s.out * 8 + batch * s.in_ * 2 + batch * s.out * y_bytes + (1 << s.b) * 4


def read_figures(path):
    """`name = number` lines of a profile summary (the figures this script quotes rather than measures)."""
    figs = {}
    if os.path.exists(path):
        for line in open(path):
            m = re.match(r"^\s*([A-Za-z0-9_ .x=]+?)\s*=\s*([0-9.eE+-]+)\s*$", line)
            if m:
                figs[m.group(1).strip()] = float(m.group(2))
    return figs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--repeats", type=int, default=5, help="the timed K-step region is run this many times in a row")
    ap.add_argument("--layers", type=int, default=40, help="distinct weight copies walked by consecutive steps")
    ap.add_argument("--mode", choices=["graph", "stream"], default="graph")
    ap.add_argument("--launches", choices=["grouped", "separate"], default="grouped",
                    help="grouped: the projections of a decoder layer that share their input (q, k, v; gate, up) go "
                         "through btc_gemv_multi, one launch per group; separate: seven btc_gemv calls")
    ap.add_argument("--gemm-m", type=int, default=2048)
    ap.add_argument("--gemm-iters", type=int, default=10)
    ap.add_argument("--gemm-warmup-ms", type=float, default=40.0, help="the GEMM legs repeat a call untimed for this long first")
    ap.add_argument("--no-compare", action="store_true", help="do not also time the other way of launching the step")
    ap.add_argument("--no-gemm", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-transform", action="store_true", help="skip the btc_transform / btc_assign timings")
    ap.add_argument("--no-other", action="store_true", help="skip the 7B (batch 1/4/16) and 70B decode sweeps")
    ap.add_argument("--profile-case", default=None,
                    help="run 24 calls of one case and exit (for rocprofv3 counter runs): gemv,out,in,v,K,batch | "
                         "gemm,out,in,v,K,M | gemm_aq,out,in,v,K,M | assign,N,v,K")
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
    if args.profile_case:
        f = args.profile_case.split(",")
        kind, nums = f[0], [int(a) for a in f[1:]]
        if kind == "assign":
            N, v_, K_ = nums
            g = torch.Generator(device=dev)
            g.manual_seed(0)
            vec = torch.randint(0, 2 ** v_, (N,), dtype=torch.int32, device=dev, generator=g)
            cbk = torch.randint(0, 2 ** v_, (K_,), dtype=torch.int32, device=dev, generator=g)
            zz = torch.empty(N, dtype=torch.int32, device=dev)
            for _ in range(6):
                B.btc_assign(vec, N, v_, cbk, K_, zz, None)
        else:
            o, i, v_, K_, rows = nums
            layer, x = S.make_case(0, o, i, v_, K_, 1 if kind == "multi" else rows,
                                   x_dtype="f16" if kind in ("gemv", "multi") else "bf16")
            s = B.btc_shape_init(o, i, v_, K_)
            packed = torch.empty(o * s.words_per_row, dtype=torch.int32, device=dev)
            B.btc_pack(s, torch.from_numpy(layer.idx).to(dev), packed, torch.zeros(64, dtype=torch.uint8, device=dev))
            cb = np.zeros(1 << s.b, dtype=np.uint32)
            cb[:K_] = layer.codebook
            cb_d = torch.from_numpy(cb.view(np.int32)).to(dev)
            al, mu = torch.from_numpy(layer.alpha).to(dev), torch.from_numpy(layer.mu).to(dev)
            xd = torch.from_numpy(x.view(np.int16)).to(dev)
            if kind == "gemv":   # cold: 24 distinct copies
                y = torch.empty(rows * o, dtype=torch.float16, device=dev)
                ws = torch.zeros(B.btc_workspace_bytes(s, rows, False), dtype=torch.uint8, device=dev)
                pk = packed.view(o, s.words_per_row)
                copies = [torch.roll(pk, shifts=(c * 37 + 1) % o, dims=0).contiguous() for c in range(24)]
                for c in copies:
                    B.btc_gemv(s, c, cb_d, al, mu, xd, rows, y, B.BTC_F16, ws)
            elif kind == "multi":   # cold: 24 launches of `rows` distinct copies each, on one activation row
                ys = [torch.empty(o, dtype=torch.float16, device=dev) for _ in range(rows)]
                ws = torch.zeros(B.btc_workspace_bytes(s, 1, False), dtype=torch.uint8, device=dev)
                pk = packed.view(o, s.words_per_row)
                copies = [torch.roll(pk, shifts=(c * 37 + 1) % o, dims=0).contiguous() for c in range(24 * rows)]
                for c in range(24):
                    B.btc_gemv_multi(s, copies[c * rows:(c + 1) * rows], [cb_d] * rows, [al] * rows, [mu] * rows, xd, ys,
                                     B.BTC_F16, ws)
            elif kind == "gemm":
                Y = torch.empty(rows * o, dtype=torch.float32, device=dev)
                ws = torch.zeros(B.btc_workspace_bytes(s, rows, True), dtype=torch.uint8, device=dev)
                for _ in range(6):
                    B.btc_gemm(s, packed, cb_d, al, mu, xd, B.BTC_BF16, rows, Y, B.BTC_F32, ws)
            else:
                Y = torch.empty(rows * o, dtype=torch.float32, device=dev)
                Qc = torch.empty(rows * i, dtype=torch.uint8, device=dev)
                lo_d = torch.empty(max(rows, 4), dtype=torch.float32, device=dev)
                st_d = torch.empty(max(rows, 4), dtype=torch.float32, device=dev)
                wsum = torch.empty(o, dtype=torch.float32, device=dev)
                ws1 = torch.zeros(B.btc_aq_workspace_bytes(s, 1), dtype=torch.uint8, device=dev)
                ws = torch.zeros(B.btc_aq_workspace_bytes(s, rows), dtype=torch.uint8, device=dev)
                B.btc_weight_rowsums(s, packed, cb_d, al, mu, wsum, ws1)
                for _ in range(6):
                    B.btc_quantize_rows(xd, B.BTC_BF16, rows, i, 8, Qc, lo_d, st_d)
                    B.btc_gemm_aq(s, packed, cb_d, al, mu, wsum, Qc, lo_d, st_d, rows, Y, B.BTC_F32, ws)
        torch.cuda.synchronize()
        print(json.dumps({"profile_case": args.profile_case}))
        return
    figures = read_figures(PROFILE_FIGURES)
    kernel_us = read_figures(PROFILE_KERNEL_US)

    def events():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def device_case(case, x_dtype=None):
        """One seeded layer of the recipe, packed on the GPU through btc_pack."""
        kw = dict(case)
        if x_dtype is not None:
            kw["x_dtype"] = x_dtype
        layer, x = S.make_case(**kw)
        s = B.btc_shape_init(layer.out, layer.n_in, layer.v, layer.K)
        idx_d = torch.from_numpy(layer.idx).to(dev)
        packed = torch.empty(layer.out * s.words_per_row, dtype=torch.int32, device=dev)
        B.btc_pack(s, idx_d, packed, torch.zeros(64, dtype=torch.uint8, device=dev))
        cb = np.zeros(1 << s.b, dtype=np.uint32)
        cb[:layer.K] = layer.codebook
        return dict(s=s, layer=layer, batch=case["batch"], packed=packed.view(layer.out, s.words_per_row),
                    codebook=torch.from_numpy(cb.view(np.int32)).to(dev),
                    alpha=torch.from_numpy(layer.alpha).to(dev), mu=torch.from_numpy(layer.mu).to(dev),
                    x=torch.from_numpy(x.view(np.int16)).to(dev), x_host=x)

    def rotated(p, n):
        """n distinct copies of a packed matrix: the rows rotated by a copy-specific offset."""
        out = p["s"].out
        return [torch.roll(p["packed"], shifts=((i * 7 + 1) * 37) % out, dims=0).contiguous() for i in range(n)]

    # ---- config 2: one seeded layer per 13B shape
    t_setup = time.time()
    protos = []
    for case in S.config_cases(2):
        p = device_case(case)
        p["count"] = SHAPES_13B_COUNT[(case["out"], case["n_in"])]
        protos.append(p)
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

    def run_layer_separate(L):
        for c in calls_per_layer[L]:
            p = c["p"]
            B.btc_gemv(p["s"], c["packed"], p["codebook"], p["alpha"], p["mu"], p["x"], 1, c["y"], B.BTC_F16, ws)

    # q, k, v (calls 0..2) and gate, up (calls 4, 5) share their input: one launch per group
    GROUPS = [(0, 3), (3, 4), (4, 6), (6, 7)]

    def run_layer_grouped(L):
        calls = calls_per_layer[L]
        for (a, b) in GROUPS:
            p = calls[a]["p"]
            if b - a == 1:
                B.btc_gemv(p["s"], calls[a]["packed"], p["codebook"], p["alpha"], p["mu"], p["x"], 1, calls[a]["y"],
                           B.BTC_F16, ws)
            else:
                grp = calls[a:b]
                B.btc_gemv_multi(p["s"], [c["packed"] for c in grp], [p["codebook"]] * (b - a), [p["alpha"]] * (b - a),
                                 [p["mu"]] * (b - a), p["x"], [c["y"] for c in grp], B.BTC_F16, ws)

    def time_step(run_fn):
        """Warm-up, then exactly `steps` layers `repeats` times in a row; returns (ms per step, per repeat)."""
        for i in range(max(args.warmup, 1)):
            run_fn(i % args.layers)
        torch.cuda.synchronize()
        reps_ = max(1, args.repeats)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(reps_ + 1)]
        if args.mode == "graph":
            full_sweeps, rest = divmod(args.steps, args.layers)
            g_full = g_rest = None
            if full_sweeps:
                g_full = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g_full):
                    for L in range(args.layers):
                        run_fn(L)
                g_full.replay()
            if rest:
                g_rest = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g_rest):
                    for L in range(rest):
                        run_fn(L)
                g_rest.replay()
            torch.cuda.synchronize()
            marks[0].record()
            for r in range(reps_):
                for _ in range(full_sweeps):
                    g_full.replay()
                if g_rest is not None:
                    g_rest.replay()
                marks[r + 1].record()
        else:
            torch.cuda.synchronize()
            marks[0].record()
            for r in range(reps_):
                for i in range(args.steps):
                    run_fn(i % args.layers)
                marks[r + 1].record()
        torch.cuda.synchronize()
        return (marks[0].elapsed_time(marks[reps_]) / (args.steps * reps_),
                [marks[r].elapsed_time(marks[r + 1]) / args.steps for r in range(reps_)])

    repeats = max(1, args.repeats)
    run_layer = run_layer_grouped if args.launches == "grouped" else run_layer_separate
    ms_per_step, ms_repeats = time_step(run_layer)
    # the other way of launching the same step, for comparison
    other_fn = run_layer_separate if args.launches == "grouped" else run_layer_grouped
    ms_other = float("nan") if args.no_compare else time_step(other_fn)[0]
    n_launches = len(GROUPS) if args.launches == "grouped" else n_calls
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    us_per_call = ms_per_step * 1e3 / n_calls
    fp16_equiv = sum(2 * c["p"]["s"].out * c["p"]["s"].in_ for c in calls_per_layer[0]) / (ms_per_step * 1e-3) / 1e9

    def time_decode(p, min_calls=200):
        """Cold / warm / single-launch times of btc_gemv on one seeded layer."""
        s, batch = p["s"], p["batch"]
        nbytes = s.out * s.words_per_row * 4
        ncopies = int(min(1200, max(8, -(-(1 << 30) // nbytes))))
        copies = rotated(p, ncopies)
        y = torch.empty(batch * s.out, dtype=torch.float16, device=dev)
        wsd = torch.zeros(B.btc_workspace_bytes(s, batch, False), dtype=torch.uint8, device=dev)
        call = lambda w: B.btc_gemv(s, w, p["codebook"], p["alpha"], p["mu"], p["x"], batch, y, B.BTC_F16, wsd)
        for w in copies[:8]:
            call(w)
        torch.cuda.synchronize()
        by = gemv_bytes(s, batch)
        # cold, amortised over a graph of all copies
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for w in copies:
                call(w)
        g.replay()
        torch.cuda.synchronize()
        reps = max(2, -(-min_calls // ncopies))
        e0, e1 = events()
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        cold = e0.elapsed_time(e1) * 1e3 / (reps * ncopies)
        # warm: the same buffer again and again
        gw = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gw):
            for _ in range(50):
                call(copies[0])
        gw.replay()
        torch.cuda.synchronize()
        e0, e1 = events()
        e0.record()
        for _ in range(4):
            gw.replay()
        e1.record()
        torch.cuda.synchronize()
        warm = e0.elapsed_time(e1) * 1e3 / 200
        # one launch between two events, on a copy not touched recently
        singles = []
        for i in range(min(ncopies, 24)):
            e0, e1 = events()
            e0.record()
            call(copies[-1 - i])
            e1.record()
            torch.cuda.synchronize()
            singles.append(e0.elapsed_time(e1) * 1e3)
        del copies, g, gw
        single = float(np.median(singles))
        row = dict(bytes=by, cold_us=round(cold, 2), warm_us=round(warm, 2), single_launch_us=round(single, 2),
                   eff_GBps=round(by / cold / 1e3, 1), frac_hbm=round(by / cold / 1e3 / HBM_PEAK_GBS, 4),
                   frac_measured_peak=round(by / cold / 1e3 / HBM_MEASURED_GBS, 4),
                   warm_GBps=round(by / warm / 1e3, 1), cold_copies=ncopies)
        k_us = kernel_us.get(f"in_kernel_us {s.out}x{s.in_} v={s.v} K={s.K} batch={batch}")
        if k_us is not None:
            row["in_kernel_us"] = k_us
        return row

    def time_pair(p, min_calls=80):
        """Cold time of ONE btc_gemv_multi launch over two distinct copies of a matrix (the k, v or the gate, up
        projections of a layer), amortised over a graph of such launches."""
        s = p["s"]
        nbytes = s.out * s.words_per_row * 4
        npairs = int(min(600, max(4, -(-(1 << 29) // nbytes))))
        copies = rotated(p, 2 * npairs)
        ys = [torch.empty(s.out, dtype=torch.float16, device=dev) for _ in range(2)]
        wsd = torch.zeros(B.btc_workspace_bytes(s, 1, False), dtype=torch.uint8, device=dev)
        call = lambda i: B.btc_gemv_multi(s, [copies[2 * i], copies[2 * i + 1]], [p["codebook"]] * 2, [p["alpha"]] * 2,
                                          [p["mu"]] * 2, p["x"], ys, B.BTC_F16, wsd)
        call(0)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(npairs):
                call(i)
        g.replay()
        torch.cuda.synchronize()
        reps = max(2, -(-min_calls // npairs))
        e0, e1 = events()
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * npairs)
        by = 2 * gemv_bytes(s, 1)
        del copies, g
        return dict(us_per_launch=round(us, 2), bytes=by, eff_GBps=round(by / us / 1e3, 1),
                    frac_hbm=round(by / us / 1e3 / HBM_PEAK_GBS, 4))

    def time_qkv(pq, pkv, min_calls=80):
        """Cold time of ONE btc_gemv_multi_shapes launch over q (pq's shape) and k, v (two distinct copies of pkv's
        shape: fewer rows under grouped-query attention), amortised over a graph of such launches."""
        sq, sk = pq["s"], pkv["s"]
        nbytes = (sq.out + 2 * sk.out) * sq.words_per_row * 4
        n = int(min(300, max(4, -(-(1 << 29) // nbytes))))
        cq, ck = rotated(pq, n), rotated(pkv, 2 * n)
        ys = [torch.empty(o, dtype=torch.float16, device=dev) for o in (sq.out, sk.out, sk.out)]
        wsd = torch.zeros(max(B.btc_workspace_bytes(sq, 1, False), B.btc_workspace_bytes(sk, 1, False)),
                          dtype=torch.uint8, device=dev)
        call = lambda i: B.btc_gemv_multi_shapes([sq, sk, sk], [cq[i], ck[2 * i], ck[2 * i + 1]],
                                                 [pq["codebook"], pkv["codebook"], pkv["codebook"]],
                                                 [pq["alpha"], pkv["alpha"], pkv["alpha"]],
                                                 [pq["mu"], pkv["mu"], pkv["mu"]], pq["x"], ys, B.BTC_F16, wsd)
        call(0)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n):
                call(i)
        g.replay()
        torch.cuda.synchronize()
        reps = max(2, -(-min_calls // n))
        e0, e1 = events()
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * n)
        by = gemv_bytes(sq, 1) + 2 * gemv_bytes(sk, 1)
        del cq, ck, g
        return dict(us_per_launch=round(us, 2), bytes=by, eff_GBps=round(by / us / 1e3, 1),
                    frac_hbm=round(by / us / 1e3 / HBM_PEAK_GBS, 4))

    def time_gemm_steady(fn, first=None):
        """ms per call in the steady state: the calls are repeated untimed until --gemm-warmup-ms have gone by (the
        clock of a chip that has been idle or under light load takes tens of milliseconds of this load to settle:
        the first ten calls run 5 to 15 % slower than the hundredth), then the median of three timed runs of
        --gemm-iters calls.  first: a dict that receives the ms per call of the very first run, before the warm-up."""
        def run():
            e0, e1 = events()
            e0.record()
            for _ in range(args.gemm_iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.gemm_iters
        fn()
        torch.cuda.synchronize()
        t_first = run()
        if first is not None:
            first["ms_first_run"] = round(t_first, 4)
        spent = t_first * args.gemm_iters
        while spent < args.gemm_warmup_ms:
            spent += run() * args.gemm_iters
        return sorted(run() for _ in range(3))[1]

    # per-shape timing of the headline shapes
    per_shape = {f"{p['s'].out}x{p['s'].in_}": time_decode(p) for p in protos}

    # ---- the other decode configurations of the benchmark spec
    other, roof70 = None, None
    if not args.no_other:
        other = {}
        seven = {}
        for case in S.config_cases(1):     # 7B shapes, 0.9 bit, 1 % outlier channels, batch 1 / 4 / 16
            p = device_case(case)
            seven.setdefault(f"{case['out']}x{case['n_in']}", {})[f"batch{case['batch']}"] = time_decode(p)
            del p
        other["llama2-7b v=10 K=512 (0.9 bit), outlier channels"] = seven
        tags = {(9, 1024): "1.11 bit", (10, 512): "0.9 bit", (10, 128): "0.7 bit"}
        layers70 = {}
        for case in S.config_cases(4):     # 70B shapes at three settings
            p = device_case(case)
            key = f"llama2-70b v={case['v']} K={case['K']} ({tags[(case['v'], case['K'])]})"
            d = layers70.setdefault(key, dict(per_shape={}, us=0.0, bytes=0))
            r = time_decode(p, min_calls=80)
            cnt = COUNT_70B[(case["out"], case["n_in"])]
            d["per_shape"][f"{case['out']}x{case['n_in']}"] = r
            d["us"] += cnt * r["cold_us"]
            d["bytes"] += cnt * r["bytes"]
            # q, k, v share their input (k and v have an eighth of q's rows): one launch through btc_gemv_multi_shapes;
            # gate, up: one launch through btc_gemv_multi; o and down stay single calls
            shp = (case["out"], case["n_in"])
            if shp == (8192, 8192):
                d["us_grouped"] = d.get("us_grouped", 0.0) + r["cold_us"]          # o
                d["q_proto"] = p                                                    # kept until k, v arrive
                continue
            if shp == (1024, 8192):
                pr = time_pair(p)
                d.setdefault("pairs", {})[f"2 x {case['out']}x{case['n_in']}"] = pr
                qkv = time_qkv(d.pop("q_proto"), p)
                d["pairs"]["8192x8192 + 2 x 1024x8192 (q, k, v)"] = qkv
                d["us_grouped"] = d.get("us_grouped", 0.0) + qkv["us_per_launch"]
            elif shp == (28672, 8192):
                pr = time_pair(p)
                d.setdefault("pairs", {})[f"2 x {case['out']}x{case['n_in']}"] = pr
                d["us_grouped"] = d.get("us_grouped", 0.0) + pr["us_per_launch"]
            else:
                d["us_grouped"] = d.get("us_grouped", 0.0) + cnt * r["cold_us"]
            del p
        for key, d in layers70.items():
            gbs = d["bytes"] / d["us"] / 1e3
            gbs_g = d["bytes"] / d["us_grouped"] / 1e3
            other[key] = dict(per_shape=d["per_shape"], layer_us=round(d["us"], 1), layer_eff_GBps=round(gbs, 1),
                              layer_frac_hbm=round(gbs / HBM_PEAK_GBS, 4),
                              layer_frac_measured_peak=round(gbs / HBM_MEASURED_GBS, 4),
                              pairs_one_launch=d.get("pairs"), layer_us_grouped=round(d["us_grouped"], 1),
                              layer_eff_GBps_grouped=round(gbs_g, 1),
                              layer_frac_hbm_grouped=round(gbs_g / HBM_PEAK_GBS, 4))
        key09 = "llama2-70b v=10 K=512 (0.9 bit)"
        big = other[key09]["per_shape"]["28672x8192"]
        roof70 = {"bound": "hbm", "achieved": big["eff_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                  "frac": big["frac_hbm"], "frac_measured_peak": big["frac_measured_peak"],
                  "traffic": figures.get("traffic_bytes_per_call 28672x8192 v=10 K=512"),
                  "layer_frac": other[key09]["layer_frac_hbm"],
                  "layer_frac_grouped": other[key09]["layer_frac_hbm_grouped"],
                  "gate_up_one_launch": dict(other[key09]["pairs_one_launch"]["2 x 28672x8192"],
                                             traffic=figures.get("traffic_bytes_per_launch 2x28672x8192 v=10 K=512"),
                                             in_kernel_us=kernel_us.get("in_kernel_us 2x28672x8192 v=10 K=512 one launch")),
                  "note": "btc_gemv on 28672x8192 at 0.9 bit, batch 1, cold: algorithmic bytes of a call "
                          f"({big['bytes']}) / graph-amortised time of a call; layer_frac = the seven matrices of "
                          "a 70B-shaped decoder layer"}
        # the long-vector settings of the paper's vector-length study (codebook itself in LDS, or gathered)
        longc = {}
        for (o, i, v_, K_) in [(4096, 4096, 16, 65536), (4096, 4096, 20, 65536), (4096, 4096, 16, 7132),
                               (11008, 4096, 16, 65536), (8192, 8192, 16, 65536)]:
            p = device_case(dict(seed=0, out=o, n_in=i, v=v_, K=K_, batch=1))
            longc[f"{o}x{i} v={v_} K={K_}"] = time_decode(p, min_calls=80)
            del p
        other["long_vectors_large_codebooks"] = longc
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
            if M > 16:            # compute-bound sizes: both sides in the steady state (see time_gemm_steady)
                def one_pass():
                    for w in Ws:
                        torch.matmul(xd, w.t())
                us = time_gemm_steady(one_pass) * 1e3 / ncopies
                del Ws
                return us
            reps = 8
            e0, e1 = events()
            e0.record()
            for _ in range(reps):
                for w in Ws:
                    torch.matmul(xd, w.t())
            e1.record()
            torch.cuda.synchronize()
            del Ws
            return e0.elapsed_time(e1) * 1e3 / (reps * ncopies)

        def time_gemm_call(p, M):
            s = p["s"]
            X2 = torch.randn(M, s.in_, device=dev).bfloat16()
            Y2 = torch.empty(M, s.out, dtype=torch.bfloat16, device=dev)
            ws2 = torch.zeros(B.btc_workspace_bytes(s, M, True), dtype=torch.uint8, device=dev)
            f = lambda: B.btc_gemm(s, p["packed"], p["codebook"], p["alpha"], p["mu"], X2, B.BTC_BF16, M, Y2,
                                   B.BTC_BF16, ws2)
            return time_gemm_steady(f) * 1e3

        mlp = {}
        o_, i_ = 8192, 28672
        for M in (1, 16):
            dense_us = time_dense(o_, i_, M, torch.float16)
            row = {"torch_fp16_us": round(dense_us, 1)}
            for (v_, K_, tag) in [(10, 512, "0.9 bit"), (10, 256, "0.8 bit"), (10, 128, "0.7 bit")]:
                p = device_case(dict(seed=0, out=o_, n_in=i_, v=v_, K=K_, batch=M))
                us = time_decode(p, min_calls=40)["cold_us"]
                row[tag] = dict(us=us, speedup_over_fp16=round(dense_us / us, 2))
                del p
            mlp[f"M{M}"] = row
        p = device_case(dict(seed=0, out=o_, n_in=i_, v=10, K=256, batch=1))
        for M in (32, 64, 96, 128, 256, 512, 2048):        # btc_gemm, bf16 activations
            dense_us = time_dense(o_, i_, M, torch.bfloat16)
            us = time_gemm_call(p, M)
            mlp[f"M{M}"] = {"torch_bf16_us": round(dense_us, 1),
                            "0.8 bit": dict(us=round(us, 1), speedup_over_bf16=round(dense_us / us, 2),
                                            tflops=round(2.0 * M * o_ * i_ / us / 1e6, 1))}
        del p
        other["mlp_8192x28672_vs_dense_torch"] = mlp

    # ---- prefill GEMM, config 3 (uniform indices, bf16 activations, fp32 output): btc_gemm = one contraction
    # kernel per call, plus a second pass when the call is split along k
    gemm = None
    if not args.no_gemm:
        gemm = {}
        cases3 = {}
        for case in S.config_cases(3):
            cases3.setdefault(case["batch"], []).append(case)
        for M in sorted({args.gemm_m, 512}, reverse=True):
            per, tot_flop, tot_ms, tot_ms_b, tot_ms_first = {}, 0.0, 0.0, 0.0, 0.0
            for case in cases3.get(M) or [dict(c, batch=M) for c in cases3[2048]]:
                p = device_case(case)
                s = p["s"]
                X = p["x"]
                Y = torch.empty(M * s.out, dtype=torch.float32, device=dev)
                wsg = torch.zeros(B.btc_workspace_bytes(s, M, True), dtype=torch.uint8, device=dev)
                call = lambda: B.btc_gemm(s, p["packed"], p["codebook"], p["alpha"], p["mu"], X, B.BTC_BF16, M, Y,
                                          B.BTC_F32, wsg)
                first = {}
                ms = time_gemm_steady(call, first)
                flop = 2.0 * M * s.out * s.in_
                cnt = SHAPES_13B_COUNT[(s.out, s.in_)]
                per[f"{s.out}x{s.in_}"] = dict(ms=round(ms, 4), tflops=round(flop / ms / 1e9, 1),
                                               tflops_first_run=round(flop / first["ms_first_run"] / 1e9, 1))
                tot_flop += flop * cnt
                tot_ms += ms * cnt
                tot_ms_first += first["ms_first_run"] * cnt
                # the same call with the output rounded to bf16 (half the bytes written by the epilogue)
                Yb = torch.empty(M * s.out, dtype=torch.bfloat16, device=dev)
                callb = lambda: B.btc_gemm(s, p["packed"], p["codebook"], p["alpha"], p["mu"], X, B.BTC_BF16, M, Yb,
                                           B.BTC_BF16, wsg)
                msb = time_gemm_steady(callb)
                per[f"{s.out}x{s.in_}"]["tflops_bf16_out"] = round(flop / msb / 1e9, 1)
                tot_ms_b += msb * cnt
                del X, Y, Yb, p
            tf = tot_flop / tot_ms / 1e9
            gemm[f"M{M}"] = dict(M=M, x_dtype="bf16", y_dtype="f32", per_shape=per, layer_tflops=round(tf, 1),
                                 layer_tflops_bf16_out=round(tot_flop / tot_ms_b / 1e9, 1),
                                 layer_tflops_first_run=round(tot_flop / tot_ms_first / 1e9, 1),
                                 timing=f"steady state: median of 3 runs of {args.gemm_iters} calls after "
                                        f"{args.gemm_warmup_ms:g} ms of the same call; first_run: the first "
                                        f"{args.gemm_iters} calls after the decode legs (clock not settled yet)",
                                 frac_mfma_peak=round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                                 frac_measured_peak=round(tf / MFMA_BF16_MEASURED_TFLOPS, 4))

    # ---- the layer on 8-bit activation codes (W0.8A8): quantise + product, prefill rows on the integer matrix
    # cores, one decode row through the decode engines
    act_quant = None
    if not args.no_gemm:
        act_quant = {}
        for M in (args.gemm_m, 1):
            per, tot_op, tot_ms = {}, 0.0, 0.0
            for case in S.config_cases(2):
                p = device_case(dict(case, batch=M, x_dtype="bf16" if M > 1 else "f16"))
                s = p["s"]
                Qc = torch.empty(M * s.in_, dtype=torch.uint8, device=dev)
                lo_d = torch.empty(max(M, 4), dtype=torch.float32, device=dev)
                st_d = torch.empty(max(M, 4), dtype=torch.float32, device=dev)
                Y = torch.empty(M * s.out, dtype=torch.float32, device=dev)
                wsq = torch.zeros(B.btc_aq_workspace_bytes(s, M), dtype=torch.uint8, device=dev)
                ws1 = torch.zeros(B.btc_aq_workspace_bytes(s, 1), dtype=torch.uint8, device=dev)
                wsum = torch.empty(s.out, dtype=torch.float32, device=dev)
                B.btc_weight_rowsums(s, p["packed"], p["codebook"], p["alpha"], p["mu"], wsum, ws1)
                xdt = B.BTC_BF16 if M > 1 else B.BTC_F16

                def call():
                    B.btc_quantize_rows(p["x"], xdt, M, s.in_, 8, Qc, lo_d, st_d)
                    B.btc_gemm_aq(s, p["packed"], p["codebook"], p["alpha"], p["mu"], wsum, Qc, lo_d, st_d, M, Y,
                                  B.BTC_F32, wsq)
                call()
                torch.cuda.synchronize()
                if M > 1:
                    ms = time_gemm_steady(call)
                else:
                    reps = 50
                    e0, e1 = events()
                    e0.record()
                    for _ in range(reps):
                        call()
                    e1.record()
                    torch.cuda.synchronize()
                    ms = e0.elapsed_time(e1) / reps
                ops = 2.0 * M * s.out * s.in_
                cnt = SHAPES_13B_COUNT[(s.out, s.in_)]
                per[f"{s.out}x{s.in_}"] = dict(us=round(ms * 1e3, 1), tops=round(ops / ms / 1e9, 1))
                if M == 1:
                    # one decode row is a few small launches: also timed the way the headline is, replayed from a graph
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        for _ in range(20):
                            call()
                    g.replay()
                    torch.cuda.synchronize()
                    e0, e1 = events()
                    e0.record()
                    for _ in range(5):
                        g.replay()
                    e1.record()
                    torch.cuda.synchronize()
                    per[f"{s.out}x{s.in_}"]["us_graph"] = round(e0.elapsed_time(e1) * 1e3 / 100, 1)
                    del g
                tot_op += ops * cnt
                tot_ms += ms * cnt
                del p, Qc, Y, wsq
            row = dict(M=M, bits=8, per_shape=per, note="btc_quantize_rows + btc_gemm_aq, warm, stream-timed" + (" (us) and replayed from a graph of 20 (us_graph)" if M == 1 else ""))
            if M > 1:
                tp = tot_op / tot_ms / 1e9
                row.update(layer_tops=round(tp, 1), frac_int8_peak=round(tp / 5000.0, 4))
            act_quant[f"M{M}"] = row

    # ---- the storage variant with several (alpha, mu) groups per weight row (btc_gemv_groups), one decode row,
    # three groups drawn uniformly; bytes = index stream + group map (2 bits per weight) + per-row constants
    groups = None
    if not args.no_other:
        groups = {}
        ng = 3
        for case in S.config_cases(2):
            p = device_case(dict(case, batch=1))
            s = p["s"]
            rng = np.random.Generator(np.random.PCG64(7))
            fields = rng.integers(0, ng, size=(s.out, 16 * ((s.in_ + 15) // 16)), dtype=np.uint32)
            fields[:, s.in_:] = 0
            gm = np.zeros((s.out, fields.shape[1] // 16), dtype=np.uint32)
            for t in range(16):
                gm |= fields[:, t::16] << np.uint32(2 * t)
            gm_d = torch.from_numpy(gm.view(np.int32)).to(dev)
            al = torch.rand(s.out * ng, dtype=torch.float32, device=dev) * 0.02
            mu_g = torch.randn(s.out * ng, dtype=torch.float32, device=dev) * 0.002
            Y = torch.empty(s.out, dtype=torch.float32, device=dev)
            call = lambda: B.btc_gemv_groups(s, p["packed"], p["codebook"], al, mu_g, gm_d, ng, p["x"], Y, B.BTC_F32)
            call()
            torch.cuda.synchronize()
            e0, e1 = events()
            e0.record()
            for _ in range(50):
                call()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / 50 * 1e3
            nbytes = p["packed"].numel() * 4 + gm.nbytes + s.out * ng * 8
            groups[f"{s.out}x{s.in_}"] = dict(groups=ng, us=round(us, 1), stored_bytes=int(nbytes),
                                             gbs=round(nbytes / us / 1e3, 1))
            del p, gm_d, Y

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
                e0, e1 = events()
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
        e0, e1 = events()
        e0.record()
        for _ in range(5):
            gt.replay()
        e1.record()
        torch.cuda.synchronize()
        transform["decoder_layer_decode_with_4_transforms_us"] = round(e0.elapsed_time(e1) * 1e3 / (5 * args.layers), 2)
        ms_sep = ms_other if args.launches == "grouped" else ms_per_step     # seven separate btc_gemv calls
        if args.no_compare and args.launches == "grouped":
            ms_sep = time_step(run_layer_separate)[0]
        transform["decoder_layer_decode_without_us"] = round(ms_sep * 1e3, 2)
        # the same layer through btc_gemv_transformed: the first consumer of a transformed row computes it inside
        # its own kernel (every workgroup, on the matrix cores, factors prepared once) and hands it to the others;
        # factor sizes without a fused kernel (the input of down) run as the two launches inside the call
        prep = {}
        for n, (n1, n2, bd, p1d, p2d, xt) in tr.items():
            nb = B.btc_transform_prepared_bytes(n1, n2)
            prep[n] = None
            if nb:
                prep[n] = torch.empty(nb, dtype=torch.uint8, device=dev)
                B.btc_transform_prepare(n1, n2, p1d, p2d, prep[n])

        def run_layer_f(L):
            calls = calls_per_layer[L]
            for (a, b) in GROUPS:
                p = calls[a]["p"]
                n1, n2, bd, p1d, p2d, xt = tr[p["s"].in_]
                grp = calls[a:b] if args.launches == "grouped" else calls[a:a + 1]
                k = len(grp)
                B.btc_gemv_transformed_multi(p["s"], [c["packed"] for c in grp], [p["codebook"]] * k, [p["alpha"]] * k,
                                             [p["mu"]] * k, p["x"], n1, n2, bd, p1d, p2d, prep[p["s"].in_],
                                             [c["y"] for c in grp], B.BTC_F16, ws, xt_out=xt)
                if args.launches != "grouped":
                    for c in calls[a + 1:b]:      # the other consumers of the row: plain calls
                        B.btc_gemv(p["s"], c["packed"], p["codebook"], p["alpha"], p["mu"], xt, 1, c["y"], B.BTC_F16, ws)

        run_layer_f(0)
        torch.cuda.synchronize()
        gf = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gf):
            for L in range(args.layers):
                run_layer_f(L)
        gf.replay()
        torch.cuda.synchronize()
        e0, e1 = events()
        e0.record()
        for _ in range(5):
            gf.replay()
        e1.record()
        torch.cuda.synchronize()
        fused_us = e0.elapsed_time(e1) * 1e3 / (5 * args.layers)
        transform["decoder_layer_decode_fused_us"] = round(fused_us, 2)
        ms_same = ms_per_step                      # the plain step launched the same way as the fused one
        transform["decoder_layer_decode_fused_launches"] = args.launches
        transform["decoder_layer_decode_without_same_launches_us"] = round(ms_same * 1e3, 2)
        transform["fused_over_without"] = round(fused_us / (ms_same * 1e3), 3)
        transform["two_launches_over_without"] = round(
            transform["decoder_layer_decode_with_4_transforms_us"] / (ms_sep * 1e3), 3)

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
            e0, e1 = events()
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
            else:   # 3.5 vector-ALU instructions per (vector, centroid) pair, counted with SQ_INSTS_VALU
                    # (profiles/assign_kernel_trace.md), on 256 x 64 lanes at 2.4 GHz
                row.update(route="all pairs", lane_ops_per_s=round(3.5 * N * K_ / us * 1e6, -9),
                           frac_alu=round(3.5 * N * K_ / us * 1e6 / 39.3e12, 4))
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

    # ---- CPU oracle on the host cores, bounded sample of the same workload: whole passes over one matrix of
    # each 13B shape with all cores, then the same with one thread, each split into its three stages
    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.build()
        omp = ctypes.CDLL("libgomp.so.1")
        all_threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        for p in protos:
            p["packed_h"] = oracle.pack(p["layer"].idx, p["layer"].K)

        def oracle_pass(split):
            """One pass over one matrix of each 13B shape; the three stages timed one by one."""
            for p in protos:
                lay = p["layer"]
                t0 = time.perf_counter()
                oracle.unpack(p["packed_h"], p["s"].nchunks, lay.K)
                t1 = time.perf_counter()
                W = oracle.materialise(p["packed_h"], lay.codebook, lay.alpha, lay.mu, lay.n_in, lay.v, lay.K)
                t2 = time.perf_counter()
                oracle.matmul(W, oracle.widen(np.atleast_2d(p["x_host"]), "f16"))
                t3 = time.perf_counter()
                split["unpack_s"] += t1 - t0
                split["materialise_s"] += t2 - t1
                split["multiply_s"] += t3 - t2
            return sum(gemv_bytes(p["s"], 1) for p in protos)

        def timed(threads, budget_s):
            omp.omp_set_num_threads(threads)
            split = dict(unpack_s=0.0, materialise_s=0.0, multiply_s=0.0)
            t0, done, reps = time.perf_counter(), 0, 0
            while time.perf_counter() - t0 < budget_s:
                done += oracle_pass(split)
                reps += 1
            el = time.perf_counter() - t0
            return dict(value=round(done / el / 1e9, 4), passes=reps, seconds=round(el, 1),
                        split_s_per_pass={k: round(v / reps, 4) for k, v in split.items()})

        many = timed(all_threads, 8.0)
        one = timed(1, 8.0)
        omp.omp_set_num_threads(all_threads)
        cpu = dict(value=many["value"], unit="GB/s", cores=all_threads, kind="oracle",
                   sample=f"{many['passes']} pass(es) over one matrix of each 13B shape (unpack, materialise fp64, "
                          f"multiply; each stage timed by itself), {many['seconds']} s with {all_threads} threads; "
                          f"then {one['passes']} pass(es) in {one['seconds']} s with one thread",
                   split_s_per_pass=many["split_s_per_pass"],
                   single_thread=dict(value=one["value"], unit="GB/s", cores=1,
                                      split_s_per_pass=one["split_s_per_pass"]))

    traffic = figures.get("traffic_bytes_per_step" if args.launches == "grouped" else "traffic_bytes_per_step separate")
    out = {
        "metric": "btc_gemv effective weight GB/s (13B shapes, 0.8-bit, batch 1, cold)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "ms_per_step_repeats": [round(m, 5) for m in ms_repeats],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 in / f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "llama2-13b decoder-layer projections (4x5120x5120, 2x13824x5120, 1x5120x13824), "
                               "v=10 K=256 (0.8 bit), Zipf(1.1) indices, batch-1 GEMV, "
                               f"{args.layers} distinct weight copies ({total_weight_bytes / 1e9:.2f} GB) walked cold",
                   "step": "one decoder layer = 7 projections" + (
                       ", 4 launches: btc_gemv_multi for q/k/v and for gate/up (shared input), btc_gemv for o and down"
                       if args.launches == "grouped" else ", 7 btc_gemv calls"), "launch": args.mode,
                   "timed": f"{repeats} x {args.steps} steps"},
        "us_per_call": round(us_per_call, 3),
        "launches_per_step": n_launches,
        ("separate_launches" if args.launches == "grouped" else "grouped_launches"): None if args.no_compare else {
            "ms_per_step": round(ms_other, 5), "value": round(step_bytes / (ms_other * 1e-3) / 1e9, 1), "unit": "GB/s",
            "launches_per_step": n_calls if args.launches == "grouped" else len(GROUPS)},
        "fp16_equivalent_GBps": round(fp16_equiv, 1),
        "frac_measured_peak": round(value / HBM_MEASURED_GBS, 4),
        "per_shape": per_shape,
        "gemm": gemm,
        "other_decode_configs": other,
        "roofline": {"bound": "hbm", "achieved": round(value, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(value / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "note": "algorithmic bytes of the 7 projections of a step / event-timed duration of a step "
                             f"({n_launches} launches); "
                             "traffic = HBM bytes per step (fetched + written) read from "
                             "profiles/gemv_13b_hbm_traffic.md (rocprofv3 counter runs), algorithmic bytes per step "
                             f"{step_bytes}"},
        "roofline_gemv_70b": roof70,
        "roofline_gemm": None if gemm is None else {
            "bound": "mfma", "achieved": gemm[f"M{args.gemm_m}"]["layer_tflops"], "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": gemm[f"M{args.gemm_m}"]["frac_mfma_peak"],
            "frac_measured_peak": gemm[f"M{args.gemm_m}"]["frac_measured_peak"], "traffic": None,
            "achieved_first_run": gemm[f"M{args.gemm_m}"]["layer_tflops_first_run"],
            "note": f"2*M*out*in flop of the 7 projections at M={args.gemm_m} / event-timed btc_gemm calls "
                    "(whole calls); " + gemm[f"M{args.gemm_m}"]["timing"]},
        "act_quant": act_quant,
        "gemv_groups": groups,
        "transform": transform,
        "assign": assign,
        "cpu_baseline": cpu,
        "setup_s": round(t_setup, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
