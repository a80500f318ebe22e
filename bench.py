#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: compress + sparse integer GEMMs of one BERT-base
encoder layer (QKV, attention output, FFN up, FFN down; 2:4 sparsity, int8 weights, 4096 tokens).

One step = for each of the four layers in turn, nm_compress of its fp32 weight matrix and then
nm_gemm against it (bias + bf16 output), all on one stream with inputs resident in HBM.  Prints one JSON line:
dense-equivalent int8 TOPS of the whole step, the roofline position of the dominant kernel, and
the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_DENSE_PEAK_TOPS = 5000.0        # MI355X dense int8 MFMA peak (sparsity not counted)
HBM_PEAK_GBS = 8000.0
# HBM bytes per nm_gemm launch (bf16 output, tiled layout) of the benchmark's four layers, from rocprofv3
# FETCH_SIZE and WRITE_SIZE passes scaled by what the same counters read on a plain 256 MiB copy.  Counters
# cannot be read from inside this process: the figures are those of the file named here and go stale with
# any change of the tiling (the file states the commit it was measured at).
TRAFFIC_PROFILE = "profiles/bert_base_2of4_int8_counters.txt"
MEASURED_HBM_BYTES_BF16 = {"qkv": 31.25e6, "attn_out": 12.59e6, "ffn_up": 40.54e6, "ffn_down": 30.88e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--out-dtype", choices=["bf16", "f32", "i8"], default="bf16",
                    help="i8: nm_gemm_q8, the layer output as int8 codes for the next layer (not the headline configuration)")
    ap.add_argument("--layout", choices=["tiled", "rows"], default="tiled",
                    help="layout of the packed weights: tiled (what the fast kernels read; the benchmark) or rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-streaming-leg", action="store_true",
                    help="skip the second timed leg (buffer sets rotated over more than the 256 MB Infinity Cache)")
    ap.add_argument("--no-power-leg", action="store_true",
                    help="skip the leg that runs the dominant GEMM's shape with a 16 times longer reduction for about two seconds and "
                         "reads board power and shader clock from rocm-smi meanwhile (what the K loop costs per step, and what bounds it)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    ap.add_argument("--workload", choices=["bert_base", "bert_large", "hetero", "table4", "table3", "single", "copy"], default="bert_base",
                    help="bert_base: the four GEMMs of a BERT-base layer at 4096 tokens (the benchmark); "
                         "bert_large: those of a BERT-large layer at 32x384 = 12288 tokens (the third workload of the "
                         "task's list; not the headline configuration); "
                         "hetero: the 48 GEMMs of a 12-layer BERT-base encoder with a seeded mix of 2:4 / 1:4 / 2:8 and "
                         "int8 / int4 schemes at 4096 tokens (the fifth workload of the task's list); "
                         "table4: the 72 GEMMs (query, key, value separately) of a 12-layer BERT-base encoder under one of the "
                         "configurations the paper's search chose (Sec. 5.4: dense and 2:4 components, 4- and 8-bit), see --task; "
                         "table3: the batch x sequence sweep of the paper's inference table (Sec. 5.3) on BERT-large, the 96 "
                         "GEMMs of 24 layers enqueued back to back for every token count; "
                         "single: one 768x768 layer at 128 tokens (the skinny shape, for profiling); "
                         "copy: a plain 256 MiB device copy (calibrates the HBM traffic counters)")
    ap.add_argument("--task", default="MNLI", help="row of the Sec. 5.4 table for --workload table4 (MNLI, SST-2, QNLI, QQP, CoLA, STS-B, MRPC, RTE)")
    ap.add_argument("--qkv", choices=["grouped", "separate"], default="grouped",
                    help="--workload table4: query, key and value layers of one scheme share a launch (nm_gemm_batch), or every layer "
                         "has its own nm_gemm call")
    ap.add_argument("--tokens", type=int, default=None,
                    help="token count for the bert_base / bert_large layer sets instead of the workload's own (batch x "
                         "sequence length of the paper's inference table, e.g. 128 x 384 = 49152): a sweep, not the benchmark")
    ap.add_argument("--only", default=None,
                    help="restrict the bert_base workload to one layer (qkv, attn_out, ffn_up, ffn_down): used by "
                         "the counter passes, which can tell dispatches apart only by kernel name and grid")
    ap.add_argument("--compress", choices=["batched", "per_layer"], default="batched",
                    help="batched: the step compresses all weight matrices with one nm_compress_batch call per scheme and "
                         "then runs the GEMMs; per_layer: nm_compress and nm_gemm alternate, layer by layer")
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph",
                    help="graph: the launches of a step are captured once in a HIP graph and replayed")
    return ap.parse_args()


def table3_sweep(args, lib, layout):
    """Sec. 5.3's inference table as a workload: BERT-large, batch {1, 32, 64, 128} x sequence {128, 384}, linear layers only.
    For every token count the 96 nm_gemm calls of 24 encoder layers (each layer with weight matrices of its own, compressed
    beforehand as at deployment; bias, bf16 output; activations handed on through one buffer per width) are captured in one
    HIP graph and replayed.  Prints one JSON line: the time of the 24-layer stack per token count."""
    import dataclasses
    import torch

    import paper_2206_15014_amd as nm
    from paper_2206_15014_amd import synth
    from paper_2206_15014_amd.binding import NM_OUT_BF16

    dev = torch.device("cuda:0")
    layers = 24
    shapes = synth.config3()
    gen = torch.Generator(device=dev)
    gen.manual_seed(3)
    packed = []                                             # [layer][gemm] -> (vals, meta, scales, bias)
    for _ in range(layers):
        row = []
        for g in shapes:
            W = torch.randn((g.O, g.K), generator=gen, device=dev, dtype=torch.float32) * 0.02
            v, m, sc = nm.nm_compress(W, g.N, g.M, g.bits, layout=layout)
            row.append((v, m, sc, torch.randn(g.O, generator=gen, device=dev, dtype=torch.float32) * 0.02))
        packed.append(row)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    sweep = []
    token_counts = [args.tokens] if args.tokens else [1 * 128, 1 * 384, 32 * 128, 64 * 128, 32 * 384, 128 * 128, 64 * 384, 128 * 384]
    for T in token_counts:
        X = {K: torch.randint(-127, 128, (T, K), generator=gen, device=dev, dtype=torch.int8) for K in (1024, 4096)}
        out = {g.name: torch.empty((T, g.O), dtype=torch.bfloat16, device=dev) for g in shapes}

        def enqueue(st):
            for row in packed:
                for g, (v, m, sc, b) in zip(shapes, row):
                    rc = lib.nm_gemm(X[g.K].data_ptr(), T, g.K, g.K, 0.05, None, v.data_ptr(), m.data_ptr(), sc.data_ptr(), g.O, g.N, g.M,
                                     g.bits, layout, b.data_ptr(), None, out[g.name].data_ptr(), NM_OUT_BF16, g.O, st)
                    if rc != 0:
                        raise RuntimeError("nm_gemm failed: %s" % nm.nm_status_string(rc))

        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            enqueue(side.cuda_stream)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                enqueue(side.cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(max(args.warmup // 10, 2)):
            graph.replay()
        torch.cuda.synchronize()
        reps = max(args.steps // 10, 5)
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / reps
        ops = layers * sum(dataclasses.replace(g, T=T).dense_ops for g in shapes)
        sweep.append({"tokens": T, "ms_24_layers": round(ms, 4), "us_per_gemm": round(ms * 1e3 / (4 * layers), 2),
                      "dense_equiv_tops": round(ops / (ms * 1e-3) / 1e12, 1)})
        del graph, X, out
    head = [r for r in sweep if r["tokens"] == 32 * 384] or sweep[-1:]
    print(json.dumps({
        "metric": "dense-equivalent int8 TOPS of N:M sparse GEMM (BERT shapes) + % of int8 roofline",
        "value": head[0]["dense_equiv_tops"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head[0]["ms_24_layers"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "BERT-large, 24 encoder layers x (QKV, attn-out, FFN-up, FFN-down) = 96 nm_gemm calls back to back in one HIP "
                               "graph, 2:4 int8, bias, bf16 out, %s layout; step = the 24-layer stack at 32x384=12288 tokens; sweep = the "
                               "batch x sequence grid of the paper's inference table (Sec. 5.3)" % args.layout},
        "pct_of_int8_dense_peak": round(100.0 * head[0]["dense_equiv_tops"] / INT8_DENSE_PEAK_TOPS, 2),
        "sweep": sweep}))


def smi_read():
    """(socket power in watts, shader clock in MHz, power limit in watts) as rocm-smi reports them now; None where it does not say."""
    import re
    import subprocess
    try:
        out = subprocess.run(["rocm-smi", "-a", "--json"], capture_output=True, text=True, timeout=30).stdout
        card = json.loads(out)
        card = card[sorted(card)[0]]
        m = re.search(r"(\d+)\s*Mhz", str(card.get("sclk clock speed:", "")), re.I)

        def num(key):
            try:
                return float(card.get(key))
            except (TypeError, ValueError):
                return None
        return (num("current_socket_power (W)"), int(m.group(1)) if m else None, num("Max Graphics Package Power (W)"))
    except Exception:
        return None


def k_loop_leg(args, lib, nm, torch, gd, Xd, layout, out_torch, out_code, timed_launches, check, dev):
    side = torch.cuda.Stream()
    mult = 16
    while mult > 2 and gd.T * gd.K * mult > (192 << 20):
        mult //= 2
    us = {}
    keep = None
    for m in (mult // 2, mult):
        K = gd.K * m
        W = torch.randn((gd.O, K), dtype=torch.float32, device=dev) * 0.02
        X = Xd.repeat(1, m).contiguous()      # the layer's own activations side by side: the loop's rate depends on the data (power)
        vals, meta, scales = nm.nm_compress(W, gd.N, gd.M, gd.bits, layout=layout)
        del W
        bias = torch.zeros(gd.O, dtype=torch.float32, device=dev)
        out = torch.empty((gd.T, gd.O), dtype=out_torch, device=dev)
        a = (X.data_ptr(), gd.T, K, K, 0.01, None, vals.data_ptr(), meta.data_ptr(), scales.data_ptr(), gd.O, gd.N, gd.M, gd.bits,
             layout, bias.data_ptr(), None, out.data_ptr(), out_code, gd.O, torch.cuda.current_stream().cuda_stream)
        us[m] = timed_launches(lib.nm_gemm, a, 10)
        keep = (a, X, vals, meta, scales, bias, out)
    steps_long, steps_half = gd.K * mult // 128, gd.K * mult // 256
    us_per_step = (us[mult] - us[mult // 2]) / (steps_long - steps_half)
    in_loop_tops = 2.0 * gd.T * gd.O * 128 / us_per_step / 1e6
    # about three seconds of the long launch in one go; two rocm-smi readings while they run
    a = keep[0]
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        b = a[:-1] + (side.cuda_stream,)
        check(lib.nm_gemm(*b))
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for _ in range(20):
                check(lib.nm_gemm(*b))
    torch.cuda.current_stream().wait_stream(side)
    replays = max(1, int(3.2e6 / (20 * us[mult])))
    import threading
    readings = []

    def sampler():
        for wait in (0.9, 0.9):
            time.sleep(wait)
            readings.append((smi_read(), not torch.cuda.current_stream().query()))
    th = threading.Thread(target=sampler)
    th.start()
    for _ in range(replays):
        g.replay()
    torch.cuda.synchronize()
    th.join()
    watts = sclk = cap = None
    good = [r for r, busy in readings if r is not None and busy]
    if good:
        watts, sclk, cap = good[-1]
    return {"shape": "%d tokens, K = %d and %d (%d and %d times the layer's, its activations repeated side by side), %d outputs" % (gd.T, gd.K * mult // 2, gd.K * mult, mult // 2, mult, gd.O),
            "us_long": round(us[mult], 2), "us_half": round(us[mult // 2], 2),
            "us_per_128_column_step": round(us_per_step, 4),
            "dense_equiv_tops_in_loop": round(in_loop_tops, 1),
            "frac_dense_peak_in_loop": round(in_loop_tops / INT8_DENSE_PEAK_TOPS, 4),
            "board_power_w": watts, "board_power_limit_w": cap, "sclk_mhz_in_loop": sclk,
            "note": "board power and shader clock: rocm-smi's readings about two seconds into three seconds of that launch repeated "
                    "back to back (null: rocm-smi gave nothing, or the launches had ended before the reading)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard over tokens or over output "
              "rows with no exchange between GPUs); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2206_15014_amd as nm
    from paper_2206_15014_amd import binding, synth
    from paper_2206_15014_amd.binding import NM_LAYOUT_ROWS, NM_LAYOUT_TILED, NM_OUT_BF16, NM_OUT_F32
    layout = NM_LAYOUT_TILED if args.layout == "tiled" else NM_LAYOUT_ROWS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.workload == "copy":
        n = 256 << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(max(args.steps, 1)):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"workload": "copy", "bytes_read_per_launch": n, "bytes_written_per_launch": n,
                          "launches": max(args.steps, 1)}))
        return
    lib = binding.raw()
    if args.workload == "table3":
        table3_sweep(args, lib, layout)
        return
    if args.workload == "single":
        g1 = synth.config1_tensors()[0]
        gemms = [synth.Gemm("single", g1.T, g1.K, g1.O, g1.N, g1.M, g1.bits, (1, 0, 0), outliers=False)]
        workload_name = "single 768x768 linear layer, 128 tokens, 2:4 int8"
    elif args.workload == "table4":
        gemms = synth.table4_encoder(args.task)
        workload_name = ("12-layer BERT-base encoder under the configuration chosen for %s in the paper's Sec. 5.4 table (%s for query, key, "
                         "value, attention output, FFN 1, FFN 2; Q = dense, S = 2:4), 72 GEMMs, 32x128=4096 tokens, activation and output "
                         "buffers shared between layers" % (args.task, " ".join(synth.TABLE4[args.task])))
    elif args.workload == "hetero":
        gemms = synth.config5()
        workload_name = ("heterogeneous 12-layer BERT-base encoder, 48 GEMMs, schemes drawn from {2:4 i8, 1:4 i8, 2:4 i4, "
                         "1:4 i4, 2:8 i4} by a seeded sampler, 32x128=4096 tokens, activation and output buffers shared between layers")
    else:
        gemms = synth.config3() if args.workload == "bert_large" else synth.config2()
        if args.tokens is not None:
            import dataclasses
            assert args.tokens > 0
            gemms = [dataclasses.replace(g, T=args.tokens) for g in gemms]
        if args.only is not None:
            gemms = [g for g in gemms if g.name == args.only]
            assert gemms, "--only names no layer of the workload"
        workload_name = ("BERT-large encoder layer linear set (QKV, attn-out, FFN-up, FFN-down), 2:4 int8, "
                         "32x384=12288 tokens" if args.workload == "bert_large" else
                         "BERT-base encoder layer linear set (QKV, attn-out, FFN-up, FFN-down), 2:4 int8, "
                         "32x128=4096 tokens")
        if args.tokens is not None:
            workload_name = workload_name[:workload_name.rindex(",") + 1] + " %d tokens" % args.tokens
    out_code = NM_OUT_BF16 if args.out_dtype == "bf16" else NM_OUT_F32
    out_torch = {"bf16": torch.bfloat16, "f32": torch.float32, "i8": torch.int8}[args.out_dtype]
    out_bytes = {"bf16": 2, "f32": 4, "i8": 1}[args.out_dtype]

    # ---- resident inputs and preallocated outputs -------------------------------------------
    host = []
    jobs = []
    # The 12-layer encoder keeps one activation buffer per reduction width and one output buffer per
    # layer shape, as an encoder does whose layers hand their activations on; the one-layer sets
    # give every GEMM its own.
    shared = args.workload in ("hetero", "table4")
    acts, outs = {}, {}
    for g in gemms:
        W = synth.weights(g)
        if not shared or g.K not in acts:
            Xq, sx = synth.activations(g)
            acts[g.K] = (Xq, sx, torch.from_numpy(Xq).to(dev))
        Xq, sx, Xd = acts[g.K]
        if not shared or g.name not in outs:
            outs[g.name] = torch.empty((g.T, g.O), dtype=out_torch, device=dev)
        b = synth.bias(g)
        host.append((g, W, Xq, sx, b))
        vb, mb, _ = nm.nm_packed_sizes(g.O, g.K, g.N, g.M, g.bits, layout)
        jobs.append(dict(
            g=g, sx=float(sx),
            W=torch.from_numpy(W).to(dev), X=Xd, bias=torch.from_numpy(b).to(dev),
            vals=torch.empty(vb, dtype=torch.uint8, device=dev), meta=torch.empty(mb, dtype=torch.uint8, device=dev),
            scales=torch.empty(g.O, dtype=torch.float32, device=dev),
            out=outs[g.name],
            absmax=torch.zeros(1, dtype=torch.float32, device=dev)))
    stream = torch.cuda.current_stream().cuda_stream

    def compress_args(j):
        g = j["g"]
        return (j["W"].data_ptr(), g.O, g.K, g.K, g.N, g.M, g.bits, layout, j["vals"].data_ptr(), j["meta"].data_ptr(),
                j["scales"].data_ptr(), stream)

    gemm_fn = lib.nm_gemm_q8 if args.out_dtype == "i8" else lib.nm_gemm

    def gemm_args(j):
        g = j["g"]
        if args.out_dtype == "i8":         # any positive scale times the same: 1/16 keeps most codes inside the range
            return (j["X"].data_ptr(), g.T, g.K, g.K, j["sx"], None, j["vals"].data_ptr(), j["meta"].data_ptr(),
                    j["scales"].data_ptr(), g.O, g.N, g.M, g.bits, layout, j["bias"].data_ptr(), 0.0625, None, j["out"].data_ptr(),
                    g.O, j["absmax"].data_ptr(), stream)
        return (j["X"].data_ptr(), g.T, g.K, g.K, j["sx"], None, j["vals"].data_ptr(), j["meta"].data_ptr(),
                j["scales"].data_ptr(), g.O, g.N, g.M, g.bits, layout, j["bias"].data_ptr(), None, j["out"].data_ptr(),
                out_code, g.O, stream)

    cargs = [compress_args(j) for j in jobs]
    gargs = [gemm_args(j) for j in jobs]

    def check(rc):
        if rc != 0:
            raise RuntimeError("libnm call failed: %s" % nm.nm_status_string(rc))

    # one nm_compress_batch call per weight scheme (a single one for the homogeneous layer sets)
    batches = []
    for scheme in sorted({(j["g"].N, j["g"].M, j["g"].bits) for j in jobs}):
        js = [j for j in jobs if (j["g"].N, j["g"].M, j["g"].bits) == scheme]
        items = binding.compress_items([j["W"] for j in js], [(j["vals"], j["meta"], j["scales"]) for j in js])
        batches.append((items, len(js)) + scheme + (layout,))

    # The GEMM launches of a step: one nm_gemm per layer, except that the query / key / value layers of an
    # attention block that share a scheme (and their input) go through one nm_gemm_batch call.
    units = [(gemm_fn, ga[:-1]) for ga in gargs]
    unit_members = [[k] for k in range(len(gargs))]          # which layers each launch of the step computes
    grouped_launches = 0
    if args.workload == "table4" and args.qkv == "grouped" and args.out_dtype != "i8":
        units, unit_members, keep_items, i = [], [], [], 0
        scheme = lambda j: (j["g"].N, j["g"].M, j["g"].bits, j["g"].K, j["X"].data_ptr())
        while i < len(jobs):
            block = [i]
            if jobs[i]["g"].name == "query":      # the three projections of one attention block are independent of each other
                while i + len(block) < len(jobs) and jobs[i + len(block)]["g"].name in ("key", "value"):
                    block.append(i + len(block))
            done = set()
            for k in block:
                if k in done:
                    continue
                run = [m for m in block if m not in done and scheme(jobs[m]) == scheme(jobs[k])]
                done.update(run)
                if len(run) > 1:
                    g = jobs[k]["g"]
                    items = binding.gemm_items([dict(X=jobs[m]["X"], act_scale=jobs[m]["sx"], vals=jobs[m]["vals"], meta=jobs[m]["meta"],
                                                     scales=jobs[m]["scales"], O=jobs[m]["g"].O, bias=jobs[m]["bias"], out=jobs[m]["out"])
                                                for m in run])
                    keep_items.append(items)
                    units.append((lib.nm_gemm_batch, (items, len(run), g.N, g.M, g.bits, layout, out_code)))
                    unit_members.append(list(run))
                    grouped_launches += 1
                else:
                    units.append((gemm_fn, gargs[k][:-1]))
                    unit_members.append([k])
            i += len(block)

    def run_step(st, mode=None):
        """The launches of one step on stream `st`."""
        if (mode or args.compress) == "batched":
            for b in batches:
                check(lib.nm_compress_batch(*b, st))
            for fn, ua in units:
                check(fn(*(ua + (st,))))
        else:
            for ca, ga in zip(cargs, gargs):
                check(lib.nm_compress(*(ca[:-1] + (st,))))
                check(gemm_fn(*(ga[:-1] + (st,))))

    def step():
        run_step(stream)

    side = torch.cuda.Stream()

    def timed_launches(fn, a, reps):
        """Microseconds per launch: `reps` launches captured into one HIP graph on a side stream and replayed
        back to back, HIP events around the replays.  (Issued one by one from Python, launches this short
        would be bound by the host, more so under a profiler.)  With --launch eager no graph is built
        anywhere in the run and the launches are issued one by one."""
        if args.launch == "eager":
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for _ in range(3):
                check(fn(*a))
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                check(fn(*a))
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps
        g = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            b = a[:-1] + (side.cuda_stream,)
            for _ in range(3):
                check(fn(*b))
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                for _ in range(reps):
                    check(fn(*b))
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = 5
        e0.record()
        for _ in range(n):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (n * reps)

    # ---- warm-up, and which kernel dominates the step ---------------------------------------
    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    per_gemm_us = [timed_launches(gemm_fn, a, 40) for a in gargs]
    per_comp_us = [timed_launches(lib.nm_compress, a, 40) for a in cargs]
    batch_comp_us = sum(timed_launches(lib.nm_compress_batch, b + (stream,), 40) for b in batches)
    # The dominant kernel: a kernel trace lists the step's launches by kernel name, i.e. by the tile variant the
    # library chose for each launch (a measurement hook of the library reports it).  The dominant kernel is the
    # variant whose launches take the largest share of the step's GEMM time; the roofline is priced on the longest
    # of its launches (a launch of nm_gemm_batch counts with all the layers it computes).
    def moved_bytes(g):
        kc = g.K // g.M * g.N
        return g.T * g.K + g.O * kc * (g.bits + synth.index_bits(g.N, g.M)) // 8 + 8 * g.O + g.T * g.O * out_bytes
    unit_us, unit_variant = [], []
    for (fn, ua), mem in zip(units, unit_members):
        check(fn(*(ua + (stream,))))
        g = gemms[mem[0]]
        unit_variant.append((lib.nm_bench_last_gemm_tile(), g.N, g.M, g.bits, len(mem)))
        unit_us.append(per_gemm_us[mem[0]] if len(mem) == 1 else timed_launches(fn, ua + (stream,), 40))
    torch.cuda.synchronize()
    share = {}
    for v, u in zip(unit_variant, unit_us):
        share[v] = share.get(v, 0.0) + u
    top = max(share, key=lambda v: share[v])
    dom_unit = max((i for i, v in enumerate(unit_variant) if v == top),
                   key=lambda i: (unit_us[i], sum(moved_bytes(gemms[m]) for m in unit_members[i])))
    dom_members = unit_members[dom_unit]
    dom = dom_members[0]

    # ---- timed region -----------------------------------------------------------------------
    # The launches of a step are short (4-20 us each), so they are captured once into a HIP
    # graph and the graph is replayed; the eager mode issues them one by one from Python.
    graph = None
    # Several steps per graph (the largest divisor of --steps up to 20), so that the cost of starting
    # a graph replay is not paid once per 70 us step.
    steps_per_graph = max(d for d in range(1, 21) if args.steps % d == 0) if args.launch == "graph" else 1
    if args.launch == "graph":
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            cap_stream = side.cuda_stream
            with torch.cuda.graph(graph, stream=side):
                for _ in range(steps_per_graph):
                    run_step(cap_stream)
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(3):
            graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        for k in range(args.steps // steps_per_graph):
            graph.replay()
    else:
        for k in range(args.steps):
            step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    # The same work with the other arrangement of the compress calls, timed the same way and reported beside it.
    other_mode = "per_layer" if args.compress == "batched" else "batched"
    other_ms = None
    if graph is not None:
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2, stream=side):
                for _ in range(steps_per_graph):
                    run_step(side.cuda_stream, other_mode)
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(3):
            g2.replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for k in range(args.steps // steps_per_graph):
            g2.replay()
        torch.cuda.synchronize()
        other_ms = (time.perf_counter() - t2) * 1e3 / args.steps
    # Launch duration of the dominant kernel: HIP events around back-to-back (graph-replayed) launches
    # of that same kernel, right after the timed steps; a rocprofv3 kernel trace of this command
    # reports the same kernel about a microsecond shorter (the gap between two launches).
    dom_us = timed_launches(units[dom_unit][0], units[dom_unit][1] + (stream,), 40)

    # ---- second timed leg: the same step over buffer sets rotated through more than the Infinity Cache holds ----
    # Every set has its own weights, packed buffers, activations and outputs (copies of the first set), so
    # a step finds none of its operands in the 256 MB Infinity Cache or the L2s: the HBM-streaming figure
    # beside the cache-hot one above (whose whole footprint stays resident between steps).
    streaming = None
    if not args.no_streaming_leg and args.launch == "graph" and args.workload in ("bert_base", "bert_large"):
        set_bytes = sum(j[k].numel() * j[k].element_size() for j in jobs for k in ("W", "X", "vals", "meta", "out"))
        nsets = max(2, -(-(320 << 20) // set_bytes))
        sets = []
        for _ in range(nsets):
            js2 = [dict(j, W=j["W"].clone(), X=j["X"].clone(), vals=torch.empty_like(j["vals"]), meta=torch.empty_like(j["meta"]),
                        scales=torch.empty_like(j["scales"]), out=torch.empty_like(j["out"])) for j in jobs]
            items = binding.compress_items([j["W"] for j in js2], [(j["vals"], j["meta"], j["scales"]) for j in js2])
            g0 = js2[0]["g"]
            sets.append((js2, (items, len(js2), g0.N, g0.M, g0.bits, layout), [gemm_args(j) for j in js2]))
        reps = max(1, 20 // nsets)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _, b, gas in sets:                      # warm-up outside the capture
                check(lib.nm_compress_batch(*b, side.cuda_stream))
                for ga in gas:
                    check(gemm_fn(*(ga[:-1] + (side.cuda_stream,))))
            side.synchronize()
            g3 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g3, stream=side):
                for _ in range(reps):
                    for _, b, gas in sets:
                        check(lib.nm_compress_batch(*b, side.cuda_stream))
                        for ga in gas:
                            check(gemm_fn(*(ga[:-1] + (side.cuda_stream,))))
        torch.cuda.current_stream().wait_stream(side)
        g3.replay()
        torch.cuda.synchronize()
        n_rep = max(1, args.steps // (reps * nsets))
        t4 = time.perf_counter()
        for _ in range(n_rep):
            g3.replay()
        torch.cuda.synchronize()
        st_ms = (time.perf_counter() - t4) * 1e3 / (n_rep * reps * nsets)
        streaming = {"ms_per_step": round(st_ms, 5), "buffer_sets": nsets, "footprint_MB": round(nsets * set_bytes / 1e6, 1),
                     "note": "HBM-streaming: every step works on another of %d buffer sets (weights, packed buffers, "
                             "activations, outputs), %d MB in all, more than the 256 MB Infinity Cache" % (nsets, nsets * set_bytes // 1000000)}
        del sets

    # ---- the matrix pipe on its own: register-resident loop of the sparse MFMA, and the shader clock under it ----
    counters = torch.zeros(4, dtype=torch.int64, device=dev)
    probe_blocks, probe_iters = 256 * 8, 4096
    check(lib.nm_bench_smfmac_probe(probe_blocks, probe_iters, counters.data_ptr(), stream))
    torch.cuda.synchronize()
    pe0, pe1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pe0.record()
    check(lib.nm_bench_smfmac_probe(probe_blocks, probe_iters, counters.data_ptr(), stream))
    pe1.record()
    torch.cuda.synchronize()
    probe_s = pe0.elapsed_time(pe1) * 1e-3
    cyc, ticks = int(counters[0].item()), int(counters[1].item())
    sclk_mhz = cyc / max(ticks, 1) * 100.0
    smfmac_peak_tops = probe_blocks * 4 * probe_iters * 8 * (2 * 16 * 16 * 128) / probe_s / 1e12

    dense_ops = sum(g.dense_ops for g in gemms)
    value = dense_ops / (ms_per_step * 1e-3) / 1e12

    # ---- the K loop on its own, and what the board does under it --------------------------------------------
    # The dominant GEMM's token count and output width with a reduction 16 and 8 times as long: the difference of
    # the two durations is the cost of the K steps alone (launch, first loads and stores cancel).  While the long
    # one runs for about three seconds, rocm-smi's socket power and shader clock are read twice: the loop runs
    # at the board's power limit with the clock pulled down, which - not the L2s, the LDS or the matrix pipe -
    # is what sets its rate when every CU is busy.
    k_loop = None
    if not args.no_power_leg and args.launch == "graph" and args.workload in ("bert_base", "bert_large") and args.out_dtype != "i8":
        k_loop = k_loop_leg(args, lib, nm, torch, gemms[dom], jobs[dom]["X"], layout, out_torch, out_code, timed_launches, check, dev)

    gd = gemms[dom]
    names = [g.name for g in gemms]
    if len(set(names)) < len(names):       # several layers: say which layer and scheme
        names = ["L%02d.%s %d:%d i%d" % (g.seed[1], g.name, g.N, g.M, g.bits) for g in gemms]
    achieved = sum(gemms[m].dense_ops for m in dom_members) / (dom_us * 1e-6) / 1e12
    # int8 operations the method performs (pruned products never formed), and the bytes one launch has to move
    # (layers of one nm_gemm_batch launch that read the same activations read them once)
    real_ops = sum(2 * gemms[m].T * gemms[m].O * (gemms[m].K // gemms[m].M * gemms[m].N) for m in dom_members)
    alg_bytes = sum(moved_bytes(gemms[m]) for m in dom_members)
    seen_x = set()
    for m in dom_members:
        if jobs[m]["X"].data_ptr() in seen_x:
            alg_bytes -= gemms[m].T * gemms[m].K
        seen_x.add(jobs[m]["X"].data_ptr())
    frac_real = real_ops / (dom_us * 1e-6) / 1e12 / INT8_DENSE_PEAK_TOPS
    frac_hbm = alg_bytes / (dom_us * 1e-6) / 1e9 / HBM_PEAK_GBS
    hbm_bound = frac_hbm >= frac_real
    comp_bytes = sum(g.O * g.K * 4 + g.O * (g.K // g.M * g.N) * (g.bits + synth.index_bits(g.N, g.M)) // 8 + g.O * 4 for g in gemms)
    result = {
        "metric": "dense-equivalent int8 TOPS of N:M sparse GEMM (BERT shapes) + % of int8 roofline",
        "value": round(value, 2),
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": workload_name + "; step = %s (bias, %s out), %s launch%s"
                               % ("nm_compress_batch over the %d weight matrices (%d call%s), then the %d nm_gemm calls"
                                  % (len(gemms), len(batches), "" if len(batches) == 1 else "s, one per scheme", len(gemms))
                                  if args.compress == "batched" else
                                  "%d x (nm_compress, nm_gemm) layer by layer" % len(gemms), args.out_dtype, args.launch,
                                  " (%d steps per graph)" % steps_per_graph if graph is not None else ""),
                   "tokens": gemms[0].T, "hidden": min(g.K for g in gemms), "pattern": "/".join(sorted({"%d:%d" % (g.N, g.M) for g in gemms})),
                   "weight_bits": "/".join(sorted({str(g.bits) for g in gemms})), "out_dtype": args.out_dtype},
        "pct_of_int8_dense_peak": round(100.0 * value / INT8_DENSE_PEAK_TOPS, 2),
        "same_work_with_%s_compress" % other_mode: None if other_ms is None else {
            "ms_per_step": round(other_ms, 5), "value": round(dense_ops / (other_ms * 1e-3) / 1e12, 2)},
        "streaming_leg": streaming,
        "k_loop_leg": k_loop,
        "gemm_launches_per_step": len(units),
        "dominant_kernel": {"tile_variant": top[0], "pattern": "%d:%d int%d" % top[1:4], "layers_per_launch": top[4], "launches_per_step": sum(1 for v in unit_variant if v == top),
                            "us_of_gemm_us": [round(share[top], 2), round(sum(unit_us), 2)],
                            "note": "the step's nm_gemm launches grouped by the kernel variant the library chose for them (as a kernel trace groups "
                                    "them by name); the group with the largest share of the time; `roofline` is its longest launch"},
        "grouped_qkv_launches": grouped_launches,
        "roofline": {
            # the roof that binds this kernel: the larger of its two fractions, both from the method's own work
            "bound": "hbm" if hbm_bound else "mfma",
            "achieved": round(alg_bytes / (dom_us * 1e-6) / 1e9, 1) if hbm_bound else round(real_ops / (dom_us * 1e-6) / 1e12, 1),
            "peak": HBM_PEAK_GBS if hbm_bound else INT8_DENSE_PEAK_TOPS,
            "unit": "GB/s" if hbm_bound else "TFLOP/s",
            "frac": round(max(frac_hbm, frac_real), 4),
            "frac_hbm": round(frac_hbm, 4),                  # algorithmic bytes / duration against 8 TB/s
            "frac_real_ops": round(frac_real, 4),            # 2*T*O*kc int8 ops / duration against the dense int8 MFMA peak
            "frac_dense_equiv": round(achieved / INT8_DENSE_PEAK_TOPS, 4),   # 2*T*O*K (pruned zeros counted): the reading of the task's 50 % target
            "dense_equiv_tops": round(achieved, 1),
            "traffic": MEASURED_HBM_BYTES_BF16.get(gd.name) if (args.workload == "bert_base" and args.out_dtype == "bf16" and args.layout == "tiled") else None,
            "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated on a copy); a stored figure from " + TRAFFIC_PROFILE,
            "algorithmic_bytes": alg_bytes,
            "real_int8_ops": real_ops,
            "kernel": "%s %s %dx%d->%s %d:%d int%d" % ("nm_gemm" if len(dom_members) == 1 else "nm_gemm_batch", "+".join(gemms[m].name for m in dom_members),
                                                       gd.T, gd.K, "+".join(str(gemms[m].O) for m in dom_members), gd.N, gd.M, gd.bits),
            "note": "duration = HIP events around 200 back-to-back launches of this kernel (5 replays of a 40-launch graph) after "
                    "the timed steps; operands cache-hot (one buffer set)",
            "duration_us": round(dom_us, 2),
            "measured_smfmac_peak_tops": round(smfmac_peak_tops, 1),   # register-resident sparse-MFMA loop, dense-equivalent
            "sclk_mhz": round(sclk_mhz, 0),                  # shader clock under that loop (cycle counter against the 100 MHz clock)
        },
        "kernels": {
            "gemm_us_back_to_back": {n: round(u, 2) for n, u in zip(names, per_gemm_us)},
            "gemm_dense_equiv_tops": {n: round(g.dense_ops / u / 1e6, 1) for n, g, u in zip(names, gemms, per_gemm_us)},
            "compress_us_back_to_back": {n: round(u, 2) for n, u in zip(names, per_comp_us)},
            "compress_batch_us_back_to_back": round(batch_comp_us, 2),
            "compress_batch_GBps": round(comp_bytes / (batch_comp_us * 1e-6) / 1e9, 1),
            "compress_GBps": round(comp_bytes / (sum(per_comp_us) * 1e-6) / 1e9, 1),
            "compress_frac_of_hbm_peak": round(comp_bytes / (sum(per_comp_us) * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        },
    }

    # ---- the skinny shape (one 768x768 layer, 128 tokens): latency-bound, reported as HBM GB/s ------
    if args.workload == "bert_base" and args.only is None:
        gs, Ws, Xs, sxs = synth.config1_tensors()
        js = dict(g=gs, sx=float(sxs), W=torch.from_numpy(Ws).to(dev), X=torch.from_numpy(Xs).to(dev),
                  bias=torch.zeros(gs.O, dtype=torch.float32, device=dev))
        vb, mb, _ = nm.nm_packed_sizes(gs.O, gs.K, gs.N, gs.M, gs.bits, layout)
        js.update(vals=torch.empty(vb, dtype=torch.uint8, device=dev), meta=torch.empty(mb, dtype=torch.uint8, device=dev),
                  scales=torch.empty(gs.O, dtype=torch.float32, device=dev),
                  out=torch.empty((gs.T, gs.O), dtype=out_torch, device=dev),
                  absmax=torch.zeros(1, dtype=torch.float32, device=dev))
        check(lib.nm_compress(*compress_args(js)))
        us = timed_launches(gemm_fn, gemm_args(js), 40)
        esz = out_bytes
        nbytes = gs.T * gs.K + vb + mb + 8 * gs.O + gs.T * gs.O * esz
        result["kernels"]["skinny_gemm_128x768x768"] = {
            "us_back_to_back": round(us, 2), "algorithmic_bytes": nbytes, "GBps": round(nbytes / us / 1e3, 1),
            "dense_equiv_tops": round(gs.dense_ops / us / 1e6, 1)}

    # ---- fp32 activations of the first layer's shape -> int8 codes (statistic, scale, codes; all on the device) ----
    if args.workload in ("bert_base", "bert_large") and args.only is None:
        g0 = gemms[0]
        Xf = torch.randn((g0.T, g0.K), dtype=torch.float32, device=dev)
        Xq8 = torch.empty((g0.T, g0.K), dtype=torch.int8, device=dev)
        amax = torch.zeros(1, dtype=torch.float32, device=dev)
        s_x = torch.ones(1, dtype=torch.float32, device=dev)

        def act_chain(X, T, K, am, sc, Q, st):
            return (lib.nm_absmax_to_scale(am, sc, 1, st) or lib.nm_absmax_f32(X, T, K, K, am, st)
                    or lib.nm_absmax_to_scale(am, sc, 0, st) or lib.nm_quantize_act(X, T, K, K, 0.0, sc, Q, K, st))
        a_chain = (Xf.data_ptr(), g0.T, g0.K, amax.data_ptr(), s_x.data_ptr(), Xq8.data_ptr(), stream)
        us_chain = timed_launches(act_chain, a_chain, 20)
        us_q = timed_launches(lib.nm_quantize_act, (Xf.data_ptr(), g0.T, g0.K, g0.K, 0.0, s_x.data_ptr(), Xq8.data_ptr(), g0.K, stream), 20)
        result["kernels"]["act_quantize_%dx%d" % (g0.T, g0.K)] = {
            "us_statistic_scale_codes": round(us_chain, 2), "algorithmic_bytes": 9 * g0.T * g0.K,
            "GBps": round(9 * g0.T * g0.K / us_chain / 1e3, 1),
            "us_codes_only": round(us_q, 2), "GBps_codes_only": round(5 * g0.T * g0.K / us_q / 1e3, 1),
            "note": "fp32 -> int8 with the tensor's own max|x|/127: the statistic is reset and recomputed in every repetition "
                    "(four launches); back to back, the tensor stays in the Infinity Cache"}

    # ---- CPU oracle on a bounded sample of the same workload --------------------------------
    if not args.no_cpu_baseline:
        import oracle
        n = min(args.cpu_sample_tokens, gemms[0].T, 4096 if len(gemms) <= 4 else 512)   # 48 GEMMs: a smaller token sample
        ops = 0
        c0 = time.perf_counter()
        for g, W, Xq, sx, b in host:
            v, m, s = oracle.compress(W, g.N, g.M, g.bits)
            acc = oracle.gemm_sparse(Xq[:n], v, m, g.O, g.N, g.M, g.bits)
            oracle.dequant(acc, float(sx), s, b)
            ops += 2 * n * g.K * g.O
        c1 = time.perf_counter()
        result["cpu_baseline"] = {
            "value": round(ops / (c1 - c0) / 1e12, 6), "unit": "TOPS (dense-equivalent int8)",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "all %d weight matrices compressed in full, GEMM + dequant on the first %d of %d tokens "
                      "of each layer (%.1f s)" % (len(host), n, gemms[0].T, c1 - c0),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
