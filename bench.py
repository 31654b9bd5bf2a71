#!/usr/bin/env python3
"""Benchmark of the feature-loading path on one MI355X.

A *step* is one minibatch launch-set of the per-iteration path: decode the
input-node rows (gather_dequant) and, for every hop's sampled block, the fused
gather + decode + neighbourhood mean (gather_mean), all against the packed
table resident in HBM.  ``--batches-per-step L`` concatenates L independently
sampled minibatches into each launch (what a prefetching loader hands over);
L = 1 is one 1,024-seed minibatch per launch.  The one-time fit + quantize pass
that builds the table runs before the timed region and is reported separately
under "preprocess".

Prints ONE JSON line on stdout: metric / value / unit (whole-step rows per
second), ms_per_step, config (the workload), "roofline" for the fused
gather + decode + mean kernel on the outermost block (algorithmic bytes over its
HIP-event duration against the 8 TB/s HBM peak; "traffic" = counter-measured
bytes per launch when a profile summary for this workload is present), "kernels"
(the same for every call of the step), "cpu_baseline" (the CPU oracle on the host cores, a bounded sample)
and "preprocess"; with ``--scale-profile LAYERS`` also "scale_profile" (the
aggregation scale factors of the workload's codes on a graph of its family).
Progress lines go to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="largest4",
                    choices=["tiny", "mid", "large", "largest1", "largest4", "vq", "vq2k", "log2", "log4", "log1"])
    ap.add_argument("--rows", type=int, default=0, help="override N (debugging)")
    ap.add_argument("--batches", type=int, default=0, help="distinct pre-sampled launch-sets")
    ap.add_argument("--batches-per-step", type=int, default=0)
    ap.add_argument("--chunk-rows", type=int, default=1 << 20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (counter calibration under rocprofv3)")
    ap.add_argument("--mean-slots", type=int, default=0)
    ap.add_argument("--mean-blocks", type=int, default=0)
    ap.add_argument("--max-blocks", type=int, default=0)
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE",
                    help="library launch option (bifeat_set_option), repeatable")
    ap.add_argument("--no-degree-hint", action="store_true",
                    help="do not tell the library the sampler's fan-out (it then also scans for longer lists)")
    ap.add_argument("--graph", action="store_true",
                    help="replay each launch-set's step from a captured HIP graph (whole-step "
                         "timing; per-kernel figures still come from an eager pass)")
    ap.add_argument("--no-two-hop", action="store_true",
                    help="skip the two-round aggregation leg (fused call against the two-call chain)")
    ap.add_argument("--scale-profile", type=int, default=0, metavar="LAYERS",
                    help="after the timed region, also run the aggregation scale profile (error and "
                         "feature scale after 1..LAYERS rounds of neighbourhood averaging, and their "
                         "ratio) of this workload's codes on a materialised graph of the same family")
    ap.add_argument("--profile-nodes", type=int, default=1 << 20,
                    help="nodes (= leading rows of the table) of the scale-profile graph")
    ap.add_argument("--row-align", type=int, default=16, choices=[16, 128],
                    help="row stride of the packed table: 16 = rows back to back, 128 = line-aligned rows "
                         "(a 96-byte row then costs one 128-byte line per gather instead of 1.5)")
    ap.add_argument("--idx32", action="store_true",
                    help="pass the blocks' list entries as int32 (bifeat_gather_mean_i32): 4 instead of 8 "
                         "index bytes per entry, in the traffic and in the algorithmic bytes")
    ap.add_argument("--aggregator", default="mean", choices=["mean", "sum"],
                    help="which fused aggregation the hops run (the metric's workload is mean)")
    return ap.parse_args()


def traffic_from_profile(workload: str, kernel: str):
    """HBM bytes per launch of a kernel, from the committed rocprofv3 --pmc
    summary for this workload (None if there is none)."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}.md")
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch\s*[:=]\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def say(msg: str):
    """Progress line (stderr): the one JSON result line stays alone on stdout."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures the one-GPU path only: this build has no multi-GPU leg "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2207_14696_amd as bf
    from bifeat_inputs import WORKLOADS, BATCHES_PER_STEP, make_graph, launch_set, feature_rows
    from bifeat_inputs.device import DeviceTable

    w = WORKLOADS[args.workload]
    if args.rows:
        w = w.scaled(args.rows)
    L = args.batches_per_step or BATCHES_PER_STEP[w.name.split("@")[0]]
    B = args.batches or 8
    torch.cuda.set_device(0)
    dev = "cuda"

    # ------------------------------------------------------------ the table
    kind = {"uniform": bf.UNIFORM, "log": bf.LOG, "vq": bf.VQ}[w.kind]
    q = bf.Quantizer(bf.Scheme(kind, w.bits, w.vq_width if w.kind == "vq" else 0,
                               w.vq_length if w.kind == "vq" else 0,
                               bf.VQ_COSINE if w.vq_metric == "cosine" else bf.VQ_L2), w.D,
                     row_align=args.row_align)
    for opt in ("mean_slots", "mean_blocks", "max_blocks"):
        if getattr(args, opt):
            q.set_option(opt, getattr(args, opt))
    for kv in args.opt:
        name, value = kv.split("=")
        q.set_option(name, int(value))
    table = DeviceTable(w.spec)
    stride = q.row_bytes                       # bytes from row to row in the resident table
    rb = bf.Quantizer(bf.Scheme(kind, w.bits, w.vq_width if w.kind == "vq" else 0,
                                w.vq_length if w.kind == "vq" else 0), w.D).row_bytes  # bytes of codes per row
    codes = torch.empty((w.N, stride), dtype=torch.uint8, device=dev)
    chunk_rows = min(args.chunk_rows, w.N)
    buf = torch.empty((chunk_rows, w.D), dtype=table.torch_dtype, device=dev)
    esz = 4 if w.dtype == "f32" else 2
    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    pre = {}
    if w.kind == "vq":
        # codebooks: 10 Lloyd rounds on the GPU over a 65 536-row sample (rows of the
        # synthetic table are i.i.d., so its first rows are a uniform sample)
        ns = min(w.N, 1 << 16)
        sample = table.chunk(0, ns)
        a, b = ev(), ev()
        a.record()
        q.fit_update(sample)
        q.fit_finalize()
        b.record()
        b.synchronize()
        pre["vq_train_ms"] = a.elapsed_time(b)
        pre["vq_train_rows"] = ns
        del sample
        say(f"codebooks trained on {ns} rows")
    else:
        fit_ms = gen_ms = 0.0
        if w.kind == "log" and w.log_clip > 0:
            q.fit_set_log_clip(w.log_clip)      # exact clipped range: three passes over the table
        q.fit_reset()
        again, passes = True, 0
        while again:
            for r0 in range(0, w.N, chunk_rows):
                n = min(chunk_rows, w.N - r0)
                g0, a, b = ev(), ev(), ev()
                g0.record()
                table.chunk(r0, n, buf[:n])
                a.record()
                q.fit_update(buf[:n])
                b.record()
                b.synchronize()
                gen_ms += g0.elapsed_time(a)
                fit_ms += a.elapsed_time(b)
                if (r0 // chunk_rows) % 64 == 63:
                    say(f"fit pass {passes + 1}: {r0 + n} of {w.N} rows")
            again = q.fit_finalize()
            passes += 1
        pre["fit_GBps"] = passes * w.N * w.D * esz / fit_ms / 1e6
        pre["fit_passes"] = passes
        pre["chunk_generation_ms_per_pass"] = gen_ms / passes
    quant_ms = 0.0
    for r0 in range(0, w.N, chunk_rows):
        n = min(chunk_rows, w.N - r0)
        table.chunk(r0, n, buf[:n])
        a, b = ev(), ev()
        a.record()
        q.quantize(buf[:n], codes, r0)
        b.record()
        b.synchronize()
        quant_ms += a.elapsed_time(b)
        if (r0 // chunk_rows) % 64 == 63:
            say(f"quantize pass: {r0 + n} of {w.N} rows")
    say(f"table built: {w.N} rows x {stride} B")
    pre["quantize_GBps"] = (w.N * w.D * esz + w.N * rb) / quant_ms / 1e6
    pre["quantize_rows_per_s"] = w.N / quant_ms * 1e3
    pre["table_GB"] = w.N * stride / 1e9
    del buf
    if w.kind == "uniform" or (w.kind == "log" and w.log_clip == 0):
        # the same preprocessing with the table produced inside the library's kernels (the
        # synthetic generator as a row source, include/bifeat_produce.hpp): the raw chunk is
        # never written or read, only codes reach memory.  A second handle is fitted that way
        # and re-encodes the resident table in place - to the same bytes.
        q2 = bf.Quantizer(q.scheme, w.D, row_align=args.row_align)
        head = codes[:min(w.N, 1 << 18)].clone()
        tail = codes[-min(w.N, 1 << 18):].clone()
        q2.fit_reset()
        a, b, c = ev(), ev(), ev()
        a.record()
        for r0 in range(0, w.N, 16 * chunk_rows):
            table.fit_into(q2, r0, min(16 * chunk_rows, w.N - r0))
        q2.fit_finalize()
        b.record()
        for r0 in range(0, w.N, 16 * chunk_rows):
            table.quantize_into(q2, codes, r0, min(16 * chunk_rows, w.N - r0))
        c.record()
        c.synchronize()
        same = (q2.params_get_uniform() if w.kind == "uniform" else q2.params_get_log()[:2])
        ref = (q.params_get_uniform() if w.kind == "uniform" else q.params_get_log()[:2])
        same = all(np.array_equal(x, y) for x, y in zip(same, ref)) and bool(
            torch.equal(head, codes[:head.shape[0]]) and torch.equal(tail, codes[-tail.shape[0]:]))
        pre["produced_fit_ms"] = a.elapsed_time(b)
        pre["produced_quantize_ms"] = b.elapsed_time(c)
        pre["produced_fit_Gvalues_per_s"] = w.N * w.D / a.elapsed_time(b) / 1e6
        pre["produced_quantize_Gvalues_per_s"] = w.N * w.D / b.elapsed_time(c) / 1e6
        pre["produced_quantize_written_GBps"] = w.N * stride / b.elapsed_time(c) / 1e6
        pre["produced_equals_chunked"] = 1.0 if same else 0.0
        pre["chunked_fit_ms"] = fit_ms
        pre["chunked_quantize_ms"] = quant_ms
        del q2, head, tail
        say(f"produced-table pass: fit {pre['produced_fit_ms']:.1f} ms, encode {pre['produced_quantize_ms']:.1f} ms, "
            f"same parameters and codes: {same}")

    # ------------------------------------------------- pre-sampled launch-sets
    g = make_graph(w)
    sets = []
    for si in range(B):
        hops, inputs = launch_set(w, g, si, L)
        sets.append({"hops": hops, "inputs": inputs})
        say(f"launch-set {si + 1} of {B} sampled")
    for s in sets:
        s["d_inputs"] = torch.from_numpy(s["inputs"]).to(dev)
        s["d_hops"] = [(torch.from_numpy(a).to(dev),
                        torch.from_numpy(b.astype(np.int32) if args.idx32 else b).to(dev)) for a, b in s["hops"]]
        s["rows"] = int(s["inputs"].shape[0] + sum(b.shape[0] for _, b in s["hops"]))
    max_in = max(s["inputs"].shape[0] for s in sets)
    max_v = [max(s["hops"][h][0].shape[0] - 1 for s in sets) for h in range(len(w.fanouts))]
    out_in = torch.empty((max_in, w.D), dtype=torch.float32, device=dev)
    out_h = [torch.empty((v, w.D), dtype=torch.float32, device=dev) for v in max_v]
    outer = len(w.fanouts) - 1

    aggregate = q.gather_sum if args.aggregator == "sum" else q.gather_mean

    def step(i, timed=None):
        s = sets[i % B]
        if timed is not None:
            timed[0].record()
        q.gather_dequant(codes, s["d_inputs"], out_in[:s["d_inputs"].shape[0]])
        if timed is not None:
            timed[1].record()
        for h, (dp, di) in enumerate(s["d_hops"]):
            if timed is not None and h == outer:
                timed[2].record()
            # the sampler's contract: no list of hop h is longer than its fan-out
            q.set_option("mean_max_degree", 0 if args.no_degree_hint else w.fanouts[h])
            aggregate(codes, dp, di, out_h[h][:dp.shape[0] - 1])
        if timed is not None:
            timed[3].record()

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = [tuple(ev() for _ in range(4)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    if args.graph:
        # launch-bound steps (one minibatch per launch): the same launches replayed from
        # captured graphs, one per launch-set; the eager pass above keeps the per-kernel events
        graphs = []
        for i in range(B):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                step(i)
            graphs.append(gr)
        for i in range(args.warmup):
            graphs[i % B].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % B].replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    say(f"timed region done: {args.steps} steps in {wall * 1e3:.1f} ms")
    rows_total = sum(sets[i % B]["rows"] for i in range(args.steps))
    ms_per_step = wall / args.steps * 1e3

    # ------------------------------------------ roofline per kernel, dominant one first
    # algorithmic bytes (what the method must move): gather_dequant, per row
    # 8 (index) + row_bytes + 4*D; gather_mean, per block 8*(V+1) + 8*E + row_bytes*U
    # + 4*D*V with U = distinct source rows of the launch (compulsory reads).
    for s in sets:
        M = s["inputs"].shape[0]
        s["bytes_dequant"] = M * (8 + rb + 4 * w.D)
        bm = []
        for indptr, indices in s["hops"]:
            V, E = indptr.shape[0] - 1, indices.shape[0]
            U = np.unique(indices).shape[0]
            ib = 4 if args.idx32 else 8      # bytes per list entry
            bm.append((8 * (V + 1) + ib * E + rb * U + 4 * w.D * V, V, E, U,
                       8 * (V + 1) + ib * E + rb * E + 4 * w.D * V))
        s["bytes_mean"] = bm
    t_deq = sum(e[0].elapsed_time(e[1]) for e in events)
    t_inner = sum(e[1].elapsed_time(e[2]) for e in events)
    t_outer = sum(e[2].elapsed_time(e[3]) for e in events)
    b_deq = sum(sets[i % B]["bytes_dequant"] for i in range(args.steps))
    b_outer = sum(sets[i % B]["bytes_mean"][outer][0] for i in range(args.steps))
    b_inner = sum(sum(x[0] for x in sets[i % B]["bytes_mean"][:outer]) for i in range(args.steps))

    # what this machine streams at best, measured here: a 1 GiB fill (writes only) and a 1 GiB
    # copy (as many bytes read as written), for the fraction beside the one of the 8 TB/s peak
    big = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    big2 = torch.empty_like(big)
    ceil = {}
    for name, fn, nb in (("fill", lambda: big.fill_(1.0), big.numel() * 4),
                         ("copy", lambda: big2.copy_(big), big.numel() * 8)):
        fn()
        a, b = ev(), ev()
        a.record()
        for _ in range(5):
            fn()
        b.record()
        b.synchronize()
        ceil[name + "_GBps"] = round(nb * 5 / a.elapsed_time(b) / 1e6, 1)
    del big, big2

    def roof(name, nbytes, ms, rows, extra=None, profiled=True):
        ach = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        r = {"bound": "hbm", "kernel": name, "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS,
             "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
             "frac_of_fill": round(ach / ceil["fill_GBps"], 4),
             "frac_of_copy": round(ach / ceil["copy_GBps"], 4),
             "traffic": traffic_from_profile(args.workload, name) if profiled else None,
             "avg_kernel_us": round(ms / args.steps * 1e3, 2),
             "algorithmic_bytes_per_launch": int(nbytes / args.steps),
             "rows_per_s": round(rows / (ms * 1e-3), 1) if ms > 0 else 0.0}
        if extra:
            r.update(extra)
        return r

    o = [sets[i % B]["bytes_mean"][outer] for i in range(args.steps)]
    r_deq = sum(sets[i % B]["inputs"].shape[0] for i in range(args.steps))
    r_outer = sum(x[2] for x in o)
    r_inner = sum(sum(x[2] for x in sets[i % B]["bytes_mean"][:outer]) for i in range(args.steps))
    per_edge = sum(x[4] for x in o)
    kernels = {
        "gather_dequant": roof("gather_dequant", b_deq, t_deq, r_deq,
                               {"rows_per_launch": int(np.mean([s["inputs"].shape[0] for s in sets]))}),
        # per_edge_*: a packed row counted for every list entry instead of once per distinct row;
        # caches serve part of it, so this rate may exceed what HBM delivers
        "gather_mean": roof("gather_mean", b_outer, t_outer, r_outer,
                            {"block": "outermost hop", "dst_per_launch": int(np.mean([x[1] for x in o])),
                             "edges_per_launch": int(np.mean([x[2] for x in o])),
                             "distinct_rows_per_launch": int(np.mean([x[3] for x in o])),
                             "per_edge_bytes_per_launch": int(per_edge / args.steps),
                             "per_edge_GBps": round(per_edge / (t_outer * 1e-3) / 1e9, 1)}),
    }
    if outer > 0:
        kernels["gather_mean_inner_hops"] = roof("gather_mean", b_inner, t_inner, r_inner,
                                                 {"block": f"{outer} inner hop(s), one launch each"},
                                                 profiled=False)
    # the graded kernel: the fused gather + decode + mean of the outermost block (the first
    # GNN layer's input); gather_dequant and the inner hops are listed under "kernels"
    roofline = kernels["gather_mean"]

    # ------------------------------------------------------------ CPU baseline
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, g, args.cpu_seconds)

    sp = scale_profile_leg(args, w, q, codes, table) if args.scale_profile > 0 else None
    two = two_hop_leg(w, q, codes, g, L) if len(w.fanouts) >= 2 and not args.no_two_hop else None

    value = rows_total / wall
    res = {
        "metric": "sampled rows gathered+dequantized/s", "value": round(value, 1), "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "D": w.D, "scheme": w.kind,
                   "bits": w.bits if w.kind != "vq" else None,
                   "vq": [w.vq_width, w.vq_length, w.vq_metric] if w.kind == "vq" else None,
                   "row_bytes": rb, "row_stride": stride, "graph": w.graph, "avg_degree": w.avg_degree,
                   "fanouts": list(w.fanouts), "batch": w.batch, "batches_per_step": L,
                   "seed_mode": w.seed_mode, "seed": w.seed, "distinct_launch_sets": B,
                   "aggregator": args.aggregator, "hip_graph": bool(args.graph),
                   "index_bits": 32 if args.idx32 else 64},
        "rows_per_step": int(rows_total / args.steps),
        "uncompressed_equiv_GBps": round(value * w.D * esz / 1e9, 1),
        "roofline": roofline,
        "stream_ceiling": ceil,
        "kernels": kernels,
        "cpu_baseline": cpu,
        "preprocess": {k: round(v, 3) for k, v in pre.items()},
    }
    if sp is not None:
        res["scale_profile"] = sp
    if two is not None:
        res["two_hop"] = two
    print(json.dumps(res))


def two_hop_leg(w, q, codes, g, L):
    """Two rounds of the neighbourhood mean with nothing in between (Appendix A.1's linear
    propagation) over the two outermost blocks of L minibatches: ``bifeat_gather_mean_2hop``
    against ``bifeat_gather_mean`` + ``bifeat_aggregate_rows``, outside the timed region."""
    import torch
    import paper_2207_14696_amd as bf
    from bifeat_inputs import two_round_set

    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    H = len(w.fanouts)
    # the outer block's lists hold table rows, the seed-side block's lists positions among
    # the outer block's destinations
    p1, i1, p2, i2 = two_round_set(w, g, 0, L)
    V1, V2 = p1.shape[0] - 1, p2.shape[0] - 1
    d = lambda a: torch.from_numpy(a).cuda()
    dp1, di1, dp2, di2 = d(p1), d(i1), d(p2), d(i2)
    h1 = torch.empty((V1, w.D), dtype=torch.float32, device="cuda")
    h2 = torch.empty((V2, w.D), dtype=torch.float32, device="cuda")
    hf = torch.empty_like(h2)

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps * 1e3

    q.set_option("mean_max_degree", w.fanouts[H - 1])
    t1 = timed(lambda: q.gather_mean(codes, dp1, di1, h1))
    t2 = timed(lambda: bf.aggregate_rows(h1, dp2, di2, out=h2))
    q.set_option("mean_max_degree", max(w.fanouts[H - 1], w.fanouts[H - 2]))
    tf = timed(lambda: q.gather_mean_2hop(codes, dp1, di1, dp2, di2, hf))
    ok = q.poll_status(wait=True)
    diff = float((hf - h2).abs().max().item())
    q.set_option("mean_max_degree", 0)
    tu = timed(lambda: q.gather_mean_2hop(codes, dp1, di1, dp2, di2, hf), reps=5)
    fetches = int(np.diff(p1)[i2].sum())
    say(f"two rounds: chain {t1:.1f} + {t2:.1f} us, one call {tf:.1f} us")
    return {"dst": V2, "entries": int(i2.shape[0]), "outer_dst": V1, "outer_edges": int(i1.shape[0]),
            "chain_us": round(t1 + t2, 1), "chain_layer1_us": round(t1, 1), "chain_layer2_us": round(t2, 1),
            "fused_us": round(tf, 1), "fused_without_bound_us": round(tu, 1), "fused_row_fetches": fetches,
            "fused_fetched_GBps": round(fetches * q.row_bytes / tf / 1e3, 1),
            "intermediate_MB_avoided": round(V1 * w.D * 4 / 1e6, 1),
            "max_abs_diff_to_chain": diff, "status_ok": bool(ok)}


def scale_profile_leg(args, w, q, codes, table):
    """The aggregation scale profile for this workload's codes: how much of the
    actual quantisation error (decoded minus raw rows) and of the unit-length
    features survives 1..LAYERS rounds of neighbourhood averaging over a whole
    graph of the workload's family (lists include the node itself), and the
    ratio of the two, the factor that bounds the tolerable error.  Also times
    the fp32-row aggregation it is built from."""
    import torch
    import paper_2207_14696_amd as bf
    from bifeat_inputs import PowerLawGraph, UniformGraph, full_csr
    layers = args.scale_profile
    n = min(w.N, args.profile_nodes)
    g = UniformGraph(n, int(w.avg_degree), w.seed) if w.graph == "uniform" \
        else PowerLawGraph(n, w.avg_degree, 2.1, min(w.cap, n - 1), w.seed)
    indptr, indices = full_csr(g)
    E = int(indices.shape[0])
    say(f"scale profile: graph of {n} nodes, {E} list entries materialised")
    dptr, dind = torch.from_numpy(indptr).cuda(), torch.from_numpy(indices).cuda()
    x = table.chunk(0, n).float()
    dec = q.gather_dequant(codes, torch.arange(n, dtype=torch.int64, device="cuda"))
    err = dec - x
    del dec
    unit = x / x.norm(dim=1, keepdim=True).clamp_min(1e-30)
    del x
    work = torch.empty(min(layers, 2) * n * w.D, dtype=torch.float32, device="cuda")
    t0 = time.perf_counter()
    ce = bf.scale_profile(err, dptr, dind, layers, work=work)
    profile_ms = (time.perf_counter() - t0) * 1e3
    cf = bf.scale_profile(unit, dptr, dind, layers, work=work)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    err.normal_(generator=gen)
    ci = bf.scale_profile(err, dptr, dind, layers, work=work)
    # the fp32-row aggregation on its own: rows are read once each (compulsory) and written once
    out = work[:n * w.D].view(n, w.D)
    bf.aggregate_rows(unit, dptr, dind, out=out)
    reps = 5
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        bf.aggregate_rows(unit, dptr, dind, out=out)
    b.record()
    b.synchronize()
    us = a.elapsed_time(b) / reps * 1e3
    nbytes = 8 * (n + 1) + 8 * E + 2 * 4 * w.D * n
    requested = 8 * (n + 1) + 8 * E + 4 * w.D * E + 4 * w.D * n
    rel = lambda c: [round(float(v / c[0]), 6) if c[0] > 0 else 0.0 for v in c]  # noqa: E731
    c_e, c_f, c_i = rel(ce), rel(cf), rel(ci)
    return {"nodes": n, "list_entries": E, "self_loops": True, "layers": layers,
            "error_row_length": float(ce[0]),
            "C_e": c_e, "C_f": c_f, "C_hat": [round(e / f, 6) if f > 0 else None for e, f in zip(c_e, c_f)],
            "C_e_independent_noise": c_i,
            "profile_ms": round(profile_ms, 3),
            # algorithmic bytes: every row read once and written once; "requested" counts a row
            # per list entry, which caches serve in part (it can exceed the HBM peak)
            "aggregate_rows": {"bound": "hbm", "avg_kernel_us": round(us, 2),
                               "algorithmic_bytes_per_launch": nbytes,
                               "achieved": round(nbytes / us / 1e3, 1), "peak": HBM_PEAK_GBPS,
                               "unit": "GB/s", "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4),
                               "traffic": traffic_from_profile(args.workload, "aggregate_rows")
                               if (not args.rows and args.profile_nodes == 1 << 20) else None,
                               "requested_bytes_per_launch": requested,
                               "requested_GBps": round(requested / us / 1e3, 1),
                               "list_entries_per_s": round(E / us * 1e6, 1)}}


def cpu_baseline(w, g, seconds: float):
    """The oracle timed on this machine's host cores on single minibatches of the
    same workload.  It runs on a compact sub-table holding only the rows a
    minibatch touches (the full table is not built on the host), which flatters
    the CPU's caches."""
    import oracle as orc
    from bifeat_inputs import draw_seeds, sample_blocks, feature_rows
    rows_done, spent, nb, last, total_passes = 0, 0.0, 0, 0.0, 0
    bi = 10_000
    wall0 = time.perf_counter()
    note = ""
    # the untimed set-up of a minibatch (regenerate + quantize its rows) is bounded too
    while spent < seconds and nb < 64 and time.perf_counter() - wall0 < 6 * seconds:
        seeds = draw_seeds(g, w.batch, w.seed, bi, w.seed_mode)
        blocks, inputs = sample_blocks(g, seeds, w.fanouts, w.seed, bi)
        x = feature_rows(w.spec, inputs).astype(np.float32)     # inputs is sorted & unique
        remap = lambda ids: np.searchsorted(inputs, ids)        # noqa: E731
        if w.kind == "uniform":
            mn, mx = orc.fit_minmax(x)
            scale, inv = orc.uniform_params(mn, mx, w.bits)
            s = orc.Scheme.uniform(mn, scale, w.bits)
            codes = orc.pack(orc.uniform_encode(x, w.bits, mn, inv), w.bits)
        elif w.kind == "log":
            rng_e = orc.log_range_clipped(x, w.log_clip) if w.log_clip > 0 else orc.log_range(orc.log_fit(x))
            T, V = orc.log_tables(*rng_e, w.bits)
            s = orc.Scheme.log(w.D, V, w.bits)
            codes = orc.pack(orc.log_encode(x, w.bits, T), w.bits)
        else:
            P = (w.D + w.vq_width - 1) // w.vq_width
            cb = np.ascontiguousarray(
                x[:w.vq_length].reshape(w.vq_length, P, w.vq_width).transpose(1, 0, 2))
            s = orc.Scheme.vq(w.D, cb)
            # nearest-entry search of every touched row would take minutes per minibatch on
            # the host; the timed gathers do not depend on the code values
            head = orc.vq_assign(x[:4096], w.vq_width, cb, metric=w.vq_metric)
            rest = np.random.default_rng(bi).integers(0, w.vq_length, (x.shape[0] - head.shape[0], P))
            codes = orc.pack(np.concatenate([head, rest.astype(head.dtype)]),
                             orc.vq_code_bits(w.vq_length))
            note = "; vector codes beyond each sub-table's first 4096 rows drawn at random"
        idx = np.arange(inputs.shape[0], dtype=np.int64)
        csr = [(b.indptr, remap(b.indices)) for b in blocks]
        # setting a minibatch up costs far more than the oracle's pass over it, so the pass is
        # repeated until this minibatch has had its share (1/64) of the time budget
        passes, mine = 0, 0.0
        while passes == 0 or (mine < seconds / 64 and spent + mine < seconds):
            t0 = time.perf_counter()
            orc.gather_dequant(s, codes, idx)
            for indptr, indices in csr:
                orc.gather_mean(s, codes, indptr, indices)
            last = time.perf_counter() - t0
            mine += last
            passes += 1
        spent += mine
        total_passes += passes
        rows_done += passes * (inputs.shape[0] + sum(b.E for b in blocks))
        nb += 1
        bi += 1
        if nb % 8 == 0 or spent >= seconds:
            say(f"cpu baseline: minibatch {nb}, {spent:.1f} s of oracle time")
    # the last minibatch once more on one thread, if that stays within the time bound
    single = None
    cores = orc.max_threads()
    if nb > 0 and last * cores < 3 * seconds:
        orc.set_threads(1)
        t0 = time.perf_counter()
        orc.gather_dequant(s, codes, idx)
        for indptr, indices in csr:
            orc.gather_mean(s, codes, indptr, indices)
        single = round((inputs.shape[0] + sum(b.E for b in blocks)) / (time.perf_counter() - t0), 1)
        orc.set_threads(cores)
        say(f"cpu baseline: one thread, {single:.3g} rows/s")
    return {"value": round(rows_done / spent, 1), "unit": "rows/s", "cores": cores,
            "kind": "oracle", "single_thread_value": single,
            "sample": f"{nb} single minibatches (gather_dequant of the input rows + gather_mean per "
                      f"hop), each on a compact sub-table of the rows it touches, {total_passes} "
                      f"passes in all; "
                      f"{spent:.1f} s of oracle time{note}"}


if __name__ == "__main__":
    main()
