#!/usr/bin/env python3
"""Throughput of the EDEN hot path on one MI355X.

One step = encode of all n senders + the receiver's round (decode of all n messages, sum, division by n:
eden_decode_mean, which equals zero + eden_decode_accumulate + eden_finalize_mean bit for bit) on one synthetic
batch that is already resident in device memory.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def coords_of(n: int, D: int) -> float:
    return 2.0 * n * D


def passes_of(log2D: int) -> int:
    """HBM passes of the transform in the byte model the metric is defined on (2^12 on-chip block)."""
    return max(1, -(-log2D // 12))


def model_bytes(n, d, D, budgets):
    """Kernel-minimum traffic of one step: per sender encode 4d + 8D(P-1) + bD/8, decode bD/8 + 8D(P-1),
    plus 4d once for the mean."""
    P = passes_of(D.bit_length() - 1)
    total = 0.0
    for b in budgets:
        payload = D * (b / 256.0) / 8.0
        total += 4 * d + 8 * D * (P - 1) + payload          # encode
        total += payload + 8 * D * (P - 1)                  # decode
    return total + 4 * d


def kernel_bytes(kind, senders, d, D, mean_bits, narrow, fused_mean=False):
    """Algorithmic bytes one launch of a kernel kind must move (what its role reads + what it writes).
    The contiguous pass works on whole tiles of 2^12 (D <= 2^18) or 2^14 coordinates and only touches the tiles
    that hold part of the first d coordinates; the strided passes read / write the rest as implicit zeros.
    `narrow`: the decode workspace of this workload is fp16 (every sender has b <= 1 and 2^13 <= D <= 2^24).
    `fused_mean`: the last decode pass stores the mean (4 d) instead of a read-modify-write of the accumulator."""
    log2D = D.bit_length() - 1
    lo = 12 if log2D <= 18 else 14

    def ru(bits):                                     # d rounded up to whole tiles of 2^bits, at most D
        return min(D, -(-d >> bits) << bits)

    payload = D * mean_bits / 8.0
    ws = 2 if narrow else 4                           # decode workspace bytes per element
    top = ru(lo) if log2D <= 24 else ru(24)           # what the pass next to the payload reads (encode) / writes (decode)
    per_sender = {
        "enc_first": 4 * d + 4 * ru(lo),              # x in, workspace out
        "mid": 4 * ru(14) + 4 * ru(24),               # workspace in and out (three-pass sizes)
        "enc_last": 4 * top + payload,                # workspace in, packed indices out
        "dec_first": payload + ws * top,              # packed indices in, workspace out
        "dec_last": ws * ru(lo),                      # workspace in (per sender) ...
    }
    if kind == "dec_last":
        return senders * per_sender[kind] + (4 if fused_mean else 8) * d     # ... plus the accumulator (or the mean)
    if kind == "finalize_mean":
        return 8 * d
    return senders * per_sender.get(kind, 0.0)


def measured_traffic(workload: str, kind: str):
    """HBM bytes per launch of one kernel kind as rocprofv3 counted them (FETCH_SIZE and WRITE_SIZE, scaled by what the
    same counters read for a plain copy), from the tracked profiler summary of this workload: lines of the form
    `traffic_bytes <workload> <kind> <bytes>`.  None when the summary has no such line: the figure is a stored
    measurement of the build that the summary names, never a constant of this script."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_cfg4_bench.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 4 and parts[0] == "traffic_bytes" and parts[1] == workload and parts[2] == kind:
                    return float(parts[3])
    except OSError:
        pass
    return None


def graph_replay_ms(step, torch, steps):
    """ms per step when the whole step is one captured HIP graph (the library's calls only launch kernels): what is left
    when the host's launch path is taken out.  Reported beside the eager figure, never as `value`."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_config(k, eden, synth, torch, steps=20, warmup=3):
    """ms per step and Gcoords/s of synthetic configuration k (same step as the headline)."""
    w = synth.config(k)
    n, d = w.n, w.d
    D = 1 << (d - 1).bit_length()
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.alloc_messages(d, w.b_q8)
    acc = torch.zeros(d, dtype=torch.float32, device="cuda")
    bitmaps = [ctx.make_loss_bitmap(w.seed, w.client_ids[c], D, w.drop_q32) for c in range(n)] if w.drop_q32 else None

    def step():
        ctx.encode(xs, w.client_ids, w.b_q8, w.seed, msgs=msgs)
        ctx.decode_mean(msgs, w.client_ids, w.b_q8, d, w.seed, acc, bitmaps)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    assert ctx.last_device_status() == 0
    graph_ms = graph_replay_ms(step, torch, steps)
    res = {"workload": w.name, "ms_per_step": round(ms, 4), "Gcoords_per_s": round(2.0 * n * D / (ms * 1e-3) / 1e9, 2),
           "model_frac_of_peak": round(model_bytes(n, d, D, w.b_q8) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "graph_replay_ms_per_step": round(graph_ms, 4)}
    ctx.close()
    del xs, msgs, acc, ctx
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20, help="untimed steps first (the clocks of a fresh box settle within about ten)")
    ap.add_argument("--config", type=int, default=4, help="synthetic configuration 1..5 (4 = the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short timing of the other four synthetic configurations")
    ap.add_argument("--profile-all", action="store_true", help="time every kernel kind, print a table to stderr")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (each box has one); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2108_08842_amd import eden, synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    eden.lib()                                              # fails loudly if the HIP library is not built
    w = synth.config(args.config)
    n, d = w.n, w.d
    D = 1 << (d - 1).bit_length()
    log2D = D.bit_length() - 1
    mean_bits = sum(w.b_q8) / len(w.b_q8) / 256.0
    narrow = all(b <= 256 for b in w.b_q8) and 13 <= log2D <= 24

    xs_host = [synth.client_vector(w, c) for c in range(n)]
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.alloc_messages(d, w.b_q8)
    acc = torch.zeros(d, dtype=torch.float32, device="cuda")
    mean = torch.empty_like(acc)
    bitmaps = None
    if w.drop_q32:
        bitmaps = [ctx.make_loss_bitmap(w.seed, w.client_ids[c], D, w.drop_q32) for c in range(n)]

    def step():
        ctx.encode(xs, w.client_ids, w.b_q8, w.seed, msgs=msgs)
        ctx.decode_mean(msgs, w.client_ids, w.b_q8, d, w.seed, mean, bitmaps)

    def three_call_step():                                  # the receiver's round as three calls (not the headline)
        acc.zero_()
        ctx.encode(xs, w.client_ids, w.b_q8, w.seed, msgs=msgs)
        ctx.decode_accumulate(msgs, w.client_ids, w.b_q8, d, w.seed, acc, bitmaps)
        ctx.finalize_mean(acc, n, out=mean)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # find the dominant kernel with every kind timed (untimed region), then time only that one
    all_kinds = [k for k in eden.KERNEL_KINDS]
    ctx.profile_enable(all_kinds, 4096)
    step()
    torch.cuda.synchronize()
    per_kind = {}
    for kind, senders, ms in ctx.profile_collect():
        per_kind.setdefault(kind, []).append((senders, ms))
    dominant = max(per_kind, key=lambda k: sum(ms for _, ms in per_kind[k]))
    fused = "finalize_mean" not in per_kind                 # the last decode pass stored the mean itself
    step_alg_bytes = sum(kernel_bytes(kind, s_, d, D, mean_bits, narrow, fused) for kind, recs_ in per_kind.items() for s_, _ in recs_)
    if args.profile_all:
        for kind, recs in sorted(per_kind.items(), key=lambda kv: -sum(ms for _, ms in kv[1])):
            tot = sum(ms for _, ms in recs)
            byts = sum(kernel_bytes(kind, s, d, D, mean_bits, narrow, fused) for s, _ in recs)
            print(f"  {kind:14s} launches={len(recs):3d} total={tot:8.3f} ms  alg={byts / 1e9:7.3f} GB  "
                  f"{byts / 1e6 / max(tot, 1e-9):8.1f} GB/s", file=sys.stderr)
    ctx.profile_enable([dominant], 4096)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    status = ctx.last_device_status()
    assert status == 0, f"device status {status}"

    recs = ctx.profile_collect()
    ctx.profile_enable([], 0)

    def timed(fn):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / args.steps

    enc_ms = timed(lambda: ctx.encode(xs, w.client_ids, w.b_q8, w.seed, msgs=msgs))

    dec_ms = timed(lambda: ctx.decode_mean(msgs, w.client_ids, w.b_q8, d, w.seed, mean, bitmaps))
    three_ms = timed(three_call_step)
    graph_ms = graph_replay_ms(step, torch, args.steps)
    dom_ms = [ms for _, _, ms in recs]
    dom_bytes = [kernel_bytes(k, s, d, D, mean_bits, narrow, fused) for k, s, _ in recs]
    avg_ms = sum(dom_ms) / len(dom_ms)
    achieved = (sum(dom_bytes) / len(dom_bytes)) / (avg_ms * 1e-3) / 1e9

    coords = 2.0 * n * D
    value = coords / (ms_per_step * 1e-3) / 1e9
    mbytes = model_bytes(n, d, D, w.b_q8)
    model_gbs = mbytes / (ms_per_step * 1e-3) / 1e9

    out = {
        "metric": "encode+decode Gcoords/s (2*n*D coordinates per step)",
        "value": round(value, 3),
        "unit": "Gcoords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n": n, "d": d, "D": D, "b": mean_bits, "dist": w.dist,
                   "loss": w.drop_q32 / 2 ** 32},
        "value_counting_d": round(2.0 * n * d / (ms_per_step * 1e-3) / 1e9, 3),
        "encode_only": {"ms": round(enc_ms, 4), "Gcoords_per_s": round(n * D / (enc_ms * 1e-3) / 1e9, 1)},
        "decode_only": {"ms": round(dec_ms, 4), "Gcoords_per_s": round(n * D / (dec_ms * 1e-3) / 1e9, 1)},
        "three_call_step": {"ms_per_step": round(three_ms, 4),
                            "note": "zero + eden_decode_accumulate + eden_finalize_mean instead of eden_decode_mean"},
        "graph_replay": {"ms_per_step": round(graph_ms, 4), "Gcoords_per_s": round(coords_of(n, D) / (graph_ms * 1e-3) / 1e9, 1),
                         "note": "the same step replayed as one captured HIP graph; not the headline value"},
        "hbm_model": {"bytes_per_step": mbytes, "GBps": round(model_gbs, 1),
                      "frac_of_peak": round(model_gbs / HBM_PEAK_GBS, 4),
                      "note": "byte model of the metric (2^12 on-chip block, every pass moves all D "
                              "coordinates) / step time / 8 TB/s; the kernels skip the zero padding, so they move less"},
        "hbm_kernels": {"bytes_per_step": step_alg_bytes, "GBps": round(step_alg_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                        "frac_of_peak": round(step_alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                        "note": "algorithmic bytes of the kernels as built (padding tiles skipped, fp16 decode "
                                "workspace for b <= 1) / step time / 8 TB/s"},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(w.name, dominant),
                     "traffic_source": "profiles/hbm_traffic_cfg4_bench.txt (rocprofv3 counters of an own run)",
                     "algorithmic_bytes": sum(dom_bytes) / len(dom_bytes),
                     "avg_launch_ms": round(avg_ms, 4), "launches": len(dom_ms),
                     "timing": "HIP events around every launch of this kernel inside the timed region, on the launch stream"},
        "timing": "wall clock (perf_counter) around the K steps between two device synchronisations",
    }

    if not args.no_other_configs and args.config == 4:
        # the same vectors under other bit budgets, a few steps each (not the headline; parity tests cover them)
        def time_budget(name, b):
            bq = [b] * n
            m2 = ctx.alloc_messages(d, bq)

            def step2():
                ctx.encode(xs, w.client_ids, bq, w.seed, msgs=m2)
                ctx.decode_mean(m2, w.client_ids, bq, d, w.seed, mean)

            for _ in range(10):
                step2()
            ms2 = timed(step2)
            assert ctx.last_device_status() == 0
            return {"budget": name, "ms_per_step": round(ms2, 4)}

        out["other_budgets"] = [time_budget(name, b) for name, b in (
            ("b=1/2 (sub-sampled after the rotation)", 128), ("b=1/2 (pairs before the rotation)", eden.B_HALF_PRE),
            ("b=6/64 (6 of every 64 before the rotation)", eden.B_SPARSE(6)), ("b=2", 512), ("b=4", 1024))]
        # the other synthetic configurations, a few steps each (not the headline; parity tests cover them)
        del xs, msgs, acc, mean, ctx
        torch.cuda.empty_cache()
        out["other_configs"] = [time_config(k, eden, synth, torch) for k in (1, 2, 3, 5)]

    if not args.no_cpu_baseline:
        from oracle import eden_oracle as o
        # bounded sample: the first senders of the same workload, full dimension, through the float64 oracle,
        # as many as fit in about 15 s of CPU time (at least one)
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):                        # "cores: 1" is meant literally: numpy's own pools too
            t0 = time.perf_counter()
            omsgs = []
            for c in range(n):
                omsgs.append(o.encode(xs_host[c].astype(np.float64), w.seed, w.client_ids[c], w.b_q8[c]))
                if (time.perf_counter() - t0) * (c + 2) / (c + 1) > 8.0:     # encode is about half of the work
                    break
            k = len(omsgs)
            _ = o.decode_mean(omsgs, d)
            dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(2.0 * k * D / dt / 1e9, 5), "unit": "Gcoords/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"{k} of {n} senders at full d, encode+decode+mean, numpy float64, {dt:.1f} s"}
        # the same oracle on all host cores: every sender of the workload, one thread each (numpy releases the
        # interpreter lock in its loops), at most as many threads as cores
        from concurrent.futures import ThreadPoolExecutor
        threads = max(1, min(n, os.cpu_count() or 1))
        if threads > 1:
            t0 = time.perf_counter()
            with ThreadPoolExecutor(threads) as pool:
                tm = list(pool.map(lambda c: o.encode(xs_host[c].astype(np.float64), w.seed, w.client_ids[c], w.b_q8[c]),
                                   range(n)))
                dec = list(pool.map(lambda m: o.decode(m, d), tm))
            _ = sum(dec) / n
            dtm = time.perf_counter() - t0
            out["cpu_baseline_threads"] = {"value": round(2.0 * n * D / dtm / 1e9, 5), "unit": "Gcoords/s",
                                           "cores": threads, "kind": "oracle",
                                           "sample": f"all {n} senders at full d, {threads} threads, {dtm:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
