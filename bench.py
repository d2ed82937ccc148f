#!/usr/bin/env python3
"""Benchmark of the BRACE aggregation hot path on one MI355X.

One step = one pass of the whole path (sign quantisation, share-reduce vote, consensus
threshold, gather into the global update) over one synthetic batch of n client updates
already resident in HBM.  Prints ONE JSON line on stdout; progress goes to stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-cpu-baseline]
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

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published peak

# HBM bytes per launch read from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (KiB per
# dispatch, scaled by the same counters' reading for a copy kernel of known size).
# Filled from the summaries kept under profiles/; None = not measured for that workload.
MEASURED_TRAFFIC_BYTES = {
    # profiles/stream_kernel_VoteOp_cfg3_n100_d25M.md: FETCH 10,000,307,000 B + WRITE 3,126,600 B
    "cfg3_n100_d25M_lie": 10_003_433_600,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def pick_workload(name: str):
    from paper_2501_17392_amd import synth
    for w in synth.WORKLOADS:
        if w.name == name or w.name.startswith(name + "_") or w.name.split("_")[0] == name:
            return w
    raise SystemExit(f"unknown workload {name!r}; choose from {[w.name for w in synth.WORKLOADS]}")


def cpu_baseline(upd, w, lam, gpu_out, sample_cols):
    """Time the plain-C oracle on the host cores over the first `sample_cols` columns of the
    same input bytes, and check the GPU result against it on those columns."""
    import numpy as np
    from oracle import c_oracle

    c_oracle.load()
    k1 = min(w.d, sample_cols)
    t0 = time.perf_counter()
    host = upd[:, :k1].contiguous().cpu().numpy()
    t_copy = time.perf_counter() - t0
    threads = c_oracle.threads(0)
    t0 = time.perf_counter()
    want, _, _ = c_oracle.brace_direct(host, lam, 0, want_sums=False, want_bits=False, nthreads=0)
    t_all = time.perf_counter() - t0
    k1_single = max(1, k1 // 8)
    t0 = time.perf_counter()
    c_oracle.brace_direct(host[:, :k1_single], lam, 0, want_sums=False, want_bits=False, nthreads=1)
    t_one = time.perf_counter() - t0
    match = bool(np.array_equal(gpu_out[:k1].cpu().numpy(), want))
    return {
        "value": k1 / t_all,
        "unit": "coords/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"first {k1} of {w.d} coordinates x all {w.n} clients of the same input "
                  f"({4 * w.n * k1 / 1e9:.2f} GB), plain-C definition loop with OpenMP over "
                  f"coordinates; D2H copy ({t_copy:.1f} s) excluded",
        "seconds": t_all,
        "value_1thread": k1_single / t_one,
        "gpu_matches_oracle_on_sample": match,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--lam", type=float, default=5.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-cols", type=int, default=25_000_000)
    ap.add_argument("--no-probe", dest="probe", action="store_false",
                    help="skip the plain read / copy kernels on 1 GiB (counter calibration and "
                         "linear-access bandwidth, reported under 'probe')")
    ap.add_argument("--probe", dest="probe", action="store_true", help=argparse.SUPPRESS)
    ap.set_defaults(probe=True)
    ap.add_argument("--no-next-rows", dest="next_rows", action="store_false",
                    help="skip timing the other entry points (sum/mean, fused update, bit planes)")
    ap.set_defaults(next_rows=True)
    ap.add_argument("--tuning", default="",
                    help="vec,cols,unroll,nontemporal,pipeline,split_writes,rowsplit,stage_writes (default: library "
                         "defaults)")
    args = ap.parse_args()

    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU only (no collectives, no second "
                         "device); run with --gpus 1")

    import torch
    from paper_2501_17392_amd import binding as B
    from paper_2501_17392_amd import synth

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs the MI355X (torch.cuda.is_available() is False)")
    B.lib()                                   # fail loudly if the HIP library is not built
    if args.tuning:
        B.brace_set_tuning(*[int(x) for x in args.tuning.split(",")])
    dev = "cuda:0"
    w = pick_workload(args.workload)
    log(f"[bench] workload {w.name}: n={w.n} f={w.f} d={w.d} ({w.input_bytes / 1e9:.2f} GB), "
        f"lambda={args.lam}, tuning={B.brace_get_tuning()}")

    t0 = time.perf_counter()
    upd = synth.generate(w, dev)
    torch.cuda.synchronize()
    log(f"[bench] generated inputs in {time.perf_counter() - t0:.1f} s")
    out = torch.empty(w.d, device=dev, dtype=torch.float32)
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        B.brace_aggregate(upd, w.f, args.lam, out=out, stream=stream)
    torch.cuda.synchronize()

    K = args.steps
    events = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        events[i].record(stream)
        B.brace_aggregate(upd, w.f, args.lam, out=out, stream=stream)
    events[K].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    per_step_ms = sorted(events[i].elapsed_time(events[i + 1]) for i in range(K))
    step_ms = events[0].elapsed_time(events[K]) / K
    ms_per_step = wall * 1e3 / K
    step_bytes = 4 * w.n * w.d + 4 * w.d          # read n*d fp32 once, write d fp32
    step_gbs = step_bytes / (step_ms * 1e-3) / 1e9

    # The dominant kernel on its own: the streaming vote kernel reads the n x d matrix and
    # emits one bit per coordinate (the fp32 vector is then written by the small expand
    # kernel).  Same kernel, same launch shape as inside the step; timed with events on the
    # launch stream.
    bits = torch.empty((w.d + 31) // 32, device=dev, dtype=torch.int32)
    for _ in range(2):
        B.brace_aggregate(upd, w.f, args.lam, out=None, out_bits=bits, stream=stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    for i in range(K):
        ev[i].record(stream)
        B.brace_aggregate(upd, w.f, args.lam, out=None, out_bits=bits, stream=stream)
    ev[K].record(stream)
    torch.cuda.synchronize()
    vote_ms = ev[0].elapsed_time(ev[K]) / K
    vote_each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(K))
    vote_bytes = 4 * w.n * w.d + 4 * ((w.d + 31) // 32)
    achieved = vote_bytes / (vote_ms * 1e-3) / 1e9
    log(f"[bench] {K} steps: wall {ms_per_step:.3f} ms/step, on-stream {step_ms:.3f} ms "
        f"(min {per_step_ms[0]:.3f}, median {per_step_ms[K // 2]:.3f}) -> {step_gbs:.0f} GB/s "
        f"= {step_gbs / HBM_PEAK_GBS:.1%} of {HBM_PEAK_GBS:.0f} GB/s over the whole step")
    log(f"[bench] vote kernel alone: avg {vote_ms:.3f} ms (min {vote_each[0]:.3f}) -> "
        f"{achieved:.0f} GB/s = {achieved / HBM_PEAK_GBS:.1%} of peak")

    result = {
        "metric": "aggregated coordinates/sec and achieved HBM GB/s (% of peak), n=100 d=25M fp32",
        "value": w.d / (ms_per_step * 1e-3),
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name, "n": w.n, "f": w.f, "d": w.d, "lambda": args.lam,
            "input_bytes": w.input_bytes, "client_coords_per_s": w.n * w.d / (ms_per_step * 1e-3),
            "launch": B.brace_get_tuning(), "input_checksum": synth.checksum(upd[:, : min(w.d, 1 << 20)]),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
            "kernel": "brace_dev::stream_kernel<VoteOp, ...> (the streaming vote kernel)",
            "algorithmic_bytes_per_launch": vote_bytes,
            "kernel_ms_avg": vote_ms,
            "kernel_ms_min": vote_each[0],
            "kernel_ms_median": vote_each[K // 2],
            "whole_step": {
                "kernels": "stream_kernel<VoteOp, ...> + brace_expand_kernel",
                "algorithmic_bytes": step_bytes,
                "ms_avg": step_ms, "ms_min": per_step_ms[0], "ms_median": per_step_ms[K // 2],
                "achieved": step_gbs, "frac": step_gbs / HBM_PEAK_GBS,
            },
        },
    }
    if args.next_rows:
        # The widened rows, each timed alone with events on the launch stream and priced with
        # its own algorithmic bytes (read the matrix once + what it must write / re-read).
        rw = B.brace_packed_row_words(w.d)
        signs = torch.empty(w.n, rw, device=dev, dtype=torch.int32)
        model = torch.zeros(w.d, device=dev, dtype=torch.float32)
        vw = B.brace_1bit_row_words(w.d)
        votes = torch.empty(w.n, vw, device=dev, dtype=torch.int32)
        # 8 partial sign-sums (one per device of an 8-device ring), values as 12-13 clients give
        parts = torch.randint(-13, 14, (8, w.d), device=dev, dtype=torch.int16)
        nd4 = 4 * w.n * w.d
        rows = (
            ("rar_mean", lambda: B.brace_rar_aggregate(upd, out, mean=True, stream=stream),
             nd4 + 4 * w.d),
            ("update_with_bits", lambda: B.brace_aggregate_update(upd, w.f, model, 1e-3, args.lam,
                                                                  out_bits=bits, stream=stream),
             nd4 + 8 * w.d + 2 * 4 * ((w.d + 31) // 32)),
            ("update_direct", lambda: B.brace_aggregate_update(upd, w.f, model, 1e-3, args.lam,
                                                               stream=stream), nd4 + 8 * w.d),
            ("quantize", lambda: B.brace_quantize(upd, signs, stream=stream), nd4 + 4 * w.n * rw),
            ("vote_packed", lambda: B.brace_vote_packed(signs, w.d, w.f, args.lam, out=out,
                                                        stream=stream),
             4 * w.n * rw + 4 * w.d + 2 * 4 * ((w.d + 31) // 32)),
            ("expand_bits", lambda: B.brace_expand_bits(bits, w.d, out, stream=stream),
             4 * w.d + 4 * ((w.d + 31) // 32)),
            ("apply_bits", lambda: B.brace_apply_bits(bits, w.d, 1e-3, model, stream=stream),
             8 * w.d + 4 * ((w.d + 31) // 32)),
            ("quantize_1bit", lambda: B.brace_quantize_1bit(upd, 1, votes, stream=stream),
             nd4 + 4 * w.n * vw),
            ("vote_1bit", lambda: B.brace_vote_1bit(votes, w.d, w.f, args.lam, out=out, stream=stream),
             4 * w.n * vw + 4 * w.d + 2 * 4 * ((w.d + 31) // 32)),
            ("consensus_sums_g8", lambda: B.brace_consensus_sums(parts, args.lam, out=out,
                                                                 stream=stream),
             2 * 8 * w.d + 4 * w.d),
        )
        extra = {}
        for name, fn, nbytes in rows:
            for _ in range(2):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = max(5, K // 3)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            gbs = nbytes / (ms * 1e-3) / 1e9
            extra[name] = {"ms": ms, "algorithmic_bytes": nbytes, "achieved_GBps": gbs,
                           "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
            log(f"[bench] {name}: {ms:.3f} ms, {gbs:.0f} GB/s ({gbs / HBM_PEAK_GBS:.1%})")
        result["next_rows"] = extra
        del signs, model
    if args.probe:
        nel = (1 << 30) // 4
        src = torch.randn(nel, device=dev)
        dst = torch.empty_like(src)
        sink = torch.zeros(4, device=dev)
        probe = {"bytes": nel * 4}
        for name, fn, moved in (("read", lambda: B.brace_probe_read(src, sink, 1, stream), nel * 4),
                                ("copy", lambda: B.brace_probe_copy(dst, src, stream), 2 * nel * 4)):
            for _ in range(2):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            probe[name + "_GBps"] = moved / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9
        result["probe"] = probe
        log(f"[bench] probe: {probe}")
        del src, dst
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a sample ...")
        result["cpu_baseline"] = cpu_baseline(upd, w, args.lam, out, args.cpu_sample_cols)
        # reported for context only: the roofline fraction, not this ratio, rates the kernel
        result["cpu_baseline"]["gpu_over_cpu"] = result["value"] / result["cpu_baseline"]["value"]
        result["cpu_baseline"]["gpu_over_cpu_1thread"] = \
            result["value"] / result["cpu_baseline"]["value_1thread"]
        log(f"[bench] oracle: {result['cpu_baseline']['value']:.3e} coords/s on "
            f"{result['cpu_baseline']['cores']} threads; GPU matches oracle on the sample: "
            f"{result['cpu_baseline']['gpu_matches_oracle_on_sample']}")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
