#!/usr/bin/env python3
"""Benchmark of the BRACE aggregation hot path on one MI355X.

One step = one pass of the whole path (sign quantisation, share-reduce vote, consensus
threshold, gather into the global update) over one synthetic batch of n client updates
already resident in HBM.  Prints ONE JSON line on stdout; progress goes to stderr.
The headline is workload cfg3 (n = 100, d = 25 M); the same run also times the other
workloads (`per_config`), the per-chunk entry point and the widened rows (`next_rows`),
and checks every timed vote against the CPU oracle on a sample.  A mismatch is fatal: the
line is still printed, the exit status is 1.

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

# HBM bytes per launch of the streaming vote kernel, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs (units per dispatch, scaled by the same counters' reading for a copy of
# known size).  These are readings of earlier profiler runs, not of this run: each entry
# names the summary that holds it.  A workload without a counter run reports null.
PROFILED_TRAFFIC = {
    "cfg3_n100_d25M_lie": {
        "bytes": 10_003_400_806,
        "source": "profiles/stream_kernel_VoteOp_cfg3_n100_d25M.md (FETCH 10,000,269,107 B + "
                  "WRITE 3,131,699 B per launch; algorithmic 10,003,125,000 B)",
    },
    "cfg4_n64_d100M_sparse_mix": {
        "bytes": 25_612_765_594,
        "source": "profiles/stream_kernel_VoteOp_cfg2_cfg4.md (algorithmic 25,612,500,000 B)",
    },
    "cfg2_n50_d11173962_inversion": {
        "bytes": 2_298_051_481,
        "source": "profiles/stream_kernel_VoteOp_cfg2_cfg4.md (algorithmic 2,236,189,148 B; rows "
                  "are 40 mod 128 bytes apart, so the lines at the ends of every wave's run are "
                  "fetched twice)",
    },
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def pick_workload(name: str):
    from paper_2501_17392_amd import synth
    for w in synth.WORKLOADS:
        if w.name == name or w.name.startswith(name + "_") or w.name.split("_")[0] == name:
            return w
    raise SystemExit(f"unknown workload {name!r}; choose from {[w.name for w in synth.WORKLOADS]}")


def time_on_stream(fn, reps, stream, warm=2):
    """Average and per-call times (ms) of `reps` calls of fn, from events on the launch stream."""
    import torch
    for _ in range(warm):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    for i in range(reps):
        ev[i].record(stream)
        fn()
    ev[reps].record(stream)
    torch.cuda.synchronize()
    each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
    return ev[0].elapsed_time(ev[reps]) / reps, each


def warm_for(fn, seconds):
    """Untimed calls for at least `seconds`: after a stretch with the GPU idle (the CPU oracle
    leg, the launch-bound small workloads) a 0.3 ms kernel runs several per cent slow until
    the clocks are back up, which takes longer than a fixed handful of calls."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()


def sample_windows(d, cols):
    """Column windows the oracle is run on: the first `cols` coordinates and the last ones
    (the ragged end of the vector), merged when they touch."""
    if d <= 2 * cols:
        return [(0, d)]
    return [(0, cols), (d - cols, d)]


def oracle_matches(upd, lam, gpu_out, windows):
    """True when the GPU result equals the plain-C oracle on every window of columns (same
    input bytes: the oracle reads a host copy of the device matrix)."""
    import numpy as np
    from oracle import c_oracle

    ok = True
    for lo, hi in windows:
        host = upd[:, lo:hi].contiguous().cpu().numpy()
        want, _, _ = c_oracle.brace_direct(host, lam, 0, want_sums=False, want_bits=False,
                                           nthreads=0)
        ok = ok and bool(np.array_equal(gpu_out[lo:hi].cpu().numpy(), want))
    return ok


def cpu_baseline(upd, w, lam, gpu_sample, sample_cols):
    """Time the plain-C oracle on the host cores over the first `sample_cols` columns of the
    same input bytes, and check the GPU result (`gpu_sample`, a host copy of those columns
    taken right after the timed steps) against it."""
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
    match = bool(np.array_equal(gpu_sample[:k1], want))
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


def bench_large(B, synth, w, lam, steps, stream, dev, check_cols):
    """One HBM-sized workload other than the headline: whole step and vote kernel alone,
    with an oracle check of the timed output on sampled columns."""
    import torch
    t0 = time.perf_counter()
    upd = synth.generate(w, dev)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    out = torch.empty(w.d, device=dev, dtype=torch.float32)
    bits = torch.empty((w.d + 31) // 32, device=dev, dtype=torch.int32)
    warm_for(lambda: B.brace_aggregate(upd, w.f, lam, out=out, stream=stream), 0.1)
    step_ms, each = time_on_stream(
        lambda: B.brace_aggregate(upd, w.f, lam, out=out, stream=stream), steps, stream)
    match = oracle_matches(upd, lam, out, sample_windows(w.d, check_cols))
    vote_ms, _ = time_on_stream(
        lambda: B.brace_aggregate(upd, w.f, lam, out=None, out_bits=bits, stream=stream),
        steps, stream)
    step_bytes = 4 * w.n * w.d + 4 * w.d
    vote_bytes = 4 * w.n * w.d + 4 * ((w.d + 31) // 32)
    row = {
        "workload": w.name, "n": w.n, "f": w.f, "d": w.d, "steps": steps,
        "ms_per_step": step_ms, "ms_min": each[0],
        "coords_per_s": w.d / (step_ms * 1e-3),
        "GBps": step_bytes / (step_ms * 1e-3) / 1e9,
        "frac": step_bytes / (step_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "vote_kernel_ms": vote_ms,
        "vote_kernel_GBps": vote_bytes / (vote_ms * 1e-3) / 1e9,
        "vote_kernel_frac": vote_bytes / (vote_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "vote_kernel_traffic": (PROFILED_TRAFFIC.get(w.name) or {}).get("bytes"),
        "vote_kernel_traffic_source": (PROFILED_TRAFFIC.get(w.name) or {}).get(
            "source", "no counter run for this workload"),
        "gpu_matches_oracle_on_sample": match,
        "oracle_sample": f"first and last {min(check_cols, w.d)} coordinates x all clients",
        "generate_s": gen_s,
    }
    log(f"[bench] {w.name}: {step_ms:.3f} ms/step = {row['GBps']:.0f} GB/s ({row['frac']:.1%}); "
        f"vote kernel alone {vote_ms:.3f} ms ({row['vote_kernel_frac']:.1%}); oracle match {match}")
    del upd, out, bits
    torch.cuda.empty_cache()
    return row


def bench_small(B, synth, w, lam, stream, dev):
    """A launch-bound workload: per-call latency of the whole call, issued directly and
    replayed from a HIP graph; checked against the numpy oracle in full.  No roofline claim."""
    import numpy as np
    import torch
    from oracle import brace_oracle as O

    upd = synth.generate(w, dev)
    out = torch.empty(w.d, device=dev, dtype=torch.float32)
    reps = 200
    B.brace_init_device()
    for _ in range(5):
        B.brace_aggregate(upd, w.f, lam, out=out, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        B.brace_aggregate(upd, w.f, lam, out=out, stream=stream)
    torch.cuda.synchronize()
    direct_us = (time.perf_counter() - t0) / reps * 1e6
    want = O.brace_direct(upd.cpu().numpy(), lam).out
    match = bool(np.array_equal(out.cpu().numpy(), want))

    # The same call captured once and replayed: the launch cost leaves the loop.
    side = torch.cuda.Stream()
    out_g = torch.empty_like(out)
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for _ in range(10):
                B.brace_aggregate(upd, w.f, lam, out=out_g, stream=side)
    torch.cuda.synchronize()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps // 10):
        graph.replay()
    torch.cuda.synchronize()
    graph_us = (time.perf_counter() - t0) / reps * 1e6
    match_g = bool(np.array_equal(out_g.cpu().numpy(), want))
    row = {
        "workload": w.name, "n": w.n, "f": w.f, "d": w.d,
        "latency_us_direct": direct_us, "latency_us_hip_graph": graph_us,
        "roofline": "none claimed: launch-bound / resident in the memory-side cache",
        "gpu_matches_oracle": match and match_g,
        "oracle_sample": "whole vector, numpy definition",
    }
    log(f"[bench] {w.name}: {direct_us:.1f} us per call, {graph_us:.1f} us in a HIP graph; "
        f"oracle match {match and match_g}")
    return row


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
    ap.add_argument("--no-per-config", dest="per_config", action="store_false",
                    help="skip the other workloads and the per-chunk sequence")
    ap.set_defaults(per_config=True)
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
    # `out` receives the timed steps' result and nothing else ever writes it; every other
    # leg of this run has buffers of its own.
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
    # What the timed steps produced, kept on the host for the oracle check further down.
    k_check = min(w.d, args.cpu_sample_cols)
    timed_result = out[:k_check].cpu().numpy()

    per_step_ms = sorted(events[i].elapsed_time(events[i + 1]) for i in range(K))
    step_ms = events[0].elapsed_time(events[K]) / K
    ms_per_step = wall * 1e3 / K
    step_bytes = 4 * w.n * w.d + 4 * w.d          # read n*d fp32 once, write d fp32
    step_gbs = step_bytes / (step_ms * 1e-3) / 1e9

    # The dominant kernel on its own: the streaming vote kernel reads the n x d matrix and
    # emits one bit per coordinate (inside a step the fp32 vector is then written by the small
    # expand kernel).  Same kernel and launch shape as inside the step, launched K more times
    # right after the timed region and timed with events on the launch stream.
    bits = torch.empty((w.d + 31) // 32, device=dev, dtype=torch.int32)
    vote_ms, vote_each = time_on_stream(
        lambda: B.brace_aggregate(upd, w.f, args.lam, out=None, out_bits=bits, stream=stream),
        K, stream)
    vote_bytes = 4 * w.n * w.d + 4 * ((w.d + 31) // 32)
    achieved = vote_bytes / (vote_ms * 1e-3) / 1e9
    log(f"[bench] {K} steps: wall {ms_per_step:.3f} ms/step, on-stream {step_ms:.3f} ms "
        f"(min {per_step_ms[0]:.3f}, median {per_step_ms[K // 2]:.3f}) -> {step_gbs:.0f} GB/s "
        f"= {step_gbs / HBM_PEAK_GBS:.1%} of {HBM_PEAK_GBS:.0f} GB/s over the whole step")
    log(f"[bench] vote kernel alone: avg {vote_ms:.3f} ms (min {vote_each[0]:.3f}) -> "
        f"{achieved:.0f} GB/s = {achieved / HBM_PEAK_GBS:.1%} of peak")

    traffic = PROFILED_TRAFFIC.get(w.name)
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
            "launch": B.brace_get_tuning(),
            "input_checksum": f"{synth.checksum(upd[:, : min(w.d, 1 << 20)]):#018x}",
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic["bytes"] if traffic else None,
            "traffic_source": traffic["source"] if traffic else
            "no counter run for this workload",
            "kernel": "brace_dev::stream_kernel<VoteOp, V, COLS, RU, NT, PIPE, RS> (the streaming vote "
                      "kernel; <VoteOp, 2, 8, 2, true, true, false> on the headline workload)",
            "measured_on": f"{K} launches of the kernel alone (bit output) right after the timed "
                           "steps, same launch shape as inside a step",
            "algorithmic_bytes_per_launch": vote_bytes,
            "kernel_ms_avg": vote_ms,
            "kernel_ms_min": vote_each[0],
            "kernel_ms_median": vote_each[K // 2],
            "step_frac": step_gbs / HBM_PEAK_GBS,
            "whole_step": {
                "kernels": "stream_kernel<VoteOp, ...> + brace_expand_kernel, the timed steps",
                "algorithmic_bytes": step_bytes,
                "ms_avg": step_ms, "ms_min": per_step_ms[0], "ms_median": per_step_ms[K // 2],
                "achieved": step_gbs, "frac": step_gbs / HBM_PEAK_GBS,
            },
        },
    }
    ok = True
    if args.per_config:
        # The per-chunk entry point: the n ring chunks one call each, the whole sequence timed.
        chunked = torch.empty(w.d, device=dev, dtype=torch.float32)

        def all_chunks():
            for c in range(w.n):
                B.brace_aggregate_chunk(upd, w.f, c, args.lam, out=chunked, stream=stream)

        seq_ms, seq_each = time_on_stream(all_chunks, max(3, K // 5), stream, warm=1)
        same = bool(torch.equal(chunked, out))
        ok = ok and same
        result["per_chunk_sequence"] = {
            "workload": w.name, "calls": w.n, "ms": seq_ms, "ms_min": seq_each[0],
            "GBps": step_bytes / (seq_ms * 1e-3) / 1e9,
            "frac": step_bytes / (seq_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "equals_whole_call": same,
        }
        log(f"[bench] {w.n} per-chunk calls: {seq_ms:.3f} ms (whole call {step_ms:.3f} ms), "
            f"equal to the whole call: {same}")
        del chunked
    if args.next_rows:
        # The widened rows, each timed alone with events on the launch stream and priced with
        # its own algorithmic bytes (read the matrix once + what it must write / re-read).
        # The planes use the recommended row pitch (rows start on 128-byte lines).
        rw = B.brace_packed_row_words(w.d)
        rp = B.brace_packed_row_pitch(w.d)
        signs = torch.empty(w.n, rp, device=dev, dtype=torch.int32)[:, :rw]
        model = torch.zeros(w.d, device=dev, dtype=torch.float32)
        vw = B.brace_1bit_row_words(w.d)
        vp = B.brace_1bit_row_pitch(w.d)
        votes = torch.empty(w.n, vp, device=dev, dtype=torch.int32)[:, :vw]
        other = torch.empty(w.d, device=dev, dtype=torch.float32)
        # 8 partial sign-sums (one per device of an 8-device ring), values as 12-13 clients give
        parts = torch.randint(-13, 14, (8, w.d), device=dev, dtype=torch.int16)
        nd4 = 4 * w.n * w.d
        wb = 4 * ((w.d + 31) // 32)
        rows = (
            ("rar_mean", lambda: B.brace_rar_aggregate(upd, other, mean=True, stream=stream),
             nd4 + 4 * w.d),
            ("rar_sum_ring_order_fp32",
             lambda: B.brace_rar_aggregate(upd, other, order=1, stream=stream), nd4 + 4 * w.d),
            ("update_with_bits", lambda: B.brace_aggregate_update(upd, w.f, model, 1e-3, args.lam,
                                                                  out_bits=bits, stream=stream),
             nd4 + 8 * w.d + 2 * wb),
            ("update_direct", lambda: B.brace_aggregate_update(upd, w.f, model, 1e-3, args.lam,
                                                               stream=stream), nd4 + 8 * w.d),
            ("update_noalloc", lambda: B.brace_aggregate_update_noalloc(upd, w.f, model, 1e-3,
                                                                        args.lam, stream=stream),
             nd4 + 8 * w.d + 2 * wb),
            ("quantize", lambda: B.brace_quantize(upd, signs, stream=stream), nd4 + 4 * w.n * rw),
            ("vote_packed", lambda: B.brace_vote_packed(signs, w.d, w.f, args.lam, out=other,
                                                        stream=stream),
             4 * w.n * rw + 4 * w.d + 2 * wb),
            ("vote_packed_bits_only",
             lambda: B.brace_vote_packed(signs, w.d, w.f, args.lam, out_bits=bits, stream=stream),
             4 * w.n * rw + wb),
            ("expand_bits", lambda: B.brace_expand_bits(bits, w.d, other, stream=stream),
             4 * w.d + wb),
            ("apply_bits", lambda: B.brace_apply_bits(bits, w.d, 1e-3, model, stream=stream),
             8 * w.d + wb),
            ("quantize_1bit", lambda: B.brace_quantize_1bit(upd, 1, votes, stream=stream),
             nd4 + 4 * w.n * vw),
            ("vote_1bit", lambda: B.brace_vote_1bit(votes, w.d, w.f, args.lam, out=other,
                                                    stream=stream),
             4 * w.n * vw + 4 * w.d + 2 * wb),
            ("vote_1bit_bits_only",
             lambda: B.brace_vote_1bit(votes, w.d, w.f, args.lam, out_bits=bits, stream=stream),
             4 * w.n * vw + wb),
            ("consensus_sums_g8", lambda: B.brace_consensus_sums(parts, args.lam, out=other,
                                                                 stream=stream),
             2 * 8 * w.d + 4 * w.d),
        )
        extra = {}
        for name, fn, nbytes in rows:
            ms, _ = time_on_stream(fn, max(5, K // 3), stream)
            gbs = nbytes / (ms * 1e-3) / 1e9
            extra[name] = {"ms": ms, "algorithmic_bytes": nbytes, "achieved_GBps": gbs,
                           "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
            log(f"[bench] {name}: {ms:.3f} ms, {gbs:.0f} GB/s ({gbs / HBM_PEAK_GBS:.1%})")
        result["next_rows"] = extra
        del signs, model, votes, other, parts
    if args.probe:
        nel = (1 << 30) // 4
        src = torch.randn(nel, device=dev)
        dst = torch.empty_like(src)
        sink = torch.zeros(4, device=dev)
        probe = {"bytes": nel * 4}
        for name, fn, moved in (("read", lambda: B.brace_probe_read(src, sink, 1, stream), nel * 4),
                                ("copy", lambda: B.brace_probe_copy(dst, src, stream), 2 * nel * 4)):
            ms, _ = time_on_stream(fn, 10, stream)
            probe[name + "_GBps"] = moved / (ms * 1e-3) / 1e9
        result["probe"] = probe
        log(f"[bench] probe: {probe}")
        del src, dst
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a sample ...")
        result["cpu_baseline"] = cpu_baseline(upd, w, args.lam, timed_result, args.cpu_sample_cols)
        # reported for context only: the roofline fraction, not this ratio, rates the kernel
        result["cpu_baseline"]["gpu_over_cpu"] = result["value"] / result["cpu_baseline"]["value"]
        result["cpu_baseline"]["gpu_over_cpu_1thread"] = \
            result["value"] / result["cpu_baseline"]["value_1thread"]
        ok = ok and result["cpu_baseline"]["gpu_matches_oracle_on_sample"]
        log(f"[bench] oracle: {result['cpu_baseline']['value']:.3e} coords/s on "
            f"{result['cpu_baseline']['cores']} threads; GPU matches oracle on the sample: "
            f"{result['cpu_baseline']['gpu_matches_oracle_on_sample']}")
    del upd, out, bits
    torch.cuda.empty_cache()
    if args.per_config:
        # The other workloads, one matrix resident at a time.  HBM-sized ones get the same
        # figures as the headline; the two small ones a latency and no roofline claim.
        per = []
        for other_w in synth.WORKLOADS:
            if other_w.name == w.name:
                continue
            if other_w.input_bytes < (1 << 30):
                row = bench_small(B, synth, other_w, args.lam, stream, dev)
                ok = ok and row["gpu_matches_oracle"]
            else:
                row = bench_large(B, synth, other_w, args.lam, K, stream, dev, 1 << 20)
                ok = ok and row["gpu_matches_oracle_on_sample"]
            per.append(row)
        result["per_config"] = per
    result["all_oracle_checks_passed"] = bool(ok)
    print(json.dumps(result), flush=True)
    if not ok:
        log("[bench] FAILED: a GPU result differs from the oracle (see the *_matches_* fields)")
        sys.exit(1)


if __name__ == "__main__":
    main()
