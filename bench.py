#!/usr/bin/env python3
"""Benchmark of the search path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5] [--queries Q] [--n N]

A *step* is one pass of the whole hot path over one batch of Q queries of the chosen
configuration (default: the 100M-code configuration, the one the headline metric is quoted
on), with every input already resident in HBM:

    distance tables -> linear ADC scan + top-R -> coarse ranking -> inverted-index scan + top-R
    -> subset (gathered) scan + top-R -> the Alg. 3 query procedure on the whole database.

It prints ONE JSON line.  `value` is the number of PQ codes scored per second over the whole
step.  Three roofline objects:

`roofline` -- the one-query-per-launch linear scan of the configuration's own data (k_scan_w,
bound by HBM), timed with HIP events recorded around that kernel on its stream.  `frac` is the
rate of bytes the kernel really moved (`traffic`, from the tallies the kernel keeps in the same
launches: first plane streamed, second-plane lines fetched on demand or streamed) against the
8 TB/s peak, so it cannot exceed 1; the method's own M bytes per code are reported beside it
(`algorithmic_bytes_per_launch`, `algorithmic_gbs`, `moved_over_algorithmic`).
`roofline_no_pruning` -- the same kernel over N independent uniform code bytes, where nearly every
128-byte line of second halves has a row that is still open half-way, so the kernel ends up
fetching (nearly) every byte: moved = algorithmic.
`roofline_batched` -- the batched launch of the timed steps (k_scan_w4: four queries share each
code byte, so the bound is the LDS look-up rate; `achieved` counts the look-ups the kernel really
made -- it abandons part of them -- and `peak` is the best rate of conflict-free 8-byte LDS reads
over several occupancies, measured in the same run; the rate of the scan's inner loop alone at the
kernel's own occupancy is given beside it).
`cpu_baseline` is the CPU oracle's linear scan timed single-threaded on a bounded sample of the
same codes (and, beside it, on all host threads with one query each).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# Occupancies the LDS look-up ceiling is measured at: (blocks, threads per block, LDS bytes per
# block).  The ceiling reported is the best of them.
LDS_CEILING_SHAPES = [(256, 1024, 150 * 1024), (512, 1024, 64 * 1024), (1024, 1024, 64 * 1024), (2048, 512, 64 * 1024)]


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


class HipEvents:
    """A pair of raw HIP events (created through the HIP runtime torch has loaded)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.start, self.stop = ctypes.c_void_p(), ctypes.c_void_p()
        assert self.hip.hipEventCreate(ctypes.byref(self.start)) == 0
        assert self.hip.hipEventCreate(ctypes.byref(self.stop)) == 0

    def elapsed_ms(self) -> float:
        assert self.hip.hipEventSynchronize(self.stop) == 0
        ms = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(ms), self.start, self.stop) == 0
        return float(ms.value)


SWEEP_SHAPES = [  # (M, N): every one with the (Q, topk) pairs below
    (32, 100_000_000), (64, 50_000_000), (16, 10_000_000), (64, 5_000_000),
]
SWEEP_BATCHES = [(1, 100), (1, 129), (1, 256), (1, 1024), (64, 100), (64, 256), (64, 1024), (1024, 100), (1024, 1024)]


def sweep(rii, np, torch):
    """Launch time of rii_adc_scan_linear by shape (best of three calls, torch events around the
    call; uniform random codes and Gaussian code books, so nothing is pruned by the data)."""
    from paper_1808_03969_amd import binding
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for M, N in SWEEP_SHAPES:
        rng = np.random.default_rng(5 + M)
        index = rii.Index(rng.normal(size=(M, 256, 2)).astype(np.float32))
        if M == 32:
            index.set_option(binding.RII_OPT_GATHER_COPY, 0)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(5 + M)
        for r0 in range(0, N, 10_000_000):
            n = min(N, r0 + 10_000_000) - r0
            index.add(torch.randint(0, 256, (n, M), dtype=torch.uint8, device="cuda", generator=gen))
        lut = rii.rii_build_lut(index, torch.from_numpy(rng.normal(size=(1024, 2 * M)).astype(np.float32)).cuda())
        for Q, topk in SWEEP_BATCHES:
            if Q * N > 12_000_000_000 and (topk > 100 or M == 64):
                continue  # (seconds per call on the one-query-per-block paths)
            l = lut[:Q].contiguous()
            qpb, chunks = binding.rii_scan_linear_plan(index, Q, topk)
            rii.rii_adc_scan_linear(index, l, topk)
            torch.cuda.synchronize()
            best = float("inf")
            for _ in range(3):
                a.record()
                rii.rii_adc_scan_linear(index, l, topk)
                b.record()
                torch.cuda.synchronize()
                best = min(best, a.elapsed_time(b))
            print(json.dumps({"M": M, "N": N, "Q": Q, "topk": topk, "queries_per_block": qpb, "row_chunks": chunks,
                              "ms": round(best, 4), "codes_per_s": round(Q * N / (best * 1e-3), 1),
                              "algorithmic_gbs": round(Q * N * M / (best * 1e-3) / 1e9, 1)}), flush=True)
        index.close()
        del index, lut
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c4", "c5"])
    ap.add_argument("--queries", type=int, default=None, help="batch size Q (default: the configuration's)")
    ap.add_argument("--n", type=int, default=None, help="database size override (for quick runs)")
    ap.add_argument("--subset", type=int, default=1_000_000, help="|S| of the subset scan")
    ap.add_argument("--nprobe", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-uniform-leg", action="store_true", help="skip roofline_no_pruning (the scan of uniform random codes)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain streaming kernel of known size (1 GiB read + 1 GiB written) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the bench step: time rii_adc_scan_linear over uniform random codes for a set of "
                         "(M, N, Q, topk) shapes, including those outside the fast kernels' reach (M = 64, topk > 128); "
                         "one JSON line per shape")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; there is no multi-GPU path (queries and codes would shard "
              "over GPUs with a top-k merge, which is not built). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1808_03969_amd as rii
    from paper_1808_03969_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    rii.load_library()
    torch.cuda.set_device(0)
    if args.sweep:
        sweep(rii, np, torch)
        return
    cfg = workloads.CONFIGS[args.workload]
    t_setup = time.time()
    w = workloads.build(cfg, log=log, N=args.n, Q=args.queries)
    index, q, N, Q = w["index"], w["q"], w["N"], w["Q"]
    M, K, R = cfg.M, cfg.K, cfg.topk
    S = min(args.subset, N)
    nprobe = min(args.nprobe, K) if K else 0
    t0 = time.time()
    tids, toff = workloads.subsets(cfg, N, Q, S)
    torch.cuda.synchronize()
    log(f"{Q} target subsets of size {S} in {time.time() - t0:.1f}s; setup total {time.time() - t_setup:.1f}s")
    info = index.info()
    _, list_off, _, _ = index.get_lists() if K else (None, None, None, None)
    L_query = max(1, nprobe * (N // K)) if K else 1
    index.set_threshold(0)

    lut = torch.empty((Q, M, 256), dtype=torch.float32, device="cuda")
    out_lin = (torch.empty((Q, R), dtype=torch.int32, device="cuda"), torch.empty((Q, R), dtype=torch.float32, device="cuda"))
    out_ivf = (torch.empty_like(out_lin[0]), torch.empty_like(out_lin[1]))
    out_sub = (torch.empty_like(out_lin[0]), torch.empty_like(out_lin[1]))
    out_qry = (torch.empty_like(out_lin[0]), torch.empty_like(out_lin[1]))
    ev = HipEvents()
    rii.rii_index_set_scan_events(index, ev.start.value, ev.stop.value)
    stage_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(6)]
    probe_holder = {}

    def step(timed: bool):
        se = stage_ev
        se[0][0].record(); rii.rii_build_lut(index, q, out=lut); se[0][1].record()
        se[1][0].record(); rii.rii_adc_scan_linear(index, lut, R, out=out_lin); se[1][1].record()
        if K:
            se[2][0].record(); probe, _ = rii.rii_coarse_assign(index, lut, nprobe, want_d0=False); se[2][1].record()
            probe_holder["p"] = probe
            se[3][0].record(); rii.rii_adc_scan_ivf(index, lut, probe, R, out=out_ivf); se[3][1].record()
        se[4][0].record(); rii.rii_adc_scan_subset(index, lut, tids, toff, S, R, out=out_sub); se[4][1].record()
        if K:
            se[5][0].record(); rii.rii_query(index, q, R, L=L_query, out=out_qry); se[5][1].record()

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    from paper_1808_03969_amd import binding
    binding.rii_index_read_scan_counters(index)  # reset: count the timed steps only
    scan_ms, stage_ms = [], np.zeros(6)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
        torch.cuda.synchronize()
        scan_ms.append(ev.elapsed_ms())
        for i, (a, b) in enumerate(stage_ev):
            if K or i in (0, 1, 4):
                stage_ms[i] += a.elapsed_time(b)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    stage_ms /= args.steps
    counters = binding.rii_index_read_scan_counters(index)
    slices, abandoned = counters[0], counters[1]
    rii.rii_index_set_scan_events(index, None, None)

    # codes scored in one step
    probed = 0
    if K:
        lens = np.diff(list_off)
        pl = probe_holder["p"].cpu().numpy()
        probed = int(lens[pl].sum())
        probed_query = int(np.minimum(lens[pl].sum(axis=1), L_query).sum())
    scored = Q * N + Q * S + (probed + probed_query + 2 * Q * K if K else 0)
    value = scored / (ms_per_step * 1e-3)

    def one_query_leg(idx, n_rows, lut1, what, launches=12):
        """One query per launch over `idx`: launch time from the events around the kernel, bytes
        moved from the kernel's own tallies of the same launches."""
        rii.rii_index_set_scan_events(idx, ev.start.value, ev.stop.value)
        for i in range(2):                                   # warm-up (also sizes the scratch)
            rii.rii_adc_scan_linear(idx, lut1[i % len(lut1):i % len(lut1) + 1], R)
        torch.cuda.synchronize()
        binding.rii_index_read_scan_counters(idx)
        ms = []
        for i in range(launches):
            rii.rii_adc_scan_linear(idx, lut1[i % len(lut1):i % len(lut1) + 1], R)
            torch.cuda.synchronize()
            ms.append(ev.elapsed_ms())
        c = binding.rii_index_read_scan_counters(idx)
        rii.rii_index_set_scan_events(idx, None, None)
        launch_ms = float(np.mean(ms))
        algorithmic = float(n_rows) * M                      # M bytes per code and query pass
        if M == 32:
            # two planes of 16 bytes per row: the first is streamed whole; of the second, the
            # 128-byte lines the kernel asked for
            moved = n_rows * 16.0 + 128.0 * c[2] / launches
        else:
            moved = algorithmic
        moved = min(moved, algorithmic)                      # (rows re-read at block seams are cache hits)
        gbs = moved / (launch_ms * 1e-3) / 1e9
        return {
            "bound": "hbm", "kernel": f"k_scan_w<{M},linear>, one query per launch, {what}",
            "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
            "traffic": moved, "traffic_source": "kernel tallies of the timed launches (first plane streamed + second-plane lines fetched)"
                                               if M == 32 else "every code byte is read once",
            "launch_ms": round(launch_ms, 4), "launch_ms_min_max": [round(min(ms), 4), round(max(ms), 4)],
            "algorithmic_bytes_per_launch": algorithmic,
            "algorithmic_gbs": round(algorithmic / (launch_ms * 1e-3) / 1e9, 1),
            "moved_over_algorithmic": round(moved / algorithmic, 4),
            "codes_per_s": round(n_rows / (launch_ms * 1e-3), 1),
        }

    # one query per pass: the HBM-roofline number for the scan kernel, on the configuration's own data ...
    roofline = one_query_leg(index, N, lut, f"{cfg.name} data")
    scan_avg_ms = float(np.mean(scan_ms))
    # ... and on independent uniform code bytes, where half-way abandoning saves nothing
    no_pruning = None
    if not args.no_uniform_leg:
        t0 = time.time()
        uni = rii.Index(w["cb"])
        if M == 32:
            uni.set_option(binding.RII_OPT_GATHER_COPY, 0)   # this index is only ever scanned in sequence
        gen = torch.Generator(device="cuda")
        gen.manual_seed(7000 + cfg.c)
        for r0 in range(0, N, 10_000_000):
            n = min(N, r0 + 10_000_000) - r0
            uni.add(torch.randint(0, 256, (n, M), dtype=torch.uint8, device="cuda", generator=gen))
        torch.cuda.synchronize()
        log(f"{N} uniform random codes stored in {time.time() - t0:.1f}s")
        no_pruning = one_query_leg(uni, N, lut, "independent uniform code bytes")
        uni.close()

    # The batched launch: look-ups, not bytes, are what bounds it.
    batched = None
    qpb, row_chunks = binding.rii_scan_linear_plan(index, Q, R)
    if qpb == 4:
        groups = (Q + 3) // 4
        lookups = float(groups) * N * M            # one 8-byte LDS read per code byte and group of four queries
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def best_rate(launch):
            best = 0.0
            for _ in range(3):
                a.record()
                n = launch()
                b.record()
                torch.cuda.synchronize()
                best = max(best, n / (a.elapsed_time(b) * 1e-3))
            return best

        # Two ceilings, each at several occupancies: the LDS pipe's own rate of conflict-free 8-byte
        # reads (nothing but reads), and the rate of the scan's inner loop alone (address permute,
        # 8-byte read, add -- what the vector pipe lets through).  `peak` is the first at its best.
        reads, loops = {}, {}
        for blocks, threads, lds in LDS_CEILING_SHAPES:
            iters = max(1, 4000 * 256 * 1024 // (blocks * threads))
            name = f"{blocks}x{threads}thr,{lds // 1024}KB"
            reads[name] = round(best_rate(lambda: binding.rii_bench_lds_reads(8, blocks, threads, iters * 4, lds)) / 1e9, 1)
            loops[name] = round(best_rate(lambda: binding.rii_bench_lds_lookups(8, blocks, threads, iters, lds)) / 1e9, 1)
        ceiling = max(reads.values()) * 1e9
        own_shape = f"{LDS_CEILING_SHAPES[0][0]}x{LDS_CEILING_SHAPES[0][1]}thr,{LDS_CEILING_SHAPES[0][2] // 1024}KB"
        # a slice is 64 rows x M look-ups; `abandoned` slices stopped after M/2 at the latest, `quarter` of
        # them after M/4 already, `late` ones after 3M/4 (the last two at M = 32 only)
        quarter, late = counters[3], counters[4]
        executed = 64.0 * (slices * M - abandoned * (M // 2) - quarter * (M // 4) - late * (M // 4)) / args.steps
        ach = executed / (scan_avg_ms * 1e-3)
        batched = {
            "bound": "lds", "kernel": f"k_scan_w4<{M}>, {Q} queries per launch, {row_chunks} row chunk(s)", "achieved": round(ach / 1e9, 1),
            "bound_note": "the unit of work is an 8-byte LDS read per code byte and group of four queries; SQ counters "
                          "(profiles/k_scan_w4_k_scan_w_c5_instruction_mix_pmc.txt) show the vector pipe, not the LDS pipe, "
                          "as the busiest unit of this kernel",
            "peak": round(ceiling / 1e9, 1), "unit": "G look-ups/s", "frac": round(ach / ceiling, 4),
            "peak_source": "best rate of conflict-free 8-byte LDS reads (rii_bench_lds_reads) over the launch shapes listed, "
                           "measured in this run",
            "lds_read_rate_by_launch_shape": reads, "inner_loop_rate_by_launch_shape": loops,
            "frac_of_inner_loop_rate_at_own_occupancy": round(ach / (loops[own_shape] * 1e9), 4),
            "lookups_executed_per_launch": executed, "lookups_algorithmic_per_launch": lookups,
            "algorithmic_lookup_rate": round(lookups / (scan_avg_ms * 1e-3) / 1e9, 1),
            "algorithmic_frac": round(lookups / (scan_avg_ms * 1e-3) / ceiling, 4),
            "abandoned_slice_fraction": round(abandoned / max(slices, 1), 4),
            "abandoned_after_a_quarter_fraction": round(quarter / max(slices, 1), 4),
            "abandoned_after_three_quarters_fraction": round(late / max(slices, 1), 4),
            "launch_ms": round(scan_avg_ms, 3),
            "algorithmic_bytes_per_launch": float(Q) * N * M,
            "algorithmic_gbs": round(float(Q) * N * M / (scan_avg_ms * 1e-3) / 1e9, 1),
        }

        # The fp16-table variant of the same kernel (same rows, same results), timed beside it.
        out_h = (torch.empty_like(out_lin[0]), torch.empty_like(out_lin[1]))
        binding.rii_bench_scan_linear_half(index, lut, R, out=out_h)
        torch.cuda.synchronize()
        rii.rii_index_set_scan_events(index, ev.start.value, ev.stop.value)
        binding.rii_index_read_scan_counters(index)
        half_ms = []
        for _ in range(max(2, min(args.steps, 3))):
            binding.rii_bench_scan_linear_half(index, lut, R, out=out_h)
            torch.cuda.synchronize()
            half_ms.append(ev.elapsed_ms())
        ch = binding.rii_index_read_scan_counters(index)
        rii.rii_index_set_scan_events(index, None, None)
        batched["half_precision_table_variant"] = {
            "kernel": f"k_scan_w4<{M},half>", "launch_ms": round(float(np.mean(half_ms)), 3),
            "over_integer_table": round(float(np.mean(half_ms)) / scan_avg_ms, 4),
            "abandoned_slice_fraction": round(ch[1] / max(ch[0], 1), 4),
            "abandoned_after_a_quarter_fraction": round(ch[3] / max(ch[0], 1), 4),
            "results_equal": bool(torch.equal(out_h[0], out_lin[0]) and torch.equal(out_h[1], out_lin[1])),
        }
        del out_h

    # The subset scan gathers rows of M bytes out of 128-byte memory lines: bytes it needs against
    # the bytes of the lines they lie in (counted from the identifiers of a sample of the queries).
    toff_h = toff[:17].cpu().numpy()
    rows_per_line = max(1, 128 // M)
    n_lines = 0
    for i in range(len(toff_h) - 1):
        n_lines += int(torch.unique(tids[toff_h[i]:toff_h[i + 1]] // rows_per_line).numel())
    sampled = int(toff_h[-1] - toff_h[0])
    useful = float(Q) * S * (M + 4)
    in_lines = (n_lines * 128.0 / max(sampled, 1) + 4.0) * Q * S
    subset = {
        "kernel": f"k_scan_w<{M},subset>, {Q} queries x {S} target identifiers", "launch_ms": round(float(stage_ms[4]), 3),
        "useful_bytes": useful, "useful_gbs": round(useful / (stage_ms[4] * 1e-3) / 1e9, 1),
        "bytes_of_the_lines_touched": in_lines, "line_gbs": round(in_lines / (stage_ms[4] * 1e-3) / 1e9, 1),
        "note": "a gathered row brings its whole 128-byte line (identifiers: 4 bytes each, read in sequence); when the "
                "code array fits the caches (small N) the lines come from there and line_gbs can exceed the HBM rate",
    }

    if args.pmc_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)  # elementwise kernel: reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        import oracle  # the CPU oracle, timed beside the GPU path (never used by it)
        n_s = min(N, 25_000_000)
        codes_h = index.get_codes(0, n_s)
        A = lut[:2].cpu().numpy()
        got_i, got_d = out_lin[0][:2].cpu().numpy(), out_lin[1][:2].cpu().numpy()
        t0 = time.perf_counter()
        nq = 0
        for i in range(2):
            ref_i, ref_d = oracle.linear_scan(A[i], codes_h, R)
            nq += 1
            if n_s == N:
                assert np.array_equal(ref_i, got_i[i]) and np.array_equal(ref_d, got_d[i]), "GPU result differs from the oracle"
        dt = time.perf_counter() - t0
        cpu = {"value": round(nq * n_s / dt, 1), "unit": "codes/s", "cores": 1, "kind": "oracle",
               "sample": f"Alg. 1 linear scan of the first {n_s} codes for {nq} queries, top-{R}, single thread",
               "ms_per_query_full_scan": round(dt / nq * 1e3 * (N / n_s), 1)}
        # The same single-threaded oracle function on P host threads, one query each (independent
        # queries; the call releases the interpreter lock).
        from concurrent.futures import ThreadPoolExecutor
        P = max(1, min(Q, int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)))
        Ap = lut[:P].cpu().numpy()
        with ThreadPoolExecutor(P) as pool:
            t0 = time.perf_counter()
            list(pool.map(lambda i: oracle.linear_scan(Ap[i], codes_h, R), range(P)))
            dtp = time.perf_counter() - t0
        cpu["all_threads"] = {"value": round(P * n_s / dtp, 1), "unit": "codes/s", "cores": P,
                              "sample": f"the same scan for {P} queries, one per thread"}

    line = {
        "metric": "ADC codes scanned/sec (% of HBM peak) + queries/sec at top-k=100, 1 MI355X", "value": round(value, 1), "unit": "codes/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "N": N, "D": cfg.D, "M": M, "Ks": 256, "nlist": K, "Q": Q, "topk": R,
                   "nprobe": nprobe, "subset_size": S, "L_query": L_query},
        "queries_per_s": {
            "whole_step": round(Q / (ms_per_step * 1e-3), 1),
            "linear_scan": round(Q / (stage_ms[1] * 1e-3), 1),
            "ivf_nprobe": round(Q / ((stage_ms[2] + stage_ms[3]) * 1e-3), 1) if K else None,
            "subset_scan": round(Q / (stage_ms[4] * 1e-3), 1),
            "query_alg3": round(Q / (stage_ms[5] * 1e-3), 1) if K else None,
        },
        "stage_ms": {"lut": round(stage_ms[0], 3), "linear": round(stage_ms[1], 3), "coarse": round(stage_ms[2], 3),
                     "ivf": round(stage_ms[3], 3), "subset": round(stage_ms[4], 3), "query": round(stage_ms[5], 3)},
        "codes_scored_per_step": scored,
        "roofline": roofline,
        "roofline_no_pruning": no_pruning,
        "roofline_batched": batched,
        "subset_scan": subset,
        "cpu_baseline": cpu,
        "index": {"paper_bytes": info["paper_bytes"], "device_bytes": info["device_bytes"],
                  "device_over_paper": round(info["device_bytes"] / info["paper_bytes"], 3),
                  # with RII_OPT_GATHER_COPY = 0 (M = 32: no whole-row copy for gathered scans) the handle holds N * M bytes less
                  "device_over_paper_without_gather_copy": round((info["device_bytes"] - (N * M if M == 32 else 0)) / info["paper_bytes"], 3),
                  "setup_s": w["timings"]},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
