#!/usr/bin/env python3
"""Benchmark of the search path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5] [--queries Q] [--n N]

A *step* is one pass of the whole hot path over one batch of Q queries of the chosen
configuration (default: the 100M-code configuration, the one the headline metric is quoted
on), with every input already resident in HBM:

    distance tables -> linear ADC scan + top-R -> coarse ranking -> inverted-index scan + top-R
    -> subset (gathered) scan + top-R -> the Alg. 3 query procedure on the whole database.

It prints ONE JSON line.  `value` is the number of PQ codes scored per second over the whole
step.  `roofline` is the one-query-per-pass linear scan (k_scan_w: M algorithmic bytes per code, bound
by HBM; with early abandoning over the two-plane layout of M = 32 it moves about half of them, see
`moved_gbs`), timed with HIP events recorded around that kernel on its stream;
`roofline_batched` is the batched launch of the timed steps (k_scan_w4: four queries share each
code byte, so the bound is the LDS look-up rate; `achieved` counts the look-ups the kernel really
made -- it abandons part of them -- and the ceiling is measured live with the library's
look-up-only kernel).  `cpu_baseline` is the CPU oracle's linear scan timed single-threaded on a
bounded sample of the same codes (and, beside it, on all host threads with one query each).
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

# HBM-side bytes per launch from the rocprofv3 PMC runs summarised in
# profiles/k_scan_w_k_scan_w4_c5_hbm_traffic_pmc.txt (FETCH_SIZE
# x 2.000 + WRITE_SIZE x 1.000 KiB, the factors found with a plain streaming kernel of known
# size).  Reported only for the exact configuration they were measured on.
MEASURED_TRAFFIC = {
    ("c5_billion_shard", 100_000_000, 10_000): {
        # k_scan_w, one query: 797,079 KiB fetched x 2, 1,155 KiB written
        "single": 797_079 * 2.0 * 1024 + 1_155 * 1024,
        # k_scan_w4, 10,000 queries: 974,001,968 KiB fetched x 2, 10,593 KiB written
        "batched": 974_001_968 * 2.0 * 1024 + 10_593 * 1024,
    },
}

# LDS look-up ceiling from unit counts: 256 CUs x 128 B/clk of LDS bandwidth at 2.4 GHz; an
# 8-byte look-up (ds_read_b64) therefore at most 16 lanes per clock and CU.
LDS_SPEC_LOOKUPS_PER_S = 256 * 16 * 2.4e9


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
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain streaming kernel of known size (1 GiB read + 1 GiB written) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
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
    slices, abandoned = binding.rii_index_read_scan_counters(index)
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

    # one query per pass: the plain HBM-roofline number for the scan kernel
    rii.rii_index_set_scan_events(index, ev.start.value, ev.stop.value)
    single = []
    for i in range(12):
        rii.rii_adc_scan_linear(index, lut[i % Q:i % Q + 1], R)
        torch.cuda.synchronize()
        single.append(ev.elapsed_ms())
    rii.rii_index_set_scan_events(index, None, None)
    single_ms = float(np.mean(single[2:]))

    scan_avg_ms = float(np.mean(scan_ms))
    traffic = MEASURED_TRAFFIC.get((cfg.name, N, Q), {})
    single_gbs = N * M / (single_ms * 1e-3) / 1e9   # M algorithmic bytes per code and query pass
    roofline = {
        "bound": "hbm", "kernel": f"k_scan_w<{M},linear> (seeds its bound itself), one query per launch",
        "achieved": round(single_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(single_gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get("single"),
        "launch_ms": round(single_ms, 4), "algorithmic_bytes_per_launch": float(N) * M,
        "codes_per_s": round(N / (single_ms * 1e-3), 1),
    }
    if traffic.get("single"):
        # For M = 32 the kernel skips the second 16-byte plane of slices it settles after 16
        # look-ups, so it moves fewer bytes than the algorithmic count and `frac` can exceed 1;
        # the rate at which it really moves bytes is reported beside it.
        moved = traffic["single"] / (single_ms * 1e-3) / 1e9
        roofline["moved_gbs"] = round(moved, 1)
        roofline["moved_frac_of_peak"] = round(moved / HBM_PEAK_GBS, 4)
    # The batched launch: look-ups, not bytes, are what bounds it.
    batched = None
    qpb, row_chunks = binding.rii_scan_linear_plan(index, Q, R)
    if qpb == 4:
        groups = (Q + 3) // 4
        lookups = float(groups) * N * M            # one 8-byte LDS read per code byte and group of four queries
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ceil_ms = []
        for _ in range(4):
            a.record()
            n_lk = binding.rii_bench_lds_lookups(8, 256, 4000, 150 * 1024)   # one block per CU, as k_scan_w4 runs
            b.record()
            torch.cuda.synchronize()
            ceil_ms.append(a.elapsed_time(b))
        ceiling = n_lk / (min(ceil_ms[1:]) * 1e-3)
        # look-ups the kernel actually made: a slice is 64 rows x M look-ups, an abandoned one stops after M/2
        executed = 64.0 * (slices * M - abandoned * (M // 2)) / args.steps
        ach = executed / (scan_avg_ms * 1e-3)
        batched = {
            "bound": "lds", "kernel": f"k_scan_w4<{M}>, {Q} queries per launch, {row_chunks} row chunk(s)", "achieved": round(ach / 1e9, 1),
            "peak": round(ceiling / 1e9, 1), "unit": "G look-ups/s", "frac": round(ach / ceiling, 4),
            "peak_source": "measured live: rii_bench_lds_lookups(width 8, 256 blocks x 1024 threads)",
            "spec_peak": round(LDS_SPEC_LOOKUPS_PER_S / 1e9, 1), "frac_of_spec": round(ach / LDS_SPEC_LOOKUPS_PER_S, 4),
            "lookups_executed_per_launch": executed, "lookups_algorithmic_per_launch": lookups,
            "abandoned_slice_fraction": round(abandoned / max(slices, 1), 4),
            "algorithmic_lookup_rate": round(lookups / (scan_avg_ms * 1e-3) / 1e9, 1),
            "traffic": traffic.get("batched"), "launch_ms": round(scan_avg_ms, 3),
            "algorithmic_bytes_per_launch": float(Q) * N * M,
            "algorithmic_gbs": round(float(Q) * N * M / (scan_avg_ms * 1e-3) / 1e9, 1),
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
        "hbm_frac_of_peak": roofline["frac"],
        "roofline": roofline,
        "roofline_batched": batched,
        "cpu_baseline": cpu,
        "index": {"paper_bytes": info["paper_bytes"], "device_bytes": info["device_bytes"], "setup_s": w["timings"]},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
