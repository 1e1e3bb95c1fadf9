#!/usr/bin/env python3
"""Benchmark of the RNN-Descent build hot path on one MI355X.

A "step" is one complete rnnd_build (RandomGraph + T1*T2 UpdateNeighbors rounds + T1-1
AddReverseEdges) over one synthetic database that is already resident in HBM.  The default
workload is cfg3 of workloads.py (N = 1,000,000, d = 128, uint8, S=20 R=96 T1=4 T2=15), the
one the "1M-vector graph build time" metric is quoted on; next to it the other four
configurations (cfg1, cfg2: small uint8; cfg4: 1M x 96 and cfg5: 1M x 960 float32) are measured
the same way (the 1M float ones with two steps) and reported under "workloads".  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--also none] [--no-cpu-baseline]
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

# HBM bytes per scan launch (one round's scan kernels together) measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE (two runs, each scaled by what the same counter reads for a plain 1 GiB copy in the same run);
# see profiles/update_scan_cfg{3,4,5}_hbm_traffic.txt.  Keyed by (workload, kernel variant); None where it
# has not been measured.
TRAFFIC_PER_LAUNCH = {("cfg3", 2): 1.0224e9, ("cfg4", 3): 8.544e9, ("cfg5", 3): 8.3522e10}


def host_cpu():
    """Model name and core counts of the host the oracle is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        usable = os.cpu_count()
    return {"model": model, "logical_cpus": os.cpu_count(), "usable_cpus": usable}


def cpu_baseline(cfg, X, sample_n, gpu_algo_evals):
    """The oracle as it stands (plain C, gcc -O2, one thread), timed on the first sample_n rows with the same
    S, R, T1, T2.  A bounded sample: the full run takes minutes (2.5 at 1M x 128 uint8, 15 at 1M x 960).  The
    value is the sample's time scaled to the workload's size by the number of distance evaluations Alg. 4
    makes (the GPU's count at full size, which the parity tests prove equal to the oracle's, over the sample's)
    -- an extrapolation, and an optimistic one: at full size the oracle's lists and rows no longer fit the
    host's caches."""
    import oracle
    oracle.build()
    Xs = X[:sample_n].copy()
    if Xs.dtype.itemsize == 2:      # half-precision storage: the oracle works on the floats the halves stand for
        Xs = Xs.astype("float32")
    t0 = time.perf_counter()
    res = oracle.build_sync(Xs, cfg.S, cfg.R, cfg.T1, cfg.T2, 2310)
    dt = time.perf_counter() - t0
    evals = int(res.init_evals + res.round_evals.sum())
    full = sample_n >= cfg.N
    scale = 1.0 if full else gpu_algo_evals / evals
    return {
        "value": dt * scale, "unit": "s", "cores": 1, "kind": "oracle",
        "extrapolated": not full,
        "sample": ("the full workload" if full else
                   "oracle build on the first %d rows of the same workload (same S,R,T1,T2): %.2f s, %d distance "
                   "evaluations; value = that time x (evaluations of the full-size build / of the sample) = x %.2f; "
                   "measured at full size once, inside the GPU parity test of cfg3: 152 s"
                   % (sample_n, dt, evals, scale)),
        "sample_rows": sample_n, "sample_seconds": dt, "distance_evals_per_s": evals / dt,
        "host": host_cpu(),
    }


def u8_scan_kernels(cfg):
    """The launches that make up one round's uint8 matrix-core scan (the library's rule: by R and N)."""
    ks = cfg.d // 32
    if cfg.R <= 32:
        return "k_update_scan_mfma_u8_small<%d> (one launch per round)" % ks
    if cfg.N <= 524288:
        return "k_update_scan_mfma_u8_all<%d,NC> (one launch per round for all degree classes)" % ks
    if cfg.R <= 64 or cfg.N > 2097152:
        return ("k_update_scan_mfma_u8_small<%d> + k_update_scan_mfma_u8<NG,%d>, NG = 2 .. %d (one round's scan launches, back "
                "to back)" % (ks, ks, (cfg.R + 31) // 32))
    return ("k_update_scan_mfma_u8_small<%d> + k_update_scan_mfma_u8_all<%d,NC,3> (one round's scan launches: lists of at "
            "most 32 entries, then the longer classes; back to back)" % (ks, ks))


def exact_top10(Xd, Qd):
    """Exact 10 nearest neighbours of every query (ties by id): test tooling, a double-precision matmul on
    the GPU in chunks whose distance matrix stays below 16 GB."""
    import numpy as np
    import torch
    Xf = Xd.double()
    xn = (Xf * Xf).sum(1)
    nq = Qd.shape[0]
    out = np.zeros((nq, 10), np.int64)
    step = max(1, min(500, int(2e9 // Xd.shape[0])))
    for q0 in range(0, nq, step):
        Qf = Qd[q0:q0 + step].double()
        d2 = (Qf * Qf).sum(1)[:, None] + xn[None, :] - 2.0 * (Qf @ Xf.T)
        cand = torch.topk(d2, 32, dim=1, largest=False)
        cv, ci = cand.values.cpu().numpy(), cand.indices.cpu().numpy()
        for q in range(cv.shape[0]):
            out[q0 + q] = ci[q][np.lexsort((ci[q], cv[q]))][:10]
    return out


def search_quality(cfg, rn, Xd, graph, degree, nq, L=64, K=32, sweep=False):
    """Search on the graph just built, by the library's own GPU search (Alg. 1 with the cap K): queries per
    second, recall@10 and R@1 against the exact neighbours.  sweep: also the grid of L and K of Sec. 5.4 (Eq. 4 is in Sec. 4.4)."""
    import time
    import numpy as np
    import torch
    import workloads as wl
    Q = wl.make_queries(cfg, nq)
    Qd = torch.from_numpy(Q).cuda().to(Xd.dtype).contiguous()
    truth = exact_top10(Xd, Qd)

    def one(L, K):
        rn.rnnd_search(Xd, graph, degree, Qd[:64].contiguous(), L, K, min(10, L), 7)      # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ids, _, evals = rn.rnnd_search(Xd, graph, degree, Qd, L, K, min(10, L), 7)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        got = ids.cpu().numpy()
        hit = sum(len(set(truth[q].tolist()) & set(got[q].tolist())) for q in range(nq))
        return {"queries": nq, "L": L, "K": K, "k": min(10, L), "seconds": dt, "queries_per_s": nq / dt,
                "recall_at_10": hit / (10.0 * nq), "r_at_1": float((got[:, 0] == truth[:, 0]).mean()),
                "distance_evals_per_query": evals / nq}

    res = one(L, K)
    if sweep:
        res["sweep"] = [one(l, k) for l in (16, 32, 64, 128) for k in (16, 32, 48, 64, 96, 128)]
    return res


def load_workload(cfg, storage):
    """(host array the oracle would see, device tensor as the library gets it, element size, 16-bit storage or None)."""
    import numpy as np
    import torch
    import workloads as wl
    X = wl.make_data(cfg)
    half = storage in ("f16", "bf16") and cfg.dtype != "u8"
    st16 = storage if half else None
    if st16 == "f16":
        X = X.astype(np.float16)
        Xd = torch.from_numpy(X).cuda()
    elif st16 == "bf16":
        Xb = torch.from_numpy(X).to(torch.bfloat16)      # round to nearest even
        X = Xb.float().numpy()                             # the floats the stored numbers stand for (host side)
        Xd = Xb.cuda()
    else:
        Xd = torch.from_numpy(X).cuda()
    torch.cuda.synchronize()
    return X, Xd, (1 if cfg.dtype == "u8" else 2 if half else 4), st16


def measure(rn, cfg, X, Xd, esz, st16, steps, warmup, args, with_search=True, with_ceiling=True):
    """`warmup` untimed and `steps` timed complete builds of one workload; everything the line reports about it."""
    import torch
    import workloads as wl
    half = st16 is not None

    def step():
        if args.merge_cap:
            return rn.rnnd_build_wide(Xd, cfg.S, cfg.R, args.merge_cap, cfg.T1, cfg.T2, wl.BUILD_SEED, want_keys=False)
        if args.blocks:
            return rn.rnnd_build_blocks(Xd, cfg.S, cfg.R, cfg.T1, cfg.T2, wl.BUILD_SEED, args.blocks, want_keys=False)
        return rn.rnnd_build_ex(Xd, cfg.S, cfg.R, cfg.T1, cfg.T2, wl.BUILD_SEED, want_keys=False)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph, degree, _, st = step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1000.0 * wall / steps

    s = st.as_dict()
    rounds = s["rounds"]
    algo = s["init_evals"] + sum(s["algo_evals"])
    execd = s["init_evals"] + sum(s["exec_evals"])
    # The timed builds take their per-round times from the device's own clock (free: a build with statistics is as
    # fast as one without).  The roofline's launch duration comes from HIP events attached to the scan launches on
    # the build's stream, in extra builds right after the timed ones: such an event holds the queue for 4-7
    # microseconds after its kernel, three per round, which would add about 1 ms to each timed cfg3 build.
    scan_ms_clock = sum(s["scan_ms"])
    scan_ms_events = None
    if args.event_steps > 0 and not args.blocks:
        rn.rnnd_set_event_timing(True)
        try:
            for _ in range(args.event_steps):
                _, _, _, st_ev = step()
            scan_ms_events = sum(st_ev.as_dict()["scan_ms"])
        finally:
            rn.rnnd_set_event_timing(False)
    # dominant kernel: the UpdateNeighbors scan (the class launches of one round taken together).
    # Algorithmic bytes of one launch = rows of X it must gather (d*esz each) + the list entries it reads
    # (8 B) and writes back (8 B) + the redirected edges it emits (16 B); summed over the T1*T2 launches of
    # the last timed build, durations by HIP events on the build's stream.
    scan_bytes = sum(g * (cfg.d * esz + 16) + 16 * p for g, p in zip(s["gathered_rows"], s["proposals"]))
    scan_ms = scan_ms_events if scan_ms_events else scan_ms_clock
    hbm_gbs = scan_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    kv = s["kernel_variant"]
    kname = {1: "k_update_scan",
             2: u8_scan_kernels(cfg),
             3: "k_update_scan_mfma_f32<NG,CH,NRC,fast> (one launch per degree class, back to back per round; "
                "%s MFMA Gram tiles, undecided pairs by exact distances)" % (st16 if half else "fp32")}[kv]
    traffic = None if half or args.merge_cap or args.blocks else TRAFFIC_PER_LAUNCH.get((cfg.name, kv))
    if kv == 3:
        # float rows: the Gram tiles run on the fp32 matrix cores (157.3 TFLOP/s dense; 16-bit rows: on the
        # f16 ones, 2,500 TFLOP/s), the rows are gathered from HBM; the kernel is reported against whichever
        # of the two it sits closer to, with both fractions in the line.  executed flops = computed pair
        # distances * 2 d
        mfma_peak = 2500.0 if half else 157.3
        flops = sum(s["exec_evals"]) * 2.0 * cfg.d
        tflops = flops / (scan_ms * 1e-3) / 1e12 if scan_ms > 0 else 0.0
        extra = {"launches": rounds, "avg_launch_ms": scan_ms / max(1, rounds),
                 "flops_per_launch": flops / max(1, rounds), "mfma_TFLOPs": tflops, "mfma_peak_TFLOPs": mfma_peak,
                 "mfma_frac": tflops / mfma_peak, "hbm_algorithmic_GBps": hbm_gbs,
                 "hbm_frac": hbm_gbs / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": scan_bytes / max(1, rounds)}
        if hbm_gbs / HBM_PEAK_GBS >= tflops / mfma_peak:
            roof = dict({"bound": "hbm", "kernel": kname, "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": hbm_gbs / HBM_PEAK_GBS, "traffic": traffic}, **extra)
        else:
            roof = dict({"bound": "mfma", "kernel": kname, "achieved": tflops, "peak": mfma_peak, "unit": "TFLOP/s",
                         "frac": tflops / mfma_peak, "traffic": None}, **extra)
    else:
        roof = {"bound": "hbm", "kernel": kname, "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": hbm_gbs / HBM_PEAK_GBS, "traffic": traffic,
                "launches": rounds, "avg_launch_ms": scan_ms / max(1, rounds),
                "algorithmic_bytes_per_launch": scan_bytes / max(1, rounds)}
    roof["launch_timing"] = ("HIP events attached to the first and last scan launch of every round, %d extra build(s) after "
                             "the timed ones" % args.event_steps) if scan_ms_events else "device clock, the timed builds"
    roof["avg_launch_ms_device_clock"] = scan_ms_clock / max(1, rounds)    # over the timed builds (last one)
    if traffic:
        roof["traffic_over_algorithmic"] = traffic / (scan_bytes / max(1, rounds))
    if with_ceiling:
        # what a kernel that only gathers random whole rows of X reaches on this GPU (same access pattern)
        ceiling = rn.rnnd_probe_gather(Xd, max(1, int(8e9 // (cfg.d * esz))))
        roof["gather_ceiling_GBps"] = ceiling
        roof["frac_of_gather_ceiling"] = (hbm_gbs / ceiling) if ceiling > 0 else None
    if args.blocks:      # the scan launches of a run are not timed one by one
        roof = dict(roof, achieved=None, frac=None, avg_launch_ms=None, traffic=None,
                    note="per-launch scan times are measured for the synchronous build only")
    out = {
        "value": ms_per_step / 1000.0, "unit": "s", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "dtype": "u8" if cfg.dtype == "u8" else "f32",
        "storage": st16 if half else cfg.dtype,
        "arithmetic": ("uint8 rows, int8 MFMA Gram tiles, exact int32 distances" if cfg.dtype == "u8" else
                       "%s rows; decisions from %s MFMA Gram tiles with an error bound, exact f64-accumulated distances "
                       "for undecided pairs and for every stored distance (rounded once to float32)"
                       % (({"f16": "float16", "bf16": "bfloat16"}[st16], st16) if half else ("float32", "fp32"))),
        "config": {"workload": "%s: N=%d d=%d %s, S=%d R=%d T1=%d T2=%d, seeded %s mixture"
                               % (cfg.name, cfg.N, cfg.d, cfg.dtype, cfg.S, cfg.R, cfg.T1, cfg.T2, cfg.kind),
                   "kernel_variant": args.variant,
                   "update_order": ("block-sequential, %d runs per pass" % args.blocks) if args.blocks
                   else "synchronous rounds",
                   "row_width": args.merge_cap or cfg.R},
        "distance_evals_per_s": algo / (ms_per_step * 1e-3),
        "executed_distance_evals_per_s": execd / (ms_per_step * 1e-3),
        "algorithmic_distance_evals": algo, "executed_distance_evals": execd,
        "gpu_ms": {"total": s["total_ms"], "init": s["init_ms"], "rounds": sum(s["round_ms"]),
                   "scan": scan_ms_clock, "reverse": sum(s["reverse_ms"])},      # of the last timed build
        "mean_degree": float(degree.float().mean().item()), "max_degree": int(degree.max().item()),
        # list entries the merges dropped because a row was full (the paper's UpdateNeighbors never drops one)
        "dropped_entries": int(sum(s["dropped"])),
        # out-degrees 0, 1-8, 9-16, 17-32, 33-64, 65-96, 97-128
        "degree_histogram": torch.histc(degree.float(), bins=1, min=-0.5, max=0.5).int().tolist()
        + [int(((degree > lo) & (degree <= hi)).sum().item()) for lo, hi in
           ((0, 8), (8, 16), (16, 32), (32, 64), (64, 96), (96, 128))],
        "data_stats": dict(wl.describe(X), sha256=wl.sha256_of(X)[:16]),
        "roofline": roof,
    }
    if with_search:
        try:
            sq = search_quality(cfg, rn, Xd, graph, degree, min(cfg.n_queries, args.queries), sweep=args.search_sweep)
            out["recall_at_10"] = sq["recall_at_10"]
            out["search"] = sq
        except Exception as e:  # reporting only; never hides the build measurement
            out["recall_at_10"] = None
            out["recall_error"] = repr(e)
    return out, algo


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--also", default="auto",
                    help="comma-separated further workloads measured with fewer steps and reported under "
                         "\"workloads\" (auto: cfg1,cfg2,cfg4,cfg5 next to the default cfg3, none otherwise; 'none')")
    ap.add_argument("--event-steps", type=int, default=1,
                    help="extra builds after the timed ones whose scan launches carry HIP events (roofline's launch duration); "
                         "0: take it from the device clock of the timed builds")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-recall", action="store_true")
    ap.add_argument("--queries", type=int, default=10000, help="queries of the search-quality leg (at most the config's)")
    ap.add_argument("--variant", type=int, default=0, help="UpdateNeighbors kernel: 0 auto, 1 generic, 2 auto with the float scan in double precision")
    ap.add_argument("--cpu-sample", type=int, default=0, help="rows of the oracle's timed sample (default: about 20 s of work)")
    ap.add_argument("--cpu-full", action="store_true", help="time the oracle on the full workload (minutes)")
    ap.add_argument("--n", type=int, default=0, help="override the workload's N (same generator; scale checks)")
    ap.add_argument("--storage", choices=["native", "f16", "bf16"], default="native",
                    help="f16 / bf16: float workloads are stored as IEEE half precision (RNND_F16) or bfloat16 "
                         "(RNND_BF16); the graph is the one of the rounded data")
    ap.add_argument("--search-sweep", action="store_true",
                    help="search-quality leg over L in {16,32,64,128} x K in {16,...,96, no cap} (Sec. 5.4)")
    ap.add_argument("--merge-cap", type=int, default=0,
                    help="rows this many slots wide (R <= M <= 128): UpdateNeighbors merges cut to M, only "
                         "AddReverseEdges cuts to R (rnnd_build_wide); 0 = fixed-width rows, the build the metric "
                         "is quoted on")
    ap.add_argument("--blocks", type=int, default=0,
                    help="block-sequential passes with this many runs of consecutive ids per pass "
                         "(rnnd_build_blocks; 0 = the synchronous build the metric is quoted on)")
    ap.add_argument("--gather-maps", action="store_true",
                    help="instead of a build: the rate of random whole-row gathers from a matrix of the workload's shape "
                         "(random bytes; --n overrides the rows) for 1, 2, 4 and 8 lanes per row, one JSON line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (scale for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not "
                 "supported, run with --gpus 1" % args.gpus)

    import torch
    import workloads as wl
    import paper_2310_20419_amd as rn

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the hot path has no CPU fallback")
    rn.load_library()
    rn.rnnd_set_kernel_variant(args.variant)
    cfg = wl.CONFIGS[args.workload]
    if args.n:
        import dataclasses
        cfg = dataclasses.replace(cfg, N=args.n, name="%s_n%d" % (cfg.name, args.n))
    if args.gather_maps:
        # which lane -> address map gathers rows fastest (the operand layout of a matrix instruction fixes it)
        row_bytes = cfg.d * (1 if cfg.dtype == "u8" else 4)
        M = torch.empty((cfg.N, row_bytes), dtype=torch.uint8, device="cuda").random_()
        n_gather = max(1, int(8e9 // row_bytes))
        rates = {}
        for lanes in (1, 2, 4, 8):
            if (row_bytes // 16) % lanes == 0 and (row_bytes // 16) // lanes in (1, 2, 4, 8):
                rates[str(lanes)] = max(rn.rnnd_probe_gather_map(M, n_gather, lanes, seed=s) for s in (1, 2, 3))
        print(json.dumps({"mode": "gather-maps", "rows": cfg.N, "row_bytes": row_bytes, "matrix_GB": cfg.N * row_bytes / 1e9,
                          "rows_gathered": n_gather, "GBps_by_lanes_per_row": rates}))
        return
    t0 = time.perf_counter()
    X, Xd, esz, st16 = load_workload(cfg, args.storage)
    gen_s = time.perf_counter() - t0

    if args.copy_calibration:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        a.fill_(3)
        torch.cuda.synchronize()
        b.copy_(a)          # the calibration kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    head, algo = measure(rn, cfg, X, Xd, esz, st16, args.steps, args.warmup, args, with_search=not args.no_recall)
    out = {"metric": "1M-vector graph build time" if cfg.N == 1_000_000 else "graph build time",
           "value": head["value"], "unit": "s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head["ms_per_step"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
           "dtype": head["dtype"], "data": "synthetic"}
    out.update({k: v for k, v in head.items() if k not in out})
    out["data_gen_s"] = gen_s
    if not args.no_cpu_baseline:
        n_s = cfg.N if args.cpu_full else (args.cpu_sample or min(cfg.N, 250_000 if cfg.d <= 128 else 20_000))
        out["cpu_baseline"] = cpu_baseline(cfg, X, n_s, algo)
    # the other 1M configurations of the metric (float rows), fewer steps, same measurement
    also = args.also
    if also == "auto":
        also = "cfg1,cfg2,cfg4,cfg5" if (args.workload == "cfg3" and not (args.n or args.merge_cap or args.blocks)) else "none"
    names = [w for w in also.split(",") if w and w != "none" and w != args.workload]
    if names:
        del X, Xd
        rn.rnnd_release_workspace()
        torch.cuda.empty_cache()
        out["workloads"] = {}
        for name in names:
            c2 = wl.CONFIGS[name]
            t0 = time.perf_counter()
            X2, Xd2, esz2, st2 = load_workload(c2, args.storage)
            g2 = time.perf_counter() - t0
            # the small configurations build in milliseconds: the same number of steps; the 1M float ones: two
            k2 = args.steps if c2.N < 1_000_000 else max(1, min(args.steps, 2))
            sub, _ = measure(rn, c2, X2, Xd2, esz2, st2, k2, 1 if c2.N >= 1_000_000 else max(1, args.warmup), args,
                             with_search=not args.no_recall)
            sub["data_gen_s"] = g2
            sub["metric"] = "1M-vector graph build time" if c2.N == 1_000_000 else "graph build time"
            out["workloads"][name] = sub
            del X2, Xd2
            rn.rnnd_release_workspace()
            torch.cuda.empty_cache()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
