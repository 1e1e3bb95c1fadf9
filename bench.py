#!/usr/bin/env python3
"""Benchmark of the RNN-Descent build hot path on one MI355X.

A "step" is one complete rnnd_build (RandomGraph + T1*T2 UpdateNeighbors rounds + T1-1
AddReverseEdges) over one synthetic database that is already resident in HBM.  The default
workload is cfg3 of workloads.py (N = 1,000,000, d = 128, uint8, S=20 R=96 T1=4 T2=15), the
one the "1M-vector graph build time" metric is quoted on.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-cpu-baseline]
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

# HBM bytes per scan launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs, scaled by
# a plain 1 GiB copy in the same run); see profiles/update_scan_cfg3_hbm_traffic.txt and
# profiles/update_scan_cfg5_hbm_traffic.txt.  Keyed by (workload, kernel variant); None where it has
# not been measured.
TRAFFIC_PER_LAUNCH = {("cfg3", 2): 1.022e9, ("cfg5", 3): 8.337e10}


def cpu_baseline(cfg, X, sample_n):
    """The oracle as it stands, single-threaded, on the first sample_n rows (same S, R, T1, T2)."""
    import oracle
    oracle.build()
    Xs = X[:sample_n].copy()
    if Xs.dtype.itemsize == 2:      # half-precision storage: the oracle works on the floats the halves stand for
        Xs = Xs.astype("float32")
    t0 = time.perf_counter()
    res = oracle.build_sync(Xs, cfg.S, cfg.R, cfg.T1, cfg.T2, 2310)
    dt = time.perf_counter() - t0
    evals = int(res.init_evals + res.round_evals.sum())
    return {
        "value": dt * (cfg.N / sample_n), "unit": "s", "cores": 1, "kind": "oracle",
        "sample": "oracle build on the first %d rows of the same workload (same S,R,T1,T2): %.2f s, "
                  "%d distance evaluations; value = that time scaled by N/%d"
                  % (sample_n, dt, evals, sample_n),
        "sample_seconds": dt, "distance_evals_per_s": evals / dt,
    }


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-recall", action="store_true")
    ap.add_argument("--queries", type=int, default=10000, help="queries of the search-quality leg (at most the config's)")
    ap.add_argument("--variant", type=int, default=0, help="UpdateNeighbors kernel: 0 auto, 1 generic, 2 auto with the float scan in double precision")
    ap.add_argument("--cpu-sample", type=int, default=0)
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
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (scale for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not "
                 "supported, run with --gpus 1" % args.gpus)

    import numpy as np
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
    t0 = time.perf_counter()
    X = wl.make_data(cfg)
    gen_s = time.perf_counter() - t0
    half = args.storage in ("f16", "bf16") and cfg.dtype != "u8"
    st16 = args.storage if half else None
    if st16 == "f16":
        X = X.astype(np.float16)
        Xd = torch.from_numpy(X).cuda()
    elif st16 == "bf16":
        Xb = torch.from_numpy(X).to(torch.bfloat16)      # round to nearest even
        X = Xb.float().numpy()                             # the floats the stored numbers stand for (host side)
        Xd = Xb.cuda()
    else:
        Xd = torch.from_numpy(X).cuda()
    esz = 1 if cfg.dtype == "u8" else 2 if half else 4
    torch.cuda.synchronize()

    if args.copy_calibration:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        a.fill_(3)
        torch.cuda.synchronize()
        b.copy_(a)          # the calibration kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    def step():
        if args.merge_cap:
            return rn.rnnd_build_wide(Xd, cfg.S, cfg.R, args.merge_cap, cfg.T1, cfg.T2, wl.BUILD_SEED, want_keys=False)
        if args.blocks:
            return rn.rnnd_build_blocks(Xd, cfg.S, cfg.R, cfg.T1, cfg.T2, wl.BUILD_SEED, args.blocks, want_keys=False)
        return rn.rnnd_build_ex(Xd, cfg.S, cfg.R, cfg.T1, cfg.T2, wl.BUILD_SEED, want_keys=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph, degree, _, st = step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1000.0 * wall / args.steps

    s = st.as_dict()
    rounds = s["rounds"]
    algo = s["init_evals"] + sum(s["algo_evals"])
    execd = s["init_evals"] + sum(s["exec_evals"])
    # dominant kernel: the UpdateNeighbors scan (the class launches of one round taken together).
    # Algorithmic bytes of one launch = rows of X it must gather (d*esz each) + the list entries it reads
    # (8 B) and writes back (8 B) + the redirected edges it emits (16 B); summed over the T1*T2 launches of
    # the last timed build, durations by HIP events on the build's stream.
    scan_bytes = sum(g * (cfg.d * esz + 16) + 16 * p for g, p in zip(s["gathered_rows"], s["proposals"]))
    scan_ms = sum(s["scan_ms"])
    hbm_gbs = scan_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    kv = s["kernel_variant"]
    kname = {1: "k_update_scan",
             2: "k_update_scan_mfma_u8_small<%d> + k_update_scan_mfma_u8<NG,%d>, NG = 2,3 (one round's scan launches, "
                "back to back)" % (cfg.d // 32, cfg.d // 32),
             3: "k_update_scan_mfma_f32<NG,CH,NRC,fast> (one launch per degree class, back to back per round; "
                "%s MFMA Gram tiles, undecided pairs by exact distances)" % (st16 if half else "fp32")}[kv]
    if kv == 3:
        # float rows: the Gram tiles run on the fp32 matrix cores (157.3 TFLOP/s dense; 16-bit rows: on the
        # f16 ones, 2,500 TFLOP/s), the rows are gathered from HBM; the kernel is reported against whichever
        # of the two it sits closer to.  executed flops = computed pair distances * 2 d
        mfma_peak = 2500.0 if half else 157.3
        flops = sum(s["exec_evals"]) * 2.0 * cfg.d
        tflops = flops / (scan_ms * 1e-3) / 1e12 if scan_ms > 0 else 0.0
        extra = {"launches": rounds, "avg_launch_ms": scan_ms / max(1, rounds),
                 "flops_per_launch": flops / max(1, rounds), "mfma_TFLOPs": tflops, "mfma_peak_TFLOPs": mfma_peak,
                 "mfma_frac": tflops / mfma_peak, "hbm_algorithmic_GBps": hbm_gbs,
                 "hbm_frac": hbm_gbs / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": scan_bytes / max(1, rounds)}
        if hbm_gbs / HBM_PEAK_GBS >= tflops / mfma_peak:
            roof = dict({"bound": "hbm", "kernel": kname, "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": hbm_gbs / HBM_PEAK_GBS,
                         "traffic": None if half else TRAFFIC_PER_LAUNCH.get((cfg.name, kv))}, **extra)
        else:
            roof = dict({"bound": "mfma", "kernel": kname, "achieved": tflops, "peak": mfma_peak, "unit": "TFLOP/s",
                         "frac": tflops / mfma_peak, "traffic": None}, **extra)
    else:
        roof = {"bound": "hbm", "kernel": kname, "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": hbm_gbs / HBM_PEAK_GBS, "traffic": TRAFFIC_PER_LAUNCH.get((cfg.name, kv)),
                "launches": rounds, "avg_launch_ms": scan_ms / max(1, rounds),
                "algorithmic_bytes_per_launch": scan_bytes / max(1, rounds)}
    # what a kernel that only gathers random whole rows of X reaches on this GPU (same access pattern)
    ceiling = rn.rnnd_probe_gather(Xd, max(1, int(8e9 // (cfg.d * esz))))
    roof["gather_ceiling_GBps"] = ceiling
    roof["frac_of_gather_ceiling"] = (hbm_gbs / ceiling) if ceiling > 0 else None
    if args.blocks:      # the scan launches of a run are not timed one by one
        roof = dict(roof, achieved=None, frac=None, avg_launch_ms=None, traffic=None,
                    note="per-launch scan times are measured for the synchronous build only")
    out = {
        "metric": "1M-vector graph build time" if cfg.N == 1_000_000 else "graph build time",
        "value": ms_per_step / 1000.0, "unit": "s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8" if cfg.dtype == "u8" else "f32",
        "storage": st16 if half else cfg.dtype,
        "arithmetic": ("uint8 rows, int8 MFMA Gram tiles, exact int32 distances" if cfg.dtype == "u8" else
                       "%s rows; decisions from %s MFMA Gram tiles with an error bound, exact f64-accumulated distances "
                       "for undecided pairs and for every stored distance (rounded once to float32)"
                       % (({"f16": "float16", "bf16": "bfloat16"}[st16], st16) if half else ("float32", "fp32"))),
        "data": "synthetic",
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
                   "scan": scan_ms, "reverse": sum(s["reverse_ms"])},
        "mean_degree": float(degree.float().mean().item()), "max_degree": int(degree.max().item()),
        # out-degrees 0, 1-8, 9-16, 17-32, 33-64, 65-96, 97-128
        "degree_histogram": torch.histc(degree.float(), bins=1, min=-0.5, max=0.5).int().tolist()
        + [int(((degree > lo) & (degree <= hi)).sum().item()) for lo, hi in
           ((0, 8), (8, 16), (16, 32), (32, 64), (64, 96), (96, 128))],
        "data_stats": dict(wl.describe(X), sha256=wl.sha256_of(X)[:16]),
        "roofline": roof,
        "data_gen_s": gen_s,
    }
    if not args.no_recall:
        try:
            sq = search_quality(cfg, rn, Xd, graph, degree, min(cfg.n_queries, args.queries), sweep=args.search_sweep)
            out["recall_at_10"] = sq["recall_at_10"]
            out["search"] = sq
        except Exception as e:  # reporting only; never hides the build measurement
            out["recall_at_10"] = None
            out["recall_error"] = repr(e)
    if not args.no_cpu_baseline:
        n_s = args.cpu_sample or min(cfg.N, 200_000 if cfg.d <= 128 else 20_000)
        out["cpu_baseline"] = cpu_baseline(cfg, X, n_s)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
