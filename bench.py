#!/usr/bin/env python3
"""Benchmark of the LDA Gibbs sweep on one MI355X (default), and with --workload gmm of the
Gaussian-mixture sweep.

A step is one whole sweep (sample_z, count_accumulate, resample theta, resample phi) over a
synthetic corpus that is already resident in HBM.  Prints ONE JSON line: whole-sweep tokens/s,
the HBM-roofline figures of the dominant kernel (sample_z) from HIP events recorded on the
library's stream inside the timed region, and the oracle's throughput on this machine's host cores
(bounded sample) as cpu_baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per sample_z launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by
# the factors a plain 1 GiB copy shows for the same counters (reads x 2.0, writes x 1.0); the
# runs and figures are in profiles/lda_large_and_medium_kernel_trace_and_hbm_traffic.md.  None for workloads
# that have not been measured.
MEASURED_TRAFFIC_BYTES = {"large": (7_112_850 * 2.0 + 1_503_585 * 1.0) * 1024,
                          "medium": (75_375 * 2.0 + 26_395 * 1.0) * 1024,
                          "widek": (6_892_705 * 2.0 + 159_196 * 1.0) * 1024}


def sample_z_algorithmic_bytes(N, D, K):
    """Per launch: every token reads its word id, its phi row and writes z; every document reads
    its theta row and its two offsets and (K <= 256, where the kernel also builds the document
    count table and the byte copy of z for the word table) writes its row of n_dk and a byte a
    token."""
    return N * (8 + 4 * K) + D * (4 * K + 8) + (D * 4 * K + N if K <= 256 else 0)


def cpu_baseline(cfg, corpus, budget_s=20.0):
    """Oracle sweeps on a bounded sample of the same corpus (its first documents, full
    vocabulary), single thread."""
    import numpy as np
    from oracle import oracle as O
    target_tokens = 1_500_000 if cfg["K"] <= 256 else 300_000
    doc_len = corpus["doc_len"]
    cum = np.cumsum(doc_len.astype(np.int64))
    nd = int(min(len(doc_len), np.searchsorted(cum, target_tokens) + 1))
    ntok = int(cum[nd - 1])
    o = O.OracleLDA(nd, cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], cfg["seed"], doc_len[:nd],
                    corpus["w"][:ntok])
    sweeps, t0 = 0, time.perf_counter()
    while True:
        o.sweep(1)
        sweeps += 1
        el = time.perf_counter() - t0
        if sweeps >= 2 and (el > budget_s / 2 or sweeps >= 5):
            break
    return {"value": ntok * sweeps / el, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"first {nd} documents ({ntok} tokens) of the same corpus, full V={cfg['V']} "
                      f"and K={cfg['K']}, {sweeps} whole sweeps, single thread of {os.cpu_count()} visible"}


FP64_VECTOR_PEAK_TFLOPS = 78.6  # MI355X published fp64 vector peak


def gmm_z_flops(N, dim, K):
    """Floating-point operations the z step of the mixture needs per launch, counted on the
    formulas: per (point, component) dim subtractions and dim multiply-adds (2 dim) for the
    distance plus 2 for the log-weight, one exponential counted as 1, and 2 for the running sums;
    (3 dim + 5) K per point.  What the exponential really costs in instructions is not counted."""
    return N * K * (3 * dim + 5)


def bench_gmm(args, unknown_var):
    """One step = one sweep of the Gaussian mixture (z, statistics, weights, means[, variances])
    over the BASELINE configuration's point cloud, resident in HBM."""
    import numpy as np
    import torch
    from paper_1312_3613_amd import binding as B, synth
    cfg = synth.GMM_CONFIG
    steps = args.steps if args.steps is not None else cfg["sweeps"]
    t0 = time.perf_counter()
    d = synth.gmm_points(**cfg)
    t_gen = time.perf_counter() - t0
    N, dim, K = cfg["N"], cfg["dim"], cfg["K"]
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    x = torch.as_tensor(d["x"]).cuda()
    torch.cuda.synchronize()
    kw = dict(var_shape=1.0, var_scale=1.0) if unknown_var else {}
    h = B.GMM(K, cfg["alpha"], cfg["prior_sd"], cfg["sigma"], cfg["seed"], x, stream=stream,
              device_ptrs=True, **kw)
    h.sweep(args.warmup)
    h.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms = h.sweep_profile(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    lj = h.loglik()
    h.close()
    t_z = ms["sample_z"] / steps * 1e-3
    flops = gmm_z_flops(N, dim, K)
    achieved = flops / t_z / 1e12
    out = {
        "metric": "Gibbs sweep points/sec (Gaussian mixture N=1e6, R^8, K=16)",
        "value": N * steps / elapsed, "unit": "points/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": elapsed / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"GMM: N={N} dim={dim} K={K} alpha={cfg['alpha']} prior_sd={cfg['prior_sd']} "
                               + ("variances unknown, InverseGamma(1,1)" if unknown_var else f"sigma={cfg['sigma']}")
                               + f", points from the mixture's generative process (seed {cfg['seed']}), resident in HBM"},
        "roofline": {"bound": "alu", "kernel": "gmm_sample_z", "achieved": achieved,
                     "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / FP64_VECTOR_PEAK_TFLOPS, "traffic": None,
                     "algorithmic_flops_per_launch": flops, "avg_launch_ms": t_z * 1e3},
        "kernel_ms_per_sweep": {k: v / steps for k, v in ms.items()},
        "log_joint_per_point": lj / N,
        "setup_s": {"generate_points": t_gen},
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        n = 200_000
        xs = d["x"][:n]
        o = (O.OracleGMMUV(K, cfg["alpha"], cfg["prior_sd"], 1.0, 1.0, cfg["seed"], xs) if unknown_var
             else O.OracleGMM(K, cfg["alpha"], cfg["prior_sd"], cfg["sigma"], cfg["seed"], xs))
        sweeps, t0 = 0, time.perf_counter()
        while True:
            o.sweep(1)
            sweeps += 1
            el = time.perf_counter() - t0
            if sweeps >= 2 and (el > 10.0 or sweeps >= 20):
                break
        out["cpu_baseline"] = {"value": n * sweeps / el, "unit": "points/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {n} points of the same cloud, {sweeps} whole sweeps, "
                                         f"single thread of {os.cpu_count()} visible"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="large",
                    choices=["tiny", "medium", "large", "widek", "paper_shape", "gmm", "gmm_unknown_variance"])
    ap.add_argument("--topics", type=int, default=None,
                    help="infer with this many topics instead of the number the corpus was drawn with")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="build the word-count table on the main stream instead of beside the theta step")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a reference of known "
                         "size for scaling rocprofv3's FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    if args.workload.startswith("gmm"):
        bench_gmm(args, args.workload == "gmm_unknown_variance")
        return

    import numpy as np
    import torch
    from paper_1312_3613_amd import binding as B, synth

    cfg = synth.LDA_CONFIGS[args.workload]
    steps = args.steps if args.steps is not None else cfg["sweeps"]
    t0 = time.perf_counter()
    corpus = synth.lda_corpus(**cfg)
    t_gen = time.perf_counter() - t0
    if args.topics is not None:
        cfg = dict(cfg, K=args.topics)
    N, D, V, K = corpus["N"], cfg["D"], cfg["V"], cfg["K"]

    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    doc_len_d = torch.as_tensor(corpus["doc_len"]).cuda()
    w_d = torch.as_tensor(corpus["w"]).cuda()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    h = B.LDA(D, V, K, cfg["alpha"], cfg["beta"], cfg["seed"], doc_len_d, w_d, stream=stream,
              device_ptrs=True)
    t_create = time.perf_counter() - t0
    if args.no_overlap:
        h.set_overlap(False)

    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        src.fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)          # the probe: reads and writes copy_probe_mib MiB
        torch.cuda.synchronize()
        del src, dst

    h.sweep(args.warmup)
    h.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms = h.sweep_profile(steps)  # the timed region; HIP events on the library's stream inside
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    lj, lm = h.loglik()
    degenerate = h.get_degenerate()
    h.close()

    t_z = ms["sample_z"] / steps * 1e-3
    bytes_z = sample_z_algorithmic_bytes(N, D, K)
    achieved = bytes_z / t_z / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload)
    out = {
        "metric": "Gibbs sweep tokens/sec (LDA K=100/200) + achieved HBM GB/s vs peak",
        "value": N * steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"LDA {args.workload}: D={D} V={V} K={K} N={N} alpha={cfg['alpha']} "
                               f"beta={cfg['beta']}, corpus from the LDA generative process "
                               f"(seed {cfg['seed']}), inputs resident in HBM"},
        "roofline": {"bound": "hbm", "kernel": "lda_sample_z", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "algorithmic_bytes_per_launch": bytes_z,
                     "avg_launch_ms": t_z * 1e3,
                     # the measured traffic over the same launch time: what actually passes the L2
                     # (the phi-row gathers are served by L1/L2 three times out of four)
                     "traffic_GBs": None if traffic is None else traffic / t_z / 1e9,
                     "traffic_frac": None if traffic is None else traffic / t_z / 1e9 / HBM_PEAK_GBS},
        "kernel_ms_per_sweep": {k: v / steps for k, v in ms.items()},
        "overlap_word_counts_with_theta": not args.no_overlap,
        "log_marginal_per_token": lm / max(N, 1),
        "degenerate_tokens": degenerate,
        "setup_s": {"generate_corpus": t_gen, "create": t_create},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, corpus)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
