#!/usr/bin/env python3
"""Benchmark of the LDA Gibbs sweep on one MI355X (default), and with --workload gmm of the
Gaussian-mixture sweep.

A step is one whole sweep (sample_z, count_accumulate, resample theta, resample phi) over a
synthetic corpus that is already resident in HBM.  Prints ONE JSON line.  For the default
workload (LDA large, K = 200) it holds

  value / ms_per_step   whole-sweep tokens/s: W warm-up sweeps, then `--repeats` timed
                        regions of exactly K sweeps each; the median region is reported
  roofline              the dominant kernel (sample_z): algorithmic bytes per launch over the
                        launch time from HIP events on the library's stream inside the timed
                        region, against the 8 TB/s HBM peak, with the HBM traffic that
                        rocprofv3 counted for the same launch (profiles/hbm_traffic.json)
  z_plus_count          sample_z and count_accumulate alone (no overlap with the Gamma steps),
                        the pair the 60 % target is stated for
  ceilings              what the memory system allows, measured in this run: a plain
                        streaming copy and a gather-only pass over the same word stream and phi
                        table; plus the instruction counters of the profiled launch
  state_f64             the sweep with theta and phi held in fp64, beside the fp32 figure
  k100                  the same figures for the K = 100 workload (LDA medium)
  cpu_baseline          the oracle on one pinned host core, per step on a bounded sample,
                        composed to the full corpus
"""
import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def sample_z_algorithmic_bytes(N, D, K):
    """Per launch: every token reads its word id, its phi row and writes z; every document reads
    its theta row and its two offsets and (K <= 256, where the kernel also builds the document
    count table and the byte copy of z for the word table) writes its row of n_dk and a byte a
    token."""
    return N * (8 + 4 * K) + D * (4 * K + 8) + (D * 4 * K + N if K <= 256 else 0)


def count_algorithmic_bytes(N, D, V, K):
    """The part of count_accumulate that is not inside the z kernel: the word table reads one
    permutation index (4 bytes) and one topic (1 byte from the byte copy when K <= 256, else 4)
    per token and writes its V x K table; above 256 topics the document table is a kernel of its
    own that reads z and writes D x K."""
    words = N * (4 + (1 if K <= 256 else 4)) + 4 * V * K
    docs = 0 if K <= 256 else N * 4 + 4 * D * K
    return words + docs


LDA_SOURCES = ["common.hpp", "lda_device.hpp", "lda_sample_z.hpp", "lda_count.hpp", "lda_gamma.hpp",
               "lda_loglik.hpp", "lda.hip"]


def lda_source_digest():
    """Digest of the sources of the LDA kernels: the traffic file names the one it was measured at."""
    h = hashlib.sha256()
    for name in LDA_SOURCES:
        with open(os.path.join(ROOT, "paper_1312_3613_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_counters(workload):
    """rocprofv3 figures of earlier runs (HBM bytes per sample_z launch, instruction counters),
    with the commit and the digest of the kernel source they were measured at.  They cannot be
    measured inside a timed run: counters perturb timing and need the profiler around the
    process."""
    try:
        with open(TRAFFIC_FILE) as f:
            data = json.load(f)
    except (OSError, ValueError):
        return None
    entry = data.get("workloads", {}).get(workload)
    if entry is None:
        return None
    digest = lda_source_digest()
    out = dict(entry)
    out["measured_at_commit"] = data.get("measured_at_commit")
    out["kernel_source_changed_since"] = digest != data.get("lda_sources_sha256_16")
    return out


def host_description():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return model


def oracle_per_step(cfg, corpus, target_tokens, z_reps):
    """Times the oracle's four steps separately on the first documents of the corpus (about
    target_tokens tokens) with the full vocabulary, on one pinned core, and composes the time of
    a sweep over the WHOLE corpus: z and counting scale with the tokens, theta with the
    documents, and the phi step (V x K Gamma draws, whatever the number of tokens) is taken as
    measured."""
    import numpy as np
    from oracle import oracle as O
    doc_len = corpus["doc_len"]
    cum = np.cumsum(doc_len.astype(np.int64))
    nd = int(min(len(doc_len), np.searchsorted(cum, target_tokens) + 1))
    ntok = int(cum[nd - 1])
    N, D = corpus["N"], len(doc_len)
    old = os.sched_getaffinity(0)
    core = min(old)
    os.sched_setaffinity(0, {core})
    try:
        o = O.OracleLDA(nd, cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], cfg["seed"], doc_len[:nd],
                        corpus["w"][:ntok])

        def timed(fn, reps=1):
            best = None
            for _ in range(reps):
                t0 = time.perf_counter()
                fn()
                dt = time.perf_counter() - t0
                best = dt if best is None else min(best, dt)
            return best
        t_z = timed(o.step_sample_z, z_reps)
        t_c = timed(o.step_count)
        t_th = timed(o.step_resample_theta)
        t_ph = timed(o.step_resample_phi)
    finally:
        os.sched_setaffinity(0, old)
    full = t_z * N / ntok + t_c * N / ntok + t_th * D / nd + t_ph
    return {"value": N / full, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"oracle steps timed one by one on the first {nd} documents ({ntok} tokens) of the "
                      f"same corpus with the full V={cfg['V']} and K={cfg['K']}, composed to the whole corpus "
                      f"(N={N}, D={D}): sweep = (z + count) * N/{ntok} + theta * D/{nd} + phi; one thread "
                      f"pinned to core {core}",
            "sample_seconds": {"sample_z": t_z, "count": t_c, "resample_theta": t_th, "resample_phi": t_ph},
            "composed_sweep_seconds": full,
            "per_step_rates": {"sample_z_tokens_per_s": ntok / t_z, "count_tokens_per_s": ntok / t_c,
                               "theta_draws_per_s": nd * cfg["K"] / t_th,
                               "phi_draws_per_s": cfg["V"] * cfg["K"] / t_ph},
            "host": {"cpu_model": host_description(), "nproc": os.cpu_count(),
                     "usable_cores": len(old)}}


def run_lda(name, cfg, corpus, steps, warmup, repeats, with_ceilings, overlap=True, topics=None,
            with_f64=True):
    """All GPU measurements of one LDA workload.  Returns (fields of the main line, extras)."""
    import torch
    from paper_1312_3613_amd import binding as B
    if topics is not None:
        cfg = dict(cfg, K=topics)
    N, D, V, K = corpus["N"], cfg["D"], cfg["V"], cfg["K"]
    stream = torch.cuda.Stream()
    doc_len_d = torch.as_tensor(corpus["doc_len"]).cuda()
    w_d = torch.as_tensor(corpus["w"]).cuda()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    h = B.LDA(D, V, K, cfg["alpha"], cfg["beta"], cfg["seed"], doc_len_d, w_d, stream=stream,
              device_ptrs=True)
    t_create = time.perf_counter() - t0
    h.set_overlap(overlap)

    h.sweep(warmup)
    h.sync()
    # Timed regions of exactly `steps` sweeps each, of two kinds: sweep(), the call a user makes
    # (the library replays the sweep as a recorded HIP graph on this stream), by the wall clock;
    # and sweep_profile(), the same kernels launched directly with HIP events on the library's
    # stream around every step, which gives the kernels' durations.
    walls = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        h.sweep(steps)
        h.sync()
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - t0)
    regions = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ms = h.sweep_profile(steps)
        torch.cuda.synchronize()
        regions.append((time.perf_counter() - t0, ms))
    regions.sort(key=lambda r: r[0])
    profiled_elapsed, ms = regions[len(regions) // 2]          # the median region
    elapsed = sorted(walls)[len(walls) // 2]
    t_z = ms["sample_z"] / steps * 1e-3
    bytes_z = sample_z_algorithmic_bytes(N, D, K)
    achieved = bytes_z / t_z / 1e9
    counters = measured_counters(name) if topics is None else None
    traffic = None if counters is None else counters.get("sample_z_hbm_bytes")
    roofline = {"bound": "hbm", "kernel": "lda_sample_z", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "algorithmic_bytes_per_launch": bytes_z, "avg_launch_ms": t_z * 1e3,
                "note": "achieved = algorithmic bytes / launch time; 98 % of them are phi-row gathers that "
                        "L1/L2/Infinity Cache serve, so it can exceed the HBM peak and is no ceiling "
                        "fraction; traffic is what rocprofv3 counted past the L2 for one launch, "
                        "traffic_frac its rate against the HBM peak; see ceilings for the bounds "
                        "measured in this run",
                "traffic_GBs": None if traffic is None else traffic / t_z / 1e9,
                "traffic_frac": None if traffic is None else traffic / t_z / 1e9 / HBM_PEAK_GBS}
    if counters is not None:
        roofline["traffic_source"] = {"file": "profiles/hbm_traffic.json",
                                      "measured_at_commit": counters["measured_at_commit"],
                                      "kernel_source_changed_since": counters["kernel_source_changed_since"]}
    main = {"value": N * steps / elapsed, "ms_per_step": elapsed / steps * 1e3, "roofline": roofline}
    extra = {"repeats_ms_per_step": [x / steps * 1e3 for x in sorted(walls)],
             "profiled_ms_per_step": profiled_elapsed / steps * 1e3,
             "timing_note": "value and ms_per_step: median of %d regions of %d sweeps through sweep() (recorded "
                            "graph), wall clock around the region with a device synchronisation on both sides; "
                            "kernel_ms_per_sweep and the roofline's launch time: median of %d regions of %d sweeps "
                            "through sweep_profile() (direct launches, HIP events on the library's stream), "
                            "whose wall time per sweep is profiled_ms_per_step" % (repeats, steps, repeats, steps),
             "kernel_ms_per_sweep": {k: v / steps for k, v in ms.items()},
             "overlap_word_counts_with_theta": overlap}

    if with_ceilings:
        # sample_z and count_accumulate alone: the same sweeps with every kernel on one stream
        h.set_overlap(False)
        h.sweep(1)
        alone = []
        for _ in range(repeats):
            alone.append(h.sweep_profile(steps))
        h.set_overlap(overlap)
        med = {k: statistics.median(a[k] for a in alone) / steps for k in alone[0]}
        t_pair = (med["sample_z"] + med["count_accumulate"]) * 1e-3
        bytes_pair = bytes_z + count_algorithmic_bytes(N, D, V, K)
        extra["z_plus_count"] = {
            "sample_z_ms": med["sample_z"], "count_accumulate_ms": med["count_accumulate"],
            "note": "median of %d regions of %d sweeps with every kernel on one stream; up to 256 topics "
                    "sample_z also builds the document table and count_accumulate is the word table"
                    % (repeats, steps),
            "tokens_per_s": N / t_pair, "algorithmic_bytes": bytes_pair,
            "algorithmic_GBs": bytes_pair / t_pair / 1e9,
            "frac_of_hbm_peak": bytes_pair / t_pair / 1e9 / HBM_PEAK_GBS,
            "resample_theta_ms": med["resample_theta"], "resample_phi_ms": med["resample_phi"],
            "serial_sweep_ms": med["sweep"]}
        # what the memory system allows: a streaming copy and a gather-only pass
        n_copy = 1 << 28                                       # 1 GiB of floats
        src = torch.empty(n_copy, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        copy_ms = B.probe_stream_copy(src, dst, reps=10, stream=stream)
        del src, dst
        gather_ms = h.probe_gather(5)
        ceil = {"hbm_copy_GBs": 2 * 4 * n_copy / (copy_ms * 1e-3) / 1e9,
                "hbm_copy_note": "plain device copy of 1 GiB (read + write bytes over its time)",
                "gather_only_ms": gather_ms,
                "gather_only_note": "the z kernel's walk over the same word stream with every phi row loaded "
                                    "from memory (a quad per token, 64 bytes a load), no arithmetic, random "
                                    "numbers or stores: the floor that the texture addresser sets for that "
                                    "load shape; the resident form of the z kernel reads the rows of the most "
                                    "frequent words from LDS instead and can be faster",
                "gather_only_algorithmic_GBs": bytes_z / (gather_ms * 1e-3) / 1e9,
                "sample_z_ms": t_z * 1e3, "gather_only_over_sample_z": gather_ms / (t_z * 1e3)}
        if counters is not None:
            for k in ("valu_instr_per_token", "valu_busy", "texture_addresser_busy", "lds_busy", "l1_hit_rate",
                      "l2_hit_rate", "scratch_bytes_per_lane"):
                if k in counters:
                    ceil[k] = counters[k]
            ceil["counters_source"] = "rocprofv3 --pmc run recorded in profiles/hbm_traffic.json"
        extra["ceilings"] = ceil

    if with_f64:
        # the same sweep with theta and phi held in fp64 (the precision of the paper's own runs)
        f_steps = max(1, min(steps, 10))
        t0 = time.perf_counter()
        h64 = B.LDA(D, V, K, cfg["alpha"], cfg["beta"], cfg["seed"], doc_len_d, w_d, stream=stream,
                    device_ptrs=True, state_f64=True)
        t_create64 = time.perf_counter() - t0
        h64.set_overlap(overlap)
        h64.sweep(warmup)
        h64.sync()
        walls64 = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            h64.sweep(f_steps)
            h64.sync()
            torch.cuda.synchronize()
            walls64.append(time.perf_counter() - t0)
        ms64 = h64.sweep_profile(f_steps)
        e64 = sorted(walls64)[len(walls64) // 2]
        extra["state_f64"] = {
            "ms_per_step": e64 / f_steps * 1e3, "value": N * f_steps / e64, "unit": "tokens/s",
            "steps": f_steps, "over_f32_sweep": e64 / f_steps / (elapsed / steps),
            "kernel_ms_per_sweep": {k: v / f_steps for k, v in ms64.items()},
            "log_marginal_per_token": h64.loglik()[1] / max(N, 1), "create_s": t_create64,
            "note": "theta and phi stored and multiplied as fp64 (AUGUR_STATE_F64); same protocol as value "
                    "(median of %d regions of %d sweeps through sweep()); the z kernel of this mode is a plain "
                    "one written for checking against the fp64 oracle" % (repeats, f_steps)}
        h64.close()

    lj, lm = h.loglik()
    extra["log_marginal_per_token"] = lm / max(N, 1)
    extra["degenerate_tokens"] = h.get_degenerate()
    extra["setup_s"] = {"create": t_create}
    h.close()
    del doc_len_d, w_d
    return main, extra


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
    walls = []
    for _ in range(args.repeats):                     # sweep(): the recorded graph, by the wall clock
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        h.sweep(steps)
        h.sync()
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - t0)
    elapsed = sorted(walls)[len(walls) // 2]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms = h.sweep_profile(steps)                       # direct launches with events: kernel durations
    torch.cuda.synchronize()
    profiled_elapsed = time.perf_counter() - t0
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
        "repeats_ms_per_step": [x / steps * 1e3 for x in sorted(walls)],
        "profiled_ms_per_step": profiled_elapsed / steps * 1e3,
        "log_joint_per_point": lj / N,
        "setup_s": {"generate_points": t_gen},
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        n = 200_000
        xs = d["x"][:n]
        old = os.sched_getaffinity(0)
        os.sched_setaffinity(0, {min(old)})
        try:
            o = (O.OracleGMMUV(K, cfg["alpha"], cfg["prior_sd"], 1.0, 1.0, cfg["seed"], xs) if unknown_var
                 else O.OracleGMM(K, cfg["alpha"], cfg["prior_sd"], cfg["sigma"], cfg["seed"], xs))
            sweeps, t0 = 0, time.perf_counter()
            while True:
                o.sweep(1)
                sweeps += 1
                el = time.perf_counter() - t0
                if sweeps >= 2 and (el > 10.0 or sweeps >= 20):
                    break
        finally:
            os.sched_setaffinity(0, old)
        out["cpu_baseline"] = {"value": n * sweeps / el, "unit": "points/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {n} points of the same cloud, {sweeps} whole sweeps (every step "
                                         f"scales with the points), one pinned thread of {os.cpu_count()} visible",
                               "host": {"cpu_model": host_description(), "nproc": os.cpu_count()}}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--repeats", type=int, default=3,
                    help="timed regions of --steps sweeps each; the median one is reported")
    ap.add_argument("--workload", default="large",
                    choices=["tiny", "medium", "large", "widek", "paper_shape", "gmm", "gmm_unknown_variance"])
    ap.add_argument("--topics", type=int, default=None,
                    help="infer with this many topics instead of the number the corpus was drawn with")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="build the word-count table on the main stream instead of beside the theta step")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="leave out the z + count leg and the copy and gather probes")
    ap.add_argument("--no-state-f64", action="store_true",
                    help="leave out the sweep with theta and phi held in fp64")
    ap.add_argument("--no-k100", action="store_true",
                    help="with the default workload: leave out the K = 100 (LDA medium) block")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    if args.workload.startswith("gmm"):
        bench_gmm(args, args.workload == "gmm_unknown_variance")
        return

    import torch
    from paper_1312_3613_amd import synth

    cfg = synth.LDA_CONFIGS[args.workload]
    steps = args.steps if args.steps is not None else cfg["sweeps"]
    t0 = time.perf_counter()
    corpus = synth.lda_corpus(**cfg)
    t_gen = time.perf_counter() - t0
    torch.cuda.set_device(0)
    main_fields, extra = run_lda(args.workload, cfg, corpus, steps, args.warmup, args.repeats,
                                 not args.no_ceilings, overlap=not args.no_overlap, topics=args.topics,
                                 with_f64=not args.no_state_f64)
    K = args.topics if args.topics is not None else cfg["K"]
    out = {
        "metric": "Gibbs sweep tokens/sec (LDA K=100/200) + achieved HBM GB/s vs peak",
        "value": main_fields["value"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": main_fields["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"LDA {args.workload}: D={cfg['D']} V={cfg['V']} K={K} N={corpus['N']} "
                               f"alpha={cfg['alpha']} beta={cfg['beta']}, corpus from the LDA generative process "
                               f"(seed {cfg['seed']}), inputs resident in HBM"},
        "roofline": main_fields["roofline"],
    }
    out.update(extra)
    out["setup_s"]["generate_corpus"] = t_gen
    out["environment"] = {"gpu": torch.cuda.get_device_name(0), "rocm": getattr(torch.version, "hip", None),
                          "torch": torch.__version__, "cpu_model": host_description(),
                          "nproc": os.cpu_count()}
    if not args.no_cpu_baseline:
        # a bounded sample: about ten seconds of oracle work at the default workload
        out["cpu_baseline"] = oracle_per_step(dict(cfg, K=K), corpus,
                                              10_000_000 if K <= 256 else 2_000_000, z_reps=2)

    if args.workload == "large" and args.topics is None and not args.no_k100:
        # the K = 100 half of the metric: LDA medium, its own sweep count, same protocol
        mcfg = synth.LDA_CONFIGS["medium"]
        t0 = time.perf_counter()
        mcorpus = synth.lda_corpus(**mcfg)
        t_mgen = time.perf_counter() - t0
        mmain, mextra = run_lda("medium", mcfg, mcorpus, mcfg["sweeps"], args.warmup, args.repeats,
                                not args.no_ceilings, overlap=not args.no_overlap,
                                with_f64=not args.no_state_f64)
        k100 = {"config": {"workload": f"LDA medium: D={mcfg['D']} V={mcfg['V']} K={mcfg['K']} N={mcorpus['N']} "
                                       f"alpha={mcfg['alpha']} beta={mcfg['beta']} (seed {mcfg['seed']}), "
                                       f"inputs resident in HBM"},
                "steps": mcfg["sweeps"], "value": mmain["value"], "unit": "tokens/s",
                "ms_per_step": mmain["ms_per_step"], "roofline": mmain["roofline"]}
        k100.update(mextra)
        k100["setup_s"]["generate_corpus"] = t_mgen
        if not args.no_cpu_baseline:
            k100["cpu_baseline"] = oracle_per_step(mcfg, mcorpus, 3_000_000, z_reps=2)
        out["k100"] = k100
    print(json.dumps(out))


if __name__ == "__main__":
    main()
