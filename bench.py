#!/usr/bin/env python3
"""Benchmark: sampled tokens/sec per iteration of collapsed Gibbs sampling for LDA on one
MI355X (the paper's metric, Eq. 2), on a synthetic corpus shaped like the paper's larger
workload, plus the sampling kernel's HBM roofline fraction and the CPU oracle timed
beside it.

A "step" is one whole iteration: sampling, rebuild of phi and n_k, rebuild of theta and
the log-likelihood of the new state.  Inputs are resident in HBM before the timed region.
Prints ONE JSON line on stdout; progress goes to stderr.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak

# HBM bytes per sampling launch from rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE, scaled by a
# copy kernel of known size); filled in from the summaries under profiles/ per workload.
# (FETCH_SIZE KiB, WRITE_SIZE KiB) per launch; FETCH_SIZE under-reports a plain copy by 2.000 on
# this chip, WRITE_SIZE by 1.000 (same summaries).
FETCH_SCALE, WRITE_SCALE = 2.000, 1.000
MEASURED_TRAFFIC_KIB = {
    ("C4", "init"): (7.18155e7, 1.66019e6, "profiles/sample_kernel_C4.md"),
    ("C3", "init"): (1.22944e7, 2.24598e5, "profiles/sample_kernel_C3_C5.md"),
    ("C5", "init"): (2.89505e7, 1.38495e6, "profiles/sample_kernel_C3_C5.md"),
}
# VALU wave-instructions per sampling launch (SQ_INSTS_VALU, same summaries): the sampler's other
# limit is instruction issue, 1024 SIMDs x 2.4 GHz / 4 cycles per wave-instruction
MEASURED_VALU_INSTS = {("C4", "init"): 1.65364e10, ("C3", "init"): 4.18612e9, ("C5", "init"): 6.47468e9}
VALU_ISSUE_PEAK = 256 * 4 * 2.4e9 / 4.0


# The paper's own single-GPU rates (its Table 4, mean of the first 100 iterations) on the
# collections that C3 and C4 are shaped like: context, never a baseline for `vs_baseline`.
PAPER_CONTEXT = {
    "C3": "paper, NYTimes: 173.6 M tokens/s on TITAN X (Maxwell), 208.0 M on Titan Xp, 633.0 M on V100",
    "C4": "paper, PubMed: 155.6 M tokens/s on TITAN X (Maxwell), 213.0 M on Titan Xp, 686.2 M on V100",
}


def paper_unshared_accounting(k_d, k, int_bytes=4, float_bytes=4):
    """The paper's Table 1: flops and bytes per token of the four sampler steps when nothing
    is shared between samplers (32-bit integers and floats).  Returns {step: (flops, bytes)}."""
    return {
        "compute_S": (4 * k_d, 3 * int_bytes * k_d),
        "compute_Q": (2 * k, 2 * int_bytes * k),
        "sample_p1": (6 * k_d, (3 * int_bytes + 2 * float_bytes) * k_d),
        "sample_p2": (3 * k, (2 * int_bytes + 2 * float_bytes) * k),
    }


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def oracle_pass_rate(sample, cfg, seed, z, it, threads):
    """tokens/s of one whole oracle iteration (resample, recount, theta CSR, log-likelihood)
    from the state z."""
    import oracle
    n_wk, n_k = oracle.count_word_topic(sample.word_ids, z, cfg.V, cfg.K)
    t0 = time.perf_counter()
    z1 = oracle.iteration(sample.doc_ptr, sample.word_ids, z, cfg.V, cfg.K, cfg.alpha, cfg.beta,
                          seed, it, n_wk, n_k, threads=threads)
    n_wk, n_k = oracle.count_word_topic(sample.word_ids, z1, cfg.V, cfg.K)
    oracle.doc_topic_csr(sample.doc_ptr, z1, cfg.K)
    oracle.loglik(sample.doc_ptr, z1, cfg.V, cfg.K, cfg.alpha, cfg.beta, n_wk, n_k)
    return sample.T / (time.perf_counter() - t0)


def cpu_baseline(cfg, seed, target_tokens):
    """The oracle's full pass, as it stands, on a bounded sample of the same workload (the
    first documents of the same configuration as a corpus of their own), from two states:
    random topics (dense theta rows, the first iteration) and the topics the corpus was
    generated with (sparse rows, a late iteration); the figure is the mean of the two.
    Timed on all host threads and, on a sixteenth of the sample, on one thread."""
    import corpus_synth
    import oracle
    threads = oracle.max_threads()
    t_start = time.perf_counter()
    scale = min(1.0, target_tokens / (cfg.D * cfg.mean_len))
    sample = corpus_synth.generate(cfg, scale=scale)
    small = corpus_synth.generate(cfg, scale=scale / 16.0)
    rates = {}
    for label, corpus, n_threads in (("all", sample, threads), ("one", small, 1)):
        z_random = oracle.init_topics(corpus.T, cfg.K, seed)
        rates[label] = [oracle_pass_rate(corpus, cfg, seed, z_random, 1, n_threads),
                        oracle_pass_rate(corpus, cfg, seed, corpus.z_true, 1, n_threads)]
    mean_all = sum(rates["all"]) / 2.0
    mean_one = sum(rates["one"]) / 2.0
    return {
        "value": mean_all, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": "whole oracle iterations (resample + recount + theta CSR + log-likelihood) on the "
                  "first %d documents (%d tokens) of the same configuration, mean of two start "
                  "states (random topics %.4g tokens/s, generated topics %.4g tokens/s); sampling "
                  "uses %d OpenMP threads, the recounts one"
                  % (len(sample.doc_ptr) - 1, sample.T, rates["all"][0], rates["all"][1], threads),
        "single_thread": {
            "value": mean_one, "unit": "tokens/s", "cores": 1,
            "sample": "the same on the first %d documents (%d tokens), one thread"
                      % (len(small.doc_ptr) - 1, small.T),
        },
        "seconds": time.perf_counter() - t_start,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C4", help="C1..C5 (default C4, the largest single-GPU workload)")
    ap.add_argument("--state", default="init", choices=["init", "generated"],
                    help="start from random topics (as the paper does) or from the topics the corpus "
                         "was generated with (a converged-like, sparse theta)")
    ap.add_argument("--chunks", type=int, default=1,
                    help="above 1: stream the corpus through the GPU in this many chunks every "
                         "iteration (Algorithm 1, WorkSchedule2); the rate then includes the PCIe "
                         "transfers and is not the headline value")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=float, default=0.0)
    ap.add_argument("--copy-calibration-gib", type=float, default=0.0,
                    help="also run a plain device copy of this many GiB three times, so that a "
                         "rocprofv3 --pmc run holds a kernel of known HBM traffic to scale "
                         "FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (--gpus 1); the multi-GPU phi "
                 "reduction of the paper's Section 5.2 is not part of it")
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: launched with WORLD_SIZE > 1, but this build runs on ONE GPU only")

    import numpy as np
    import torch
    import corpus_synth
    import paper_1803_04631_amd as mlda

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cfg = corpus_synth.CONFIGS[args.config]
    seed = corpus_synth.SAMPLER_SEED

    t0 = time.perf_counter()
    corpus = corpus_synth.generate(cfg)
    log("corpus %s: D=%d V=%d K=%d T=%d generated in %.1f s" % (cfg.name, cfg.D, cfg.V, cfg.K, corpus.T,
                                                               time.perf_counter() - t0))
    t0 = time.perf_counter()
    model = mlda.Mlda(corpus.doc_ptr, corpus.word_ids, cfg.V, cfg.K, cfg.alpha, cfg.beta, seed,
                      device="cuda:0", chunks=args.chunks)
    if args.state == "init":
        model.init_random()
    else:
        model.set_assignments(corpus.z_true, it=0)
    model.synchronize()
    T = corpus.T
    log("resident on the GPU in %.1f s (workspace %.2f GB)" % (time.perf_counter() - t0,
                                                              model.workspace.numel() / 1e9))
    corpus.word_ids = corpus.z_true = None

    if args.copy_calibration_gib > 0:
        n = int(args.copy_calibration_gib * 2**30)
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("copy calibration: 3 device copies of %d bytes (reads %d, writes %d each)" % (n, n, n))
        del src, dst
    if args.warmup > 0:
        model.step(args.warmup, loglik=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    model.step(args.steps, loglik=True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms = model.timing()                       # [steps, 4] HIP-event times on the library's stream
    algo_bytes = model.sampler_bytes()        # [steps] algorithmic bytes of each sampling launch
    ll = model.loglik()
    nnz = model.doc_topic_nnz()
    mean_ms = ms.mean(axis=0)
    sample_ms = float(mean_ms[0])
    achieved = float((algo_bytes / (ms[:, 0] * 1e-3)).mean()) / 1e9      # GB/s, per launch then mean
    measured = MEASURED_TRAFFIC_KIB.get((cfg.name, args.state)) if args.chunks == 1 else None
    valu_insts = MEASURED_VALU_INSTS.get((cfg.name, args.state)) if args.chunks == 1 else None
    traffic = traffic_source = hbm_gbs = None
    if measured:
        traffic = (measured[0] * FETCH_SCALE + measured[1] * WRITE_SCALE) * 1024.0
        traffic_source = measured[2]
        hbm_gbs = traffic / (sample_ms * 1e-3) / 1e9
    value = T * args.steps / elapsed
    log("per iteration: sample %.2f ms, phi %.2f ms, theta %.2f ms, loglik %.2f ms; wall %.2f ms"
        % (*mean_ms, elapsed / args.steps * 1e3))
    log("tokens/s %.4g; sampler %.1f GB/s algorithmic (%.1f%% of %.0f); LL/token %.4f; theta nnz/doc %.1f"
        % (value, achieved, 100 * achieved / HBM_PEAK_GBS, HBM_PEAK_GBS, ll / T, nnz / cfg.D))

    streamed = args.chunks > 1
    out = {
        "metric": "sampled tokens/sec per iteration (1 GPU)" + (", corpus streamed over PCIe" if streamed else ""),
        "value": value,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {
            "workload": "%s: D=%d V=%d K=%d T=%d, alpha=50/K, beta=0.01, %s start, iterations %d..%d%s"
                        % (cfg.name, cfg.D, cfg.V, cfg.K, T,
                           "random-topic" if args.state == "init" else "generated-topic",
                           args.warmup + 1, args.warmup + args.steps,
                           ", streamed through the GPU in %d chunks (the rate includes the PCIe transfers)"
                           % args.chunks if streamed else ""),
            "step": ("per chunk: upload, topics to word-major order, rebuild theta, sample, add to phi, "
                     "topics back to document order, rebuild theta for the log-likelihood, download; then "
                     "n_k and the log-likelihood; kernel times are sums over the chunks (ms_rebuild_theta "
                     "includes the two order changes)") if streamed
                    else "sample + rebuild phi/n_k + rebuild theta + log-likelihood",
            "ms_sample": sample_ms, "ms_rebuild_phi": float(mean_ms[1]),
            "ms_rebuild_theta": float(mean_ms[2]), "ms_loglik": float(mean_ms[3]),
            "tokens_per_s_without_loglik": T / (float(mean_ms[:3].sum()) * 1e-3),
            "loglik_per_token": ll / T,
            "theta_nnz_per_doc": nnz / cfg.D,
            "sampler_bytes_per_token": float(algo_bytes.mean()) / T,
            # context only (other hardware, the real collections, K not stated): the paper's Table 4
            "paper_context": PAPER_CONTEXT.get(cfg.name),
        },
        "roofline": {
            "kernel": "sample_kernel" + (" (sum over the chunks of an iteration)" if streamed else ""),
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "avg_launch_ms": sample_ms,
            "algorithmic_bytes_per_launch": float(algo_bytes.mean()),
            # the two rates side by side: `useful` moves the bytes the method needs (one walk of
            # its theta row per token, so rows that co-resident tiles share in cache count once
            # per token), `hbm` the bytes the memory counters saw per launch in the committed
            # profile of this command, over this run's launch time
            "useful_gbs": achieved,
            "useful_frac": achieved / HBM_PEAK_GBS,
            "hbm_gbs": hbm_gbs,
            "hbm_frac": hbm_gbs / HBM_PEAK_GBS if hbm_gbs else None,
            "traffic_source": traffic_source,
            # the unit that is busiest: VALU issue (instructions from the same committed profile
            # over this run's launch time, against the chip's issue rate)
            "valu_insts_per_launch": valu_insts,
            "valu_issue_frac": valu_insts / VALU_ISSUE_PEAK / (sample_ms * 1e-3) if valu_insts else None,
        },
    }
    model.close()
    del model
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        target = args.cpu_sample_tokens or 5.0e10 / cfg.K      # about 10-30 s of oracle work in all
        out["cpu_baseline"] = cpu_baseline(cfg, seed, target)
        log("oracle: %.4g tokens/s on %d threads, %.4g on one (%.1f s)"
            % (out["cpu_baseline"]["value"], out["cpu_baseline"]["cores"],
               out["cpu_baseline"]["single_thread"]["value"], out["cpu_baseline"]["seconds"]))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
