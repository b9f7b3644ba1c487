"""Held-out log predictive probability against the number of Gibbs samples (Sect. 5.2 and the
figure of predictive probability against time): topics are learnt on the training documents,
then phi is declared observed (the paper's second `map` call, Fig. 3) and z and theta are
inferred on the test documents; the score is the mean over the test tokens of
ln sum_k theta_d[k] phi[w][k].

    python -m paper_1312_3613_amd.heldout_curve [--topics 50] [--max-samples 512]

Synthetic stand-in for the paper's corpus (same shape: 47,556 documents, 37,276 words, about
3.2M tokens, the last 1,000 documents held out); prints one row per power of two of samples and
a JSON line at the end.  Runs on cuda:0 through the HIP library only.
"""
import argparse
import json
import time

import numpy as np

from . import binding as B
from . import synth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--topics", type=int, default=50)
    ap.add_argument("--max-samples", type=int, default=512)
    ap.add_argument("--test-docs", type=int, default=1000)
    ap.add_argument("--fold-in-sweeps", type=int, default=50)
    ap.add_argument("--seed", type=int, default=7)
    args = ap.parse_args()

    import torch
    cfg = dict(synth.LDA_CONFIGS["paper_shape"])
    c = synth.lda_corpus(**cfg)
    D, V, K = cfg["D"], cfg["V"], args.topics
    n_train = D - args.test_docs
    ntok = int(c["doc_len"][:n_train].sum())
    a, b = cfg["alpha"], cfg["beta"]
    train = B.LDA(n_train, V, K, a, b, args.seed, c["doc_len"][:n_train], c["w"][:ntok])
    test_len, test_w = c["doc_len"][n_train:], c["w"][ntok:]
    n_test = int(test_len.sum())

    def score(phi):
        # a fresh chain on the test documents every time, phi as data
        t = B.LDA(args.test_docs, V, K, a, b, args.seed + 1, test_len, test_w)
        t.set_state(phi=phi)
        t.set_observed(phi=True)
        t.sweep(args.fold_in_sweeps)
        lm = t.loglik()[1]
        t.close()
        return lm / n_test

    rows = []
    done, gpu_s = 0, 0.0
    n = 1
    print(f"K = {K}, {n_train} training documents ({ntok} tokens), {args.test_docs} test documents "
          f"({n_test} tokens), {args.fold_in_sweeps} fold-in sweeps")
    print(" samples   training time (s)   log predictive per test token")
    phi0 = train.get_state(z=False, theta=False)[2]
    rows.append((0, 0.0, score(phi0)))
    print(f"{0:8d}   {0.0:17.4f}   {rows[-1][2]:.4f}")
    while n <= args.max_samples:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        train.sweep(n - done)
        train.sync()
        gpu_s += time.perf_counter() - t0
        done = n
        phi = train.get_state(z=False, theta=False)[2]
        rows.append((n, gpu_s, score(phi)))
        print(f"{n:8d}   {gpu_s:17.4f}   {rows[-1][2]:.4f}")
        n *= 2
    train.close()
    print(json.dumps({"topics": K, "train_tokens": ntok, "test_tokens": n_test,
                      "samples": [r[0] for r in rows], "train_seconds": [round(r[1], 5) for r in rows],
                      "log_predictive_per_token": [round(r[2], 5) for r in rows]}))


if __name__ == "__main__":
    main()
