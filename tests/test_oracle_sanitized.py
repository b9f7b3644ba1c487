"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the small
LDA and mixture sweeps, the fold-in sweep, the log joints and the Metropolis-Hastings run must
finish without a finding, and give the numbers of the plain build."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r'''
import numpy as np
from oracle import oracle as O
from paper_1312_3613_amd import synth
cfg = synth.LDA_CONFIGS["tiny"]
c = synth.lda_corpus(**cfg)
o = O.OracleLDA(cfg["D"], cfg["V"], cfg["K"], cfg["alpha"], cfg["beta"], cfg["seed"], c["doc_len"], c["w"])
o.sweep(3)
lj, lm = o.loglik()
o.set_observed(phi=True)
o.sweep(1)
# ragged edges: empty documents, one token, V = 1
for lens, w, V, K in [([1], [2], 5, 3), ([0, 0, 0], [], 4, 3), ([3, 0, 2], [0, 0, 0, 0, 0], 1, 4)]:
    e = O.OracleLDA(len(lens), V, K, 0.5, 0.5, 3, np.array(lens, dtype=np.int32), np.array(w, dtype=np.int32))
    e.sweep(2)
    e.loglik()
d = synth.gmm_points(N=3001, dim=8, K=16, seed=1)
g = O.OracleGMM(16, 1.0, 10.0, 1.0, 3, d["x"])
g.sweep(3)
gj = g.loglik()
u = O.OracleGMMUV(16, 1.0, 10.0, 1.0, 1.0, 3, d["x"])
u.sweep(2)
uj = u.loglik()
print("RESULT", repr(lj), repr(lm), repr(gj), repr(uj), int(o.z.sum()), int(g.z.sum()))
'''


def _run(env_extra):
    env = dict(os.environ, **env_extra)
    r = subprocess.run([sys.executable, "-c", CHILD], cwd=ROOT, env=env, capture_output=True, text=True,
                       timeout=600)
    return r


def test_small_sweeps_are_clean_under_asan_and_ubsan():
    from oracle import build as ob
    try:
        san = ob.build_sanitized()
    except (subprocess.CalledProcessError, FileNotFoundError) as e:   # no sanitizer runtime installed
        pytest.skip(f"cannot build the oracle with sanitizers: {e}")
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan):
        pytest.skip("libasan.so not found")
    preload = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)
    r = _run({"AUGUR_ORACLE_LIB": san, "LD_PRELOAD": preload,
              # the interpreter is not instrumented: its own allocations are not this test's matter
              "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0",
              "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"})
    assert r.returncode == 0, r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    plain = _run({})
    assert plain.returncode == 0, plain.stderr[-2000:]
    res = [l for l in r.stdout.splitlines() if l.startswith("RESULT")]
    ref = [l for l in plain.stdout.splitlines() if l.startswith("RESULT")]
    assert res and res == ref       # -O1 with sanitizers and -O2 without: same arithmetic, same numbers
