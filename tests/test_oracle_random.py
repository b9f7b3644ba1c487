"""Pins for the oracle's random primitives: Philox against published known answers,
the uniform conversions against their definitions, and distribution tests against scipy."""
import os

import numpy as np
from scipy import stats

from oracle import oracle as O


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = O.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_random_block_counter_layout():
    # counter = (index lo, index hi, sweep, stream<<24 | attempt), key = seed halves
    seed, idx, sweep, stream, att = 0x123456789ABCDEF0, (7 << 32) | 99, 17, 3, 5
    got = O.random_block(seed, idx, sweep, stream, att)
    want = O.philox4x32_10([99, 7, 17, (3 << 24) | 5], [0x9ABCDEF0, 0x12345678])
    assert (got == want).all()
    # every field matters
    base = O.random_block(1, 2, 3, 1, 0)
    for other in [(2, 2, 3, 1, 0), (1, 3, 3, 1, 0), (1, 2, 4, 1, 0), (1, 2, 3, 2, 0),
                  (1, 2, 3, 1, 1), (1 + (1 << 32), 2, 3, 1, 0), (1, 2 + (1 << 32), 3, 1, 0)]:
        assert (O.random_block(*other) != base).any()


def test_uniform_conversions_exact():
    for r in [0, 1, 511, 512, 0x7FFFFFFF, 0xFFFFFFFF, 123456789]:
        u = O.uniform24(r)
        assert 0.0 < u < 1.0
        assert float(np.float32(u)) == u                      # exact in fp32
        m = u * 2 ** 24
        assert m == int(m) and int(m) % 2 == 1 and int(m) == 2 * (r >> 9) + 1
        u2 = O.uniform32(r)
        assert 0.0 < u2 < 1.0 and u2 * 2 ** 33 == 2 * r + 1   # (r + 1/2) 2^-32 exactly
    assert O.uniform24(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert O.uniform24(0) == 2.0 ** -24


def test_datum_uniforms_share_blocks():
    seed, sweep, stream = 42, 9, O.STREAM_Z
    u = O.datum_uniforms(seed, 0, 64, sweep, stream)
    for i in range(64):
        blk = O.random_block(seed, i >> 2, sweep, stream, 0)
        assert u[i] == O.uniform24(blk[i & 3])
    # a range that starts off a block boundary is the same stream
    u2 = O.datum_uniforms(seed, 5, 20, sweep, stream)
    assert (u2 == u[5:25]).all()


def test_uniformity_and_serial_pairs():
    n = 1 << 18
    u = O.datum_uniforms(7, 0, n, 1, O.STREAM_Z)
    counts = np.bincount((u * 256).astype(int), minlength=256)
    assert stats.chisquare(counts).pvalue > 1e-4
    pair = (u[:-1] * 16).astype(int) * 16 + (u[1:] * 16).astype(int)
    assert stats.chisquare(np.bincount(pair, minlength=256)).pvalue > 1e-4
    # different sweeps and streams are uncorrelated
    v = O.datum_uniforms(7, 0, n, 2, O.STREAM_Z)
    s = O.datum_uniforms(7, 0, n, 1, O.STREAM_INIT_Z)
    assert abs(np.corrcoef(u, v)[0, 1]) < 5 / np.sqrt(n)
    assert abs(np.corrcoef(u, s)[0, 1]) < 5 / np.sqrt(n)
    assert stats.kstest(u, "uniform").pvalue > 1e-4


def test_normals_against_library_cdf():
    x = O.normals(11, 0, 200_000, 3, O.STREAM_GMM_MU)
    assert stats.kstest(x, "norm").pvalue > 1e-4
    assert abs(x.mean()) < 5 / np.sqrt(x.size)
    assert abs(x.var() - 1) < 5 * np.sqrt(2 / x.size)
    # Box-Muller, cosine branch, from words 0 and 1 of the variable's block
    blk = O.random_block(11, 5, 3, O.STREAM_GMM_MU, 0)
    want = np.sqrt(-2 * np.log(O.uniform32(blk[0]))) * np.cos(2 * np.pi * O.uniform32(blk[1]))
    assert abs(x[5] - want) < 1e-12
