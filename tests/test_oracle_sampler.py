"""Pins for the oracle's neighbour sampler (sampling inference, Section 2): the generator against its published
vectors, the selection rule against brute force, and the statistical and structural properties a uniform
fan-out sample must have."""
import os

import numpy as np

from oracle import oracle, sampler
from tests.helpers import max_rel_err, random_csr

HERE = os.path.dirname(os.path.abspath(__file__))


def test_splitmix64_matches_the_published_vectors():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "splitmix64_vectors.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 9
    for seed, k, value in rows:
        assert int(sampler.splitmix64_output(int(seed), int(k))) == int(value, 16)
    # array form = scalar form; output k+1 of seed s is output 1 of seed s + golden gamma * k (the state recurrence)
    ks = np.arange(1, 50)
    arr = sampler.splitmix64_output(77, ks)
    assert all(int(arr[i]) == int(sampler.splitmix64_output(77, int(k))) for i, k in enumerate(ks))
    state = (77 + 3 * 0x9E3779B97F4A7C15) % 2**64
    assert int(sampler.splitmix64_output(state, 1)) == int(sampler.splitmix64_output(77, 4))


def brute_force_sample(indptr, indices, fanout, seed, layer):
    E = indices.size
    out_ptr, out_idx = [0], []
    for v in range(indptr.size - 1):
        a, b = int(indptr[v]), int(indptr[v + 1])
        if b - a <= fanout:
            chosen = list(range(a, b))
        else:
            key = lambda e: (int(sampler.splitmix64_output(seed, layer * E + e + 1)) >> 32, e - a)
            chosen = sorted(sorted(range(a, b), key=key)[:fanout])
        out_idx += [int(indices[e]) for e in chosen]
        out_ptr.append(len(out_idx))
    return np.array(out_ptr, dtype=np.int64), np.array(out_idx, dtype=np.int32)


def test_sampler_equals_row_by_row_selection():
    indptr, indices = random_csr(300, 6.0, seed=5, hub=(7, 90))
    for fanout, seed, layer in ((1, 0, 0), (4, 11, 0), (4, 11, 2), (10, 2**63 + 5, 1), (1000, 3, 0)):
        ip, ix = sampler.sample_csr(indptr, indices, fanout, seed, layer)
        bp, bx = brute_force_sample(indptr, indices, fanout, seed, layer)
        assert np.array_equal(ip, bp) and np.array_equal(ix, bx)


def test_sample_structure():
    indptr, indices = random_csr(2000, 8.0, seed=9, hub=(3, 500))
    deg = np.diff(indptr)
    f = 10
    ip, ix = sampler.sample_csr(indptr, indices, f, seed=42, layer=0)
    assert np.array_equal(np.diff(ip), np.minimum(deg, f))
    for v in range(2000):
        full = indices[indptr[v]:indptr[v + 1]]
        got = ix[ip[v]:ip[v + 1]]
        if deg[v] <= f:
            assert np.array_equal(got, full)
        else:  # a subsequence of the stored list: stored order kept, no edge used twice
            j = 0
            for u in full:
                if j < got.size and got[j] == u:
                    j += 1
            assert j == got.size
    # deterministic; another layer or seed draws another sample
    ip2, ix2 = sampler.sample_csr(indptr, indices, f, seed=42, layer=0)
    assert np.array_equal(ix, ix2)
    assert not np.array_equal(ix, sampler.sample_csr(indptr, indices, f, seed=42, layer=1)[1])
    assert not np.array_equal(ix, sampler.sample_csr(indptr, indices, f, seed=43, layer=0)[1])


def test_sample_is_uniform_over_the_neighbours():
    # one row with 24 in-edges, fan-out 6: every edge is kept with probability 1/4, every pair with 6*5/(24*23)
    d, f, trials = 24, 6, 6000
    indptr = np.array([0, d] + [d] * d, dtype=np.int64)
    indices = np.arange(1, d + 1, dtype=np.int32)
    counts = np.zeros(d)
    pair = 0
    for s in range(trials):
        _, ix = sampler.sample_csr(indptr, indices, f, seed=s, layer=0)
        assert ix.size == f and np.unique(ix).size == f
        counts[ix - 1] += 1
        pair += int(1 in ix and 2 in ix)
    expect = trials * f / d
    chi2 = ((counts - expect) ** 2 / (expect * (1 - f / d))).sum()   # ~ chi-square with d-1 = 23 degrees of freedom
    assert chi2 < 60.0, chi2                                         # P(chi2_23 > 60) < 1e-4
    p_pair = f * (f - 1) / (d * (d - 1))
    assert abs(pair / trials - p_pair) < 5 * np.sqrt(p_pair * (1 - p_pair) / trials)


def test_sampling_inference_special_cases():
    rng = np.random.default_rng(0)
    n = 400
    indptr, indices = random_csr(n, 5.0, seed=21, hub=(9, 60))
    X = rng.standard_normal((n, 12)).astype(np.float32)
    layers = [dict(agg="mean", act="relu", W_self=rng.standard_normal((12, 8)).astype(np.float32) * 0.3,
                   W_neigh=rng.standard_normal((12, 8)).astype(np.float32) * 0.3, bias=None),
              dict(agg="gcn", act="none", W_neigh=rng.standard_normal((8, 4)).astype(np.float32) * 0.3, bias=None)]
    # a fan-out no smaller than the largest degree is full inference
    full = oracle.infer(indptr, indices, layers, X)
    assert max_rel_err(oracle.infer_sampled(indptr, indices, layers, X, fanout=60, seed=1), full) <= 1e-6
    assert max_rel_err(oracle.infer_sampled(indptr, indices, layers, X, fanout=5, seed=1), full) > 1e-3
    # mean aggregation over identical source rows does not depend on which neighbours are drawn
    Xc = np.tile(X[:1], (n, 1))
    one = [dict(agg="mean", act="none", W_self=None, W_neigh=np.eye(12, dtype=np.float32), bias=None)]
    got = oracle.infer_sampled(indptr, indices, one, Xc, fanout=3, seed=5)
    nonempty = np.diff(indptr) > 0
    assert np.allclose(got[nonempty], X[0], rtol=1e-6) and np.all(got[~nonempty] == 0)
    # sum aggregation of all-ones features counts the kept neighbours: min(degree, fan-out)
    ones = np.ones((n, 1), dtype=np.float32)
    cnt = oracle.infer_sampled(indptr, indices, [dict(agg="sum", act="none", W_self=None, W_neigh=np.ones((1, 1), np.float32), bias=None)],
                               ones, fanout=7, seed=8)
    assert np.array_equal(cnt[:, 0], np.minimum(np.diff(indptr), 7).astype(np.float32))


def test_sampling_a_row_slice_equals_the_slice_of_the_sample():
    indptr, indices = random_csr(900, 7.0, seed=12, hub=(400, 300))
    full_ip, full_ix = sampler.sample_csr(indptr, indices, 5, seed=77, layer=2)
    a, b = 350, 620
    ip = indptr[a:b + 1] - indptr[a]
    ix = indices[indptr[a]:indptr[b]]
    sl_ip, sl_ix = sampler.sample_csr(ip, ix, 5, seed=77, layer=2, edge_base=int(indptr[a]), total_edges=indices.size)
    assert np.array_equal(sl_ip, full_ip[a:b + 1] - full_ip[a])
    assert np.array_equal(sl_ix, full_ix[full_ip[a]:full_ip[b]])
