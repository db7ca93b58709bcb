"""Small test-only helpers: tiny random CSR graphs (with duplicates and empty rows) and the error metric."""
import numpy as np


def random_csr(n, avg_deg, seed, empty_frac=0.2, duplicates=True):
    rng = np.random.default_rng(seed)
    deg = rng.poisson(avg_deg, n)
    deg[rng.random(n) < empty_frac] = 0
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    indices = rng.integers(0, n, indptr[-1]).astype(np.int32)
    if duplicates:
        for v in np.nonzero(deg >= 2)[0][:3]:  # make sure a few repeated edges exist
            indices[indptr[v] + 1] = indices[indptr[v]]
    if not duplicates:
        rows = []
        for v in range(n):
            rows.append(np.unique(indices[indptr[v]:indptr[v + 1]]))
        deg = np.array([r.size for r in rows])
        np.cumsum(deg, out=indptr[1:])
        indices = np.concatenate(rows).astype(np.int32) if rows else indices
    return indptr, indices


def dense_adjacency(indptr, indices):
    """A[v, u] = multiplicity of edge u -> v."""
    n = indptr.size - 1
    A = np.zeros((n, n), dtype=np.float64)
    for v in range(n):
        for e in range(indptr[v], indptr[v + 1]):
            A[v, indices[e]] += 1.0
    return A


def max_rel_err(got, want):
    """max_i |g_i - o_i| / max(|o_i|, RMS(o)): element-wise relative error with an RMS floor, so that
    outputs that are ~0 by cancellation (or exactly 0 after ReLU) do not blow the ratio up."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(want * want))
    floor = rms if rms > 0 else 1.0
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), floor)))


def act_np(x, act, slope=1.0):
    if act == "relu":
        return np.maximum(x, 0.0)
    if act == "elu":
        return np.where(x > 0, x, slope * np.expm1(np.minimum(x, 0)))
    if act == "leaky_relu":
        return np.where(x > 0, x, slope * x)
    return x
