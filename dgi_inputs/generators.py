"""Seeded synthetic inputs shared by the oracle tests, the GPU tests and the benchmark.

This module holds none of the inference arithmetic: it only draws graphs, features and weights.
Everything is built from torch tensor ops so that the large graphs can be generated on the GPU
(`device="cuda"`) and the small ones on the CPU; a seed fixes the result per device type.

Graph recipes (the public datasets the paper measures on are not available here; these stand in for
them, shaped after Table 1 of the paper):
  * Chung-Lu power law: node i has weight w_i ∝ (i + i0)^(-1/(gamma-1)); an edge endpoint is drawn
    with probability ∝ w.  i0 is chosen by bisection so that the largest expected degree equals
    `max_expected_degree` (i0 = 1 if that is None).  Pairs are deduplicated and self-pairs dropped.
  * Stochastic block model with power-law block sizes.
After generation the node ids are shuffled with a seeded permutation, because generator ids are
sorted by expected degree (or by block), a locality real datasets do not have.
"""
import math
import sys
import time

import torch

VERBOSE = False
_t0 = [time.perf_counter()]


def _log(msg):
    """Progress line for the long generations (a quiet multi-minute run looks hung to a job supervisor)."""
    if VERBOSE:
        print("[dgi_inputs %7.1fs] %s" % (time.perf_counter() - _t0[0], msg), file=sys.stderr, flush=True)


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def power_law_cdf(n, gamma, max_expected_degree, endpoints, device):
    """Cumulative endpoint distribution of the Chung-Lu weights (float64, length n)."""
    alpha = 1.0 / (gamma - 1.0)
    i = torch.arange(n, dtype=torch.float64, device=device)

    def top_share(i0):
        w = (i + i0).pow(-alpha)
        return float(w[0] / w.sum())

    i0 = 1.0
    if max_expected_degree is not None and top_share(1.0) * endpoints > max_expected_degree:
        lo, hi = 1.0, float(n)
        for _ in range(60):
            mid = math.sqrt(lo * hi)
            if top_share(mid) * endpoints > max_expected_degree:
                lo = mid
            else:
                hi = mid
        i0 = hi
    w = (i + i0).pow(-alpha)
    # prefix sums on the host: a device scan combines its partial sums in a timing-dependent order, which moves the
    # last bits of the CDF and with them a handful of the billions of draws from one run to the next
    cdf = torch.cumsum(w.cpu(), 0).to(device)
    return cdf / cdf[-1], i0


_CHUNK = 1 << 27


def _draw_nodes(cdf, count, gen):
    out = torch.empty(count, dtype=torch.int64, device=cdf.device)
    for lo in range(0, count, _CHUNK):
        hi = min(count, lo + _CHUNK)
        u = torch.rand(hi - lo, dtype=torch.float64, device=cdf.device, generator=gen)
        torch.searchsorted(cdf, u, out=out[lo:hi])
    return out.clamp_(max=cdf.numel() - 1)


def _systematic_subset(sorted_keys, m):
    """m of the keys, evenly spaced through the sorted list (an unbiased thinning of the edge set that
    needs no 2^31-element random permutation)."""
    total = sorted_keys.numel()
    idx = ((torch.arange(m, dtype=torch.float64, device=sorted_keys.device) + 0.5) * (total / m)).to(torch.int64)
    return sorted_keys[idx.clamp_(max=total - 1)]


def _distinct_pairs(draw, n, m, gen, undirected):
    """Draw until m distinct non-loop pairs exist; returns int64 (a, b), m entries each."""
    keys = torch.empty(0, dtype=torch.int64, device=gen.device)
    need = m
    for _ in range(64):
        k = int(need * 1.15) + 1024
        _log("drawing %d candidate pairs" % k)
        a, b = draw(k), draw(k)
        if undirected:
            lo_, hi_ = torch.minimum(a, b), torch.maximum(a, b)
            a, b = lo_, hi_
            del lo_, hi_
        new = a * n + b
        new = new[a != b]
        del a, b
        _log("deduplicating")
        keys = torch.unique(torch.cat([keys, new]))
        del new
        if keys.numel() >= m:
            break
        need = m - keys.numel()
    if keys.numel() < m:
        raise RuntimeError("could not draw enough distinct pairs")
    if keys.numel() > m:
        keys = _systematic_subset(keys, m)
    _log("%d distinct pairs" % keys.numel())
    return keys // n, keys % n


def shuffle_ids(src, dst, n, seed):
    perm = torch.randperm(n, device=src.device, generator=_gen(seed, src.device))
    return perm[src], perm[dst]


def chung_lu_directed(n, m, gamma, seed, device="cpu", max_expected_degree=None, shuffle=True):
    """m distinct directed non-loop edges; source and destination drawn independently ∝ w."""
    gen = _gen(seed, device)
    cdf, _ = power_law_cdf(n, gamma, max_expected_degree, m, device)
    src, dst = _distinct_pairs(lambda k: _draw_nodes(cdf, k, gen), n, m, gen, undirected=False)
    if shuffle:
        src, dst = shuffle_ids(src, dst, n, seed + 7919)
    return src, dst


def chung_lu_undirected(n, m_pairs, gamma, seed, device="cpu", max_expected_degree=None, self_loops=True,
                        shuffle=True):
    """m_pairs distinct undirected pairs stored in both directions, plus one self-loop per node."""
    gen = _gen(seed, device)
    cdf, _ = power_law_cdf(n, gamma, max_expected_degree, 2 * m_pairs, device)
    a, b = _distinct_pairs(lambda k: _draw_nodes(cdf, k, gen), n, m_pairs, gen, undirected=True)
    if shuffle:
        a, b = shuffle_ids(a, b, n, seed + 7919)
    src, dst = torch.cat([a, b]), torch.cat([b, a])
    if self_loops:
        loop = torch.arange(n, dtype=torch.int64, device=src.device)
        src, dst = torch.cat([src, loop]), torch.cat([dst, loop])
    return src, dst


def sbm_power_law_blocks(n, blocks, m, p_intra, seed, device="cpu", size_exponent=2.0, shuffle=True):
    """Stochastic block model: block sizes ∝ a power law (rank^(-1/(size_exponent-1)), floored so every
    block is non-empty), m distinct directed non-loop edges; each edge picks its source block ∝ block
    size, is intra-block with probability p_intra (both endpoints uniform in the block), else its
    destination is uniform over the whole graph outside the block."""
    gen = _gen(seed, device)
    r = torch.arange(1, blocks + 1, dtype=torch.float64, device=device)
    w = r.pow(-1.0 / (size_exponent - 1.0))
    floor = max(1, n // (blocks * 20))
    sizes = torch.floor(w / w.sum() * (n - floor * blocks)).to(torch.int64) + floor
    sizes[0] += n - int(sizes.sum())
    start = torch.cumsum(sizes, 0) - sizes
    size_cdf = torch.cumsum(sizes.to(torch.float64), 0) / n

    def draw_pairs(k):
        blk = torch.searchsorted(size_cdf, torch.rand(k, dtype=torch.float64, device=device, generator=gen))
        blk.clamp_(max=blocks - 1)
        s = start[blk] + (torch.rand(k, dtype=torch.float64, device=device, generator=gen) * sizes[blk]).to(torch.int64)
        intra = torch.rand(k, dtype=torch.float64, device=device, generator=gen) < p_intra
        d_in = start[blk] + (torch.rand(k, dtype=torch.float64, device=device, generator=gen) * sizes[blk]).to(torch.int64)
        # uniform over the nodes outside the block: draw in [0, n - size) and skip over the block
        off = (torch.rand(k, dtype=torch.float64, device=device, generator=gen) * (n - sizes[blk])).to(torch.int64)
        d_out = torch.where(off >= start[blk], off + sizes[blk], off)
        return s, torch.where(intra, d_in, d_out).clamp_(max=n - 1)

    keys = torch.empty(0, dtype=torch.int64, device=device)
    need = m
    for _ in range(64):
        s, d = draw_pairs(int(need * 1.1) + 1024)
        ok = s != d
        keys = torch.unique(torch.cat([keys, s[ok] * n + d[ok]]))
        if keys.numel() >= m:
            break
        need = m - keys.numel()
    if keys.numel() > m:
        keys = _systematic_subset(keys, m)
    src, dst = keys // n, keys % n
    if shuffle:
        src, dst = shuffle_ids(src, dst, n, seed + 7919)
    return src, dst


def cap_in_degree(src, dst, n, cap):
    """Drop the in-edges of any destination beyond its first `cap` in sorted source order."""
    _log("capping in-degrees at %d" % cap)
    key = dst * n + src
    key, _ = torch.sort(key)
    deg = torch.bincount(key // n, minlength=n)
    first = torch.cumsum(deg, 0) - deg                      # first edge of every destination
    rank = torch.arange(key.numel(), device=key.device) - torch.repeat_interleave(first, deg)
    key = key[rank < cap]
    return key % n, key // n


def build_csr(src, dst, n, indptr_dtype=torch.int64):
    """CSR keyed by destination, rows sorted by source id.  Returns (indptr[n+1], indices[E] int32)."""
    _log("building CSR of %d edges" % src.numel())
    key = dst.to(torch.int64) * n + src.to(torch.int64)
    key, _ = torch.sort(key)
    indices = (key % n).to(torch.int32)
    deg = torch.bincount(key // n, minlength=n)
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=key.device)
    torch.cumsum(deg, 0, out=indptr[1:])
    return indptr.to(indptr_dtype), indices


def normal_features(n, d, seed, device="cpu", dtype=torch.float32):
    x = torch.randn(n, d, dtype=torch.float32, device=device, generator=_gen(seed, device))
    return x.to(dtype)


def xavier_uniform(fan_in, fan_out, seed, device="cpu", shape=None):
    """U(-a, a), a = sqrt(6 / (fan_in + fan_out)), gain 1; shape defaults to [fan_in, fan_out]."""
    a = math.sqrt(6.0 / (fan_in + fan_out))
    shape = shape or (fan_in, fan_out)
    u = torch.rand(*shape, dtype=torch.float32, device=device, generator=_gen(seed, device))
    return (u * 2.0 - 1.0) * a
