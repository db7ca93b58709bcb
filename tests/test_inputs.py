"""The synthetic input generators: structure checks (no inference arithmetic here)."""
import numpy as np
import torch

from dgi_inputs import configs, generators as G


def _check_csr(indptr, indices, n):
    ip, ix = indptr.cpu().numpy().astype(np.int64), indices.cpu().numpy()
    assert ip[0] == 0 and ip[-1] == ix.size and (np.diff(ip) >= 0).all()
    assert ix.size == 0 or (ix.min() >= 0 and ix.max() < n)
    for v in range(0, n, max(1, n // 50)):
        row = ix[ip[v]:ip[v + 1]]
        assert (np.diff(row) > 0).all()  # sorted, deduplicated
    return ip, ix


def test_chung_lu_directed_counts_and_seed():
    src, dst = G.chung_lu_directed(5000, 40000, 2.1, seed=1)
    assert src.numel() == 40000 and (src != dst).all()
    assert torch.unique(src * 5000 + dst).numel() == 40000
    s2, d2 = G.chung_lu_directed(5000, 40000, 2.1, seed=1)
    assert torch.equal(src, s2) and torch.equal(dst, d2)
    indeg = torch.bincount(dst, minlength=5000)
    assert indeg.max() > 20 * indeg.float().mean()  # heavy tail


def test_undirected_is_symmetric_with_loops():
    n = 3000
    src, dst = G.chung_lu_undirected(n, 20000, 2.2, seed=2, max_expected_degree=300.0)
    assert src.numel() == 2 * 20000 + n
    k1 = torch.sort(src * n + dst)[0]
    k2 = torch.sort(dst * n + src)[0]
    assert torch.equal(k1, k2)
    indptr, indices = G.build_csr(src, dst, n)
    ip, ix = _check_csr(indptr, indices, n)
    assert all(v in ix[ip[v]:ip[v + 1]] for v in range(0, n, 97))
    assert np.diff(ip).max() < 3 * 300


def test_sbm_intra_fraction():
    n, blocks, m = 20000, 20, 100000
    src, dst = G.sbm_power_law_blocks(n, blocks, m, 0.9, seed=3, shuffle=False)
    assert src.numel() == m and (src != dst).all()
    r = torch.arange(1, blocks + 1, dtype=torch.float64)
    # recompute the block of each endpoint from the (unshuffled) layout
    w = r.pow(-1.0)
    floor = max(1, n // (blocks * 20))
    sizes = torch.floor(w / w.sum() * (n - floor * blocks)).to(torch.int64) + floor
    sizes[0] += n - int(sizes.sum())
    ends = torch.cumsum(sizes, 0)
    bs, bd = torch.searchsorted(ends, src, right=True), torch.searchsorted(ends, dst, right=True)
    frac = float((bs == bd).double().mean())
    assert 0.85 < frac < 0.95


def test_cap_in_degree():
    src, dst = G.chung_lu_directed(2000, 30000, 2.0, seed=4)
    s2, d2 = G.cap_in_degree(src, dst, 2000, 40)
    assert torch.bincount(d2, minlength=2000).max() <= 40
    assert s2.numel() < src.numel()


def test_configs_small_scale():
    for k, scale in [(1, 0.1), (2, 0.0005), (3, 0.0005), (4, 0.00002), (5, 0.0002)]:
        c = configs.make_config(k, scale=scale)
        _check_csr(c["indptr"], c["indices"], c["num_nodes"])
        assert c["x"].shape == (c["num_nodes"], c["layers"][0]["W_neigh"].shape[0])
        for a, b in zip(c["layers"][:-1], c["layers"][1:]):
            assert a["W_neigh"].shape[1] == b["W_neigh"].shape[0]


def test_xavier_bounds():
    w = G.xavier_uniform(100, 256, seed=5)
    a = (6.0 / 356) ** 0.5
    assert w.shape == (100, 256) and w.abs().max() <= a and w.abs().max() > 0.95 * a
    assert abs(float(w.mean())) < 0.01
