"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its host-only
planning helpers (batching rule and Eq. 2 of Section 4.1, input-set counting and reordering of
Section 4.2) behave as the paper states.  No device call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2211_15082_amd import binding as B
from tests.helpers import random_csr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dgi.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dgi_[a-z_0-9]+)\s*\(", header))
    assert {"dgi_graph_load", "dgi_layer_forward", "dgi_infer"} <= declared
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert set(B.EXPORTS) == declared
    assert B.version() == 1
    assert B._status_string(B.ERR_BAD_GRAPH) == "malformed graph"


def test_struct_sizes_match_header_layout():
    # natural alignment of the C structs in dgi.h
    assert ctypes.sizeof(B.LayerStruct) == 9 * 4 + 4 + 5 * 8 + 4 + 4
    assert ctypes.sizeof(B.OptsStruct) == 7 * 8
    assert ctypes.sizeof(B.StatsStruct) == 8 + 8 + 16 * (8 * 8 + 4 * 3) + 16
    assert ctypes.sizeof(B.GraphInfoStruct) == 5 * 8 + 8 + 8
    assert ctypes.sizeof(B.HostStatsStruct) == 8 + 8 + 16 * 8 * 8 + 4 * 8


def brute_batch_end(ip, limit, begin, n_t, n_i):
    end = begin + 1
    while end < limit and end + 1 - begin <= n_t and ip[end + 1] - ip[begin] <= n_i:
        end += 1
    return end


@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_batch_end_matches_linear_scan(dtype):
    indptr, _ = random_csr(500, 6.0, seed=1)
    indptr[301:] += 400  # one heavy row (row 300)
    ip = indptr.astype(dtype)
    rng = np.random.default_rng(0)
    for _ in range(300):
        begin = int(rng.integers(0, 500))
        n_t = int(rng.integers(1, 80))
        n_i = int(rng.integers(0, 300))
        assert B.plan_batch_end(ip, 500, begin, n_t, n_i) == brute_batch_end(indptr, 500, begin, n_t, n_i)


def test_batches_respect_both_thresholds_and_cover_all_rows():
    indptr, _ = random_csr(2000, 8.0, seed=2)
    n_t, n_i = 64, 300
    b, rows = 0, 0
    while b < 2000:
        e = B.plan_batch_end(indptr, 2000, b, n_t, n_i)
        assert b < e <= 2000 and e - b <= n_t
        edges = indptr[e] - indptr[b]
        assert edges <= n_i or e - b == 1  # a row heavier than n_i forms a batch by itself
        rows += e - b
        b = e
    assert rows == 2000


def test_eq2_threshold_update_and_oom_halving():
    # r = M / M_k: half of the expected memory used => both thresholds double
    assert B.threshold_update(1000.0, 500.0, 64, 4096) == (128, 8192)
    assert B.threshold_update(900.0, 1800.0, 64, 4096) == (32, 2048)
    assert B.threshold_update(1000.0, 1000.0, 7, 9) == (7, 9)
    assert B.threshold_update(1.0, 1e9, 5, 5) == (1, 1)       # never below one
    assert B.threshold_update(1000.0, 0.0, 5, 6) == (5, 6)    # nothing measured: unchanged
    # out of memory: halve both
    assert B.threshold_halve(64, 4097) == (32, 2048)
    assert B.threshold_halve(1, 9) == (1, 4)
    with pytest.raises(B.DgiError) as ei:
        B.threshold_halve(1, 1)
    assert ei.value.status == B.ERR_OOM


def toy_graph():
    """The toy graph of the paper's Figure 2 / Section 4.2 example: A and B both have in-neighbours
    {C, D}; C has in-neighbours {E, F}.  (The figure does not show in-edges of D; it has none here.)
    ids: A=0 B=1 C=2 D=3 E=4 F=5."""
    rows = [[2, 3], [2, 3], [4, 5], [], [], []]
    indptr = np.zeros(7, dtype=np.int64)
    np.cumsum([len(r) for r in rows], out=indptr[1:])
    return indptr, np.array([u for r in rows for u in r], dtype=np.int32)


def test_input_set_of_the_papers_toy_batches():
    indptr, indices = toy_graph()
    assert B.batch_input_set_size(indptr, indices, 0, 2) == 2   # batch {A, B} needs C, D
    # batch {A, C}: renumber so that A and C are consecutive: order A, C, B, D, E, F
    perm = np.array([0, 2, 1, 3, 4, 5], dtype=np.int32)  # new id of old id
    rows_new = [[], [], [], [], [], []]
    for old in range(6):
        rows_new[perm[old]] = sorted(perm[indices[indptr[old]:indptr[old + 1]]])
    ip2 = np.zeros(7, dtype=np.int64)
    np.cumsum([len(r) for r in rows_new], out=ip2[1:])
    ix2 = np.array([u for r in rows_new for u in r], dtype=np.int32)
    assert B.batch_input_set_size(ip2, ix2, 0, 2) == 4           # batch {A, C} needs C, D, E, F
    assert B.batch_input_set_size(indptr, indices, 0, 6) == 4
    assert B.batch_input_set_size(indptr, indices, 3, 6) == 0


@pytest.mark.parametrize("method", ["degree", "bfs_rcm", "random", "none", "community"])
def test_reorder_permutation_is_a_bijection(method):
    indptr, indices = random_csr(300, 4.0, seed=3)
    perm = B.reorder_permutation(indptr, indices, method, seed=7)
    assert sorted(perm.tolist()) == list(range(300))
    if method == "degree":
        deg = np.diff(indptr)
        order = np.argsort(perm)
        assert (np.diff(deg[order]) <= 0).all()
    if method == "none":
        assert (perm == np.arange(300)).all()
    if method == "random":
        assert (B.reorder_permutation(indptr, indices, method, seed=7) == perm).all()
        assert (B.reorder_permutation(indptr, indices, method, seed=8) != perm).any()


def _total_inputs(indptr, indices, perm, batch):
    n = indptr.size - 1
    old_of_new = np.argsort(perm)
    total = 0
    for b in range(0, n, batch):
        olds = old_of_new[b:b + batch]
        total += np.unique(np.concatenate([indices[indptr[o]:indptr[o + 1]] for o in olds] + [np.zeros(0, np.int32)])).size
    return total


def test_bfs_order_shares_inputs_on_a_community_graph():
    # 40 communities of 50 nodes, ids shuffled: batches of consecutive BFS ids should need far fewer
    # distinct inputs than batches of shuffled ids (the effect Section 4.2 is after)
    rng = np.random.default_rng(5)
    n, comm = 2000, 50
    shuffle = rng.permutation(n)
    inv = np.argsort(shuffle)
    rows = []
    for new_id in range(n):
        orig = inv[new_id]
        c = orig // comm
        nb = rng.choice(np.arange(c * comm, (c + 1) * comm), size=8, replace=False)
        rows.append(np.sort(shuffle[nb]))
    indptr = np.arange(0, 8 * n + 1, 8, dtype=np.int64)
    indices = np.concatenate(rows).astype(np.int32)
    ident = np.arange(n, dtype=np.int32)
    rcm = B.reorder_permutation(indptr, indices, "bfs_rcm")
    assert _total_inputs(indptr, indices, rcm, 50) < 0.5 * _total_inputs(indptr, indices, ident, 50)


def test_community_order_keeps_planted_communities_contiguous():
    # 30 planted communities of 40..100 nodes, 12 in-edges per node, one in eight of them leaving the community, ids
    # shuffled: label propagation leaves one label per community (a stray node with mostly outside neighbours aside), so
    # a community occupies a contiguous id range and batches of consecutive ids read far fewer distinct inputs than
    # with the shuffled ids or the BFS order
    rng = np.random.default_rng(11)
    sizes = rng.integers(40, 101, 30)
    start = np.concatenate([[0], np.cumsum(sizes)])
    n = int(start[-1])
    comm = np.repeat(np.arange(30), sizes)
    shuffle = rng.permutation(n)          # shuffled id of original node i
    rows = [None] * n
    for i in range(n):
        c = comm[i]
        nb = rng.choice(np.arange(start[c], start[c + 1]), size=12, replace=False)
        out = rng.random(12) < 0.125
        nb[out] = rng.integers(0, n, int(out.sum()))
        rows[shuffle[i]] = np.sort(shuffle[nb])
    indptr = np.arange(0, 12 * n + 1, 12, dtype=np.int64)
    indices = np.concatenate(rows).astype(np.int32)
    perm = B.reorder_permutation(indptr, indices, "community")
    assert sorted(perm.tolist()) == list(range(n))
    new_of_orig = perm[shuffle]
    runs = []
    for c in range(30):
        ids = np.sort(new_of_orig[start[c]:start[c + 1]])
        runs.append(1 + int((np.diff(ids) > 1).sum()))   # contiguous id ranges the community falls into
    assert sum(r == 1 for r in runs) >= 27 and max(runs) <= 3, runs
    ident = np.arange(n, dtype=np.int32)
    rcm = B.reorder_permutation(indptr, indices, "bfs_rcm")
    t_comm, t_rcm, t_id = (_total_inputs(indptr, indices, p_, 64) for p_ in (perm, rcm, ident))
    assert t_comm < 0.5 * t_id and t_comm < t_rcm


def test_rcm_on_a_path_is_the_path():
    # path 0-1-2-...-9 with ids scrambled: Cuthill-McKee from an end walks the path; reversed order keeps
    # neighbours adjacent
    order = np.array([3, 7, 0, 9, 4, 1, 8, 2, 6, 5])
    n = 10
    rows = [[] for _ in range(n)]
    for i in range(n - 1):
        a, b = order[i], order[i + 1]
        rows[a].append(b)
        rows[b].append(a)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum([len(r) for r in rows], out=indptr[1:])
    indices = np.array([u for r in rows for u in sorted(r)], dtype=np.int32)
    perm = B.reorder_permutation(indptr, indices, "bfs_rcm")
    pos = perm[order]
    assert (np.abs(np.diff(pos)) == 1).all()


def test_argument_validation_fails_before_any_device_work():
    # these calls must be rejected by host-side checks alone (this test runs without a GPU)
    lib = ctypes.CDLL(B.LIB_PATH)
    h = ctypes.c_void_p()
    ip = np.zeros(3, dtype=np.int64)
    args = lambda n, e, p: (ctypes.c_int64(n), ctypes.c_int64(e), p, ctypes.c_int32(B.I64), None, ctypes.c_int32(B.HOST), None, ctypes.byref(h))
    assert lib.dgi_graph_load(*args(-1, 0, ip.ctypes.data_as(ctypes.c_void_p))) == B.ERR_INVALID_ARG
    assert lib.dgi_graph_load(*args(2, 0, None)) == B.ERR_INVALID_ARG
    assert lib.dgi_graph_load(*args(2, 5, ip.ctypes.data_as(ctypes.c_void_p))) == B.ERR_INVALID_ARG   # indices NULL with edges
    assert "indices" in B.last_error()
    assert lib.dgi_graph_free(None) == B.OK
    assert lib.dgi_infer(None, None, 1, None, 0, None, 0, None, None) == B.ERR_INVALID_ARG
    assert lib.dgi_layer_forward(None, None, None, 0, None, 0, 0, 0, None, 0, None) == B.ERR_INVALID_ARG
    assert lib.dgi_infer_partial(None, None, 1, None, 0, None, 0, None, 0, None, None, None) == B.ERR_INVALID_ARG
    assert lib.dgi_infer_host(None, None, 1, None, 0, None, 0, None, None, None) == B.ERR_INVALID_ARG
    assert lib.dgi_host_alloc(ctypes.c_uint64(64), None) == B.ERR_INVALID_ARG
    assert lib.dgi_host_free(None) == B.OK
    assert lib.dgi_graph_sample(None, 10, ctypes.c_uint64(1), 0, None, None) == B.ERR_INVALID_ARG
    assert lib.dgi_infer_sampled(None, None, 1, None, 0, None, 0, 10, ctypes.c_uint64(1), None, None) == B.ERR_INVALID_ARG
    with pytest.raises(B.DgiError) as ei:
        B.plan_batch_end(np.zeros(4, np.int64), 3, 5, 1, 1)
    assert ei.value.status == B.ERR_INVALID_ARG and "begin" in str(ei.value)
    assert lib.dgi_reorder_permutation(ctypes.c_int64(2), None, None, 1, ctypes.c_uint64(0), None) == B.ERR_INVALID_ARG


def test_public_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, with no C++ or HIP types in it
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "dgi.h"\nint main(void) { dgi_infer_opts_t o; dgi_host_stats_t h; (void)o; (void)h; return (int)sizeof(dgi_layer_t) == 0; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), "-fsyntax-only", str(src)], check=True)
