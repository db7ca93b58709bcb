"""GPU parity for layer-wise inference with host-resident embeddings (Algorithm 2 with Section 4.1's batch
controller): every layer matrix lives in pinned host memory, batches load their input sets.  Compared with the
CPU oracle element by element; the transfer statistics are checked against a direct count."""
import numpy as np
import pytest
import torch

from dgi_inputs import generators as G
from oracle import oracle
from tests.helpers import max_rel_err, random_csr

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


def B():
    from paper_2211_15082_amd import binding
    return binding


def rnd(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def pinned(a, dtype=torch.float32):
    t = torch.empty(a.shape, dtype=dtype, pin_memory=True)
    t.copy_(torch.from_numpy(a).to(dtype))
    return t


def model(kind):
    if kind == "sage":
        return [dict(agg="mean", act="relu", W_self=rnd((32, 48), 2, 0.2), W_neigh=rnd((32, 48), 3, 0.2), bias=rnd((48,), 4)),
                dict(agg="sum", act="relu", W_self=rnd((48, 24), 5, 0.1), W_neigh=rnd((48, 24), 6, 0.1), bias=None),
                dict(agg="mean", act="none", W_self=rnd((24, 16), 7, 0.2), W_neigh=rnd((24, 16), 8, 0.2), bias=rnd((16,), 9))]
    if kind == "gcn":
        return [dict(agg="gcn", act="relu", W_neigh=rnd((32, 64), 2, 0.2), bias=rnd((64,), 4)),
                dict(agg="gcn", act="none", W_neigh=rnd((64, 16), 5, 0.2), bias=None)]
    if kind == "gat":
        return [dict(agg="gat", act="elu", W_neigh=rnd((32, 32), 2, 0.3), heads=2, attn_src=rnd((2, 16), 3, 0.5),
                     attn_dst=rnd((2, 16), 4, 0.5), bias=rnd((32,), 5)),
                dict(agg="gat", act="none", W_neigh=rnd((32, 16), 6, 0.3), heads=1, attn_src=rnd((1, 16), 7, 0.5),
                     attn_dst=rnd((1, 16), 8, 0.5), bias=None)]
    raise ValueError(kind)


def input_rows_by_hand(indptr, indices, ends):
    """sum over batches [b, e) of |[b, e) + sources of the batch's edges|"""
    total, b = 0, 0
    for e in ends:
        src = np.unique(indices[indptr[b]:indptr[e]])
        total += np.union1d(src, np.arange(b, e)).size
        b = e
    return total


@pytest.mark.parametrize("kind", ["sage", "gcn", "gat"])
def test_host_resident_inference_matches_the_oracle(kind):
    bd = B()
    n = 5000
    indptr, indices = random_csr(n, 4.0, seed=17, hub=(40, 2500))
    X = rnd((n, 32), 1)
    layers = model(kind)
    want = oracle.infer(indptr, indices, layers, X)
    g = bd.graph_load(indptr, indices)
    structs, keep = zip(*[bd.make_layer(L) for L in layers])
    x = pinned(X)
    # fixed batches of 700 rows: 8 batches per layer, input sets counted by hand
    out = torch.full((n, 16), 777.0, dtype=torch.float32, pin_memory=True)
    st = bd.infer_host(g, list(structs), x, out, batch_size=700, stream_always=True)
    assert max_rel_err(out.numpy(), want) <= TOL_F32
    ends = list(range(700, n, 700)) + [n]
    assert st["batches"] == [len(ends)] * len(layers)
    assert st["input_rows"] == [input_rows_by_hand(indptr, indices, ends)] * len(layers)
    assert st["input_bytes"][0] == st["input_rows"][0] * 32 * 4
    assert st["output_bytes"][-1] == n * 16 * 4
    # dynamic batches (Eq. 2) under a budget that cannot hold the graph at once
    out2 = torch.full((n, 16), 777.0, dtype=torch.float32, pin_memory=True)
    st2 = bd.infer_host(g, list(structs), x, out2, mem_budget_bytes=2_400_000, init_node_threshold=64, stream_always=True)
    assert max_rel_err(out2.numpy(), want) <= TOL_F32
    # (launch overheads dominate batches this small, so the library keeps two of them in flight: M is half the budget)
    assert st2["slots"] == 2
    # (later layers start from the thresholds the previous layer settled on, rescaled by the row width, so a layer
    # with narrow rows may need fewer batches)
    assert st2["batches"][0] >= 3 and sum(st2["batches"]) >= 5, st2["batches"]
    assert st2["peak_batch_bytes"] <= st2["budget_bytes"] == 1_200_000 // 256 * 256
    # a layer that multiplies first and whose transformed rows are clearly narrower than its input rows runs as a dense
    # pass over all rows plus batches that load the transformed rows: GCN 64 -> 16 (Z is 16 wide) and GAT 32 -> 16 with
    # one head (Z = [z | e_l | e_r] is 18 wide); GraphSAGE 48 -> 24 and 24 -> 16, whose batches gather the z_neigh block
    # only (24 and 16 wide) and read z_self for their own rows
    dense = {"sage": [0, n * (48 + 48) * 4, n * (24 + 32) * 4], "gcn": [0, n * (64 + 16) * 4], "gat": [0, n * (32 + 18) * 4]}[kind]
    assert st2["transform_bytes"] == dense and st["transform_bytes"] == [0] * len(layers)
    if kind == "gcn":
        assert st2["input_bytes"][1] == st2["input_rows"][1] * 16 * 4
    if kind == "sage":   # z_neigh rows of the input sets + z_self rows of the destination rows
        assert st2["input_bytes"][1] == (st2["input_rows"][1] + n) * 24 * 4
    # hidden layers kept in host memory although a whole layer fits a slot: one batch per layer
    out3 = torch.full((n, 16), 777.0, dtype=torch.float32, pin_memory=True)
    st3 = bd.infer_host(g, list(structs), x, out3, stream_always=True)
    assert max_rel_err(out3.numpy(), want) <= TOL_F32
    assert st3["batches"] == [1] * len(layers) and st3["input_rows"] == [n] * len(layers)
    # ample memory: one copy in, the device-resident schedule, one copy out
    out4 = torch.full((n, 16), 777.0, dtype=torch.float32, pin_memory=True)
    st4 = bd.infer_host(g, list(structs), x, out4)
    assert max_rel_err(out4.numpy(), want) <= TOL_F32
    assert st4["device_resident"] == 1 and st4["input_bytes"] == [n * 32 * 4] + [0] * (len(layers) - 1)
    assert st3["device_resident"] == 0 and st["device_resident"] == 0


def test_host_output_columns_beyond_the_layer_width_are_left_alone():
    # out_host as the first 47 columns of a 48-column pinned matrix (the library's device buffers pad 47 to 48 as well):
    # column 47 belongs to the caller and must keep its contents, in the device-resident shortcut and when streaming
    bd = B()
    n = 3000
    indptr, indices = random_csr(n, 4.0, seed=29)
    X = rnd((n, 32), 1)
    layers = [dict(agg="mean", act="relu", W_self=rnd((32, 64), 2, 0.2), W_neigh=rnd((32, 64), 3, 0.2), bias=rnd((64,), 4)),
              dict(agg="mean", act="none", W_self=rnd((64, 47), 5, 0.2), W_neigh=rnd((64, 47), 6, 0.2), bias=None)]
    want = oracle.infer(indptr, indices, layers, X)
    g = bd.graph_load(indptr, indices)
    structs, keep = zip(*[bd.make_layer(L) for L in layers])
    x = pinned(X)
    for kw in (dict(), dict(stream_always=True), dict(stream_always=True, batch_size=500)):
        wide = torch.full((n, 48), 777.0, dtype=torch.float32, pin_memory=True)
        bd.infer_host(g, list(structs), x, wide[:, :47], **kw)
        assert max_rel_err(wide[:, :47].numpy(), want) <= TOL_F32, kw
        assert bool((wide[:, 47] == 777.0).all()), kw


def test_host_resident_thresholds_are_halved_when_a_batch_does_not_fit():
    bd = B()
    n = 4000
    indptr, indices = random_csr(n, 5.0, seed=23)
    X = rnd((n, 64), 1)
    layers = [dict(agg="mean", act="relu", W_self=rnd((64, 64), 2, 0.1), W_neigh=rnd((64, 64), 3, 0.1), bias=None),
              dict(agg="mean", act="none", W_self=rnd((64, 8), 4, 0.1), W_neigh=rnd((64, 8), 5, 0.1), bias=None)]
    want = oracle.infer(indptr, indices, layers, X)
    g = bd.graph_load(indptr, indices)
    structs, keep = zip(*[bd.make_layer(L) for L in layers])
    out = torch.empty((n, 8), dtype=torch.float32, pin_memory=True)
    # the first planned batch is the whole graph (about 2.5 MB): it has to be halved a few times to fit a 250 KB slot
    st = bd.infer_host(g, list(structs), pinned(X), out, mem_budget_bytes=500_000, init_node_threshold=n, init_edge_threshold=10**9)
    assert st["oom_retries"] >= 2 and st["peak_batch_bytes"] <= st["budget_bytes"] == 250_000 // 256 * 256
    assert max_rel_err(out.numpy(), want) <= TOL_F32
    # a destination row whose own input set (about 2,100 distinct sources x 256 bytes) exceeds the budget
    indptr_h, indices_h = random_csr(n, 5.0, seed=23, hub=(5, 3000))
    gh = bd.graph_load(indptr_h, indices_h)
    with pytest.raises(bd.DgiError) as ei:
        bd.infer_host(gh, list(structs), pinned(X), out, mem_budget_bytes=200_000)
    assert ei.value.status == bd.ERR_OOM


def test_host_resident_bf16_and_argument_checks():
    bd = B()
    n = 3000
    indptr, indices = random_csr(n, 6.0, seed=29)
    X = torch.from_numpy(rnd((n, 64), 1)).to(torch.bfloat16)
    Ws, Wn = [torch.from_numpy(rnd((64, 64), s, 0.1)).to(torch.bfloat16).float().numpy() for s in (2, 3)]
    W2s, W2n = [torch.from_numpy(rnd((64, 24), s, 0.1)).to(torch.bfloat16).float().numpy() for s in (4, 5)]
    layers = [dict(agg="mean", act="relu", W_self=Ws, W_neigh=Wn, bias=None, out_storage="bf16"),
              dict(agg="mean", act="none", W_self=W2s, W_neigh=W2n, bias=None, out_storage="f32")]
    want = oracle.infer(indptr, indices, layers, X.float().numpy())
    g = bd.graph_load(indptr, indices)
    structs, keep = zip(*[bd.make_layer(L, feat_dtype="bf16") for L in layers])
    x = torch.empty((n, 64), dtype=torch.bfloat16, pin_memory=True)
    x.copy_(X)
    out = torch.empty((n, 24), dtype=torch.float32, pin_memory=True)
    st = bd.infer_host(g, list(structs), x, out, batch_size=1000, stream_always=True)
    assert st["batches"] == [3, 3]
    assert max_rel_err(out.numpy(), want) <= TOL_BF16
    # a budget that forces several batches: the 64 -> 24 layer then runs as a dense pass ([z_self | z_neigh] is 48 wide,
    # three quarters of its input) plus batches that load rows of Z, stored in bf16 like the device-resident path's Z
    out_b = torch.empty((n, 24), dtype=torch.float32, pin_memory=True)
    st_b = bd.infer_host(g, list(structs), x, out_b, mem_budget_bytes=600_000, stream_always=True)
    assert max_rel_err(out_b.numpy(), want) <= TOL_BF16
    assert st_b["transform_bytes"] == [0, n * (64 + 48) * 2] and min(st_b["batches"]) >= 2
    # an empty graph is a no-op
    g0 = bd.graph_load(np.zeros(1, np.int64), np.zeros(0, np.int32))
    st0 = bd.infer_host(g0, list(structs), torch.empty((0, 64), dtype=torch.bfloat16, pin_memory=True),
                        torch.empty((0, 24), dtype=torch.float32, pin_memory=True))
    assert st0["batches"] == [0, 0]
    # pageable host memory and device memory are refused
    with pytest.raises(bd.DgiError) as ei:
        bd.infer_host(g, list(structs), X.clone(), out)
    assert ei.value.status == bd.ERR_INVALID_ARG
    with pytest.raises(bd.DgiError) as ei:
        bd.infer_host(g, list(structs), x.cuda(), out)
    assert ei.value.status == bd.ERR_INVALID_ARG


def test_reordering_shrinks_the_input_sets_of_fixed_batches():
    # Section 4.2: with node ids that follow the graph's locality, the batches of consecutive ids share inputs.
    # A block graph (90 % of the edges inside blocks of ~400 nodes) with shuffled ids, then renumbered by BFS/RCM.
    bd = B()
    n, m = 40_000, 400_000
    src, dst = G.sbm_power_law_blocks(n, 100, m, 0.9, 5, "cpu")
    shuffle = torch.from_numpy(np.random.default_rng(1).permutation(n))
    indptr, indices = G.build_csr(shuffle[src], shuffle[dst], n, torch.int32)
    layers = [dict(agg="mean", act="none", W_self=rnd((16, 16), 2, 0.2), W_neigh=rnd((16, 16), 3, 0.2), bias=None)]
    structs, keep = zip(*[bd.make_layer(L) for L in layers])
    X = rnd((n, 16), 1)
    g = bd.graph_load(indptr.cuda(), indices.cuda())
    out = torch.empty((n, 16), dtype=torch.float32, pin_memory=True)
    st = bd.infer_host(g, list(structs), pinned(X), out, batch_size=2000, stream_always=True)
    g2, perm = bd.graph_reorder(g, "bfs_rcm", seed=0)
    p = perm.cpu().numpy()
    X2 = np.empty_like(X)
    X2[p] = X
    out2 = torch.empty((n, 16), dtype=torch.float32, pin_memory=True)
    st2 = bd.infer_host(g2, list(structs), pinned(X2), out2, batch_size=2000, stream_always=True)
    assert max_rel_err(out2.numpy()[p], out.numpy()) <= TOL_F32          # the same model output, row for row
    assert st2["input_rows"][0] < 0.85 * st["input_rows"][0], (st["input_rows"], st2["input_rows"])


def test_exactly_sized_page_locked_buffers_from_the_library():
    # dgi_host_alloc / dgi_host_free behind binding.pinned_empty: accepted by dgi_infer_host like torch's pinned tensors
    import gc
    bd = B()
    n = 2000
    indptr, indices = random_csr(n, 5.0, seed=41)
    X = rnd((n, 48), 1)
    layers = [dict(agg="mean", act="relu", W_self=rnd((48, 32), 2, 0.2), W_neigh=rnd((48, 32), 3, 0.2), bias=rnd((32,), 4)),
              dict(agg="gcn", act="none", W_neigh=rnd((32, 8), 5, 0.2), bias=None)]
    want = oracle.infer(indptr, indices, layers, X)
    g = bd.graph_load(indptr, indices)
    structs, keep = zip(*[bd.make_layer(L) for L in layers])
    x = bd.pinned_empty((n, 48), torch.float32)
    x.copy_(torch.from_numpy(X))
    out = bd.pinned_empty((n, 8), torch.float32)
    out.fill_(777.0)
    st = bd.infer_host(g, list(structs), x, out, mem_budget_bytes=700_000, stream_always=True)
    assert st["device_resident"] == 0 and max_rel_err(out.numpy(), want) <= TOL_F32
    view = out[:10]          # a view keeps the block alive after the first tensor object is gone
    del out
    gc.collect()
    assert max_rel_err(view.numpy(), want[:10]) <= TOL_F32
    del view, x
    gc.collect()
