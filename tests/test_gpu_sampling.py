"""GPU parity for sampling inference (Section 2): the device sampler against the oracle's, bit for bit, and the
sampled layer-wise inference against the oracle element by element."""
import numpy as np
import pytest
import torch

from oracle import oracle, sampler
from tests.helpers import max_rel_err, random_csr

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4


def B():
    from paper_2211_15082_amd import binding
    return binding


def rnd(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


@pytest.mark.parametrize("itype", [np.int32, np.int64])
def test_device_sampler_equals_the_oracle_sampler(itype):
    bd = B()
    n = 3000
    indptr, indices = random_csr(n, 9.0, seed=31, hub=(17, 40_000))   # one row far beyond a wavefront's 64 lanes
    g = bd.graph_load(indptr.astype(itype), indices)
    for fanout, seed, layer in ((1, 5, 0), (10, 5, 0), (10, 5, 3), (10, 2**64 - 3, 1), (64, 9, 0), (65, 9, 2), (100_000, 1, 0)):
        gs = bd.graph_sample(g, fanout, seed, layer)
        ip, ix = gs.csr()
        want_ip, want_ix = sampler.sample_csr(indptr, indices, fanout, seed, layer)
        assert np.array_equal(ip, want_ip), (fanout, seed, layer)
        assert np.array_equal(ix, want_ix), (fanout, seed, layer)
        assert gs.info()["max_in_degree"] == min(fanout, 40_000)
        gs.free()
    with pytest.raises(bd.DgiError):
        bd.graph_sample(g, 0, 1, 0)
    g0 = bd.graph_load(np.zeros(1, np.int64), np.zeros(0, np.int32))
    assert bd.graph_sample(g0, 10, 1, 0).info()["num_nodes"] == 0
    # a graph without edges, and sampling inference on an empty graph
    g1 = bd.graph_load(np.zeros(6, np.int64), np.zeros(0, np.int32))
    assert bd.graph_sample(g1, 10, 1, 0).info()["num_edges"] == 0
    ls, keep = bd.make_layer(dict(agg="mean", act="none", W_self=rnd((4, 4), 1), W_neigh=rnd((4, 4), 2), bias=None))
    bd.infer_sampled(g0, [ls], torch.empty(0, 4, device="cuda"), torch.empty(0, 4, device="cuda"), 10, 1)
    x1 = torch.ones(5, 4, device="cuda")
    o1 = torch.empty(5, 4, device="cuda")
    bd.infer_sampled(g1, [ls], x1, o1, 10, 1)   # no neighbours: out = x W_self
    assert np.allclose(o1.cpu().numpy(), np.ones((5, 4), np.float32) @ rnd((4, 4), 1), rtol=1e-5)


@pytest.mark.parametrize("kind", ["sage", "gcn", "gat"])
def test_sampling_inference_matches_the_oracle(kind):
    bd = B()
    n = 5000
    indptr, indices = random_csr(n, 14.0, seed=33, hub=(2, 3000))
    X = rnd((n, 32), 1)
    if kind == "sage":
        layers = [dict(agg="mean", act="relu", W_self=rnd((32, 48), 2, 0.2), W_neigh=rnd((32, 48), 3, 0.2), bias=rnd((48,), 4)),
                  dict(agg="sum", act="relu", W_self=rnd((48, 24), 5, 0.1), W_neigh=rnd((48, 24), 6, 0.1), bias=None),
                  dict(agg="mean", act="none", W_self=rnd((24, 16), 7, 0.2), W_neigh=rnd((24, 16), 8, 0.2), bias=rnd((16,), 9))]
    elif kind == "gcn":
        layers = [dict(agg="gcn", act="relu", W_neigh=rnd((32, 64), 2, 0.2), bias=rnd((64,), 4)),
                  dict(agg="gcn", act="relu", W_neigh=rnd((64, 64), 5, 0.2), bias=None),
                  dict(agg="gcn", act="none", W_neigh=rnd((64, 16), 6, 0.2), bias=None)]
    else:
        layers = [dict(agg="gat", act="elu", W_neigh=rnd((32, 32), 2, 0.3), heads=2, attn_src=rnd((2, 16), 3, 0.5),
                       attn_dst=rnd((2, 16), 4, 0.5), bias=rnd((32,), 5)),
                  dict(agg="gat", act="none", W_neigh=rnd((32, 16), 6, 0.3), heads=1, attn_src=rnd((1, 16), 7, 0.5),
                       attn_dst=rnd((1, 16), 8, 0.5), bias=None)]
    g = bd.graph_load(indptr, indices)
    structs, keep = zip(*[bd.make_layer(L) for L in layers])
    x = torch.from_numpy(X).cuda()
    out = torch.full((n, 16), 777.0, dtype=torch.float32, device="cuda")
    for fanout, seed in ((10, 7), (3, 8)):
        want = oracle.infer_sampled(indptr, indices, layers, X, fanout, seed)
        bd.infer_sampled(g, list(structs), x, out, fanout, seed, batch_size=0 if fanout == 10 else 1500)
        assert max_rel_err(out.cpu().numpy(), want) <= TOL_F32, (kind, fanout)
    # a fan-out that covers every row is full inference
    bd.infer_sampled(g, list(structs), x, out, 3000, 1)
    full = torch.empty_like(out)
    bd.infer(g, list(structs), x, full)
    assert max_rel_err(out.cpu().numpy(), full.cpu().numpy()) <= TOL_F32
    assert max_rel_err(out.cpu().numpy(), oracle.infer(indptr, indices, layers, X)) <= TOL_F32
