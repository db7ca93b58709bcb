"""dgi_layer_forward_static (the entry point that allocates nothing: its workspace is a static device array) against
dgi_layer_forward on the same inputs.  Both run the same kernels, so the outputs must be bit-equal; the oracle is
compared as well.  Two calls in a row share the array: the second, smaller one must not see the first one's leftovers."""
import numpy as np
import pytest
import torch

from oracle import oracle
from tests.helpers import max_rel_err, random_csr

pytestmark = pytest.mark.gpu


def _rnd(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def _case(bd, n, d_in, d_out, agg, order, seed, hub=None, storage="f32"):
    indptr, indices = random_csr(n, 6.0, seed=seed, hub=hub)
    X = _rnd((n, d_in), seed + 1)
    layer = dict(agg=agg, act="relu", order=order, W_neigh=_rnd((d_in, d_out), seed + 2, 0.2), bias=_rnd((d_out,), seed + 3))
    if agg in ("sum", "mean"):
        layer["W_self"] = _rnd((d_in, d_out), seed + 4, 0.2)
    if agg == "gat":
        layer.update(heads=2, attn_src=_rnd((2, d_out // 2), seed + 5, 0.3), attn_dst=_rnd((2, d_out // 2), seed + 6, 0.3), order="auto")
    g = bd.graph_load(indptr, indices)
    ls, keep = bd.make_layer(layer, feat_dtype=storage)
    dt = torch.bfloat16 if storage == "bf16" else torch.float32
    x = torch.from_numpy(X).cuda().to(dt)
    return dict(g=g, ls=ls, keep=keep, x=x, indptr=indptr, indices=indices, layer=layer, X=x.float().cpu().numpy(), n=n, d_out=d_out)


def _run_both(bd, c, b, e, check_mem=True):
    ref = torch.full((c["n"], c["d_out"]), 777.0, dtype=torch.float32, device="cuda")
    got = torch.full((c["n"], c["d_out"]), 777.0, dtype=torch.float32, device="cuda")
    bd.layer_forward(c["g"], c["ls"], c["x"], ref, b, e)
    free_before = torch.cuda.mem_get_info()[0]
    bd.layer_forward_static(c["g"], c["ls"], c["x"], got, b, e)
    torch.cuda.synchronize()
    # the call takes no device memory (the first use of the static array on a device is exempt: the HIP runtime
    # materialises a code object's device variables when their address is first looked up)
    assert not check_mem or torch.cuda.mem_get_info()[0] == free_before
    assert torch.equal(ref, got)
    want = oracle.layer_forward(c["indptr"], c["indices"], c["layer"], c["X"])
    tol = 2e-2 if c["x"].dtype == torch.bfloat16 else 1e-4
    assert max_rel_err(got[b:e].cpu().numpy(), want[b:e]) <= tol
    assert bool((got[:b] == 777.0).all()) and bool((got[e:] == 777.0).all())


@pytest.mark.parametrize("agg,order", [("mean", "agg_first_split"), ("mean", "agg_first_fused"), ("gcn", "transform_first"),
                                       ("sum", "transform_first"), ("gat", "auto")])
def test_static_workspace_call_equals_layer_forward_twice_in_a_row(agg, order):
    from paper_2211_15082_amd import binding as bd
    big = _case(bd, 3000, 192, 64, agg, order, seed=11, hub=(5, 2500))     # hub partials, several tiles, ragged tail
    small = _case(bd, 333, 64, 32, agg, order, seed=23)                    # smaller input right after: no leftovers seen
    _run_both(bd, big, 0, 3000, check_mem=False)
    _run_both(bd, small, 7, 301)
    _run_both(bd, big, 1000, 2999)


def test_static_workspace_bf16_and_size_limit():
    from paper_2211_15082_amd import binding as bd
    c = _case(bd, 2000, 128, 128, "mean", "agg_first_split", seed=31, storage="bf16")
    _run_both(bd, c, 0, 2000, check_mem=False)
    _run_both(bd, c, 100, 1999)
    # a transform-first layer keeps the transformed rows of all N nodes in the workspace: 200,000 x 64 floats > 32 MiB
    n = 200_000
    indptr = np.arange(n + 1, dtype=np.int64)
    indices = np.zeros(n, dtype=np.int32)
    g = bd.graph_load(indptr, indices)
    layer = dict(agg="gcn", act="none", order="transform_first", W_neigh=_rnd((128, 64), 1, 0.2), bias=None)
    ls, keep = bd.make_layer(layer)
    assert bd.layer_workspace_bytes(g, ls, 0, n) > bd.STATIC_WORKSPACE_BYTES
    x = torch.zeros(n, 128, device="cuda")
    out = torch.zeros(n, 64, device="cuda")
    with pytest.raises(bd.DgiError) as ei:
        bd.layer_forward_static(g, ls, x, out, 0, n)
    assert ei.value.status == bd.ERR_UNSUPPORTED and "static workspace" in str(ei.value)
