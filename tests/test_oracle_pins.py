"""Pins of the CPU oracle against things that are not the oracle: dense-adjacency algebra written with
numpy matrices, a library sparse product, brute-force node-wise recursion (Algorithm 1), closed forms
and invariants.  The paper prints no worked numeric example, so no value here is quoted from it."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import oracle
from tests.helpers import act_np, dense_adjacency, random_csr

TOL = 1e-6  # the oracle stores float32; its double arithmetic is checked to float32 rounding


def rnd(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def sage_dense(A, X, Ws, Wn, b, act, agg):
    """Dense-adjacency form: act(X Ws + D^-1 A X Wn + b) (mean) or with A alone (sum)."""
    X = X.astype(np.float64)
    M = A @ X
    if agg == "mean":
        deg = A.sum(1, keepdims=True)
        M = np.where(deg > 0, M / np.maximum(deg, 1.0), 0.0)
    out = M @ Wn.astype(np.float64) + b
    if Ws is not None:
        out = out + X @ Ws.astype(np.float64)
    return act_np(out, act)


def gcn_dense(A, X, W, b, act):
    d_in = np.maximum(A.sum(1), 1.0)
    d_out = np.maximum(A.sum(0), 1.0)
    An = A / np.sqrt(d_in)[:, None] / np.sqrt(d_out)[None, :]
    return act_np(An @ X.astype(np.float64) @ W.astype(np.float64) + b, act)


def gat_dense(A, X, W, a_src, a_dst, heads, slope, b, act, act_slope=1.0):
    n = A.shape[0]
    Z = X.astype(np.float64) @ W.astype(np.float64)
    F = Z.shape[1] // heads
    out = np.zeros_like(Z)
    for h in range(heads):
        Zh = Z[:, h * F:(h + 1) * F]
        el = Zh @ a_src[h].astype(np.float64)
        er = Zh @ a_dst[h].astype(np.float64)
        S = er[:, None] + el[None, :]          # S[v, u]
        S = np.where(S > 0, S, slope * S)
        S = np.where(A > 0, S, -np.inf)
        with np.errstate(invalid="ignore"):
            mx = S.max(1, keepdims=True)
            P = np.where(A > 0, A * np.exp(S - mx), 0.0)   # multiplicity counts repeated edges
            den = P.sum(1, keepdims=True)
            alpha = np.where(den > 0, P / np.where(den > 0, den, 1.0), 0.0)
        out[:, h * F:(h + 1) * F] = alpha @ Zh
    return act_np(out + b, act, act_slope)


@pytest.mark.parametrize("agg", ["sum", "mean"])
@pytest.mark.parametrize("act", ["none", "relu"])
def test_sage_matches_dense_adjacency(agg, act):
    indptr, indices = random_csr(48, 3.0, seed=11)
    A = dense_adjacency(indptr, indices)
    assert (A.sum(1) == 0).any() and A.max() >= 2  # has empty rows and a repeated edge
    X, Ws, Wn, b = rnd((48, 7), 1), rnd((7, 5), 2), rnd((7, 5), 3), rnd((5,), 4)
    got = oracle.layer_forward(indptr, indices, dict(agg=agg, act=act, W_self=Ws, W_neigh=Wn, bias=b), X)
    np.testing.assert_allclose(got, sage_dense(A, X, Ws, Wn, b, act, agg), rtol=TOL, atol=TOL)
    got = oracle.layer_forward(indptr, indices, dict(agg=agg, act=act, W_self=None, W_neigh=Wn, bias=None), X)
    np.testing.assert_allclose(got, sage_dense(A, X, None, Wn, 0.0, act, agg), rtol=TOL, atol=TOL)


def test_gcn_matches_dense_adjacency():
    indptr, indices = random_csr(40, 4.0, seed=5)
    A = dense_adjacency(indptr, indices)
    assert not np.allclose(A, A.T)  # directed: d_out(source) and d_in(destination) differ
    X, W, b = rnd((40, 6), 7), rnd((6, 9), 8), rnd((9,), 9)
    got = oracle.layer_forward(indptr, indices, dict(agg="gcn", act="relu", W_neigh=W, bias=b), X)
    np.testing.assert_allclose(got, gcn_dense(A, X, W, b, "relu"), rtol=TOL, atol=TOL)


@pytest.mark.parametrize("heads", [1, 2, 4])
def test_gat_matches_dense_masked_softmax(heads):
    indptr, indices = random_csr(36, 3.5, seed=21)
    A = dense_adjacency(indptr, indices)
    F = 3
    X, W, b = rnd((36, 5), 1), rnd((5, heads * F), 2), rnd((heads * F,), 3)
    a_s, a_d = rnd((heads, F), 4), rnd((heads, F), 5)
    layer = dict(agg="gat", act="elu", act_slope=1.0, W_neigh=W, bias=b, heads=heads, attn_src=a_s, attn_dst=a_d,
                 attn_slope=0.2)
    got = oracle.layer_forward(indptr, indices, layer, X)
    np.testing.assert_allclose(got, gat_dense(A, X, W, a_s, a_d, heads, 0.2, b, "elu"), rtol=TOL, atol=TOL)


def test_identity_weights_reduce_to_library_spmm():
    # W_neigh = I, no self term, no bias, no activation, SUM  =>  output = A X (CSR times dense)
    indptr, indices = random_csr(200, 6.0, seed=3)
    n, d = 200, 12
    X = rnd((n, d), 17)
    A = sp.csr_matrix((np.ones(indices.size), indices, indptr), shape=(n, n))  # duplicates add up
    got = oracle.layer_forward(indptr, indices, dict(agg="sum", act="none", W_neigh=np.eye(d, dtype=np.float32)), X)
    np.testing.assert_allclose(got, A @ X.astype(np.float64), rtol=TOL, atol=TOL)


def test_transposed_weight_would_fail():
    # h W with W [in x out] row-major: a rectangular W pins the operand order
    indptr, indices = random_csr(10, 2.0, seed=2, empty_frac=0.0)
    X = rnd((10, 3), 1)
    W = np.arange(6, dtype=np.float32).reshape(3, 2)
    got = oracle.layer_forward(indptr, indices, dict(agg="sum", act="none", W_self=W, W_neigh=np.zeros((3, 2), np.float32)), X)
    np.testing.assert_allclose(got, X.astype(np.float64) @ W, rtol=TOL, atol=TOL)


# ---- node-wise inference (Algorithm 1): recursive descent from the raw features, no memoisation ----
def nodewise(v, l, indptr, indices, layers, X, d_out):
    if l == 0:
        return X[v].astype(np.float64)
    L = layers[l - 1]
    nb = indices[indptr[v]:indptr[v + 1]]
    K = L["W_neigh"].shape[0]
    m = np.zeros(K)
    for u in nb:
        hu = nodewise(int(u), l - 1, indptr, indices, layers, X, d_out)
        c = 1.0 / np.sqrt(max(d_out[u], 1) * max(nb.size, 1)) if L["agg"] == "gcn" else 1.0
        m += c * hu
    if L["agg"] == "mean" and nb.size:
        m /= nb.size
    s = m @ L["W_neigh"].astype(np.float64) + (L["bias"] if L.get("bias") is not None else 0.0)
    if L.get("W_self") is not None:
        s = s + nodewise(v, l - 1, indptr, indices, layers, X, d_out) @ L["W_self"].astype(np.float64)
    return act_np(s, L["act"])


@pytest.mark.parametrize("agg", ["mean", "gcn"])
def test_layerwise_equals_nodewise(agg):
    # Section 2: both schemes produce the same output embedding
    indptr, indices = random_csr(30, 2.0, seed=9)
    d_out = np.bincount(indices, minlength=30)
    dims = [4, 5, 3, 2]
    layers = []
    for l in range(3):
        layers.append(dict(agg=agg, act="relu" if l < 2 else "none", W_neigh=rnd((dims[l], dims[l + 1]), 10 + l),
                           W_self=None if agg == "gcn" else rnd((dims[l], dims[l + 1]), 20 + l),
                           bias=rnd((dims[l + 1],), 30 + l)))
    X = rnd((30, 4), 99)
    got = oracle.infer(indptr, indices, layers, X)
    want = np.stack([nodewise(v, 3, indptr, indices, layers, X, d_out) for v in range(30)])
    # hidden layers are stored in float32 by the layer-wise oracle, the recursion stays in double
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=2e-6)


def test_one_layer_model_is_the_layer():
    indptr, indices = random_csr(25, 3.0, seed=4)
    X = rnd((25, 6), 5)
    layer = dict(agg="mean", act="relu", W_self=rnd((6, 4), 1), W_neigh=rnd((6, 4), 2), bias=rnd((4,), 3))
    np.testing.assert_array_equal(oracle.infer(indptr, indices, [layer], X),
                                  oracle.layer_forward(indptr, indices, layer, X))


def relabel(indptr, indices, perm_new_of_old):
    n = indptr.size - 1
    old_of_new = np.argsort(perm_new_of_old)
    rows = [np.sort(perm_new_of_old[indices[indptr[o]:indptr[o + 1]]]) for o in old_of_new]
    ip = np.zeros(n + 1, dtype=np.int64)
    np.cumsum([r.size for r in rows], out=ip[1:])
    return ip, np.concatenate(rows).astype(np.int32)


@pytest.mark.parametrize("agg", ["mean", "gcn", "gat"])
def test_permutation_equivariance(agg):
    # renumbering nodes (Section 4.2) only renumbers the output rows
    n = 60
    indptr, indices = random_csr(n, 3.0, seed=13)
    perm = np.random.default_rng(5).permutation(n).astype(np.int32)
    ip2, ix2 = relabel(indptr, indices, perm)
    X = rnd((n, 5), 8)
    X2 = np.empty_like(X)
    X2[perm] = X
    if agg == "gat":
        layers = [dict(agg="gat", act="elu", W_neigh=rnd((5, 6), 1), heads=2, attn_src=rnd((2, 3), 2),
                       attn_dst=rnd((2, 3), 3), bias=rnd((6,), 4)),
                  dict(agg="gat", act="none", W_neigh=rnd((6, 4), 5), heads=1, attn_src=rnd((1, 4), 6),
                       attn_dst=rnd((1, 4), 7), bias=None)]
    else:
        layers = [dict(agg=agg, act="relu", W_self=rnd((5, 6), 1), W_neigh=rnd((5, 6), 2), bias=rnd((6,), 3)),
                  dict(agg=agg, act="none", W_self=rnd((6, 4), 4), W_neigh=rnd((6, 4), 5), bias=None)]
    a = oracle.infer(indptr, indices, layers, X)
    b = oracle.infer(ip2, ix2, layers, X2)
    np.testing.assert_allclose(b[perm], a, rtol=1e-5, atol=1e-6)


def test_constant_features_closed_forms():
    n, d, c = 50, 4, 1.75
    indptr, indices = random_csr(n, 3.0, seed=6)
    deg = np.diff(indptr)
    X = np.full((n, d), c, dtype=np.float32)
    Ws, Wn, b = rnd((d, 3), 1), rnd((d, 3), 2), rnd((3,), 3)
    got = oracle.layer_forward(indptr, indices, dict(agg="mean", act="none", W_self=Ws, W_neigh=Wn, bias=b), X)
    full = c * (Ws.astype(np.float64).sum(0) + Wn.astype(np.float64).sum(0)) + b
    self_only = c * Ws.astype(np.float64).sum(0) + b
    np.testing.assert_allclose(got[deg > 0], np.broadcast_to(full, (int((deg > 0).sum()), 3)), rtol=TOL, atol=TOL)
    np.testing.assert_allclose(got[deg == 0], np.broadcast_to(self_only, (int((deg == 0).sum()), 3)), rtol=TOL, atol=TOL)
    # GAT: the attention weights of a row sum to one, so equal z rows aggregate to that z row
    W = rnd((d, 6), 4)
    layer = dict(agg="gat", act="none", W_neigh=W, heads=2, attn_src=rnd((2, 3), 5), attn_dst=rnd((2, 3), 6), bias=None)
    got = oracle.layer_forward(indptr, indices, layer, X)
    z = c * W.astype(np.float64).sum(0)
    np.testing.assert_allclose(got[deg > 0], np.broadcast_to(z, (int((deg > 0).sum()), 6)), rtol=TOL, atol=TOL)
    np.testing.assert_array_equal(got[deg == 0], 0.0)  # empty neighbourhood: zero vector, no NaN


def test_zero_attention_is_mean_of_projection():
    n = 40
    indptr, indices = random_csr(n, 3.0, seed=8)
    X, W = rnd((n, 5), 1), rnd((5, 8), 2)
    gat = dict(agg="gat", act="none", W_neigh=W, heads=2, attn_src=np.zeros((2, 4), np.float32),
               attn_dst=np.zeros((2, 4), np.float32), bias=None)
    mean = dict(agg="mean", act="none", W_self=None, W_neigh=W, bias=None)
    np.testing.assert_allclose(oracle.layer_forward(indptr, indices, gat, X),
                               oracle.layer_forward(indptr, indices, mean, X), rtol=TOL, atol=TOL)


def test_gcn_on_regular_graph_is_mean():
    # ring with self-loops and both directions: every node has in- and out-degree 3 => 1/sqrt(3*3) = 1/3
    n = 17
    rows = [sorted({(v - 1) % n, v, (v + 1) % n}) for v in range(n)]
    indptr = np.arange(0, 3 * n + 1, 3, dtype=np.int64)
    indices = np.array(rows, dtype=np.int32).ravel()
    X, W, b = rnd((n, 4), 1), rnd((4, 3), 2), rnd((3,), 3)
    gcn = oracle.layer_forward(indptr, indices, dict(agg="gcn", act="none", W_neigh=W, bias=b), X)
    mean = oracle.layer_forward(indptr, indices, dict(agg="mean", act="none", W_self=None, W_neigh=W, bias=b), X)
    np.testing.assert_allclose(gcn, mean, rtol=TOL, atol=TOL)


def test_star_hub_closed_form():
    # destination 0 has 50,000 in-neighbours with features 1, 2, ..., 50000
    k = 50_000
    n = k + 1
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = k
    indices = np.arange(1, n, dtype=np.int32)
    X = np.zeros((n, 2), dtype=np.float32)
    X[1:, 0] = np.arange(1, n)
    X[1:, 1] = 1.0
    I2 = np.eye(2, dtype=np.float32)
    s = oracle.layer_forward(indptr, indices, dict(agg="sum", act="none", W_neigh=I2), X, rows=[0, 1])
    assert s[0, 0] == np.float32(k * (k + 1) / 2) and s[0, 1] == k and (s[1] == 0).all()
    m = oracle.layer_forward(indptr, indices, dict(agg="mean", act="none", W_neigh=I2), X, rows=[0])
    assert m[0, 0] == np.float32((k + 1) / 2) and m[0, 1] == 1.0
    # GCN: d_out(u) = 1 for every source, d_in(0) = k  =>  sum / sqrt(k)
    g = oracle.layer_forward(indptr, indices, dict(agg="gcn", act="none", W_neigh=I2), X, rows=[0])
    np.testing.assert_allclose(g[0], [k * (k + 1) / 2 / np.sqrt(k), k / np.sqrt(k)], rtol=1e-6)


@pytest.mark.parametrize("agg", ["sum", "mean", "gcn"])
def test_linearity_without_activation(agg):
    indptr, indices = random_csr(30, 3.0, seed=12)
    layer = dict(agg=agg, act="none", W_self=rnd((4, 3), 1), W_neigh=rnd((4, 3), 2), bias=rnd((3,), 3))
    X1, X2 = rnd((30, 4), 4), rnd((30, 4), 5)
    f = lambda X: oracle.layer_forward(indptr, indices, layer, X).astype(np.float64)
    np.testing.assert_allclose(f(X1 + X2), f(X1) + f(X2) - f(np.zeros_like(X1)), rtol=1e-5, atol=1e-5)


def test_softmax_stability_and_shift_invariance():
    n = 30
    indptr, indices = random_csr(n, 4.0, seed=14, empty_frac=0.0)
    X = np.abs(rnd((n, 3), 1)) + 0.5
    W = np.abs(rnd((3, 4), 2)) + 0.1          # positive z
    big = dict(agg="gat", act="none", W_neigh=W, heads=1, attn_src=np.full((1, 4), 60.0, np.float32),
               attn_dst=np.full((1, 4), -20.0, np.float32), bias=None)
    out = oracle.layer_forward(indptr, indices, big, X)
    assert np.isfinite(out).all()
    A = dense_adjacency(indptr, indices)
    np.testing.assert_allclose(out, gat_dense(A, X, W, big["attn_src"], big["attn_dst"], 1, 0.2, 0.0, "none"),
                               rtol=1e-5, atol=1e-5)
    # all raw scores positive => LeakyReLU is the identity => adding a constant to every score of a
    # destination (a change of a_dst only) cancels in the softmax
    pos = dict(big, attn_src=np.full((1, 4), 1.0, np.float32), attn_dst=np.full((1, 4), 0.5, np.float32))
    pos2 = dict(pos, attn_dst=np.full((1, 4), 3.0, np.float32))
    np.testing.assert_allclose(oracle.layer_forward(indptr, indices, pos, X),
                               oracle.layer_forward(indptr, indices, pos2, X), rtol=1e-5, atol=1e-6)


def test_leaky_relu_score_slope_matters():
    # two in-neighbours with scores of opposite sign: closed-form two-way softmax
    indptr = np.array([0, 2, 2, 2], dtype=np.int64)
    indices = np.array([1, 2], dtype=np.int32)
    X = np.array([[0.0], [2.0], [-3.0]], dtype=np.float32)
    layer = dict(agg="gat", act="none", W_neigh=np.ones((1, 1), np.float32), heads=1,
                 attn_src=np.ones((1, 1), np.float32), attn_dst=np.zeros((1, 1), np.float32), attn_slope=0.2, bias=None)
    out = oracle.layer_forward(indptr, indices, layer, X)
    e1, e2 = 2.0, 0.2 * -3.0
    a1 = np.exp(e1) / (np.exp(e1) + np.exp(e2))
    np.testing.assert_allclose(out[0, 0], a1 * 2.0 + (1 - a1) * -3.0, rtol=1e-6)


def test_activations_and_bias_closed_values():
    indptr = np.array([0, 0], dtype=np.int64)
    indices = np.zeros(0, dtype=np.int32)
    X = np.array([[1.0]], dtype=np.float32)
    W = np.array([[-2.0, 3.0]], dtype=np.float32)
    b = np.array([0.5, -0.5], dtype=np.float32)
    base = dict(agg="sum", W_self=W, W_neigh=np.zeros((1, 2), np.float32), bias=b)
    np.testing.assert_allclose(oracle.layer_forward(indptr, indices, dict(base, act="none"), X), [[-1.5, 2.5]])
    np.testing.assert_allclose(oracle.layer_forward(indptr, indices, dict(base, act="relu"), X), [[0.0, 2.5]])
    np.testing.assert_allclose(oracle.layer_forward(indptr, indices, dict(base, act="leaky_relu", act_slope=0.1), X), [[-0.15, 2.5]])
    np.testing.assert_allclose(oracle.layer_forward(indptr, indices, dict(base, act="elu", act_slope=1.0), X),
                               [[np.expm1(-1.5), 2.5]], rtol=1e-6)


def test_bf16_storage_rounds_to_nearest_even():
    # identity layer on an isolated node: output = bf16(x).  1+2^-8 is a tie -> 1 (even); 1+3*2^-8 is a
    # tie -> 1+2^-6 (even mantissa); 1+2^-8+2^-12 is above the tie -> 1+2^-7.
    indptr = np.array([0, 0], dtype=np.int64)
    indices = np.zeros(0, dtype=np.int32)
    xs = np.array([[1 + 2.0**-8, 1 + 3 * 2.0**-8, 1 + 2.0**-8 + 2.0**-12, -(1 + 3 * 2.0**-8), 0.0, 3.0e-5]], dtype=np.float32)
    I = np.eye(6, dtype=np.float32)
    out = oracle.layer_forward(indptr, indices, dict(agg="sum", act="none", W_self=I, W_neigh=I, out_storage="bf16"), xs)
    want = [1.0, 1 + 2.0**-6, 1 + 2.0**-7, -(1 + 2.0**-6), 0.0]
    np.testing.assert_array_equal(out[0, :5], np.array(want, dtype=np.float32))
    import torch
    np.testing.assert_array_equal(out[0], torch.from_numpy(xs[0]).to(torch.bfloat16).float().numpy())
    # every output of a bf16-stored layer is representable in bfloat16
    ip, ix = random_csr(40, 3.0, seed=2)
    o = oracle.layer_forward(ip, ix, dict(agg="mean", act="relu", W_self=rnd((5, 7), 1), W_neigh=rnd((5, 7), 2),
                                          out_storage="bf16"), rnd((40, 5), 3))
    np.testing.assert_array_equal(o, torch.from_numpy(o).to(torch.bfloat16).float().numpy())


def test_rows_argument_selects_rows():
    indptr, indices = random_csr(50, 3.0, seed=15)
    X = rnd((50, 4), 1)
    layer = dict(agg="gcn", act="relu", W_neigh=rnd((4, 3), 2), bias=rnd((3,), 3))
    full = oracle.layer_forward(indptr, indices, layer, X)
    rows = [49, 0, 7, 7, 23]
    np.testing.assert_array_equal(oracle.layer_forward(indptr, indices, layer, X, rows=rows), full[rows])


def test_empty_graph_and_empty_rows():
    layer = dict(agg="mean", act="relu", W_self=rnd((3, 2), 1), W_neigh=rnd((3, 2), 2), bias=None)
    out = oracle.layer_forward(np.zeros(1, np.int64), np.zeros(0, np.int32), layer, np.zeros((0, 3), np.float32))
    assert out.shape == (0, 2)


def test_jumping_knowledge_stack_matches_dense_algebra():
    # JKNet (the paper's appendix example): the last layer reads the concatenation of all earlier layer outputs
    indptr, indices = random_csr(40, 3.0, seed=31)
    A = dense_adjacency(indptr, indices)
    X = rnd((40, 6), 1)
    l1 = dict(agg="mean", act="relu", W_self=rnd((6, 8), 2), W_neigh=rnd((6, 8), 3), bias=rnd((8,), 4))
    l2 = dict(agg="mean", act="relu", W_self=rnd((8, 4), 5), W_neigh=rnd((8, 4), 6), bias=rnd((4,), 7))
    l3 = dict(agg="gcn", act="none", W_neigh=rnd((12, 5), 8), bias=rnd((5,), 9))
    h1 = sage_dense(A, X, l1["W_self"], l1["W_neigh"], l1["bias"], "relu", "mean")
    h2 = sage_dense(A, h1.astype(np.float32), l2["W_self"], l2["W_neigh"], l2["bias"], "relu", "mean")
    want = gcn_dense(A, np.concatenate([h1, h2], axis=1).astype(np.float32), l3["W_neigh"], l3["bias"], "none")
    got = oracle.infer_jk(indptr, indices, [l1, l2, l3], X)
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=1e-5)


def test_error_report_figures_on_a_hand_made_case():
    # the parity metric and the two un-gated figures reported beside it
    from tests.helpers import error_report
    want = np.array([[3.0, -4.0], [0.0, 1e-6]])
    got = np.array([[3.0003, -4.0], [1e-5, 2e-6]])
    rep = error_report(got, want)
    rms = np.sqrt((9 + 16 + 0 + 1e-12) / 4)
    # floored: largest of 3e-4/3, 0/4, 1e-5/rms, 1e-6/rms
    assert abs(rep["max_rel_floored"] - 1e-4) < 1e-9 and 1e-5 / rms < 1e-4
    assert abs(rep["max_abs"] - 3e-4) < 1e-12
    # un-floored over the non-zero expected values: {1e-4, 0, 1.0}; the 99.9th percentile sits just under the max
    assert 0.99 < rep["p999_rel_unfloored"] <= 1.0
