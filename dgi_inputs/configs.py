"""The five benchmark configurations as seeded synthetic inputs.

`make_config(k, scale=1.0, device=...)` returns a dict with the CSR (torch tensors on `device`), the
input features and a list of layer dicts (weights as torch tensors on `device`).  `scale` < 1 shrinks
node and edge counts by that factor with identical generator parameters (used for cases the CPU oracle
must finish in seconds).  Layer dicts use the vocabulary of the oracle wrapper and the GPU binding:
agg / act / W_self / W_neigh / bias / heads / attn_src / attn_dst / attn_slope / out_storage.
"""
import torch

from . import generators as G

SEEDS = {1: (1001, 2001, 3001), 2: (1002, 2002, 3002), 3: (1002, 2002, 3003), 4: (1004, 2004, 3004),
         5: (1005, 2005, 3005)}


def _sage_layers(dims, seed, device, storage="f32", agg="mean"):
    layers = []
    for l in range(len(dims) - 1):
        last = l == len(dims) - 2
        Ws = G.xavier_uniform(dims[l], dims[l + 1], seed + 10 * l, device)
        Wn = G.xavier_uniform(dims[l], dims[l + 1], seed + 10 * l + 1, device)
        if storage == "bf16":
            Ws, Wn = Ws.to(torch.bfloat16).float(), Wn.to(torch.bfloat16).float()
        layers.append(dict(agg=agg, act="none" if last else "relu", W_self=Ws, W_neigh=Wn,
                           bias=torch.zeros(dims[l + 1], device=device), heads=1,
                           out_storage="f32" if last else storage))
    return layers


def _gcn_layers(dims, seed, device):
    layers = []
    for l in range(len(dims) - 1):
        last = l == len(dims) - 2
        layers.append(dict(agg="gcn", act="none" if last else "relu", W_self=None,
                           W_neigh=G.xavier_uniform(dims[l], dims[l + 1], seed + 10 * l, device),
                           bias=torch.zeros(dims[l + 1], device=device), heads=1, out_storage="f32"))
    return layers


def _gat_layers(spec, in_dim, seed, device):
    """spec: list of (heads, head_dim).  ELU between layers (the usual GAT choice; the paper does not say),
    no activation after the last."""
    layers = []
    d = in_dim
    for l, (heads, f) in enumerate(spec):
        last = l == len(spec) - 1
        layers.append(dict(agg="gat", act="none" if last else "elu", act_slope=1.0, W_self=None,
                           W_neigh=G.xavier_uniform(d, heads * f, seed + 10 * l, device),
                           attn_src=G.xavier_uniform(f, 1, seed + 10 * l + 1, device, shape=(heads, f)),
                           attn_dst=G.xavier_uniform(f, 1, seed + 10 * l + 2, device, shape=(heads, f)),
                           attn_slope=0.2, bias=torch.zeros(heads * f, device=device), heads=heads,
                           out_storage="f32"))
        d = heads * f
    return layers


def products_like_graph(scale, device, indptr_dtype=torch.int64):
    """Symmetrised Chung-Lu graph, exponent 2.2, with self-loops: 2.4 M nodes, 62 M undirected pairs
    (124 M directed edges) + 2.4 M loops at scale 1; largest expected degree capped at 20,000·sqrt(scale)."""
    n = max(64, int(2_400_000 * scale))
    pairs = max(128, int(62_000_000 * scale))
    src, dst = G.chung_lu_undirected(n, pairs, 2.2, SEEDS[2][0], device,
                                     max_expected_degree=max(50.0, 20000.0 * scale ** 0.5))
    indptr, indices = G.build_csr(src, dst, n, indptr_dtype)
    return n, indptr, indices


def make_config(k, scale=1.0, device="cpu", verbose=False):
    G.VERBOSE = verbose
    gs, fs, ws = SEEDS[k]
    if k == 1:
        n, m = max(64, int(10_000 * scale)), max(128, int(100_000 * scale))
        src, dst = G.chung_lu_directed(n, m, 2.1, gs, device)
        indptr, indices = G.build_csr(src, dst, n, torch.int32)
        x = G.normal_features(n, 64, fs, device)
        layers = _sage_layers([64, 64, 16], ws, device)
        name = "cfg1 GraphSAGE-mean 64-64-16"
    elif k in (2, 3):
        n, indptr, indices = products_like_graph(scale, device, torch.int32)
        x = G.normal_features(n, 100, fs, device)
        if k == 2:
            layers = _gcn_layers([100, 256, 256, 47], ws, device)
            name = "cfg2 GCN 100-256-256-47"
        else:
            layers = _gat_layers([(4, 64), (1, 47)], 100, ws, device)
            name = "cfg3 GAT 100-(4x64)-(1x47)"
    elif k == 4:
        n, m = max(64, int(111_000_000 * scale)), max(128, int(1_600_000_000 * scale))
        cap = max(50, int(50_000 * scale ** 0.5))
        src, dst = G.chung_lu_directed(n, m, 2.0, gs, device, max_expected_degree=float(cap))
        src, dst = G.cap_in_degree(src, dst, n, cap)
        indptr, indices = G.build_csr(src, dst, n, torch.int64)
        del src, dst
        G._log("features")
        x = G.normal_features(n, 128, fs, device, torch.bfloat16)
        layers = _sage_layers([128, 128, 128, 172], ws, device, storage="bf16")
        name = "cfg4 GraphSAGE-mean bf16 128-128-128-172"
    elif k == 5:
        n, m = max(256, int(20_000_000 * scale)), max(512, int(400_000_000 * scale))
        blocks = max(4, int(2000 * scale ** 0.5))
        src, dst = G.sbm_power_law_blocks(n, blocks, m, 0.9, gs, device)
        indptr, indices = G.build_csr(src, dst, n, torch.int32 if m < 2**31 - 1 else torch.int64)
        x = G.normal_features(n, 256, fs, device)
        layers = _sage_layers([256, 256, 64], ws, device)
        name = "cfg5 GraphSAGE-mean 256-256-64 (SBM)"
    else:
        raise ValueError(k)
    return dict(name=name, num_nodes=n, indptr=indptr, indices=indices, x=x, layers=layers, scale=scale)


def to_numpy_layers(layers):
    out = []
    for L in layers:
        out.append({k: (v.detach().cpu().numpy() if isinstance(v, torch.Tensor) else v) for k, v in L.items()})
    return out
