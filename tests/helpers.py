"""Small test-only helpers: tiny random CSR graphs (with duplicates and empty rows) and the error metric."""
import numpy as np


def random_csr(n, avg_deg, seed, empty_frac=0.2, duplicates=True, hub=None):
    """Poisson in-degrees, uniform sources; hub=(row, degree) plants one high-degree destination."""
    rng = np.random.default_rng(seed)
    deg = rng.poisson(avg_deg, n)
    deg[rng.random(n) < empty_frac] = 0
    if hub is not None:
        deg[hub[0]] = hub[1]
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


def error_report(got, want):
    """The three figures every parity report states: the gated one (max relative error with the RMS floor of
    max_rel_err), and, for information, the 99.9th percentile of the un-floored element-wise relative error over
    the non-zero expected values and the largest absolute error."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return dict(max_rel_floored=0.0, p999_rel_unfloored=0.0, max_abs=0.0)
    diff = np.abs(got - want)
    nz = want != 0
    p999 = float(np.percentile(diff[nz] / np.abs(want[nz]), 99.9)) if nz.any() else 0.0
    return dict(max_rel_floored=max_rel_err(got, want), p999_rel_unfloored=p999, max_abs=float(diff.max()))


def format_error_report(r):
    return ("max |g-o|/max(|o|, RMS(o)) = %.3e, 99.9th percentile of |g-o|/|o| = %.3e, max |g-o| = %.3e"
            % (r["max_rel_floored"], r["p999_rel_unfloored"], r["max_abs"]))


def act_np(x, act, slope=1.0):
    if act == "relu":
        return np.maximum(x, 0.0)
    if act == "elu":
        return np.where(x > 0, x, slope * np.expm1(np.minimum(x, 0)))
    if act == "leaky_relu":
        return np.where(x > 0, x, slope * x)
    return x


# ---- node-wise evaluation of sampled targets on a big graph (Algorithm 1, with the per-layer target sets
# V^l of Section 3.3): only index plumbing lives here, the arithmetic is the oracle's. ---------------------
def _gather_rows(indptr, indices, rows):
    """Concatenated in-neighbour lists of `rows` (torch tensors, any device) and the per-row counts."""
    import torch
    start = indptr[rows].to(torch.int64)
    cnt = indptr[rows + 1].to(torch.int64) - start
    total = int(cnt.sum())
    if total == 0:
        return indices.new_empty(0, dtype=torch.int64), cnt
    seg_first = torch.cumsum(cnt, 0) - cnt
    pos = torch.arange(total, device=indptr.device) - torch.repeat_interleave(seg_first, cnt)
    return indices[torch.repeat_interleave(start, cnt) + pos].to(torch.int64), cnt


def nodewise_oracle(indptr, indices, x, layers_np, targets, num_layers, x_is_bf16=False):
    """Final-layer rows of `targets`, computed by the CPU oracle from the targets' L-hop in-neighbourhood
    only.  indptr / indices / x: torch tensors of the FULL graph (on the GPU for the big configs);
    layers_np: numpy layer dicts.  Works for aggregators that use no global out-degree (sum, mean, gat)."""
    import numpy as np
    import torch
    from oracle import oracle
    dev = indptr.device
    n = indptr.numel() - 1
    targets = torch.as_tensor(targets, dtype=torch.int64, device=dev)
    # need[l] = nodes whose layer-l embedding is required; need[L] = targets, need[l-1] = need[l] ∪ N(need[l])
    need = [None] * (num_layers + 1)
    need[num_layers] = torch.unique(targets)
    for l in range(num_layers, 0, -1):
        nb, _ = _gather_rows(indptr, indices, need[l])
        need[l - 1] = torch.unique(torch.cat([need[l], nb]))
    U = need[0]                                   # sorted global ids of every node touched
    # sub-CSR over U: rows of need[1] are complete (all their in-neighbours are in U); other rows are empty
    interior = need[1]
    nb, cnt = _gather_rows(indptr, indices, interior)
    deg = torch.zeros(U.numel(), dtype=torch.int64, device=dev)
    deg[torch.searchsorted(U, interior)] = cnt
    sub_indptr = torch.zeros(U.numel() + 1, dtype=torch.int64, device=dev)
    torch.cumsum(deg, 0, out=sub_indptr[1:])
    # rows are written in ascending local id == ascending global id == the order of `interior`
    sub_indices = torch.searchsorted(U, nb).to(torch.int32)
    ip, ix = sub_indptr.cpu().numpy(), sub_indices.cpu().numpy()
    h = x[U].float().cpu().numpy()
    for l in range(1, num_layers + 1):
        rows_local = torch.searchsorted(U, need[l]).cpu().numpy()
        part = oracle.layer_forward(ip, ix, layers_np[l - 1], h, rows=rows_local)
        if l == num_layers:
            full = {int(g): part[i] for i, g in enumerate(need[l].cpu().numpy())}
            return np.stack([full[int(t)] for t in targets.cpu().numpy()])
        nxt = np.zeros((U.numel(), part.shape[1]), dtype=np.float32)
        nxt[rows_local] = part
        h = nxt
