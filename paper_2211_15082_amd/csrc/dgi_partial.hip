// Partial inference (Sections 2 and 3.3 of the DGI paper): output embeddings for a set of target nodes only.
//
// The per-layer target sets are annotated backwards from the user's targets: V^L = targets, and V^{l-1} =
// V^l plus the in-neighbours of V^l (a node's own previous embedding is an input of Eq. 1 as well).  As soon as
// |V^l| * d_avg >= n the sets below are taken to be all nodes (the paper's shortcut: the next set would hold most
// of the graph anyway): layers 1 .. l-1 then run on the whole graph with the ordinary schedule, and only the inputs
// of layer l, V^l plus its in-neighbours, are marked exactly.  The remaining layers run on a compact sub-problem
// whose nodes are numbered by descending depth (targets first, then V^{L-1} \ V^L, ...): the sets are nested, so
// V^l is the id range [0, |V^l|) there and layer l computes exactly those rows (infer_rows), reading the rows
// [0, |V^{l-1}|) the layer before it wrote.  Degrees in the GCN normaliser stay those of the full graph.
#include <algorithm>
#include <climits>
#include <cstring>

#include "dgi_subproblem.h"

namespace dgi {
namespace {

using namespace subp;

__global__ void mark_targets_kernel(const int32_t* targets, int64_t n, int64_t N, int32_t L, int32_t* depth, int* bad) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t t = targets[i];
        if (t < 0 || t >= N) { *bad = 1; continue; }
        depth[t] = L;  // every writer stores the same value
    }
}

// rows with depth >= l hand depth l-1 to their in-neighbours (one wavefront per row)
template <typename IdxT>
__global__ void expand_depth_kernel(const IdxT* indptr, const int32_t* indices, int64_t N, int32_t l, int32_t* depth) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; v < N; v += waves) {
        if (depth[v] < l) continue;
        const int64_t a = (int64_t)indptr[v], b = (int64_t)indptr[v + 1];
        for (int64_t e = a + lane; e < b; e += 64) atomicMax(&depth[indices[e]], l - 1);
    }
}

__global__ void local_targets_kernel(const int32_t* targets, int64_t n, const int32_t* loc, int32_t* out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) out[i] = loc[targets[i]];
}

// key[i] = L - depth[U[i]]: ascending keys put the targets first
__global__ void depth_keys_kernel(const int32_t* U, int64_t n, const int32_t* depth, int32_t L, int32_t* key) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) key[i] = L - depth[U[i]];
}

__global__ void scatter_positions_kernel(const int32_t* U, int64_t n, int32_t* loc) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) loc[U[i]] = (int32_t)i;
}

template <typename IdxT>
dgi_status_t infer_partial(const dgi_graph* g, const dgi_layer_t* layers, int32_t L, const void* x, int64_t ld_x,
                           const int32_t* targets, int64_t nt, void* out, int64_t ld_out, const dgi_infer_opts_t* opts,
                           dgi_partial_stats_t* ps, hipStream_t s) {
    const int64_t N = g->N;
    const IdxT* indptr = (const IdxT*)g->d_indptr;
    const int yb = layers[L - 1].out_dtype == DGI_BF16 ? 2 : 4;
    const int out_dim = layers[L - 1].out_dim;
    const double d_avg = N > 0 ? (double)g->E / (double)N : 0.0;
    Buf depth, bad;
    Scratch sc;
    DGI_TRY(depth.alloc(N * 4)); DGI_TRY(bad.alloc(4));
    DGI_TRY(sc.alloc(N, s));

    DGI_TRY(launch_fill_zero(bad.p, 4, s));
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(N)), dim3(kBlock), 0, s, depth.as<int32_t>(), N, -1);
    hipLaunchKernelGGL(mark_targets_kernel, dim3(grid_for(nt)), dim3(kBlock), 0, s, targets, nt, N, L, depth.as<int32_t>(), bad.as<int>());
    int h_bad = 0;
    DGI_HIP(hipMemcpyAsync(&h_bad, bad.p, 4, hipMemcpyDeviceToHost, s));
    auto count_level = [&](int32_t l, int64_t* n_out) { return sc.count_level(depth.as<int32_t>(), N, l, n_out, s); };
    int64_t set_size[DGI_MAX_LAYERS + 1] = {};
    DGI_TRY(count_level(L, &set_size[L]));
    DGI_REQUIRE(h_bad == 0, DGI_ERR_INVALID_ARG, "infer_partial: a target id is outside [0, num_nodes)");
    if (ps) { std::memset(ps, 0, sizeof(*ps)); ps->num_layers = L; ps->set_size[L] = set_size[L]; ps->all_nodes_from_layer = -1; }
    // ---- backward annotation of V^{L-1} ... V^{l0}, with the |V^l| * d_avg >= n shortcut -------------------------
    // l0 = number of leading layers that run on all nodes (0 without the shortcut).  The inputs of layer l0 + 1 are
    // marked exactly in either case: they are the node set U of the sub-problem.
    dgi_infer_opts_t o{};
    if (opts) o = *opts;
    o.perm_new_of_old = nullptr;
    o.stats = nullptr;
    int32_t l0 = 0;
    for (int32_t l = L; l >= 1; --l) {
        const bool shortcut = (double)set_size[l] * d_avg >= (double)N;
        hipLaunchKernelGGL(expand_depth_kernel<IdxT>, dim3(grid_for(N * 64)), dim3(kBlock), 0, s, indptr, g->d_indices, N, l, depth.as<int32_t>());
        DGI_TRY(count_level(l - 1, &set_size[l - 1]));
        if (ps) ps->set_size[l - 1] = set_size[l - 1];
        // (with l - 1 == 0 the inputs are rows of x: nothing runs on all nodes; a jumping-knowledge stack is one
        // unit for dgi_infer, so it is never cut)
        if (shortcut && l - 1 >= 1 && !o.jk_concat) {
            l0 = l - 1;
            if (ps) ps->all_nodes_from_layer = l0;
            break;
        }
    }

    // The marked input set holds half of the graph or more: extracting and relabelling a sub-problem of that size costs
    // more than the rows it saves, so every layer runs on the whole graph and the target rows are picked at the end
    // (the shortcut's "all nodes" taken one layer further up).
    if (set_size[l0] * 2 >= N) {
        Buf full;
        const int64_t ld_full = round_up(out_dim, 16 / yb);
        DGI_TRY(full.alloc((size_t)N * ld_full * yb));
        DGI_TRY(dgi_infer(g, layers, L, x, ld_x, full.p, ld_full, &o, s));
        DGI_TRY(launch_permute_rows(full.p, ld_full, out, ld_out, nt, out_dim, yb, targets, true, s));
        DGI_HIP(hipStreamSynchronize(s));
        if (ps) {
            ps->all_nodes_from_layer = L;
            ps->sub_nodes = N; ps->sub_edges = g->E;
            for (int32_t l = 0; l < L; ++l) ps->rows_computed[l] = N;
        }
        return DGI_OK;
    }

    // ---- layers 1 .. l0 on the whole graph (shortcut only) -------------------------------------------------------------
    Buf h_all;
    const void* src = x;
    int64_t ld_src = ld_x;
    if (l0 >= 1) {
        const int hb = layers[l0 - 1].out_dtype == DGI_BF16 ? 2 : 4;
        const int64_t ld_h = round_up(layers[l0 - 1].out_dim, 16 / hb);
        DGI_TRY(h_all.alloc((size_t)N * ld_h * hb));
        DGI_TRY(dgi_infer(g, layers, l0, x, ld_x, h_all.p, ld_h, &o, s));
        src = h_all.p; ld_src = ld_h;
        if (ps) for (int32_t l = 0; l < l0; ++l) ps->rows_computed[l] = N;
    }

    // ---- compact sub-problem over U = V^{l0} for layers l0 + 1 .. L, nodes numbered by descending depth --------------
    const int64_t n_sub = set_size[l0];
    const int32_t Ls = L - l0;
    const dgi_layer_t* sub_layers = layers + l0;
    const int sb = sub_layers[0].feat_dtype == DGI_BF16 ? 2 : 4;
    const int sub_in = sub_layers[0].in_dim;
    Buf U, U2, key, key2, sub_deg, sub_indptr, sub_indices, x_sub, out_sub, tloc, sort_tmp;
    DGI_TRY(U.alloc(n_sub * 4)); DGI_TRY(U2.alloc(n_sub * 4)); DGI_TRY(key.alloc(n_sub * 4)); DGI_TRY(key2.alloc(n_sub * 4));
    DGI_TRY(sub_deg.alloc((n_sub + 1) * 8)); DGI_TRY(sub_indptr.alloc((n_sub + 1) * 8));
    // sc.flag holds (depth >= l0) from the last count_level call: U in ascending id, then a stable sort by depth
    DGI_CUB(hipcub::DeviceSelect::Flagged(sc.tmp.p, sc.tb, hipcub::CountingInputIterator<int32_t>(0), sc.flag.as<int32_t>(), U.as<int32_t>(),
                                          sc.cnt.as<int32_t>(), (int)N, s));
    hipLaunchKernelGGL(depth_keys_kernel, dim3(grid_for(n_sub)), dim3(kBlock), 0, s, U.as<int32_t>(), n_sub, depth.as<int32_t>(), L, key.as<int32_t>());
    size_t stb = 0;
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(nullptr, stb, key.as<int32_t>(), key2.as<int32_t>(), U.as<int32_t>(), U2.as<int32_t>(), (int)n_sub, 0, 6, s));
    DGI_TRY(sort_tmp.alloc(stb));
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(sort_tmp.p, stb, key.as<int32_t>(), key2.as<int32_t>(), U.as<int32_t>(), U2.as<int32_t>(), (int)n_sub, 0, 6, s));
    int32_t* Us = U2.as<int32_t>();   // global id of local node i
    hipLaunchKernelGGL(scatter_positions_kernel, dim3(grid_for(n_sub)), dim3(kBlock), 0, s, Us, n_sub, sc.loc.as<int32_t>());
    // rows of V^{l0+1} keep their in-neighbour lists; the rest of U are inputs only
    hipLaunchKernelGGL(sub_rows_kernel<IdxT>, dim3(grid_for(n_sub)), dim3(kBlock), 0, s, Us, n_sub, indptr, depth.as<int32_t>(), l0 + 1, sub_deg.as<int64_t>());
    DGI_TRY(launch_fill_zero(sub_indptr.p, 8, s));
    DGI_CUB(hipcub::DeviceScan::InclusiveSum(sc.tmp.p, sc.tb, sub_deg.as<int64_t>(), sub_indptr.as<int64_t>() + 1, (int)n_sub, s));
    int64_t e_sub = 0;
    DGI_HIP(hipMemcpyAsync(&e_sub, sub_indptr.as<int64_t>() + n_sub, 8, hipMemcpyDeviceToHost, s));
    DGI_HIP(hipStreamSynchronize(s));
    DGI_TRY(sub_indices.alloc(e_sub * 4));
    GraphGuard sub;
    DGI_TRY(sub_graph<IdxT>(g, sc, n_sub, e_sub, Us, sub_indptr.as<int64_t>(), sub_indices.as<int32_t>(), &sub, s));
    const int64_t ld_xs = round_up(sub_in, 16 / sb), ld_os = round_up(out_dim, 16 / yb);
    int64_t row_limit[DGI_MAX_LAYERS] = {};
    for (int32_t l = 0; l < Ls; ++l) {
        row_limit[l] = set_size[l0 + 1 + l];
        if (ps) ps->rows_computed[l0 + l] = row_limit[l];
    }
    DGI_TRY(x_sub.alloc((size_t)n_sub * ld_xs * sb)); DGI_TRY(out_sub.alloc((size_t)std::max<int64_t>(row_limit[Ls - 1], 1) * ld_os * yb));
    DGI_TRY(tloc.alloc(nt * 4));
    DGI_TRY(launch_permute_rows(src, ld_src, x_sub.p, ld_xs, n_sub, sub_in, sb, Us, true, s));
    {
        // the sub-problem's schedule borrows the full graph's cached arena instead of allocating one of its own
        std::lock_guard<std::mutex> lend(g->ws_mutex);
        sub.g->ws_ptr = g->ws_ptr; sub.g->ws_bytes = g->ws_bytes;
        const dgi_status_t rc = infer_rows(sub.g, sub_layers, Ls, x_sub.p, ld_xs, out_sub.p, ld_os, &o, row_limit, s);
        g->ws_ptr = sub.g->ws_ptr; g->ws_bytes = sub.g->ws_bytes;   // (it may have been replaced by a larger one)
        sub.g->ws_ptr = nullptr; sub.g->ws_bytes = 0;
        DGI_TRY(rc);
    }
    hipLaunchKernelGGL(local_targets_kernel, dim3(grid_for(nt)), dim3(kBlock), 0, s, targets, nt, sc.loc.as<int32_t>(), tloc.as<int32_t>());
    DGI_TRY(launch_permute_rows(out_sub.p, ld_os, out, ld_out, nt, out_dim, yb, tloc.as<int32_t>(), true, s));
    DGI_HIP(hipStreamSynchronize(s));
    if (ps) { ps->sub_nodes = n_sub; ps->sub_edges = e_sub; }
    return DGI_OK;
}

}  // namespace
}  // namespace dgi

using namespace dgi;

extern "C" dgi_status_t dgi_infer_partial(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x,
                                          int64_t ld_x, const int32_t* targets, int64_t num_targets, void* out, int64_t ld_out,
                                          const dgi_infer_opts_t* opts, dgi_partial_stats_t* pstats, void* hip_stream) {
    DGI_REQUIRE(g && layers, DGI_ERR_INVALID_ARG, "infer_partial: NULL argument");
    DGI_REQUIRE(num_layers >= 1 && num_layers < DGI_MAX_LAYERS, DGI_ERR_INVALID_ARG, "infer_partial: bad layer count");
    DGI_REQUIRE(num_targets >= 0 && num_targets < (int64_t)INT_MAX, DGI_ERR_INVALID_ARG, "infer_partial: bad target count");
    DGI_REQUIRE(!(opts && opts->perm_new_of_old), DGI_ERR_UNSUPPORTED, "infer_partial: pass the graph in its own numbering (no permutation)");
    if (pstats) { std::memset(pstats, 0, sizeof(*pstats)); pstats->num_layers = num_layers; pstats->all_nodes_from_layer = -1; }
    if (num_targets == 0 || g->N == 0) return DGI_OK;
    DGI_REQUIRE(targets && x && out, DGI_ERR_INVALID_ARG, "infer_partial: NULL buffer");
    DGI_REQUIRE(ld_x >= layers[0].in_dim && ld_out >= layers[num_layers - 1].out_dim, DGI_ERR_INVALID_ARG, "infer_partial: leading dimension too small");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return g->itype == DGI_I64 ? infer_partial<int64_t>(g, layers, num_layers, x, ld_x, targets, num_targets, out, ld_out, opts, pstats, s)
                               : infer_partial<int32_t>(g, layers, num_layers, x, ld_x, targets, num_targets, out, ld_out, opts, pstats, s);
}
