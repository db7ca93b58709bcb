// Partial inference (Sections 2 and 3.3 of the DGI paper): output embeddings for a set of target nodes only.
//
// The per-layer target sets are annotated backwards from the user's targets: V^L = targets, and V^{l-1} =
// V^l plus the in-neighbours of V^l (a node's own previous embedding is an input of Eq. 1 as well).  The
// annotation stops, and all nodes are used, as soon as |V^l| * d_avg >= n (the paper's shortcut: the next
// set would hold most of the graph anyway).  Otherwise the rows of V^1 (with their complete in-neighbour
// lists) and the inputs V^0 are extracted into a compact sub-problem, relabelled, and the ordinary
// layer-wise schedule (dgi_infer) runs on it: rows outside V^l at layer l are computed too, but they have
// empty lists below V^1 and nobody reads them.  Degrees in the GCN normaliser stay those of the full graph.
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

template <typename IdxT>
dgi_status_t infer_partial(const dgi_graph* g, const dgi_layer_t* layers, int32_t L, const void* x, int64_t ld_x,
                           const int32_t* targets, int64_t nt, void* out, int64_t ld_out, const dgi_infer_opts_t* opts,
                           dgi_partial_stats_t* ps, hipStream_t s) {
    const int64_t N = g->N;
    const IdxT* indptr = (const IdxT*)g->d_indptr;
    const int xb = layers[0].feat_dtype == DGI_BF16 ? 2 : 4, yb = layers[L - 1].out_dtype == DGI_BF16 ? 2 : 4;
    const int in_dim = layers[0].in_dim, out_dim = layers[L - 1].out_dim;
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
    int64_t n_l = 0;
    DGI_TRY(count_level(L, &n_l));
    DGI_REQUIRE(h_bad == 0, DGI_ERR_INVALID_ARG, "infer_partial: a target id is outside [0, num_nodes)");
    if (ps) { std::memset(ps, 0, sizeof(*ps)); ps->num_layers = L; ps->set_size[L] = n_l; ps->all_nodes_from_layer = -1; }
    // ---- backward annotation of V^{L-1} ... V^0, with the |V^l| * d_avg >= n shortcut -----------------------
    bool use_all = false;
    for (int32_t l = L; l >= 1; --l) {
        if ((double)n_l * d_avg >= (double)N) { use_all = true; if (ps) ps->all_nodes_from_layer = l - 1; break; }
        hipLaunchKernelGGL(expand_depth_kernel<IdxT>, dim3(grid_for(N * 64)), dim3(kBlock), 0, s, indptr, g->d_indices, N, l, depth.as<int32_t>());
        DGI_TRY(count_level(l - 1, &n_l));
        if (ps) ps->set_size[l - 1] = n_l;
    }
    dgi_infer_opts_t o{};
    if (opts) o = *opts;
    o.perm_new_of_old = nullptr;

    if (use_all) {
        // the annotated sets cover (nearly) the whole graph: run full inference and pick the target rows
        Buf full;
        const int64_t ld_full = round_up(out_dim, 16 / yb);
        DGI_TRY(full.alloc((size_t)N * ld_full * yb));
        DGI_TRY(dgi_infer(g, layers, L, x, ld_x, full.p, ld_full, &o, s));
        DGI_TRY(launch_permute_rows(full.p, ld_full, out, ld_out, nt, out_dim, yb, targets, true, s));
        DGI_HIP(hipStreamSynchronize(s));
        if (ps) { ps->sub_nodes = N; ps->sub_edges = g->E; }
        return DGI_OK;
    }

    // ---- compact sub-problem over U = V^0 -----------------------------------------------------------------------
    const int64_t n_sub = n_l;  // |V^0|
    Buf U, sub_deg, sub_indptr, sub_indices, x_sub, out_sub, tloc;
    DGI_TRY(U.alloc(n_sub * 4)); DGI_TRY(sub_deg.alloc((n_sub + 1) * 8)); DGI_TRY(sub_indptr.alloc((n_sub + 1) * 8));
    // sc.flag still holds (depth >= 0) from the last count_level call
    int64_t e_sub = 0;
    DGI_TRY(sub_rows<IdxT>(g, depth.as<int32_t>(), sc, n_sub, U.as<int32_t>(), sub_deg.as<int64_t>(), sub_indptr.as<int64_t>(), &e_sub, s));
    DGI_TRY(sub_indices.alloc(e_sub * 4));
    GraphGuard sub;
    DGI_TRY(sub_graph<IdxT>(g, sc, n_sub, e_sub, U.as<int32_t>(), sub_indptr.as<int64_t>(), sub_indices.as<int32_t>(), &sub, s));
    const int64_t ld_xs = round_up(in_dim, 16 / xb), ld_os = round_up(out_dim, 16 / yb);
    DGI_TRY(x_sub.alloc((size_t)n_sub * ld_xs * xb)); DGI_TRY(out_sub.alloc((size_t)n_sub * ld_os * yb)); DGI_TRY(tloc.alloc(nt * 4));
    DGI_TRY(launch_permute_rows(x, ld_x, x_sub.p, ld_xs, n_sub, in_dim, xb, U.as<int32_t>(), true, s));
    DGI_TRY(dgi_infer(sub.g, layers, L, x_sub.p, ld_xs, out_sub.p, ld_os, &o, s));
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
