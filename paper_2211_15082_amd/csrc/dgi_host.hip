// Layer-wise inference with host-resident embeddings (Algorithm 2 with Section 4.1's dynamic batch size): the
// feature matrices stay in page-locked host memory, every batch loads the rows of its input set over the host
// link, computes one layer for its destination rows and dumps them back.  The per-batch sub-problem (input
// set, relabelled neighbour lists) is built on the device with the same steps as partial inference.
#include <chrono>
#include <climits>
#include <cstring>

#include "dgi_subproblem.h"

namespace dgi {
namespace {

using namespace subp;

// depth = 1 for the batch's destination rows (they keep their lists), else -1
__global__ void batch_depth_kernel(int32_t* depth, int64_t N, int64_t b, int64_t e) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (int64_t)gridDim.x * blockDim.x)
        depth[i] = (i >= b && i < e) ? 1 : -1;
}

// sources of the batch's edges become inputs (depth 0) unless they are destination rows already
__global__ void mark_sources_kernel(const int32_t* indices, int64_t e0, int64_t e1, int32_t* depth) {
    for (int64_t i = e0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < e1; i += (int64_t)gridDim.x * blockDim.x)
        atomicMax(&depth[indices[i]], 0);
}

struct HostBuf {  // page-locked host memory, visible to the device
    void* p = nullptr;
    ~HostBuf() { (void)hipHostFree(p); }
    dgi_status_t alloc(size_t bytes) { DGI_HIP(hipHostMalloc(&p, std::max<size_t>(bytes, 16), hipHostMallocDefault)); return DGI_OK; }
};

struct Events {
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    ~Events() { for (auto e : ev) if (e) (void)hipEventDestroy(e); }
    dgi_status_t create() { for (auto& e : ev) DGI_HIP(hipEventCreate(&e)); return DGI_OK; }
};

// the device address of page-locked host memory; an error for anything else
dgi_status_t device_view(const void* host, const char* what, void** dev) {
    hipPointerAttribute_t attr{};
    hipError_t err = hipPointerGetAttributes(&attr, host);
    if (err != hipSuccess) { (void)hipGetLastError(); set_error("infer_host: %s is not page-locked host memory", what); return DGI_ERR_INVALID_ARG; }
    DGI_REQUIRE(attr.type == hipMemoryTypeHost, DGI_ERR_INVALID_ARG, "infer_host: %s must be page-locked host memory (hipHostMalloc)", what);
    DGI_HIP(hipHostGetDevicePointer(dev, const_cast<void*>(host), 0));
    return DGI_OK;
}

template <typename IdxT>
dgi_status_t infer_host(const dgi_graph* g, const dgi_layer_t* layers, int32_t L, const void* x_host, int64_t ld_x, void* out_host,
                        int64_t ld_out, const dgi_infer_opts_t& o, dgi_host_stats_t* hs, hipStream_t s) {
    const auto t_start = std::chrono::steady_clock::now();
    const int64_t N = g->N;
    const double avg_deg = N > 0 ? (double)g->E / (double)N : 0.0;
    void* x_dev = nullptr;
    void* out_dev = nullptr;
    DGI_TRY(device_view(x_host, "x_host", &x_dev));
    DGI_TRY(device_view(out_host, "out_host", &out_dev));

    // hidden layers in host memory, used alternately
    HostBuf hid[2];
    size_t hid_bytes = 0;
    for (int l = 0; l + 1 < L; ++l) {
        const int eb = layers[l].out_dtype == DGI_BF16 ? 2 : 4;
        hid_bytes = std::max<size_t>(hid_bytes, (size_t)N * (size_t)round_up(layers[l].out_dim, 16 / eb) * eb);
    }
    const int n_hidden = L >= 3 ? 2 : (L == 2 ? 1 : 0);
    for (int i = 0; i < n_hidden; ++i) DGI_TRY(hid[i].alloc(hid_bytes));

    // N-sized device scratch and the batch arena (M of Eq. 2)
    Buf depth, arena;
    Scratch sc;
    DGI_TRY(depth.alloc(N * 4));
    DGI_TRY(sc.alloc(N, s));
    uint64_t budget = o.mem_budget_bytes;
    if (budget == 0) {
        size_t free_b = 0, total_b = 0;
        DGI_HIP(hipMemGetInfo(&free_b, &total_b));
        budget = (uint64_t)(0.9 * (double)free_b);
    }
    // no batch needs more than the whole graph at once
    uint64_t whole = 0;
    for (int l = 0; l < L; ++l) {
        const int xb = layers[l].feat_dtype == DGI_BF16 ? 2 : 4, yb = layers[l].out_dtype == DGI_BF16 ? 2 : 4;
        uint64_t ws = 0;
        DGI_TRY(dgi_layer_workspace_bytes(g, &layers[l], 0, N, &ws));
        whole = std::max<uint64_t>(whole, (uint64_t)g->E * 4 + (uint64_t)(N + 1) * 20 + (uint64_t)N * round_up(layers[l].in_dim, 16 / xb) * xb +
                                              (uint64_t)N * round_up(layers[l].out_dim, 16 / yb) * yb + 2 * ws + 8192);
    }
    const uint64_t M = std::min(budget, whole);
    DGI_REQUIRE(M >= 65536, DGI_ERR_OOM, "infer_host: memory budget %llu bytes is too small", (unsigned long long)budget);
    DGI_TRY(arena.alloc(M));
    Events ev;
    DGI_TRY(ev.create());
    if (hs) { hs->budget_bytes = (int64_t)M; }

    const void* cur = x_dev;
    int64_t ld_cur = ld_x;
    for (int l = 0; l < L; ++l) {
        const dgi_layer_t& Ly = layers[l];
        const int xb = Ly.feat_dtype == DGI_BF16 ? 2 : 4, yb = Ly.out_dtype == DGI_BF16 ? 2 : 4;
        const int64_t ld_xs = round_up(Ly.in_dim, 16 / xb), ld_os = round_up(Ly.out_dim, 16 / yb);
        const bool last = l == L - 1;
        char* dst_host = last ? static_cast<char*>(out_host) : static_cast<char*>(hid[l % 2].p);
        const int64_t ld_dst = last ? ld_out : ld_os;

        int64_t n_t = o.batch_size > 0 ? o.batch_size : (o.init_node_threshold > 0 ? o.init_node_threshold : 65536);
        int64_t n_i = o.batch_size > 0 ? INT64_MAX / 4
                                       : (o.init_edge_threshold > 0 ? o.init_edge_threshold : (int64_t)std::max(1.0, (double)n_t * std::max(avg_deg, 1.0)));
        int64_t b = 0;
        while (b < N) {
            int64_t e = 0;
            DGI_TRY(dgi_plan_batch_end(g->h_indptr.data(), DGI_I64, N, b, std::max<int64_t>(n_t, 1), std::max<int64_t>(n_i, 0), &e));
            const int64_t rows = e - b, e_b = g->h_indptr[e] - g->h_indptr[b];
            auto shrink = [&]() -> dgi_status_t {  // the out-of-memory reaction of Section 4.1
                if (hs) hs->oom_retries += 1;
                if (rows <= 1 || dgi_threshold_halve(&n_t, &n_i) != DGI_OK) {
                    set_error("infer_host: layer %d: one destination row with its input set does not fit %llu bytes", l, (unsigned long long)M);
                    return DGI_ERR_OOM;
                }
                n_t = std::min(n_t, std::max<int64_t>(rows / 2, 1));
                return DGI_OK;
            };
            // ---- (i) input set ------------------------------------------------------------------------------
            DGI_HIP(hipEventRecord(ev.ev[0], s));
            hipLaunchKernelGGL(batch_depth_kernel, dim3(grid_for(N)), dim3(kBlock), 0, s, depth.as<int32_t>(), N, b, e);
            if (e_b > 0)
                hipLaunchKernelGGL(mark_sources_kernel, dim3(grid_for(e_b)), dim3(kBlock), 0, s, g->d_indices, g->h_indptr[b], g->h_indptr[e], depth.as<int32_t>());
            int64_t n_sub = 0;
            DGI_TRY(sc.count_level(depth.as<int32_t>(), N, 0, &n_sub, s));
            // ---- device memory of this batch (M_k), carved from the arena ----------------------------------------
            uint64_t off = 0;
            auto carve = [&](uint64_t bytes) { const uint64_t at = off; off += (uint64_t)round_up((int64_t)std::max<uint64_t>(bytes, 16), 256); return at; };
            const uint64_t o_idx = carve((uint64_t)e_b * 4), o_ptr = carve((uint64_t)(n_sub + 1) * 8), o_deg = carve((uint64_t)(n_sub + 1) * 8);
            const uint64_t o_U = carve((uint64_t)n_sub * 4), o_x = carve((uint64_t)n_sub * ld_xs * xb), o_y = carve((uint64_t)rows * ld_os * yb);
            if (off > M) { DGI_TRY(shrink()); continue; }
            char* A = arena.as<char>();
            int64_t e_sub = 0;
            DGI_TRY(sub_rows<IdxT>(g, depth.as<int32_t>(), sc, n_sub, (int32_t*)(A + o_U), (int64_t*)(A + o_deg), (int64_t*)(A + o_ptr), &e_sub, s));
            DGI_REQUIRE(e_sub == e_b, DGI_ERR_DEVICE, "infer_host: sub-problem has %lld edges, expected %lld", (long long)e_sub, (long long)e_b);
            GraphGuard sub;
            DGI_TRY(sub_graph<IdxT>(g, sc, n_sub, e_sub, (const int32_t*)(A + o_U), (const int64_t*)(A + o_ptr), (int32_t*)(A + o_idx), &sub, s));
            // the batch's rows are one run of local ids: [lb, lb + rows)
            int32_t lb = 0;
            DGI_HIP(hipMemcpyAsync(&lb, sc.loc.as<int32_t>() + b, 4, hipMemcpyDeviceToHost, s));
            DGI_HIP(hipStreamSynchronize(s));
            uint64_t ws_bytes = 0;
            DGI_TRY(dgi_layer_workspace_bytes(sub.g, &Ly, lb, lb + rows, &ws_bytes));
            const uint64_t o_ws = carve(ws_bytes);
            const uint64_t M_k = off + sub.g->device_bytes;
            if (M_k > M) { DGI_TRY(shrink()); continue; }
            // ---- (ii) rows of the input set, read from host memory by the device ----------------------------------
            DGI_TRY(launch_permute_rows(cur, ld_cur, A + o_x, ld_xs, n_sub, Ly.in_dim, xb, (const int32_t*)(A + o_U), true, s));
            DGI_HIP(hipEventRecord(ev.ev[1], s));
            // ---- (iii) the layer on the sub-problem; output row v lands at (v - lb) of the batch's matrix --------------
            char* y_base = A + o_y - (int64_t)lb * ld_os * yb;
            DGI_TRY(dgi_layer_forward(sub.g, &Ly, A + o_x, ld_xs, y_base, ld_os, lb, lb + rows, A + o_ws, ws_bytes, s));
            DGI_HIP(hipEventRecord(ev.ev[2], s));
            // ---- (iv) dump the batch's rows ------------------------------------------------------------------------
            DGI_HIP(hipMemcpy2DAsync(dst_host + (size_t)b * ld_dst * yb, (size_t)ld_dst * yb, A + o_y, (size_t)ld_os * yb, (size_t)Ly.out_dim * yb,
                                     (size_t)rows, hipMemcpyDeviceToHost, s));
            DGI_HIP(hipEventRecord(ev.ev[3], s));
            DGI_HIP(hipStreamSynchronize(s));  // the arena and the sub-problem are reused by the next batch
            if (hs) {
                float t01 = 0.f, t12 = 0.f, t23 = 0.f;
                DGI_HIP(hipEventElapsedTime(&t01, ev.ev[0], ev.ev[1]));
                DGI_HIP(hipEventElapsedTime(&t12, ev.ev[1], ev.ev[2]));
                DGI_HIP(hipEventElapsedTime(&t23, ev.ev[2], ev.ev[3]));
                hs->load_ms[l] += t01; hs->compute_ms[l] += t12; hs->store_ms[l] += t23;
                hs->batches[l] += 1;
                hs->input_rows[l] += n_sub;
                hs->input_bytes[l] += n_sub * (int64_t)Ly.in_dim * xb;
                hs->output_bytes[l] += rows * (int64_t)Ly.out_dim * yb;
                hs->peak_batch_bytes = std::max<int64_t>(hs->peak_batch_bytes, (int64_t)M_k);
            }
            if (o.batch_size == 0) DGI_TRY(dgi_threshold_update((double)M, (double)M_k, &n_t, &n_i));  // Eq. 2
            b = e;
        }
        // H^{l-1} is dead from here on: its buffer takes H^{l+1}
        DGI_HIP(hipHostGetDevicePointer(const_cast<void**>(&cur), dst_host, 0));
        ld_cur = ld_dst;
    }
    if (hs) hs->total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_start).count();
    return DGI_OK;
}

}  // namespace
}  // namespace dgi

using namespace dgi;

extern "C" dgi_status_t dgi_infer_host(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x_host,
                                       int64_t ld_x, void* out_host, int64_t ld_out, const dgi_infer_opts_t* opts,
                                       dgi_host_stats_t* hstats, void* hip_stream) {
    DGI_REQUIRE(g && layers, DGI_ERR_INVALID_ARG, "infer_host: NULL argument");
    DGI_REQUIRE(num_layers >= 1 && num_layers <= DGI_MAX_LAYERS, DGI_ERR_INVALID_ARG, "infer_host: 1..%d layers supported", DGI_MAX_LAYERS);
    dgi_infer_opts_t o{};
    if (opts) o = *opts;
    DGI_REQUIRE(!o.perm_new_of_old && !o.jk_concat, DGI_ERR_UNSUPPORTED, "infer_host: permutation and jumping-knowledge options are not supported");
    DGI_REQUIRE(o.batch_size >= 0, DGI_ERR_INVALID_ARG, "infer_host: negative batch_size");
    DGI_REQUIRE(g->N < (int64_t)INT_MAX, DGI_ERR_UNSUPPORTED, "infer_host: at most 2^31 - 2 nodes");
    for (int l = 1; l < num_layers; ++l) {
        DGI_REQUIRE(layers[l].in_dim == layers[l - 1].out_dim, DGI_ERR_INVALID_ARG, "layer %d: in_dim != previous out_dim", l);
        DGI_REQUIRE(layers[l].feat_dtype == layers[l - 1].out_dtype, DGI_ERR_INVALID_ARG, "layer %d: feat_dtype != previous out_dtype", l);
    }
    if (hstats) { std::memset(hstats, 0, sizeof(*hstats)); hstats->num_layers = num_layers; }
    if (g->N == 0) return DGI_OK;
    DGI_REQUIRE(x_host && out_host, DGI_ERR_INVALID_ARG, "infer_host: NULL buffer");
    DGI_REQUIRE(ld_x >= layers[0].in_dim && ld_out >= layers[num_layers - 1].out_dim, DGI_ERR_INVALID_ARG, "infer_host: leading dimension too small");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return g->itype == DGI_I64 ? infer_host<int64_t>(g, layers, num_layers, x_host, ld_x, out_host, ld_out, o, hstats, s)
                               : infer_host<int32_t>(g, layers, num_layers, x_host, ld_x, out_host, ld_out, o, hstats, s);
}
