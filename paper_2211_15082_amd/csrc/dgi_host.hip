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

// One of two pipeline slots: the device memory of a batch, its sub-problem and the events around its three
// stages.  While one slot computes and dumps its batch on the second stream, the other builds and loads the
// next batch on the first.
struct Slot {
    char* mem = nullptr;
    GraphGuard sub;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};  // load begin, loaded, computed, stored
    bool pending = false;
    int layer = 0;
    int64_t n_sub = 0, rows = 0, in_bytes = 0, out_bytes = 0;
    uint64_t M_k = 0;
    bool dense = false;  // a row chunk of a layer's dense pass (no input set, no sub-problem)
    ~Slot() { for (auto e : ev) if (e) (void)hipEventDestroy(e); }
    dgi_status_t create() { for (auto& e : ev) DGI_HIP(hipEventCreate(&e)); return DGI_OK; }
    // wait until the slot's batch has been stored, account for it, release its sub-problem
    dgi_status_t retire(dgi_host_stats_t* hs) {
        if (!pending) return DGI_OK;
        DGI_HIP(hipEventSynchronize(ev[3]));
        if (hs) {
            float t01 = 0.f, t12 = 0.f, t23 = 0.f;
            DGI_HIP(hipEventElapsedTime(&t01, ev[0], ev[1]));
            DGI_HIP(hipEventElapsedTime(&t12, ev[1], ev[2]));
            DGI_HIP(hipEventElapsedTime(&t23, ev[2], ev[3]));
            hs->load_ms[layer] += t01; hs->compute_ms[layer] += t12; hs->store_ms[layer] += t23;
            if (dense) {
                hs->transform_bytes[layer] += in_bytes + out_bytes;
            } else {
                hs->batches[layer] += 1;
                hs->input_rows[layer] += n_sub;
                hs->input_bytes[layer] += in_bytes;
                hs->output_bytes[layer] += out_bytes;
            }
            hs->peak_batch_bytes = std::max<int64_t>(hs->peak_batch_bytes, (int64_t)M_k);
        }
        sub.reset();
        pending = false;
        return DGI_OK;
    }
};

struct StreamPair {
    hipStream_t a = nullptr, b = nullptr;
    ~StreamPair() { if (a) (void)hipStreamDestroy(a); if (b) (void)hipStreamDestroy(b); }
    dgi_status_t create() {
        DGI_HIP(hipStreamCreateWithFlags(&a, hipStreamNonBlocking));
        DGI_HIP(hipStreamCreateWithFlags(&b, hipStreamNonBlocking));
        return DGI_OK;
    }
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

// Device rows to host memory; only columns [0, width) of the destination rows are written.  Dense rows on both sides
// (width == both leading dimensions): one contiguous copy by the DMA engine.  Otherwise a kernel writes the rows
// through the mapped host address: a pitched DMA copy of sub-kilobyte rows ran at 14 GB/s here, a third of the
// link (and a contiguous copy of padded rows would write the device buffer's padding columns into the caller's).
dgi_status_t store_rows(const void* src_dev, int64_t ld_src, void* dst_host, void* dst_host_dev, int64_t ld_dst, int64_t rows, int width, int eb,
                        hipStream_t s) {
    if (rows == 0) return DGI_OK;
    if (ld_src == ld_dst && width == ld_dst) {
        DGI_HIP(hipMemcpyAsync(dst_host, src_dev, (size_t)rows * width * eb, hipMemcpyDeviceToHost, s));
        return DGI_OK;
    }
    return launch_permute_rows(src_dev, ld_src, dst_host_dev, ld_dst, rows, width, eb, nullptr, true, s);
}

template <typename IdxT>
dgi_status_t infer_host(const dgi_graph* g, const dgi_layer_t* layers, int32_t L, const void* x_host, int64_t ld_x, void* out_host,
                        int64_t ld_out, const dgi_infer_opts_t& o, dgi_host_stats_t* hs, hipStream_t s) {
    const auto t_start = std::chrono::steady_clock::now();
    std::lock_guard<std::mutex> hs_lock(g->hs_mutex);  // one dgi_infer_host at a time per graph handle
    const int64_t N = g->N;
    const double avg_deg = N > 0 ? (double)g->E / (double)N : 0.0;
    void* x_dev = nullptr;
    void* out_dev = nullptr;
    DGI_TRY(device_view(x_host, "x_host", &x_dev));
    DGI_TRY(device_view(out_host, "out_host", &out_dev));

    uint64_t budget = o.mem_budget_bytes;
    if (budget == 0) {
        size_t free_b = 0, total_b = 0;
        DGI_HIP(hipMemGetInfo(&free_b, &total_b));
        budget = (uint64_t)(0.9 * (double)(free_b + g->ws_bytes));  // the graph handle's cached arena counts as available
    }
    // When x, the output and the device-resident schedule's buffers all fit the budget, nothing needs to leave the
    // device between layers: one copy in, dgi_infer, one copy out.
    {
        const int xb = layers[0].feat_dtype == DGI_BF16 ? 2 : 4, yb = layers[L - 1].out_dtype == DGI_BF16 ? 2 : 4;
        const int64_t ld_xd = round_up(layers[0].in_dim, 16 / xb), ld_yd = round_up(layers[L - 1].out_dim, 16 / yb);
        const uint64_t io_bytes = (uint64_t)N * ld_xd * xb + (uint64_t)N * ld_yd * yb + 512;
        if (io_bytes < budget && !o.host_stream_always) {
            Buf xd, yd;
            DGI_TRY(xd.alloc((size_t)N * ld_xd * xb));
            DGI_TRY(yd.alloc((size_t)N * ld_yd * yb));
            dgi_infer_opts_t r = o;
            dgi_stats_t rs;
            r.mem_budget_bytes = budget - io_bytes;
            r.stats = &rs;
            Slot t;  // for its events
            DGI_TRY(t.create());
            DGI_HIP(hipEventRecord(t.ev[0], s));
            DGI_HIP(hipMemcpy2DAsync(xd.p, (size_t)ld_xd * xb, x_host, (size_t)ld_x * xb, (size_t)layers[0].in_dim * xb, (size_t)N, hipMemcpyHostToDevice, s));
            DGI_HIP(hipEventRecord(t.ev[1], s));
            const dgi_status_t rc = dgi_infer(g, layers, L, xd.p, ld_xd, yd.p, ld_yd, &r, s);
            if (rc == DGI_OK) {
                DGI_HIP(hipEventRecord(t.ev[2], s));
                DGI_TRY(store_rows(yd.p, ld_yd, out_host, out_dev, ld_out, N, layers[L - 1].out_dim, yb, s));
                DGI_HIP(hipEventRecord(t.ev[3], s));
                DGI_HIP(hipStreamSynchronize(s));
                if (hs) {
                    float t01 = 0.f, t23 = 0.f;
                    DGI_HIP(hipEventElapsedTime(&t01, t.ev[0], t.ev[1]));
                    DGI_HIP(hipEventElapsedTime(&t23, t.ev[2], t.ev[3]));
                    hs->load_ms[0] = t01; hs->store_ms[L - 1] = t23;
                    for (int l = 0; l < L; ++l) { hs->compute_ms[l] = rs.layer_ms[l]; hs->batches[l] = rs.batches[l]; }
                    hs->input_rows[0] = N; hs->input_bytes[0] = N * (int64_t)layers[0].in_dim * xb;
                    hs->output_bytes[L - 1] = N * (int64_t)layers[L - 1].out_dim * yb;
                    hs->budget_bytes = (int64_t)budget; hs->peak_batch_bytes = rs.workspace_bytes + (int64_t)io_bytes;
                    hs->oom_retries = rs.oom_retries; hs->device_resident = 1;
                    hs->total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_start).count();
                }
                return DGI_OK;
            }
            if (rc != DGI_ERR_OOM) return rc;
            DGI_HIP(hipStreamSynchronize(s));  // the hidden layers do not fit: stream them through host memory
        }
    }

    // hidden layers in host memory, used alternately (kept in the graph handle between calls)
    size_t hid_bytes = 0;
    for (int l = 0; l + 1 < L; ++l) {
        const int eb = layers[l].out_dtype == DGI_BF16 ? 2 : 4;
        hid_bytes = std::max<size_t>(hid_bytes, (size_t)N * (size_t)round_up(layers[l].out_dim, 16 / eb) * eb);
    }
    const int n_hidden = L >= 3 ? 2 : (L == 2 ? 1 : 0);
    if (n_hidden > 0 && (g->hs_hid_bytes < hid_bytes || (n_hidden == 2 && !g->hs_hid[1]))) {
        for (int i = 0; i < 2; ++i) { (void)hipHostFree(g->hs_hid[i]); g->hs_hid[i] = nullptr; }
        g->hs_hid_bytes = 0;
        for (int i = 0; i < n_hidden; ++i) DGI_HIP(hipHostMalloc(&g->hs_hid[i], std::max<size_t>(hid_bytes, 16), hipHostMallocDefault));
        g->hs_hid_bytes = hid_bytes;
    }
    void* const* hid = g->hs_hid;

    // N-sized device scratch and the batch arena (M of Eq. 2)
    Buf depth;
    Scratch sc;
    DGI_TRY(depth.alloc(N * 4));
    DGI_TRY(sc.alloc(N, s));
    if (o.mem_budget_bytes == 0) {  // the attempt above may have left an arena in the graph handle: give it back, measure again
        DGI_TRY(release_infer_arena(g));
        size_t free_b = 0, total_b = 0;
        DGI_HIP(hipMemGetInfo(&free_b, &total_b));
        budget = (uint64_t)(0.9 * (double)free_b);
    }
    // no batch needs more than the whole graph at once
    uint64_t whole = 0;
    int n_slots = 2;
    for (int l = 0; l < L; ++l) {
        const int xb = layers[l].feat_dtype == DGI_BF16 ? 2 : 4, yb = layers[l].out_dtype == DGI_BF16 ? 2 : 4;
        uint64_t ws = 0;
        DGI_TRY(dgi_layer_workspace_bytes(g, &layers[l], 0, N, &ws));
        whole = std::max<uint64_t>(whole, (uint64_t)g->E * 4 + (uint64_t)(N + 1) * 20 + (uint64_t)N * round_up(layers[l].in_dim, 16 / xb) * xb +
                                              (uint64_t)N * round_up(layers[l].out_dim, 16 / yb) * yb + 2 * ws + 8192);
    }
    // One slot or two?  Two slots overlap a batch's compute and dump with the next batch's load, but halve M, and
    // smaller batches load more rows in total (their input sets overlap): measured on a 2.4 M-node power-law graph,
    // half the slot size means 1.6 times the bytes over the host link (twice, once a batch's input set is most of the
    // graph).  So two slots pay off only where compute and dump are a large part of a batch's time, as on a graph
    // whose batches need little beyond their own rows.  Estimated on the first batch the two-slot plan would run
    // (host link 45 GB/s each way, gathers 5 TB/s, transforms 100 TFLOP/s, 0.2 ms of launches per layer): one slot
    // unless compute + dump exceed 0.38 of the load, the point where 1.6x the traffic costs as much as the lost
    // overlap.
    auto choose_slots = [&]() -> dgi_status_t {
#ifdef DGI_HOST_SLOTS  // measurement builds pin the number of batches in flight
        n_slots = DGI_HOST_SLOTS == 1 ? 1 : 2;
        return DGI_OK;
#endif
        if (whole <= budget) { n_slots = 1; return DGI_OK; }  // a whole layer at once: every row crosses the link once
        const int64_t n_t = o.batch_size > 0 ? o.batch_size : (o.init_node_threshold > 0 ? o.init_node_threshold : 65536);
        const int64_t n_i = o.batch_size > 0 ? INT64_MAX / 4
                                             : (o.init_edge_threshold > 0 ? o.init_edge_threshold : (int64_t)std::max(1.0, (double)n_t * std::max(avg_deg, 1.0)));
        int64_t e = 0;
        DGI_TRY(dgi_plan_batch_end(g->h_indptr.data(), DGI_I64, N, 0, std::max<int64_t>(n_t, 1), std::max<int64_t>(n_i, 0), &e));
        const int64_t e_b = g->h_indptr[e] - g->h_indptr[0];
        hipLaunchKernelGGL(batch_depth_kernel, dim3(grid_for(N)), dim3(kBlock), 0, s, depth.as<int32_t>(), N, (int64_t)0, e);
        if (e_b > 0)
            hipLaunchKernelGGL(mark_sources_kernel, dim3(grid_for(e_b)), dim3(kBlock), 0, s, g->d_indices, g->h_indptr[0], g->h_indptr[e], depth.as<int32_t>());
        int64_t n_sub = 0;
        DGI_TRY(sc.count_level(depth.as<int32_t>(), N, 0, &n_sub, s));
        double load = 0, work = 0;
        for (int l = 0; l < L; ++l) {
            const double in_row = (double)layers[l].in_dim * (layers[l].feat_dtype == DGI_BF16 ? 2 : 4);
            const double out_row = (double)layers[l].out_dim * (layers[l].out_dtype == DGI_BF16 ? 2 : 4);
            const double k_tot = (double)layers[l].in_dim * (layers[l].W_self ? 2 : 1);
            load += (double)n_sub * in_row / 45e9;
            work += (double)e_b * std::max(in_row, out_row) / 5e12 + (double)e * 2.0 * k_tot * layers[l].out_dim / 100e12 + 2e-4 +
                    (double)e * out_row / 45e9;
        }
        n_slots = work > 0.38 * load ? 2 : 1;
        return DGI_OK;
    };
    // One or two slots of M bytes each (M is Eq. 2's expected consumption of one batch); everything at once if it fits.
    if (whole > budget / 2) DGI_TRY(choose_slots());
    const bool all_fits = whole <= budget / (uint64_t)n_slots;
    const uint64_t M = (all_fits ? whole : budget / (uint64_t)n_slots) / 256 * 256;
    DGI_REQUIRE(M >= 65536, DGI_ERR_OOM, "infer_host: memory budget %llu bytes is too small", (unsigned long long)budget);
    const uint64_t arena = (uint64_t)n_slots * M;
    if (g->hs_arena_bytes < arena || g->hs_arena_bytes > arena + M / 2 + ((uint64_t)64 << 20)) {  // too small, or far beyond this call's budget
        (void)hipFree(g->hs_arena); g->hs_arena = nullptr; g->hs_arena_bytes = 0;
        DGI_HIP(hipMalloc(reinterpret_cast<void**>(&g->hs_arena), arena));
        g->hs_arena_bytes = arena;
    }
    Slot slot[2];
    StreamPair st;
    DGI_TRY(st.create());
    struct SyncOnExit {  // declared last, so on every return path the streams drain before the slots are torn down
        hipStream_t a, b;
        ~SyncOnExit() { (void)hipStreamSynchronize(a); (void)hipStreamSynchronize(b); }
    } drain{st.a, st.b};
    for (int i = 0; i < n_slots; ++i) { DGI_TRY(slot[i].create()); slot[i].mem = g->hs_arena + (uint64_t)i * M; }
    if (hs) { hs->budget_bytes = (int64_t)M; hs->slots = n_slots; }
    DGI_HIP(hipStreamSynchronize(s));  // the caller's earlier work on its stream (x_host may come from it)
    const hipStream_t sa = st.a, sb = st.b;

    const void* cur = x_dev;
    int64_t ld_cur = ld_x;
    int64_t k = 0;  // batch counter: slot k % n_slots
    // Thresholds that planned the last batch filling at least half of M, and the bytes of an input row then: the next
    // layer starts from them (rescaled by the row width) instead of climbing from the initial values again, which
    // costs a few undersized batches per layer (Eq. 2 under-predicts: an input set grows more slowly than its batch).
    int64_t carry_nt = 0, carry_ni = 0;
    double carry_row = 0.0;
    for (int l = 0; l < L; ++l) {
        const dgi_layer_t& Ly = layers[l];
        const int xb = Ly.feat_dtype == DGI_BF16 ? 2 : 4, yb = Ly.out_dtype == DGI_BF16 ? 2 : 4;
        const int64_t ld_xs = round_up(Ly.in_dim, 16 / xb), ld_os = round_up(Ly.out_dim, 16 / yb);
        const bool last = l == L - 1;
        char* dst_host = last ? static_cast<char*>(out_host) : static_cast<char*>(hid[l % 2]);
        const int64_t ld_dst = last ? ld_out : ld_os;
        char* dst_dev = nullptr;
        DGI_HIP(hipHostGetDevicePointer(reinterpret_cast<void**>(&dst_dev), dst_host, 0));

        // Transform-first across the host link.  When the layer's plan multiplies before it aggregates and a
        // transformed row is clearly narrower than an input row, the rows every batch loads for its input set should
        // be the narrow ones: a dense pass streams H^{l-1} through the device once in contiguous row chunks and
        // leaves Z = H^{l-1} W in host memory, and the batches then gather rows of Z and only aggregate.
        TransformInfo ti{};
        DGI_TRY(layer_transform_info(g, &Ly, &ti));
        const int zb = ti.z_dtype == DGI_BF16 ? 2 : 4;
        // (GraphSAGE: the batches gather only the z_neigh block of a transformed row; z_self is needed for the batch's own
        // rows alone, which are one contiguous run of Z)
        const int64_t ld_zn = round_up(Ly.out_dim, 16 / zb);
        const uint64_t gathered_row = ti.has_self ? (uint64_t)ld_zn * zb : (uint64_t)ti.z_ld * zb;
        bool two_pass = !all_fits && ti.transform_first && gathered_row * 4 <= (uint64_t)ld_xs * xb * 3;
        const char* z_rows = nullptr;   // device view of Z in host memory (two passes)
        const void* f_src = cur;        // where the batches' input rows come from
        int64_t f_ld = ld_cur, f_lds = ld_xs;
        int f_width = Ly.in_dim, f_eb = xb;
        if (two_pass) {
            const uint64_t z_bytes = (uint64_t)N * ti.z_ld * zb;
            if (g->hs_z_bytes < z_bytes) {
                (void)hipHostFree(g->hs_z); g->hs_z = nullptr; g->hs_z_bytes = 0;
                if (hipHostMalloc(&g->hs_z, (size_t)z_bytes, hipHostMallocDefault) == hipSuccess) {
                    g->hs_z_bytes = z_bytes;
                } else {  // no page-locked memory left for Z: the layer runs in one pass over its input rows
                    (void)hipGetLastError();
                    g->hs_z = nullptr;
                    two_pass = false;
                }
            }
        }
        if (two_pass) {
            char* z_host = static_cast<char*>(g->hs_z);
            char* z_dev = nullptr;
            DGI_HIP(hipHostGetDevicePointer(reinterpret_cast<void**>(&z_dev), z_host, 0));
            const uint64_t w_bytes = (uint64_t)round_up((int64_t)ti.weight_bytes, 256);
            const uint64_t per_row = (uint64_t)ld_xs * xb + (uint64_t)ti.z_ld * zb;
            DGI_REQUIRE(M > w_bytes + 1024 + per_row, DGI_ERR_OOM, "infer_host: layer %d: the packed weights and one row do not fit %llu bytes", l, (unsigned long long)M);
            const int64_t rows_c = std::max<int64_t>(1, (int64_t)((M - w_bytes - 1024) / per_row));
            for (int64_t r0 = 0; r0 < N; r0 += rows_c) {
                const int64_t n = std::min(rows_c, N - r0);
                Slot& S = slot[k % n_slots];
                DGI_TRY(S.retire(hs));
                char* A = S.mem;
                const uint64_t o_x = w_bytes, o_z = o_x + (uint64_t)round_up(n * ld_xs * xb, 256);
                DGI_HIP(hipEventRecord(S.ev[0], sa));
                DGI_TRY(launch_permute_rows(static_cast<const char*>(cur) + (size_t)r0 * ld_cur * xb, ld_cur, A + o_x, ld_xs, n, Ly.in_dim, xb, nullptr, true, sa));
                DGI_HIP(hipEventRecord(S.ev[1], sa));
                DGI_HIP(hipStreamWaitEvent(sb, S.ev[1], 0));
                DGI_TRY(layer_transform_rows(g, &Ly, A + o_x, ld_xs, n, A + o_z, A, sb));
                DGI_HIP(hipEventRecord(S.ev[2], sb));
                DGI_TRY(store_rows(A + o_z, ti.z_ld, z_host + (size_t)r0 * ti.z_ld * zb, z_dev + (size_t)r0 * ti.z_ld * zb, ti.z_ld, n, ti.z_cols, zb, sb));
                DGI_HIP(hipEventRecord(S.ev[3], sb));
                S.pending = true; S.dense = true; S.layer = l; S.n_sub = 0; S.rows = n;
                S.M_k = o_z + (uint64_t)n * ti.z_ld * zb;
                S.in_bytes = n * (int64_t)Ly.in_dim * xb; S.out_bytes = n * (int64_t)ti.z_cols * zb;
                ++k;
            }
            for (int i = 0; i < n_slots; ++i) DGI_TRY(slot[i].retire(hs));  // the batches read all of Z
            z_rows = z_dev;
            f_src = z_dev; f_ld = ti.z_ld; f_lds = ti.z_ld; f_eb = zb;
            f_width = (int)ti.z_ld;  // whole padded rows: 16-byte pieces over the link (the padding columns are never read)
            if (ti.has_self) { f_src = z_dev + (size_t)ti.z_neigh_col * zb; f_lds = ld_zn; f_width = (int)ld_zn; }
        }

        int64_t n_t = o.batch_size > 0 ? o.batch_size : (all_fits ? N : (o.init_node_threshold > 0 ? o.init_node_threshold : 65536));
        int64_t n_i = (o.batch_size > 0 || all_fits) ? INT64_MAX / 4
                                       : (o.init_edge_threshold > 0 ? o.init_edge_threshold : (int64_t)std::max(1.0, (double)n_t * std::max(avg_deg, 1.0)));
        const double row_now = (double)f_lds * f_eb;
        if (o.batch_size == 0 && !all_fits && carry_nt > 0) {
            const double sc_rows = carry_row / row_now;
            n_t = (int64_t)std::min(4.0e18, std::max(1.0, (double)carry_nt * sc_rows));
            n_i = (int64_t)std::min(4.0e18, std::max(1.0, (double)carry_ni * sc_rows));
        }
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
            Slot& S = slot[k % n_slots];
            DGI_TRY(S.retire(hs));  // its previous batch (n_slots batches ago) must have left the slot
            // ---- (i) input set, on the first stream ---------------------------------------------------------------
            DGI_HIP(hipEventRecord(S.ev[0], sa));
            hipLaunchKernelGGL(batch_depth_kernel, dim3(grid_for(N)), dim3(kBlock), 0, sa, depth.as<int32_t>(), N, b, e);
            if (e_b > 0)
                hipLaunchKernelGGL(mark_sources_kernel, dim3(grid_for(e_b)), dim3(kBlock), 0, sa, g->d_indices, g->h_indptr[b], g->h_indptr[e], depth.as<int32_t>());
            int64_t n_sub = 0;
            DGI_TRY(sc.count_level(depth.as<int32_t>(), N, 0, &n_sub, sa));
            // ---- device memory of this batch (M_k), carved from the slot -------------------------------------------------
            uint64_t off = 0;
            auto carve = [&](uint64_t bytes) { const uint64_t at = off; off += (uint64_t)round_up((int64_t)std::max<uint64_t>(bytes, 16), 256); return at; };
            const uint64_t o_idx = carve((uint64_t)e_b * 4), o_ptr = carve((uint64_t)(n_sub + 1) * 8), o_deg = carve((uint64_t)(n_sub + 1) * 8);
            const uint64_t o_U = carve((uint64_t)n_sub * 4), o_x = carve((uint64_t)n_sub * f_lds * f_eb), o_y = carve((uint64_t)rows * ld_os * yb);
            const bool split_z = two_pass && ti.has_self;
            const uint64_t o_zs = carve(split_z ? (uint64_t)rows * ld_zn * zb : 0);  // z_self of the batch's own rows
            if (off > M) { DGI_TRY(shrink()); continue; }
            char* A = S.mem;
            int64_t e_sub = 0;
            DGI_TRY(sub_rows<IdxT>(g, depth.as<int32_t>(), sc, n_sub, (int32_t*)(A + o_U), (int64_t*)(A + o_deg), (int64_t*)(A + o_ptr), &e_sub, sa));
            DGI_REQUIRE(e_sub == e_b, DGI_ERR_DEVICE, "infer_host: sub-problem has %lld edges, expected %lld", (long long)e_sub, (long long)e_b);
            DGI_TRY(sub_graph<IdxT>(g, sc, n_sub, e_sub, (const int32_t*)(A + o_U), (const int64_t*)(A + o_ptr), (int32_t*)(A + o_idx), &S.sub, sa));
            // the batch's rows are one run of local ids: [lb, lb + rows)
            int32_t lb = 0;
            DGI_HIP(hipMemcpyAsync(&lb, sc.loc.as<int32_t>() + b, 4, hipMemcpyDeviceToHost, sa));
            DGI_HIP(hipStreamSynchronize(sa));
            uint64_t ws_bytes = 0;
            if (two_pass) ws_bytes = layer_aggregate_temp_bytes(S.sub.g, &Ly, lb, lb + rows);
            else DGI_TRY(dgi_layer_workspace_bytes(S.sub.g, &Ly, lb, lb + rows, &ws_bytes));
            const uint64_t o_ws = carve(ws_bytes);
            const uint64_t M_k = off + S.sub.g->device_bytes;
            if (M_k > M) { S.sub.reset(); DGI_TRY(shrink()); continue; }
            // ---- (ii) rows of the input set, read from host memory by the device --------------------------------------
            DGI_TRY(launch_permute_rows(f_src, f_ld, A + o_x, f_lds, n_sub, f_width, f_eb, (const int32_t*)(A + o_U), true, sa));
            if (split_z)
                DGI_TRY(launch_permute_rows(z_rows + (size_t)b * ti.z_ld * zb, ti.z_ld, A + o_zs, ld_zn, rows, (int)ld_zn, zb,
                                            nullptr, true, sa));
            DGI_HIP(hipEventRecord(S.ev[1], sa));
            // ---- (iii) the layer on the sub-problem, on the second stream; the output buffer starts at row lb ----------------
            DGI_HIP(hipStreamWaitEvent(sb, S.ev[1], 0));
            if (split_z)
                DGI_TRY(layer_aggregate_rows_split(S.sub.g, &Ly, A + o_x, ld_zn, A + o_zs, ld_zn, A + o_y, ld_os, lb, lb, lb + rows, A + o_ws, ws_bytes, sb));
            else if (two_pass) DGI_TRY(layer_aggregate_rows(S.sub.g, &Ly, A + o_x, A + o_y, ld_os, lb, lb, lb + rows, A + o_ws, ws_bytes, sb));
            else DGI_TRY(layer_forward_rows(S.sub.g, &Ly, A + o_x, ld_xs, A + o_y, ld_os, lb, lb, lb + rows, A + o_ws, ws_bytes, sb));
            DGI_HIP(hipEventRecord(S.ev[2], sb));
            // ---- (iv) dump the batch's rows ------------------------------------------------------------------------------
            DGI_TRY(store_rows(A + o_y, ld_os, dst_host + (size_t)b * ld_dst * yb, dst_dev + (size_t)b * ld_dst * yb, ld_dst, rows, Ly.out_dim, yb, sb));
            DGI_HIP(hipEventRecord(S.ev[3], sb));
            S.pending = true; S.dense = false; S.layer = l; S.n_sub = n_sub; S.rows = rows; S.M_k = M_k;
            S.in_bytes = n_sub * (int64_t)f_width * f_eb + (split_z ? rows * ld_zn * zb : 0); S.out_bytes = rows * (int64_t)Ly.out_dim * yb;
            if (o.batch_size == 0 && !all_fits) {
                if (2 * M_k >= M) { carry_nt = n_t; carry_ni = n_i; carry_row = row_now; }
                DGI_TRY(dgi_threshold_update((double)M, (double)M_k, &n_t, &n_i));  // Eq. 2
            }
            b = e;
            ++k;
        }
        // layer l+1 reads what layer l dumped: both slots must have stored their batches.  H^{l-1} is dead from
        // here on: its buffer takes H^{l+1}.
        for (int i = 0; i < n_slots; ++i) DGI_TRY(slot[i].retire(hs));
        cur = dst_dev;
        ld_cur = ld_dst;
    }
    if (hs) hs->total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_start).count();
    return DGI_OK;
}

}  // namespace
}  // namespace dgi

using namespace dgi;

extern "C" dgi_status_t dgi_host_alloc(uint64_t bytes, void** ptr) {
    DGI_REQUIRE(ptr != nullptr, DGI_ERR_INVALID_ARG, "host_alloc: NULL argument");
    *ptr = nullptr;
    const hipError_t e = hipHostMalloc(ptr, (size_t)std::max<uint64_t>(bytes, 16), hipHostMallocDefault);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *ptr = nullptr;
        set_error("host_alloc: %llu bytes of page-locked memory: %s", (unsigned long long)bytes, hipGetErrorString(e));
        return DGI_ERR_OOM;
    }
    return DGI_OK;
}

extern "C" dgi_status_t dgi_host_free(void* ptr) {
    if (ptr) DGI_HIP(hipHostFree(ptr));
    return DGI_OK;
}

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
