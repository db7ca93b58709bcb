// Graph handle: device CSR keyed by destination (row v = in-neighbours N(v) of Eq. 1), degree vectors,
// the hub-row list used by the aggregation kernels, and the device side of node reordering (Section 4.2).
#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <cmath>
#include <cstring>

#include "dgi_internal.h"

namespace dgi {
namespace {

__global__ void check_and_count_kernel(const int32_t* indices, int64_t E, int64_t N, int32_t* deg_out, int* bad) {
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < E; e += (int64_t)gridDim.x * blockDim.x) {
        const int32_t u = indices[e];
        if (u < 0 || u >= N) { *bad = 1; continue; }
        atomicAdd(&deg_out[u], 1);  // integer atomics: order-independent result
    }
}

template <typename IdxT>
__global__ void inv_sqrt_degrees_kernel(const IdxT* indptr, const int32_t* deg_out, int64_t N, float* rs_in, float* rs_out) {
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= N) return;
    const float din = (float)(indptr[v + 1] - indptr[v]);
    const float dout = (float)deg_out[v];
    rs_in[v] = 1.0f / sqrtf(din < 1.f ? 1.f : din);
    rs_out[v] = 1.0f / sqrtf(dout < 1.f ? 1.f : dout);
}

// new row r = old row old_of_new[r]; sources relabelled through perm_new_of_old
template <typename IdxT>
__global__ void relabel_rows_kernel(const IdxT* indptr_old, const int32_t* indices_old, const IdxT* indptr_new,
                                    const int32_t* old_of_new, const int32_t* perm_new_of_old, int64_t N, int32_t* indices_new) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; r < N; r += waves) {
        const int64_t o = old_of_new[r];
        const int64_t src = (int64_t)indptr_old[o], dst = (int64_t)indptr_new[r];
        const int64_t deg = (int64_t)indptr_old[o + 1] - src;
        for (int64_t i = lane; i < deg; i += 64) indices_new[dst + i] = perm_new_of_old[indices_old[src + i]];
    }
}

template <typename T>
dgi_status_t dev_alloc(T** p, uint64_t count, dgi_graph* g) {
    *p = nullptr;
    const uint64_t bytes = std::max<uint64_t>(count, 1) * sizeof(T);
    DGI_HIP(hipMalloc(reinterpret_cast<void**>(p), bytes));
    g->device_bytes += bytes;
    return DGI_OK;
}

void find_hubs(dgi_graph* g) {
    g->h_hub_rows.clear();
    g->h_hub_chunk_ptr.assign(1, 0);
    g->max_in_degree = 0;
    for (int64_t v = 0; v < g->N; ++v) {
        const int64_t d = g->h_indptr[v + 1] - g->h_indptr[v];
        g->max_in_degree = std::max(g->max_in_degree, d);
        if (d > kHubDegree) {
            g->h_hub_rows.push_back(v);
            g->h_hub_chunk_ptr.push_back(g->h_hub_chunk_ptr.back() + (d + kHubChunk - 1) / kHubChunk);
        }
    }
}

// Shared tail of load / reorder: the handle already has N, E, itype, device CSR and h_indptr.
// Without count_out (library-built graphs only: their indices are known to be valid) the out-degrees are not counted
// and the handle refuses GCN layers.
dgi_status_t finish_graph(dgi_graph* g, hipStream_t stream, bool no_hubs = false, bool count_out = true, const int32_t* counted = nullptr,
                          void* node_vectors = nullptr) {
    g->has_out_degrees = count_out || counted != nullptr;
    if (node_vectors) {  // lent by the caller (a sampled graph lives for one layer: no allocation per layer)
        const uint64_t stride = (uint64_t)round_up(g->N * 4, 256);
        char* base = static_cast<char*>(node_vectors);
        g->d_deg_out = reinterpret_cast<int32_t*>(base);
        g->d_rs_in = reinterpret_cast<float*>(base + stride);
        g->d_rs_out = reinterpret_cast<float*>(base + 2 * stride);
        g->own_vectors = false;
    } else {
        DGI_TRY(dev_alloc(&g->d_deg_out, g->N, g));
        DGI_TRY(dev_alloc(&g->d_rs_in, g->N, g));
        DGI_TRY(dev_alloc(&g->d_rs_out, g->N, g));
    }
    int* d_bad = nullptr;
    DGI_HIP(hipMalloc(reinterpret_cast<void**>(&d_bad), sizeof(int)));
    dgi_status_t st = DGI_OK;
    int bad = 0;
    do {
        if ((st = launch_fill_zero(d_bad, sizeof(int), stream)) != DGI_OK) break;
        if (g->N > 0 && (st = launch_fill_zero(g->d_deg_out, (uint64_t)g->N * 4, stream)) != DGI_OK) break;
        if (counted && g->N > 0) {
            const hipError_t ce = hipMemcpyAsync(g->d_deg_out, counted, (size_t)g->N * 4, hipMemcpyDeviceToDevice, stream);
            if (ce != hipSuccess) { set_error("graph setup failed: %s", hipGetErrorString(ce)); st = DGI_ERR_DEVICE; break; }
        } else if (g->E > 0 && count_out) {
            const int64_t blocks = std::min<int64_t>((g->E + 255) / 256, 65536);
            hipLaunchKernelGGL(check_and_count_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, g->d_indices, g->E, g->N,
                               g->d_deg_out, d_bad);
        }
        if (g->N > 0) {
            const unsigned blocks = (unsigned)((g->N + 255) / 256);
            if (g->itype == DGI_I64)
                hipLaunchKernelGGL(inv_sqrt_degrees_kernel<int64_t>, dim3(blocks), dim3(256), 0, stream,
                                   (const int64_t*)g->d_indptr, g->d_deg_out, g->N, g->d_rs_in, g->d_rs_out);
            else
                hipLaunchKernelGGL(inv_sqrt_degrees_kernel<int32_t>, dim3(blocks), dim3(256), 0, stream,
                                   (const int32_t*)g->d_indptr, g->d_deg_out, g->N, g->d_rs_in, g->d_rs_out);
        }
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) e = hipMemcpyAsync(&bad, d_bad, sizeof(int), hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) { set_error("graph setup failed: %s", hipGetErrorString(e)); st = DGI_ERR_DEVICE; }
    } while (0);
    (void)hipFree(d_bad);
    DGI_TRY(st);
    DGI_REQUIRE(bad == 0, DGI_ERR_BAD_GRAPH, "indices hold a value outside [0, num_nodes)");
    if (no_hubs) { g->h_hub_rows.clear(); g->h_hub_chunk_ptr.assign(1, 0); }
    else find_hubs(g);
    const size_t nh = g->h_hub_rows.size();
    DGI_TRY(dev_alloc(&g->d_hub_rows, nh, g));
    DGI_TRY(dev_alloc(&g->d_hub_chunk_ptr, nh + 1, g));
    if (nh) DGI_HIP(hipMemcpyAsync(g->d_hub_rows, g->h_hub_rows.data(), nh * 8, hipMemcpyHostToDevice, stream));
    DGI_HIP(hipMemcpyAsync(g->d_hub_chunk_ptr, g->h_hub_chunk_ptr.data(), (nh + 1) * 8, hipMemcpyHostToDevice, stream));
    DGI_HIP(hipStreamSynchronize(stream));
    return DGI_OK;
}

dgi_status_t validate_indptr(const dgi_graph* g) {
    const auto& ip = g->h_indptr;
    DGI_REQUIRE(ip[0] == 0, DGI_ERR_BAD_GRAPH, "indptr[0] is %lld, expected 0", (long long)ip[0]);
    for (int64_t v = 0; v < g->N; ++v)
        DGI_REQUIRE(ip[v + 1] >= ip[v], DGI_ERR_BAD_GRAPH, "indptr decreases at row %lld", (long long)v);
    DGI_REQUIRE(ip[g->N] == g->E, DGI_ERR_BAD_GRAPH, "indptr[N] is %lld but num_edges is %lld", (long long)ip[g->N], (long long)g->E);
    return DGI_OK;
}

}  // namespace

// A handle over device arrays the library built itself (int64 indptr), taking the host copy of indptr and, with
// own_arrays, the device arrays too: no download, no validation of indptr.  With max_degree >= 0 and no hub rows
// possible the host scan for hubs is skipped as well; without count_out_degrees the count of out-degrees (one integer
// atomic per edge) is skipped too, and the handle then serves every aggregation but GCN.  On failure nothing is adopted: the caller still owns the arrays.
dgi_status_t graph_adopt(int64_t N, int64_t E, int64_t* d_indptr, int32_t* d_indices, std::vector<int64_t>&& h_indptr, int64_t max_degree,
                         bool own_arrays, bool count_out_degrees, hipStream_t stream, dgi_graph_t** out, const int32_t* counted_out_degrees, void* node_vectors) {
    dgi_graph* g = new dgi_graph();
    g->N = N; g->E = E; g->itype = DGI_I64;
    (void)hipGetDevice(&g->device);
    g->d_indptr = d_indptr; g->d_indices = d_indices; g->own_csr = false;
    g->device_bytes = (uint64_t)(N + 1) * 8 + (uint64_t)E * 4;
    g->h_indptr = std::move(h_indptr);
    const bool skip_hub_scan = max_degree >= 0 && max_degree <= kHubDegree;
    dgi_status_t st = finish_graph(g, stream, skip_hub_scan, count_out_degrees, counted_out_degrees, node_vectors);
    if (st != DGI_OK) { h_indptr = std::move(g->h_indptr); dgi_graph_free(g); return st; }
    if (skip_hub_scan) g->max_in_degree = max_degree;
    g->own_csr = own_arrays;
    *out = g;
    return DGI_OK;
}

}  // namespace dgi

using namespace dgi;

extern "C" dgi_status_t dgi_graph_free(dgi_graph_t* g) {
    if (!g) return DGI_OK;
    if (g->own_csr) {
        (void)hipFree(const_cast<void*>(g->d_indptr));
        (void)hipFree(const_cast<int32_t*>(g->d_indices));
    }
    if (g->own_vectors) {
        (void)hipFree(g->d_deg_out);
        (void)hipFree(g->d_rs_in);
        (void)hipFree(g->d_rs_out);
    }
    (void)hipFree(g->d_hub_rows);
    (void)hipFree(g->d_hub_chunk_ptr);
    (void)hipFree(g->ws_ptr);
    (void)hipFree(g->hs_arena);
    (void)hipHostFree(g->hs_hid[0]);
    (void)hipHostFree(g->hs_hid[1]);
    (void)hipHostFree(g->hs_z);
    (void)hipFree(g->ss_d_ip);
    (void)hipFree(g->ss_d_ix);
    (void)hipFree(g->ss_d_tmp);
    (void)hipFree(g->ss_d_deg);
    (void)hipFree(g->ss_d_vec);
    delete g;
    return DGI_OK;
}

extern "C" dgi_status_t dgi_graph_load(int64_t num_nodes, int64_t num_edges, const void* indptr, int32_t indptr_type,
                                       const int32_t* indices, int32_t where, void* hip_stream, dgi_graph_t** out) {
    DGI_REQUIRE(out != nullptr, DGI_ERR_INVALID_ARG, "graph_load: out is NULL");
    *out = nullptr;
    DGI_REQUIRE(num_nodes >= 0 && num_edges >= 0, DGI_ERR_INVALID_ARG, "graph_load: negative size");
    DGI_REQUIRE(num_nodes < ((int64_t)1 << 31) - 1, DGI_ERR_UNSUPPORTED, "graph_load: node ids must fit int32");
    DGI_REQUIRE(indptr != nullptr, DGI_ERR_INVALID_ARG, "graph_load: indptr is NULL");
    DGI_REQUIRE(indices != nullptr || num_edges == 0, DGI_ERR_INVALID_ARG, "graph_load: indices is NULL");
    DGI_REQUIRE(indptr_type == DGI_I32 || indptr_type == DGI_I64, DGI_ERR_INVALID_ARG, "graph_load: bad indptr_type");
    DGI_REQUIRE(where == DGI_HOST || where == DGI_DEVICE, DGI_ERR_INVALID_ARG, "graph_load: bad memory location");
    DGI_REQUIRE(indptr_type == DGI_I64 || num_edges < ((int64_t)1 << 31), DGI_ERR_INVALID_ARG,
                "graph_load: int32 indptr cannot address %lld edges", (long long)num_edges);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    dgi_graph* g = new dgi_graph();
    g->N = num_nodes; g->E = num_edges; g->itype = indptr_type;
    (void)hipGetDevice(&g->device);
    const size_t isz = indptr_type == DGI_I64 ? 8 : 4;
    const size_t ip_bytes = (size_t)(num_nodes + 1) * isz;
    std::vector<char> raw(ip_bytes);
    dgi_status_t st = DGI_OK;
    auto fail = [&](dgi_status_t s) { dgi_graph_free(g); return s; };
    if (where == DGI_HOST) {
        std::memcpy(raw.data(), indptr, ip_bytes);
        void* dip = nullptr; int32_t* dix = nullptr;
        if ((st = dev_alloc(reinterpret_cast<char**>(&dip), ip_bytes, g)) != DGI_OK) return fail(st);
        g->d_indptr = dip; g->own_csr = true;
        if ((st = dev_alloc(&dix, (uint64_t)num_edges, g)) != DGI_OK) return fail(st);
        g->d_indices = dix;
        hipError_t e = hipMemcpyAsync(dip, indptr, ip_bytes, hipMemcpyHostToDevice, stream);
        if (e == hipSuccess && num_edges) e = hipMemcpyAsync(dix, indices, (size_t)num_edges * 4, hipMemcpyHostToDevice, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) { set_error("graph_load: upload failed: %s", hipGetErrorString(e)); return fail(DGI_ERR_DEVICE); }
    } else {
        g->d_indptr = indptr; g->d_indices = indices; g->own_csr = false;
        hipError_t e = hipMemcpyAsync(raw.data(), indptr, ip_bytes, hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) { set_error("graph_load: indptr download failed: %s", hipGetErrorString(e)); return fail(DGI_ERR_DEVICE); }
    }
    g->h_indptr.resize((size_t)num_nodes + 1);
    if (indptr_type == DGI_I64) std::memcpy(g->h_indptr.data(), raw.data(), ip_bytes);
    else for (int64_t i = 0; i <= num_nodes; ++i) g->h_indptr[i] = reinterpret_cast<const int32_t*>(raw.data())[i];
    raw.clear(); raw.shrink_to_fit();
    if ((st = validate_indptr(g)) != DGI_OK) return fail(st);
    if ((st = finish_graph(g, stream)) != DGI_OK) return fail(st);
    *out = g;
    return DGI_OK;
}

extern "C" dgi_status_t dgi_graph_info(const dgi_graph_t* g, dgi_graph_info_t* info) {
    DGI_REQUIRE(g && info, DGI_ERR_INVALID_ARG, "graph_info: NULL argument");
    info->num_nodes = g->N; info->num_edges = g->E; info->max_in_degree = g->max_in_degree;
    info->num_hub_rows = (int64_t)g->h_hub_rows.size();
    info->num_hub_edges = 0;
    for (int64_t v : g->h_hub_rows) info->num_hub_edges += g->h_indptr[v + 1] - g->h_indptr[v]; info->indptr_type = g->itype; info->reserved = 0;
    info->device_bytes = g->device_bytes;
    return DGI_OK;
}

extern "C" dgi_status_t dgi_graph_vector(const dgi_graph_t* g, int32_t kind, void* dst) {
    DGI_REQUIRE(g && dst, DGI_ERR_INVALID_ARG, "graph_vector: NULL argument");
    if (g->N == 0) return DGI_OK;
    if (kind == 0) {
        int32_t* d = static_cast<int32_t*>(dst);
        for (int64_t v = 0; v < g->N; ++v) d[v] = (int32_t)(g->h_indptr[v + 1] - g->h_indptr[v]);
        return DGI_OK;
    }
    const void* src = kind == 1 ? (const void*)g->d_deg_out : kind == 2 ? (const void*)g->d_rs_in : kind == 3 ? (const void*)g->d_rs_out : nullptr;
    DGI_REQUIRE(src, DGI_ERR_INVALID_ARG, "graph_vector: unknown kind %d", kind);
    DGI_HIP(hipMemcpy(dst, src, (size_t)g->N * 4, hipMemcpyDeviceToHost));
    return DGI_OK;
}

extern "C" dgi_status_t dgi_graph_csr(const dgi_graph_t* g, int64_t* indptr, int32_t* indices) {
    DGI_REQUIRE(g && indptr && (indices || g->E == 0), DGI_ERR_INVALID_ARG, "graph_csr: NULL argument");
    std::memcpy(indptr, g->h_indptr.data(), (size_t)(g->N + 1) * 8);
    if (g->E) DGI_HIP(hipMemcpy(indices, g->d_indices, (size_t)g->E * 4, hipMemcpyDeviceToHost));
    return DGI_OK;
}

extern "C" dgi_status_t dgi_graph_reorder(const dgi_graph_t* g, int32_t method, uint64_t seed, void* hip_stream,
                                          dgi_graph_t** g_out, int32_t* perm_out, int32_t perm_where) {
    DGI_REQUIRE(g && g_out && perm_out, DGI_ERR_INVALID_ARG, "graph_reorder: NULL argument");
    *g_out = nullptr;
    DGI_REQUIRE(perm_where == DGI_HOST || perm_where == DGI_DEVICE, DGI_ERR_INVALID_ARG, "graph_reorder: bad perm location");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t N = g->N, E = g->E;
    std::vector<int32_t> perm((size_t)std::max<int64_t>(N, 1)), old_of_new((size_t)std::max<int64_t>(N, 1));
    int32_t* d_perm = nullptr;
    DGI_HIP(hipMalloc((void**)&d_perm, std::max<size_t>(N, 1) * 4));
    struct FreeOnExit { int32_t*& p; ~FreeOnExit() { (void)hipFree(p); p = nullptr; } } perm_guard{d_perm};
    // the permutation: on the device for DEGREE / BFS_RCM, on the host otherwise (and beyond the device limits)
    dgi_status_t pst = DGI_ERR_UNSUPPORTED;
    if (method == DGI_REORDER_DEGREE || method == DGI_REORDER_BFS_RCM || method == DGI_REORDER_COMMUNITY)
        pst = reorder_permutation_device(g, method, d_perm, stream);
    if (pst == DGI_OK) {
        if (N) DGI_HIP(hipMemcpy(perm.data(), d_perm, (size_t)N * 4, hipMemcpyDeviceToHost));
    } else if (pst == DGI_ERR_UNSUPPORTED) {
        std::vector<int32_t> h_indices((size_t)std::max<int64_t>(E, 1));
        if (E) DGI_HIP(hipMemcpy(h_indices.data(), g->d_indices, (size_t)E * 4, hipMemcpyDeviceToHost));
        DGI_TRY(reorder_permutation(N, g->h_indptr.data(), h_indices.data(), method, seed, perm.data()));
        if (N) DGI_HIP(hipMemcpy(d_perm, perm.data(), (size_t)N * 4, hipMemcpyHostToDevice));
    } else {
        return pst;
    }
    for (int64_t o = 0; o < N; ++o) old_of_new[perm[o]] = (int32_t)o;

    dgi_graph* ng = new dgi_graph();
    ng->N = N; ng->E = E; ng->itype = g->itype; ng->device = g->device; ng->own_csr = true;
    ng->h_indptr.assign((size_t)N + 1, 0);
    for (int64_t r = 0; r < N; ++r) {
        const int64_t o = old_of_new[r];
        ng->h_indptr[r + 1] = ng->h_indptr[r] + (g->h_indptr[o + 1] - g->h_indptr[o]);
    }
    dgi_status_t st = DGI_OK;
    int32_t *d_oon = nullptr, *d_unsorted = nullptr;
    void* d_tmp = nullptr;
    auto cleanup = [&]() { (void)hipFree(d_oon); (void)hipFree(d_unsorted); (void)hipFree(d_tmp); d_oon = d_unsorted = nullptr; d_tmp = nullptr; };
    auto fail = [&](dgi_status_t s) { cleanup(); dgi_graph_free(ng); return s; };
    const size_t isz = g->itype == DGI_I64 ? 8 : 4;
    void* dip = nullptr; int32_t* dix = nullptr;
    if ((st = dev_alloc(reinterpret_cast<char**>(&dip), (uint64_t)(N + 1) * isz, ng)) != DGI_OK) return fail(st);
    ng->d_indptr = dip;
    if ((st = dev_alloc(&dix, (uint64_t)E, ng)) != DGI_OK) return fail(st);
    ng->d_indices = dix;
    auto chk = [&](hipError_t e, const char* what) {
        if (e != hipSuccess) { set_error("graph_reorder: %s failed: %s", what, hipGetErrorString(e)); return false; }
        return true;
    };
    if (!chk(hipMalloc((void**)&d_oon, std::max<size_t>(N, 1) * 4), "alloc") ||
        !chk(hipMalloc((void**)&d_unsorted, std::max<size_t>(E, 1) * 4), "alloc"))
        return fail(DGI_ERR_DEVICE);
    if (g->itype == DGI_I64) {
        if (!chk(hipMemcpyAsync(dip, ng->h_indptr.data(), (N + 1) * 8, hipMemcpyHostToDevice, stream), "upload")) return fail(DGI_ERR_DEVICE);
    } else {
        std::vector<int32_t> ip32((size_t)N + 1);
        for (int64_t i = 0; i <= N; ++i) ip32[i] = (int32_t)ng->h_indptr[i];
        if (!chk(hipMemcpyAsync(dip, ip32.data(), (N + 1) * 4, hipMemcpyHostToDevice, stream), "upload") ||
            !chk(hipStreamSynchronize(stream), "sync"))
            return fail(DGI_ERR_DEVICE);
    }
    if (N) {
        if (!chk(hipMemcpyAsync(d_oon, old_of_new.data(), N * 4, hipMemcpyHostToDevice, stream), "upload"))
            return fail(DGI_ERR_DEVICE);
        const int64_t blocks = std::min<int64_t>((N * 64 + 255) / 256, (int64_t)1 << 22);  // < 2^32 threads per launch
        if (g->itype == DGI_I64)
            hipLaunchKernelGGL(relabel_rows_kernel<int64_t>, dim3((unsigned)blocks), dim3(256), 0, stream, (const int64_t*)g->d_indptr,
                               g->d_indices, (const int64_t*)dip, d_oon, d_perm, N, d_unsorted);
        else
            hipLaunchKernelGGL(relabel_rows_kernel<int32_t>, dim3((unsigned)blocks), dim3(256), 0, stream, (const int32_t*)g->d_indptr,
                               g->d_indices, (const int32_t*)dip, d_oon, d_perm, N, d_unsorted);
        if (!chk(hipGetLastError(), "relabel launch")) return fail(DGI_ERR_DEVICE);
    }
    if (E) {
        // sort every new row by source id (segmented radix sort; segment offsets are the new indptr)
        size_t tmp_bytes = 0;
        hipError_t e;
        const int bits = 32;
        if (g->itype == DGI_I64)
            e = hipcub::DeviceSegmentedRadixSort::SortKeys(nullptr, tmp_bytes, d_unsorted, dix, E, N, (const int64_t*)dip, (const int64_t*)dip + 1, 0, bits, stream);
        else
            e = hipcub::DeviceSegmentedRadixSort::SortKeys(nullptr, tmp_bytes, d_unsorted, dix, E, N, (const int32_t*)dip, (const int32_t*)dip + 1, 0, bits, stream);
        if (!chk(e, "segmented sort sizing") || !chk(hipMalloc(&d_tmp, std::max<size_t>(tmp_bytes, 16)), "alloc")) return fail(DGI_ERR_DEVICE);
        if (g->itype == DGI_I64)
            e = hipcub::DeviceSegmentedRadixSort::SortKeys(d_tmp, tmp_bytes, d_unsorted, dix, E, N, (const int64_t*)dip, (const int64_t*)dip + 1, 0, bits, stream);
        else
            e = hipcub::DeviceSegmentedRadixSort::SortKeys(d_tmp, tmp_bytes, d_unsorted, dix, E, N, (const int32_t*)dip, (const int32_t*)dip + 1, 0, bits, stream);
        if (!chk(e, "segmented sort")) return fail(DGI_ERR_DEVICE);
    }
    if (perm_where == DGI_DEVICE) {
        if (N && !chk(hipMemcpyAsync(perm_out, d_perm, N * 4, hipMemcpyDeviceToDevice, stream), "perm copy")) return fail(DGI_ERR_DEVICE);
    } else {
        std::memcpy(perm_out, perm.data(), (size_t)N * 4);
    }
    if (!chk(hipStreamSynchronize(stream), "sync")) return fail(DGI_ERR_DEVICE);
    cleanup();
    if ((st = finish_graph(ng, stream)) != DGI_OK) { dgi_graph_free(ng); return st; }
    *g_out = ng;
    return DGI_OK;
}
