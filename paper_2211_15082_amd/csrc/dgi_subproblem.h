// Extraction of a compact sub-problem from a graph: a node set U (ascending ids, relabelled 0..|U|-1), the
// complete in-neighbour lists of some of its rows, and the full graph's GCN normalisers.  Used by partial
// inference (Section 3.3: the rows of V^1 over the inputs V^0) and by host-resident inference (Algorithm 2:
// one batch of destination rows over its input set).  Internal to libdgi; every translation unit that includes
// this header gets its own copy of the kernels.
#pragma once

#include <hipcub/hipcub.hpp>

#include <algorithm>

#include "dgi_internal.h"

namespace dgi {
namespace subp {

constexpr int kBlock = 256;
inline unsigned grid_for(int64_t n) { return (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + kBlock - 1) / kBlock, (int64_t)1 << 22)); }

#define DGI_CUB(call)                                                                                              \
    do {                                                                                                           \
        hipError_t _e = (call);                                                                                    \
        if (_e != hipSuccess) { set_error("%s failed: %s", #call, hipGetErrorString(_e)); return DGI_ERR_DEVICE; } \
    } while (0)

struct Buf {
    void* p = nullptr;
    Buf() = default;
    Buf(const Buf&) = delete;
    Buf& operator=(const Buf&) = delete;
    ~Buf() { (void)hipFree(p); }
    dgi_status_t alloc(size_t bytes) { DGI_HIP(hipMalloc(&p, std::max<size_t>(bytes, 16))); return DGI_OK; }
    template <typename T> T* as() { return static_cast<T*>(p); }
};

struct GraphGuard {
    dgi_graph_t* g = nullptr;
    ~GraphGuard() { dgi_graph_free(g); }
    void reset() { dgi_graph_free(g); g = nullptr; }
};

static __global__ void fill_i32_kernel(int32_t* a, int64_t N, int32_t value) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (int64_t)gridDim.x * blockDim.x) a[i] = value;
}

static __global__ void level_flags_kernel(const int32_t* depth, int64_t N, int32_t l, int32_t* flag) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (int64_t)gridDim.x * blockDim.x)
        flag[i] = depth[i] >= l ? 1 : 0;
}

// per kept node (local id i, global id U[i]): its in-degree if the row keeps its list (depth >= keep_depth), else 0
template <typename IdxT>
static __global__ void sub_rows_kernel(const int32_t* U, int64_t n_sub, const IdxT* indptr, const int32_t* depth, int32_t keep_depth,
                                       int64_t* sub_deg) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_sub; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t v = U[i];
        sub_deg[i] = depth[v] >= keep_depth ? (int64_t)(indptr[v + 1] - indptr[v]) : 0;
    }
}

// one wavefront per kept row: copy its list, relabelled (order preserved, so sums keep their order)
template <typename IdxT>
static __global__ void sub_indices_kernel(const int32_t* U, int64_t n_sub, const IdxT* indptr, const int32_t* indices,
                                          const int64_t* sub_indptr, const int32_t* loc, int32_t* sub_indices) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; i < n_sub; i += waves) {
        const int64_t a = sub_indptr[i], d = sub_indptr[i + 1] - a;
        const int64_t src = (int64_t)indptr[U[i]];
        for (int64_t j = lane; j < d; j += 64) sub_indices[a + j] = loc[indices[src + j]];
    }
}

static __global__ void gather_f32_kernel(const float* in, const int32_t* idx, int64_t n, float* out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) out[i] = in[idx[i]];
}

// N-sized scratch shared by the steps below: flag (node is in U), loc (exclusive scan of flag = local id),
// a device counter and hipCUB's temporary storage.
struct Scratch {
    Buf flag, loc, tmp, cnt;
    size_t tb = 0;
    dgi_status_t alloc(int64_t N, hipStream_t s) {
        DGI_TRY(flag.alloc(N * 4)); DGI_TRY(loc.alloc((N + 1) * 4)); DGI_TRY(cnt.alloc(8));
        size_t t2 = 0;
        DGI_CUB(hipcub::DeviceReduce::Sum(nullptr, tb, flag.as<int32_t>(), cnt.as<int32_t>(), (int)N, s));
        DGI_CUB(hipcub::DeviceScan::ExclusiveSum(nullptr, t2, flag.as<int32_t>(), loc.as<int32_t>(), (int)N, s));
        tb = std::max(tb, t2);
        DGI_CUB(hipcub::DeviceSelect::Flagged(nullptr, t2, hipcub::CountingInputIterator<int32_t>(0), flag.as<int32_t>(), (int32_t*)nullptr, cnt.as<int32_t>(), (int)N, s));
        tb = std::max(tb, t2);
        DGI_CUB(hipcub::DeviceScan::InclusiveSum(nullptr, t2, (int64_t*)nullptr, (int64_t*)nullptr, (int)N, s));
        tb = std::max(tb, t2);
        DGI_TRY(tmp.alloc(tb));
        return DGI_OK;
    }
    // flag[i] = depth[i] >= l; returns the number of set flags (synchronises the stream)
    dgi_status_t count_level(const int32_t* depth, int64_t N, int32_t l, int64_t* n_out, hipStream_t s) {
        hipLaunchKernelGGL(level_flags_kernel, dim3(grid_for(N)), dim3(kBlock), 0, s, depth, N, l, flag.as<int32_t>());
        DGI_CUB(hipcub::DeviceReduce::Sum(tmp.p, tb, flag.as<int32_t>(), cnt.as<int32_t>(), (int)N, s));
        int32_t c = 0;
        DGI_HIP(hipMemcpyAsync(&c, cnt.p, 4, hipMemcpyDeviceToHost, s));
        DGI_HIP(hipStreamSynchronize(s));
        *n_out = c;
        return DGI_OK;
    }
};

// Step 1.  With sc.flag = (depth >= 0) and n_sub its population: U (ascending ids), sc.loc (local ids) and the
// sub-problem's indptr (int64, n_sub + 1 entries).  Returns its edge count (synchronises the stream).
template <typename IdxT>
dgi_status_t sub_rows(const dgi_graph* g, const int32_t* depth, Scratch& sc, int64_t n_sub, int32_t* U, int64_t* sub_deg,
                      int64_t* sub_indptr, int64_t* e_sub, hipStream_t s) {
    const int64_t N = g->N;
    DGI_CUB(hipcub::DeviceScan::ExclusiveSum(sc.tmp.p, sc.tb, sc.flag.as<int32_t>(), sc.loc.as<int32_t>(), (int)N, s));
    DGI_CUB(hipcub::DeviceSelect::Flagged(sc.tmp.p, sc.tb, hipcub::CountingInputIterator<int32_t>(0), sc.flag.as<int32_t>(), U, sc.cnt.as<int32_t>(), (int)N, s));
    hipLaunchKernelGGL(sub_rows_kernel<IdxT>, dim3(grid_for(n_sub)), dim3(kBlock), 0, s, U, n_sub, (const IdxT*)g->d_indptr, depth, 1, sub_deg);
    DGI_TRY(launch_fill_zero(sub_indptr, 8, s));
    DGI_CUB(hipcub::DeviceScan::InclusiveSum(sc.tmp.p, sc.tb, sub_deg, sub_indptr + 1, (int)n_sub, s));
    DGI_HIP(hipMemcpyAsync(e_sub, sub_indptr + n_sub, 8, hipMemcpyDeviceToHost, s));
    DGI_HIP(hipStreamSynchronize(s));
    return DGI_OK;
}

// Step 2.  Relabelled neighbour lists into sub_indices (e_sub entries), a graph handle over the borrowed
// arrays, and the full graph's normalisers d_out^-1/2, d_in^-1/2 for the kept nodes.
template <typename IdxT>
dgi_status_t sub_graph(const dgi_graph* g, Scratch& sc, int64_t n_sub, int64_t e_sub, const int32_t* U, const int64_t* sub_indptr,
                       int32_t* sub_indices, GraphGuard* sub, hipStream_t s) {
    hipLaunchKernelGGL(sub_indices_kernel<IdxT>, dim3(grid_for(n_sub * 64)), dim3(kBlock), 0, s, U, n_sub, (const IdxT*)g->d_indptr, g->d_indices,
                       sub_indptr, sc.loc.as<int32_t>(), sub_indices);
    DGI_HIP(hipGetLastError());
    DGI_TRY(dgi_graph_load(n_sub, e_sub, sub_indptr, DGI_I64, sub_indices, DGI_DEVICE, s, &sub->g));
    hipLaunchKernelGGL(gather_f32_kernel, dim3(grid_for(n_sub)), dim3(kBlock), 0, s, g->d_rs_out, U, n_sub, sub->g->d_rs_out);
    hipLaunchKernelGGL(gather_f32_kernel, dim3(grid_for(n_sub)), dim3(kBlock), 0, s, g->d_rs_in, U, n_sub, sub->g->d_rs_in);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

}  // namespace subp
}  // namespace dgi
