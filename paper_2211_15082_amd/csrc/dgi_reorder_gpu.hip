// Device side of node reordering (Section 4.2 of the DGI paper): the permutation itself is computed on the GPU.
//
//  DEGREE : stable radix sort of the node ids by descending in-degree.
//  BFS_RCM: level-synchronous Cuthill-McKee on the undirected structure, reversed at the end.  It yields
//           exactly the order of the sequential algorithm in dgi_reorder.cpp: a newly reached node belongs to
//           the frontier node with the smallest position that touches it (atomicMin on the parent position),
//           the children of a level are ordered by (parent position, undirected degree, id) with two stable
//           radix sorts, and every component starts at the unvisited node of smallest (degree, id).  After
//           kMaxBfsComponents components the remaining nodes are appended in (degree, id) order, as on the host.
//
//  COMMUNITY: label propagation (one wavefront per node: the labels of up to 64 neighbours at a time are counted
//           against each other with lane broadcasts), then a stable radix sort of the ids by label.  Follows the rule
//           stated in dgi_reorder.cpp exactly.
//
// Out-neighbour lists come from a radix sort of the edges by source (the CSR only stores in-neighbours).
#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <climits>
#include <vector>

#include "dgi_internal.h"

namespace dgi {
namespace {

constexpr int kBlock = 256;
inline unsigned blocks_for(int64_t n, int64_t cap = (int64_t)1 << 22) {
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + kBlock - 1) / kBlock, cap));
}

template <typename IdxT>
__global__ void in_degree_keys_kernel(const IdxT* indptr, int64_t N, uint32_t* key, int32_t* id) {
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < N; v += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t d = (uint32_t)(indptr[v + 1] - indptr[v]);
        key[v] = ~d;  // ascending sort of ~d = descending degree
        id[v] = (int32_t)v;
    }
}

__global__ void invert_order_kernel(const int32_t* order, int64_t N, int32_t* perm, int reverse) {
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < N; r += (int64_t)gridDim.x * blockDim.x)
        perm[order[r]] = (int32_t)(reverse ? N - 1 - r : r);
}

// dst[e] = destination row of stored edge e (one wavefront per row)
template <typename IdxT>
__global__ void edge_rows_kernel(const IdxT* indptr, int64_t N, int32_t* dst) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; v < N; v += waves) {
        const int64_t a = (int64_t)indptr[v], b = (int64_t)indptr[v + 1];
        for (int64_t e = a + lane; e < b; e += 64) dst[e] = (int32_t)v;
    }
}

template <typename IdxT>
__global__ void undirected_degree_kernel(const IdxT* indptr, const int32_t* deg_out, int64_t N, uint32_t* udeg, int32_t* id,
                                         int64_t* out_cnt) {
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < N; v += (int64_t)gridDim.x * blockDim.x) {
        udeg[v] = (uint32_t)(indptr[v + 1] - indptr[v]) + (uint32_t)deg_out[v];
        id[v] = (int32_t)v;
        out_cnt[v] = deg_out[v];
    }
}

__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t value) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = value;
}

// first index >= cursor in by_degree whose node is unvisited (pos < 0); result via atomicMin
__global__ void first_unvisited_kernel(const int32_t* by_degree, const int32_t* pos, int64_t N, int64_t cursor, unsigned long long* result) {
    for (int64_t i = cursor + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (int64_t)gridDim.x * blockDim.x) {
        if (pos[by_degree[i]] < 0) { atomicMin(result, (unsigned long long)i); return; }  // later indices of this thread are larger
    }
}

__global__ void frontier_degrees_kernel(const int32_t* frontier, int64_t nf, const uint32_t* udeg, int64_t* cnt) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nf) cnt[i] = udeg[frontier[i]];
}

// One wavefront per frontier node: list its in- and out-neighbours as candidates and bid for the unvisited ones.
template <typename IdxT>
__global__ void expand_kernel(const int32_t* frontier, int64_t nf, int64_t base, const int64_t* offs, const IdxT* indptr,
                              const int32_t* indices, const int64_t* out_ptr, const int32_t* out_idx, const int32_t* pos,
                              int32_t* best, int32_t* cand, int32_t* cand_parent) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; i < nf; i += waves) {
        const int64_t x = frontier[i];
        const int32_t p = (int32_t)(base + i);
        const int64_t ia = (int64_t)indptr[x], ib = (int64_t)indptr[x + 1];
        const int64_t oa = out_ptr[x], ob = out_ptr[x + 1];
        const int64_t o = offs[i];
        for (int64_t j = lane; j < (ib - ia) + (ob - oa); j += 64) {
            const int32_t y = j < ib - ia ? indices[ia + j] : out_idx[oa + (j - (ib - ia))];
            cand[o + j] = y;
            cand_parent[o + j] = p;
            if (pos[y] < 0) atomicMin(&best[y], p);
        }
    }
}

// A candidate wins if its parent is the smallest bidder; one of several identical (y, parent) slots is kept.
__global__ void claim_kernel(const int32_t* cand, const int32_t* cand_parent, int64_t nc, const int32_t* pos, const int32_t* best,
                             int32_t* claimed, uint8_t* flag) {
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < nc; s += (int64_t)gridDim.x * blockDim.x) {
        const int32_t y = cand[s];
        uint8_t f = 0;
        if (pos[y] < 0 && best[y] == cand_parent[s] && atomicCAS(&claimed[y], 0, 1) == 0) f = 1;
        flag[s] = f;
    }
}

__global__ void child_keys_kernel(const int32_t* child, int64_t n, const int32_t* best, const uint32_t* udeg, uint64_t* key) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) key[i] = ((uint64_t)(uint32_t)best[child[i]] << 32) | udeg[child[i]];
}

__global__ void assign_positions_kernel(const int32_t* nodes, int64_t n, int64_t base, int32_t* pos, int32_t* order) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { pos[nodes[i]] = (int32_t)(base + i); order[base + i] = nodes[i]; }
}

__global__ void unvisited_flags_kernel(const int32_t* by_degree, const int32_t* pos, int64_t N, uint8_t* flag) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += (int64_t)gridDim.x * blockDim.x)
        flag[i] = pos[by_degree[i]] < 0 ? 1 : 0;
}

struct DevBuf {
    void* p = nullptr;
    ~DevBuf() { (void)hipFree(p); }
    dgi_status_t alloc(size_t bytes) { DGI_HIP(hipMalloc(&p, std::max<size_t>(bytes, 16))); return DGI_OK; }
    template <typename T> T* as() { return static_cast<T*>(p); }
};

#define DGI_CUB(call)                                                                           \
    do {                                                                                        \
        hipError_t _e = (call);                                                                 \
        if (_e != hipSuccess) { set_error("%s failed: %s", #call, hipGetErrorString(_e)); return DGI_ERR_DEVICE; } \
    } while (0)

template <typename IdxT>
dgi_status_t degree_perm(const dgi_graph* g, int32_t* d_perm, hipStream_t s) {
    const int64_t N = g->N;
    DevBuf key, key2, id, id2, tmp;
    DGI_TRY(key.alloc(N * 4)); DGI_TRY(key2.alloc(N * 4)); DGI_TRY(id.alloc(N * 4)); DGI_TRY(id2.alloc(N * 4));
    hipLaunchKernelGGL(in_degree_keys_kernel<IdxT>, dim3(blocks_for(N)), dim3(kBlock), 0, s, (const IdxT*)g->d_indptr, N,
                       key.as<uint32_t>(), id.as<int32_t>());
    size_t tb = 0;
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(nullptr, tb, key.as<uint32_t>(), key2.as<uint32_t>(), id.as<int32_t>(), id2.as<int32_t>(), (int)N, 0, 32, s));
    DGI_TRY(tmp.alloc(tb));
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(tmp.p, tb, key.as<uint32_t>(), key2.as<uint32_t>(), id.as<int32_t>(), id2.as<int32_t>(), (int)N, 0, 32, s));
    hipLaunchKernelGGL(invert_order_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, id2.as<int32_t>(), N, d_perm, 0);
    DGI_HIP(hipGetLastError());
    DGI_HIP(hipStreamSynchronize(s));
    return DGI_OK;
}

template <typename IdxT>
dgi_status_t rcm_perm(const dgi_graph* g, int32_t* d_perm, hipStream_t s) {
    const int64_t N = g->N, E = g->E;
    DGI_REQUIRE(2 * E + 1 < (int64_t)INT_MAX && N < (int64_t)INT_MAX, DGI_ERR_UNSUPPORTED,
                "device BFS reordering handles up to 2^30 edges (32-bit item counts of the sort/scan primitives)");
    const IdxT* indptr = (const IdxT*)g->d_indptr;
    // ---- out-neighbour lists: sort the edges by source ---------------------------------------------------
    DevBuf dst, src_sorted, out_idx, out_cnt, out_ptr, udeg, udeg2, ids, by_degree, tmp;
    DGI_TRY(dst.alloc(E * 4)); DGI_TRY(src_sorted.alloc(E * 4)); DGI_TRY(out_idx.alloc(E * 4));
    DGI_TRY(out_cnt.alloc((N + 1) * 8)); DGI_TRY(out_ptr.alloc((N + 1) * 8));
    DGI_TRY(udeg.alloc(N * 4)); DGI_TRY(udeg2.alloc(N * 4)); DGI_TRY(ids.alloc(N * 4)); DGI_TRY(by_degree.alloc(N * 4));
    hipLaunchKernelGGL(edge_rows_kernel<IdxT>, dim3(blocks_for(N * 64)), dim3(kBlock), 0, s, indptr, N, dst.as<int32_t>());
    hipLaunchKernelGGL(undirected_degree_kernel<IdxT>, dim3(blocks_for(N)), dim3(kBlock), 0, s, indptr, g->d_deg_out, N,
                       udeg.as<uint32_t>(), ids.as<int32_t>(), out_cnt.as<int64_t>());
    size_t tb = 0, t2 = 0;
    int bits = 1;
    while (((int64_t)1 << bits) < N) ++bits;
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(nullptr, tb, g->d_indices, src_sorted.as<int32_t>(), dst.as<int32_t>(), out_idx.as<int32_t>(), (int)E, 0, bits, s));
    DGI_CUB(hipcub::DeviceScan::ExclusiveSum(nullptr, t2, out_cnt.as<int64_t>(), out_ptr.as<int64_t>(), (int)(N + 1), s));
    tb = std::max(tb, t2);
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(nullptr, t2, udeg.as<uint32_t>(), udeg2.as<uint32_t>(), ids.as<int32_t>(), by_degree.as<int32_t>(), (int)N, 0, 32, s));
    tb = std::max(tb, t2);
    // per-level scratch is bounded by all candidates of a level (<= 2E) and all nodes
    const int64_t maxc = 2 * E + 1;
    DGI_CUB(hipcub::DeviceScan::ExclusiveSum(nullptr, t2, (int64_t*)nullptr, (int64_t*)nullptr, (int)(N + 1), s));
    tb = std::max(tb, t2);
    DGI_CUB(hipcub::DeviceSelect::Flagged(nullptr, t2, (int32_t*)nullptr, (uint8_t*)nullptr, (int32_t*)nullptr, (int64_t*)nullptr, (int)std::min<int64_t>(maxc, INT_MAX), s));
    tb = std::max(tb, t2);
    DGI_CUB(hipcub::DeviceRadixSort::SortKeys(nullptr, t2, (int32_t*)nullptr, (int32_t*)nullptr, (int)N, 0, bits, s));
    tb = std::max(tb, t2);
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(nullptr, t2, (uint64_t*)nullptr, (uint64_t*)nullptr, (int32_t*)nullptr, (int32_t*)nullptr, (int)N, 0, 64, s));
    tb = std::max(tb, t2);
    DGI_TRY(tmp.alloc(tb));
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(tmp.p, tb, g->d_indices, src_sorted.as<int32_t>(), dst.as<int32_t>(), out_idx.as<int32_t>(), (int)E, 0, bits, s));
    DGI_CUB(hipcub::DeviceScan::ExclusiveSum(tmp.p, tb, out_cnt.as<int64_t>(), out_ptr.as<int64_t>(), (int)(N + 1), s));
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(tmp.p, tb, udeg.as<uint32_t>(), udeg2.as<uint32_t>(), ids.as<int32_t>(), by_degree.as<int32_t>(), (int)N, 0, 32, s));
    (void)hipFree(dst.p); dst.p = nullptr;
    (void)hipFree(src_sorted.p); src_sorted.p = nullptr;

    // ---- breadth-first enumeration -------------------------------------------------------------------------
    DevBuf pos, best, claimed, order, cnt, offs, cand, cand_parent, flag, child, child2, ckey, ckey2, nsel, first;
    DGI_TRY(pos.alloc(N * 4)); DGI_TRY(best.alloc(N * 4)); DGI_TRY(claimed.alloc(N * 4)); DGI_TRY(order.alloc(N * 4));
    DGI_TRY(cnt.alloc((N + 1) * 8)); DGI_TRY(offs.alloc((N + 1) * 8));
    DGI_TRY(cand.alloc(maxc * 4)); DGI_TRY(cand_parent.alloc(maxc * 4)); DGI_TRY(flag.alloc(std::max<int64_t>(maxc, N)));
    DGI_TRY(child.alloc(N * 4)); DGI_TRY(child2.alloc(N * 4)); DGI_TRY(ckey.alloc(N * 8)); DGI_TRY(ckey2.alloc(N * 8));
    DGI_TRY(nsel.alloc(8)); DGI_TRY(first.alloc(8));
    hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, pos.as<int32_t>(), N, -1);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, best.as<int32_t>(), N, INT_MAX);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, claimed.as<int32_t>(), N, 0);
    int64_t done = 0, cursor = 0;
    int32_t* frontier = child.as<int32_t>();   // current frontier lives in `order` itself: order[base .. base+nf)
    (void)frontier;
    for (int comp = 0; comp < kMaxBfsComponents && done < N; ++comp) {
        unsigned long long h_first = ~0ull;
        DGI_HIP(hipMemcpyAsync(first.p, &h_first, 8, hipMemcpyHostToDevice, s));
        hipLaunchKernelGGL(first_unvisited_kernel, dim3(blocks_for(N - cursor, 1024)), dim3(kBlock), 0, s, by_degree.as<int32_t>(),
                           pos.as<int32_t>(), N, cursor, first.as<unsigned long long>());
        DGI_HIP(hipMemcpyAsync(&h_first, first.p, 8, hipMemcpyDeviceToHost, s));
        DGI_HIP(hipStreamSynchronize(s));
        if (h_first == ~0ull) break;
        cursor = (int64_t)h_first + 1;
        // the start node becomes a one-node frontier at position `done`
        hipLaunchKernelGGL(assign_positions_kernel, dim3(1), dim3(kBlock), 0, s, by_degree.as<int32_t>() + h_first, (int64_t)1, done,
                           pos.as<int32_t>(), order.as<int32_t>());
        int64_t base = done, nf = 1;
        done += 1;
        while (nf > 0) {
            const int32_t* F = order.as<int32_t>() + base;
            hipLaunchKernelGGL(frontier_degrees_kernel, dim3(blocks_for(nf + 1)), dim3(kBlock), 0, s, F, nf, udeg.as<uint32_t>(), cnt.as<int64_t>());
            DGI_CUB(hipcub::DeviceScan::ExclusiveSum(tmp.p, tb, cnt.as<int64_t>(), offs.as<int64_t>(), (int)(nf + 1), s));
            int64_t nc = 0;
            DGI_HIP(hipMemcpyAsync(&nc, offs.as<int64_t>() + nf, 8, hipMemcpyDeviceToHost, s));
            DGI_HIP(hipStreamSynchronize(s));
            if (nc == 0) break;
            DGI_REQUIRE(nc <= maxc, DGI_ERR_DEVICE, "bfs reorder: candidate buffer overflow");
            hipLaunchKernelGGL(expand_kernel<IdxT>, dim3(blocks_for(nf * 64)), dim3(kBlock), 0, s, F, nf, base, offs.as<int64_t>(), indptr,
                               g->d_indices, out_ptr.as<int64_t>(), out_idx.as<int32_t>(), pos.as<int32_t>(), best.as<int32_t>(),
                               cand.as<int32_t>(), cand_parent.as<int32_t>());
            hipLaunchKernelGGL(claim_kernel, dim3(blocks_for(nc)), dim3(kBlock), 0, s, cand.as<int32_t>(), cand_parent.as<int32_t>(), nc,
                               pos.as<int32_t>(), best.as<int32_t>(), claimed.as<int32_t>(), flag.as<uint8_t>());
            DGI_CUB(hipcub::DeviceSelect::Flagged(tmp.p, tb, cand.as<int32_t>(), flag.as<uint8_t>(), child.as<int32_t>(), nsel.as<int64_t>(), (int)nc, s));
            int64_t nn = 0;
            DGI_HIP(hipMemcpyAsync(&nn, nsel.p, 8, hipMemcpyDeviceToHost, s));
            DGI_HIP(hipStreamSynchronize(s));
            if (nn == 0) break;
            // order the children by (parent position, degree, id): sort by id, then stably by the 64-bit key
            DGI_CUB(hipcub::DeviceRadixSort::SortKeys(tmp.p, tb, child.as<int32_t>(), child2.as<int32_t>(), (int)nn, 0, bits, s));
            hipLaunchKernelGGL(child_keys_kernel, dim3(blocks_for(nn)), dim3(kBlock), 0, s, child2.as<int32_t>(), nn, best.as<int32_t>(),
                               udeg.as<uint32_t>(), ckey.as<uint64_t>());
            DGI_CUB(hipcub::DeviceRadixSort::SortPairs(tmp.p, tb, ckey.as<uint64_t>(), ckey2.as<uint64_t>(), child2.as<int32_t>(), child.as<int32_t>(), (int)nn, 0, 64, s));
            hipLaunchKernelGGL(assign_positions_kernel, dim3(blocks_for(nn)), dim3(kBlock), 0, s, child.as<int32_t>(), nn, done,
                               pos.as<int32_t>(), order.as<int32_t>());
            DGI_HIP(hipGetLastError());
            base = done;
            nf = nn;
            done += nn;
        }
    }
    if (done < N) {  // leftovers in (degree, id) order
        hipLaunchKernelGGL(unvisited_flags_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, by_degree.as<int32_t>(), pos.as<int32_t>(), N, flag.as<uint8_t>());
        DGI_CUB(hipcub::DeviceSelect::Flagged(tmp.p, tb, by_degree.as<int32_t>(), flag.as<uint8_t>(), order.as<int32_t>() + done, nsel.as<int64_t>(), (int)N, s));
        int64_t nn = 0;
        DGI_HIP(hipMemcpyAsync(&nn, nsel.p, 8, hipMemcpyDeviceToHost, s));
        DGI_HIP(hipStreamSynchronize(s));
        DGI_REQUIRE(done + nn == N, DGI_ERR_DEVICE, "bfs reorder: %lld nodes enumerated, %lld expected", (long long)(done + nn), (long long)N);
    }
    hipLaunchKernelGGL(invert_order_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, order.as<int32_t>(), N, d_perm, 1);
    DGI_HIP(hipGetLastError());
    DGI_HIP(hipStreamSynchronize(s));
    return DGI_OK;
}

__global__ void iota_i32_kernel(int32_t* p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = (int32_t)i;
}

// One round of label propagation, one wavefront per node.  Nodes whose id has the parity of `round` take the most
// frequent label among their in- and out-neighbours (64 at a time, see dgi_reorder.cpp for the exact rule).
template <typename IdxT>
__global__ __launch_bounds__(256) void label_round_kernel(const IdxT* indptr, const int32_t* indices, const int64_t* out_ptr,
                                                          const int32_t* out_idx, int64_t N, const int32_t* lab, int32_t* nxt, int round) {
    const int lane = threadIdx.x & 63;
    const int64_t waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; v < N; v += waves) {
        if (((v ^ round) & 1) != 0) {
            if (lane == 0) nxt[v] = lab[v];
            continue;
        }
        const int64_t ia = (int64_t)indptr[v], din = (int64_t)indptr[v + 1] - ia;
        const int64_t oa = out_ptr[v], total = din + (out_ptr[v + 1] - oa);
        int32_t best = -1;
        int64_t cnt = 0;
        for (int64_t base = 0; base < total; base += 64) {
            const int64_t j = base + lane;
            const bool has = j < total;
            int32_t l = -1;
            if (has) l = lab[j < din ? indices[ia + j] : out_idx[oa + (j - din)]];
            int c = 0;
#pragma unroll
            for (int k = 0; k < 64; ++k) c += (__builtin_amdgcn_readlane(l, k) == l) ? 1 : 0;
            // largest count wins, ties go to the smallest label: maximise (count, 0x7fffffff - label)
            unsigned long long key = has ? (((unsigned long long)c << 32) | (unsigned)(0x7fffffff - l)) : 0ull;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)key, off, 64), hi = (unsigned)__shfl_xor((int)(unsigned)(key >> 32), off, 64);
                const unsigned long long other = ((unsigned long long)hi << 32) | lo;
                key = other > key ? other : key;
            }
            const int32_t w = (int32_t)(0x7fffffff - (unsigned)key);
            const int64_t cw = (int64_t)(key >> 32);
            if (w == best) cnt += cw;
            else if (cw > cnt) { best = w; cnt = cw; }
        }
        if (lane == 0) nxt[v] = total > 0 ? best : lab[v];
    }
}

template <typename IdxT>
dgi_status_t community_perm(const dgi_graph* g, int32_t* d_perm, hipStream_t s) {
    const int64_t N = g->N, E = g->E;
    DGI_REQUIRE(E + 1 < (int64_t)INT_MAX && N < (int64_t)INT_MAX, DGI_ERR_UNSUPPORTED,
                "device community reordering handles up to 2^31 edges (32-bit item counts of the sort/scan primitives)");
    const IdxT* indptr = (const IdxT*)g->d_indptr;
    DevBuf dst, src_sorted, out_idx, out_cnt, out_ptr, lab, nxt, ids, ids2, tmp;
    DGI_TRY(dst.alloc(E * 4)); DGI_TRY(src_sorted.alloc(E * 4)); DGI_TRY(out_idx.alloc(E * 4));
    DGI_TRY(out_cnt.alloc((N + 1) * 8)); DGI_TRY(out_ptr.alloc((N + 1) * 8));
    DGI_TRY(lab.alloc(N * 4)); DGI_TRY(nxt.alloc(N * 4)); DGI_TRY(ids.alloc(N * 4)); DGI_TRY(ids2.alloc(N * 4));
    // out-neighbour lists: a stable sort of the edges by source keeps each list in ascending destination id
    hipLaunchKernelGGL(edge_rows_kernel<IdxT>, dim3(blocks_for(N * 64)), dim3(kBlock), 0, s, indptr, N, dst.as<int32_t>());
    hipLaunchKernelGGL(undirected_degree_kernel<IdxT>, dim3(blocks_for(N)), dim3(kBlock), 0, s, indptr, g->d_deg_out, N,
                       nxt.as<uint32_t>(), ids.as<int32_t>(), out_cnt.as<int64_t>());
    size_t tb = 0, t2 = 0;
    int bits = 1;
    while (((int64_t)1 << bits) < N) ++bits;
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(nullptr, tb, g->d_indices, src_sorted.as<int32_t>(), dst.as<int32_t>(), out_idx.as<int32_t>(), (int)E, 0, bits, s));
    DGI_CUB(hipcub::DeviceScan::ExclusiveSum(nullptr, t2, out_cnt.as<int64_t>(), out_ptr.as<int64_t>(), (int)(N + 1), s));
    tb = std::max(tb, t2);
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(nullptr, t2, lab.as<int32_t>(), nxt.as<int32_t>(), ids.as<int32_t>(), ids2.as<int32_t>(), (int)N, 0, bits, s));
    tb = std::max(tb, t2);
    DGI_TRY(tmp.alloc(tb));
    if (E) DGI_CUB(hipcub::DeviceRadixSort::SortPairs(tmp.p, tb, g->d_indices, src_sorted.as<int32_t>(), dst.as<int32_t>(), out_idx.as<int32_t>(), (int)E, 0, bits, s));
    DGI_CUB(hipcub::DeviceScan::ExclusiveSum(tmp.p, tb, out_cnt.as<int64_t>(), out_ptr.as<int64_t>(), (int)(N + 1), s));
    (void)hipFree(dst.p); dst.p = nullptr;
    (void)hipFree(src_sorted.p); src_sorted.p = nullptr;
    hipLaunchKernelGGL(iota_i32_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, lab.as<int32_t>(), N);
    int32_t *a = lab.as<int32_t>(), *b = nxt.as<int32_t>();
    for (int r = 0; r < DGI_COMMUNITY_ROUNDS; ++r) {
        hipLaunchKernelGGL(label_round_kernel<IdxT>, dim3(blocks_for(N * 64)), dim3(kBlock), 0, s, indptr, g->d_indices, out_ptr.as<int64_t>(),
                           out_idx.as<int32_t>(), N, a, b, r);
        std::swap(a, b);
    }
    DGI_HIP(hipGetLastError());
    // ids by (label, old id): stable sort of 0..N-1 by label
    hipLaunchKernelGGL(iota_i32_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, ids.as<int32_t>(), N);
    DGI_CUB(hipcub::DeviceRadixSort::SortPairs(tmp.p, tb, a, b, ids.as<int32_t>(), ids2.as<int32_t>(), (int)N, 0, bits, s));
    hipLaunchKernelGGL(invert_order_kernel, dim3(blocks_for(N)), dim3(kBlock), 0, s, ids2.as<int32_t>(), N, d_perm, 0);
    DGI_HIP(hipGetLastError());
    DGI_HIP(hipStreamSynchronize(s));
    return DGI_OK;
}

}  // namespace

dgi_status_t reorder_permutation_device(const dgi_graph* g, int method, int32_t* d_perm, hipStream_t stream) {
    if (g->N == 0) return DGI_OK;
    const bool i64 = g->itype == DGI_I64;
    if (method == DGI_REORDER_DEGREE) return i64 ? degree_perm<int64_t>(g, d_perm, stream) : degree_perm<int32_t>(g, d_perm, stream);
    if (method == DGI_REORDER_BFS_RCM) return i64 ? rcm_perm<int64_t>(g, d_perm, stream) : rcm_perm<int32_t>(g, d_perm, stream);
    if (method == DGI_REORDER_COMMUNITY) return i64 ? community_perm<int64_t>(g, d_perm, stream) : community_perm<int32_t>(g, d_perm, stream);
    set_error("device reordering implements DEGREE, BFS_RCM and COMMUNITY only");
    return DGI_ERR_UNSUPPORTED;
}

}  // namespace dgi
