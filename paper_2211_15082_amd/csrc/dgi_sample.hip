// Sampling inference (Section 2 of the DGI paper: every node aggregates a sampled subset of its in-neighbours,
// fan-out 10 in the paper's experiments).  Each layer draws its own sample; layer-wise execution then runs the
// ordinary schedule on the sampled graph, so a node still reads 1-hop inputs only.
//
// Sampling rule: a row with at most `fanout` in-edges keeps them all; otherwise it keeps the `fanout` edges with
// the smallest keys, in stored order.  The key of the edge at position e of `indices` in layer l is the upper 32
// bits of output number l*E + e + 1 of SplitMix64 (Steele, Lea, Flood 2014) seeded with `seed`; equal keys are
// ordered by position in the row.  The keys are a counter-based function of (seed, layer, e), so the sample does
// not depend on scheduling, and a host implementation of the same rule reproduces it exactly.
#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <climits>
#include <mutex>
#include <thread>
#include <utility>
#include <vector>

#include "dgi_internal.h"

namespace dgi {
namespace {

__device__ __forceinline__ uint64_t splitmix64_output(uint64_t seed, uint64_t k) {
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * k;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// One wavefront (= one workgroup) per destination row, rows strided over the grid.  A long row finds its
// fanout-th smallest (key, position) pair by an 8-pass radix select over the 64-bit pair (a 256-bin histogram in
// LDS per pass), then keeps the pairs up to that threshold with an order-preserving wave compaction.
template <typename IdxT>
__global__ __launch_bounds__(64) void sample_rows_kernel(const IdxT* indptr, const int32_t* indices, int64_t N, int fanout, uint64_t seed,
                                                         uint64_t key_base /* l*E + 1 */, const int64_t* new_indptr, int32_t* new_indices,
                                                         int32_t* deg_out /* NULL, or zeroed: out-degrees of the sample are counted here */) {
    __shared__ uint32_t hist[256];
    const int lane = threadIdx.x;
    for (int64_t v = blockIdx.x; v < N; v += gridDim.x) {
        const int64_t a = (int64_t)indptr[v], d = (int64_t)indptr[v + 1] - a, o = new_indptr[v];
        if (d <= fanout) {
            for (int64_t j = lane; j < d; j += 64) {
                const int32_t u = indices[a + j];
                new_indices[o + j] = u;
                if (deg_out) atomicAdd(&deg_out[u], 1);  // integer atomics: order-independent result
            }
            continue;
        }
        auto value = [&](int64_t j) { return (splitmix64_output(seed, key_base + (uint64_t)(a + j)) & 0xFFFFFFFF00000000ull) | (uint64_t)j; };
        if (d <= 64) {  // the whole row sits in the wavefront: rank every value against the others
            const uint64_t mine = lane < d ? value(lane) : ~0ull;
            int rank = 0;
            for (int i = 0; i < (int)d; ++i) {
                const uint64_t other = ((uint64_t)__shfl((uint32_t)(mine >> 32), i, 64) << 32) | (uint32_t)i;  // the low half is the position
                rank += other < mine ? 1 : 0;
            }
            const bool keep = lane < d && rank < fanout;
            const unsigned long long m = __ballot(keep);
            if (keep) {
                const int32_t u = indices[a + lane];
                new_indices[o + __popcll(m & ((1ull << lane) - 1ull))] = u;
                if (deg_out) atomicAdd(&deg_out[u], 1);
            }
            continue;
        }
        uint64_t prefix = 0;  // the bytes of the threshold found so far (the high ones)
        uint32_t need = (uint32_t)fanout;  // rank of the threshold among the values that share `prefix`
        for (int p = 7; p >= 0; --p) {
            for (int i = lane; i < 256; i += 64) hist[i] = 0u;
            __syncthreads();
            for (int64_t j = lane; j < d; j += 64) {
                const uint64_t val = value(j);
                if (p == 7 || (val >> (8 * (p + 1))) == prefix) atomicAdd(&hist[(val >> (8 * p)) & 255u], 1u);
            }
            __syncthreads();
            const uint32_t c0 = hist[4 * lane], c1 = hist[4 * lane + 1], c2 = hist[4 * lane + 2], c3 = hist[4 * lane + 3];
            const uint32_t mine = c0 + c1 + c2 + c3;
            uint32_t incl = mine;
#pragma unroll
            for (int sft = 1; sft < 64; sft <<= 1) {
                const uint32_t up = __shfl_up(incl, sft, 64);
                if (lane >= sft) incl += up;
            }
            const uint32_t excl = incl - mine;
            // exactly one lane holds the bucket where the running count reaches `need`
            const bool here = excl < need && need <= incl;
            uint32_t bucket = 0, below = 0;
            if (here) {
                uint32_t run = excl;
                if (run + c0 >= need) { bucket = 4 * lane; below = run; }
                else if ((run += c0) + c1 >= need) { bucket = 4 * lane + 1; below = run; }
                else if ((run += c1) + c2 >= need) { bucket = 4 * lane + 2; below = run; }
                else { run += c2; bucket = 4 * lane + 3; below = run; }
            }
            const unsigned long long m = __ballot(here);
            const int src = __ffsll((long long)m) - 1;
            bucket = __shfl(bucket, src, 64);
            below = __shfl(below, src, 64);
            need -= below;
            prefix = (prefix << 8) | bucket;
            __syncthreads();
        }
        // prefix is now the fanout-th smallest value: keep what does not exceed it, in stored order
        int64_t base = o;
        for (int64_t j0 = 0; j0 < d; j0 += 64) {
            const int64_t j = j0 + lane;
            const bool keep = j < d && value(j) <= prefix;
            const unsigned long long m = __ballot(keep);
            const int64_t at = base + __popcll(m & ((1ull << lane) - 1ull));
            if (keep && at < o + fanout) {  // (exactly fanout values pass; the bound keeps a row inside its slots regardless)
                const int32_t u = indices[a + j];
                new_indices[at] = u;
                if (deg_out) atomicAdd(&deg_out[u], 1);
            }
            base += __popcll(m);
        }
    }
}

// in-degrees of the sample, as int64, at out[1 + v] (out[0] = 0): the input of the device prefix sum
template <typename IdxT>
__global__ void min_degree_kernel(const IdxT* indptr, int64_t N, int fanout, int64_t* out) {
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v <= N; v += (int64_t)gridDim.x * blockDim.x) {
        if (v == N) { out[0] = 0; continue; }
        const int64_t d = (int64_t)indptr[v + 1] - (int64_t)indptr[v];
        out[v + 1] = d < fanout ? d : fanout;
    }
}

// The sampled graph of one layer.  With `cached` the host indptr vector and the device arrays come from (and stay
// in) g's handle and the new handle borrows the device arrays; the caller must hold g->hs_mutex and hand the host
// vector back (g->ss_ip = std::move(sampled->h_indptr)) before freeing the sampled handle.
dgi_status_t sample_graph(const dgi_graph* g, int fanout, uint64_t seed, int layer, bool cached, bool count_out_degrees, hipStream_t s, dgi_graph_t** g_out) {
    const int64_t N = g->N;
    // host indptr of the sample = prefix sums of min(degree, fanout), in parallel chunks (the handle keeps a host copy
    // for batch planning); the device copy is computed on the device, so nothing crosses the host link
    // (the sample's indptr depends on the degrees and the fan-out only: with `cached`, a call with the fan-out of the
    // previous one reuses both copies — for 111 M rows the host prefix sums were 18 of a layer's 42 ms of sampling)
    std::vector<int64_t> ip;
    if (cached) ip = std::move(g->ss_ip);
    const bool reuse_ip = cached && g->ss_ip_fanout == fanout && ip.size() == (size_t)N + 1 && g->ss_d_ip != nullptr;
    if (cached) g->ss_ip_fanout = -1;  // set again once this call has succeeded
    ip.resize((size_t)N + 1);
    ip[0] = 0;
    if (!reuse_ip) {
        const int T = (int)std::max<int64_t>(1, std::min<int64_t>({(int64_t)std::thread::hardware_concurrency(), (int64_t)16, N / 65536 + 1}));
        std::vector<int64_t> chunk_sum((size_t)T + 1, 0);
        auto range = [&](int t) { return std::make_pair(N * t / T, N * (t + 1) / T); };
        auto run = [&](auto&& fn) {
            std::vector<std::thread> th;
            for (int t = 1; t < T; ++t) th.emplace_back(fn, t);
            fn(0);
            for (auto& x : th) x.join();
        };
        run([&](int t) {
            const auto r = range(t);
            int64_t sum = 0;
            for (int64_t v = r.first; v < r.second; ++v) sum += std::min<int64_t>(g->h_indptr[v + 1] - g->h_indptr[v], fanout);
            chunk_sum[t + 1] = sum;
        });
        for (int t = 0; t < T; ++t) chunk_sum[t + 1] += chunk_sum[t];
        run([&](int t) {
            const auto r = range(t);
            int64_t acc = chunk_sum[t];
            for (int64_t v = r.first; v < r.second; ++v) { acc += std::min<int64_t>(g->h_indptr[v + 1] - g->h_indptr[v], fanout); ip[v + 1] = acc; }
        });
    }
    const int64_t Es = ip[N];
    auto give_back = [&]() { if (cached) g->ss_ip = std::move(ip); };
    int64_t* d_ip = cached ? g->ss_d_ip : nullptr;
    int32_t* d_ix = cached ? g->ss_d_ix : nullptr;
    void* d_tmp = cached ? g->ss_d_tmp : nullptr;  // (cached: no allocation or release per call once the buffers exist)
    // GCN reads the sample's out-degrees: the sampling kernel counts them while it writes the kept edges (the
    // atomics hide behind its own latency-bound work; a separate pass over the sampled edges took as long as the sampling)
    int32_t* d_deg = (cached && count_out_degrees) ? g->ss_d_deg : nullptr;
    auto fail = [&](dgi_status_t st) {
        if (!cached) { (void)hipFree(d_tmp); (void)hipFree(d_deg); (void)hipFree(d_ip); (void)hipFree(d_ix); }
        give_back();
        return st;
    };
    hipError_t err = hipSuccess;
    if (!d_ip) {
        err = hipMalloc(reinterpret_cast<void**>(&d_ip), (size_t)(N + 1) * 8);
        if (err == hipSuccess && cached) g->ss_d_ip = d_ip;
    }
    if (err == hipSuccess && (!d_ix || (cached && g->ss_ix_cap < (uint64_t)Es))) {
        if (cached) { (void)hipFree(g->ss_d_ix); g->ss_d_ix = nullptr; g->ss_ix_cap = 0; }
        err = hipMalloc(reinterpret_cast<void**>(&d_ix), std::max<size_t>((size_t)Es * 4, 16));
        if (err == hipSuccess && cached) { g->ss_d_ix = d_ix; g->ss_ix_cap = (uint64_t)std::max<int64_t>(Es, 4); }
    }
    size_t tmp_bytes = 0;
    if (err == hipSuccess) err = hipcub::DeviceScan::InclusiveSum(nullptr, tmp_bytes, d_ip, d_ip, (int)(N + 1), s);
    if (err == hipSuccess && (!d_tmp || (cached && g->ss_tmp_cap < tmp_bytes))) {
        if (cached) { (void)hipFree(g->ss_d_tmp); g->ss_d_tmp = nullptr; g->ss_tmp_cap = 0; }
        err = hipMalloc(&d_tmp, std::max<size_t>(tmp_bytes, 16));
        if (err == hipSuccess && cached) { g->ss_d_tmp = d_tmp; g->ss_tmp_cap = std::max<size_t>(tmp_bytes, 16); }
    }
    if (err == hipSuccess && cached && !g->ss_d_vec)  // the N-vectors of the sampled handle, lent for its one layer
        err = hipMalloc(reinterpret_cast<void**>(&g->ss_d_vec), (size_t)(3 * round_up(N * 4, 256) + 256));
    if (err == hipSuccess && count_out_degrees && !d_deg) {
        err = hipMalloc(reinterpret_cast<void**>(&d_deg), std::max<size_t>((size_t)N * 4, 16));
        if (err == hipSuccess && cached) g->ss_d_deg = d_deg;
    }
    if (err != hipSuccess) { set_error("graph_sample: %s", hipGetErrorString(err)); return fail(err == hipErrorOutOfMemory ? DGI_ERR_OOM : DGI_ERR_DEVICE); }
    if (d_deg && N > 0) {
        const dgi_status_t zs = launch_fill_zero(d_deg, (uint64_t)N * 4, s);
        if (zs != DGI_OK) return fail(zs);
    }
    {
        const unsigned grid1 = (unsigned)std::min<int64_t>((N + 256) / 256, (int64_t)1 << 20);
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(N, (int64_t)1 << 22));
        const uint64_t key_base = (uint64_t)layer * (uint64_t)g->E + 1ull;
        if (g->itype == DGI_I64) {
            if (!reuse_ip) {
                hipLaunchKernelGGL(min_degree_kernel<int64_t>, dim3(grid1), dim3(256), 0, s, (const int64_t*)g->d_indptr, N, fanout, d_ip);
                err = hipcub::DeviceScan::InclusiveSum(d_tmp, tmp_bytes, d_ip, d_ip, (int)(N + 1), s);
            }
            if (err == hipSuccess && N > 0)
                hipLaunchKernelGGL(sample_rows_kernel<int64_t>, dim3(grid), dim3(64), 0, s, (const int64_t*)g->d_indptr, g->d_indices, N, fanout, seed, key_base,
                                   d_ip, d_ix, d_deg);
        } else {
            if (!reuse_ip) {
                hipLaunchKernelGGL(min_degree_kernel<int32_t>, dim3(grid1), dim3(256), 0, s, (const int32_t*)g->d_indptr, N, fanout, d_ip);
                err = hipcub::DeviceScan::InclusiveSum(d_tmp, tmp_bytes, d_ip, d_ip, (int)(N + 1), s);
            }
            if (err == hipSuccess && N > 0)
                hipLaunchKernelGGL(sample_rows_kernel<int32_t>, dim3(grid), dim3(64), 0, s, (const int32_t*)g->d_indptr, g->d_indices, N, fanout, seed, key_base,
                                   d_ip, d_ix, d_deg);
        }
        if (err == hipSuccess) err = hipGetLastError();
    }
    if (err == hipSuccess) err = hipStreamSynchronize(s);
    if (err != hipSuccess) { set_error("graph_sample: %s", hipGetErrorString(err)); return fail(DGI_ERR_DEVICE); }
    if (!cached) (void)hipFree(d_tmp);
    d_tmp = nullptr;
    const dgi_status_t st = graph_adopt(N, Es, d_ip, d_ix, std::move(ip), std::min<int64_t>(g->max_in_degree, fanout), !cached, false, s, g_out, d_deg,
                                        cached ? g->ss_d_vec : nullptr);
    if (st != DGI_OK) return fail(st);  // graph_adopt handed `ip` back
    if (!cached) (void)hipFree(d_deg);  // copied into the new handle
    if (cached) g->ss_ip_fanout = fanout;
    return DGI_OK;
}

}  // namespace
}  // namespace dgi

using namespace dgi;

extern "C" dgi_status_t dgi_graph_sample(const dgi_graph_t* g, int32_t fanout, uint64_t seed, int32_t layer, void* hip_stream,
                                         dgi_graph_t** g_out) {
    DGI_REQUIRE(g && g_out, DGI_ERR_INVALID_ARG, "graph_sample: NULL argument");
    *g_out = nullptr;
    DGI_REQUIRE(fanout >= 1, DGI_ERR_INVALID_ARG, "graph_sample: fan-out must be at least 1");
    DGI_REQUIRE(layer >= 0 && layer < DGI_MAX_LAYERS, DGI_ERR_INVALID_ARG, "graph_sample: bad layer index");
    DGI_REQUIRE(g->N < (int64_t)INT_MAX - 1, DGI_ERR_UNSUPPORTED, "graph_sample: at most 2^31 - 3 nodes");
    return sample_graph(g, fanout, seed, layer, false, true, static_cast<hipStream_t>(hip_stream), g_out);
}

extern "C" dgi_status_t dgi_infer_sampled(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x, int64_t ld_x,
                                          void* out, int64_t ld_out, int32_t fanout, uint64_t seed, const dgi_infer_opts_t* opts,
                                          void* hip_stream) {
    DGI_REQUIRE(g && layers, DGI_ERR_INVALID_ARG, "infer_sampled: NULL argument");
    DGI_REQUIRE(num_layers >= 1 && num_layers <= DGI_MAX_LAYERS, DGI_ERR_INVALID_ARG, "infer_sampled: 1..%d layers supported", DGI_MAX_LAYERS);
    dgi_infer_opts_t o{};
    if (opts) o = *opts;
    DGI_REQUIRE(!o.perm_new_of_old && !o.jk_concat, DGI_ERR_UNSUPPORTED, "infer_sampled: permutation and jumping-knowledge options are not supported");
    DGI_REQUIRE(fanout >= 1, DGI_ERR_INVALID_ARG, "infer_sampled: fan-out must be at least 1");
    DGI_REQUIRE(g->N < (int64_t)INT_MAX - 1, DGI_ERR_UNSUPPORTED, "infer_sampled: at most 2^31 - 3 nodes");
    o.stats = nullptr;
    for (int l = 1; l < num_layers; ++l) {
        DGI_REQUIRE(layers[l].in_dim == layers[l - 1].out_dim, DGI_ERR_INVALID_ARG, "layer %d: in_dim != previous out_dim", l);
        DGI_REQUIRE(layers[l].feat_dtype == layers[l - 1].out_dtype, DGI_ERR_INVALID_ARG, "layer %d: feat_dtype != previous out_dtype", l);
    }
    const int64_t N = g->N;
    if (N == 0) return DGI_OK;
    DGI_REQUIRE(x && out, DGI_ERR_INVALID_ARG, "infer_sampled: NULL buffer");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // Hidden layers: two buffers carved from the device memory the handle keeps for dgi_infer_host (the two calls
    // exclude each other through hs_mutex), so repeated calls allocate nothing.
    std::lock_guard<std::mutex> hs_lock(g->hs_mutex);
    size_t hid_bytes = 256;
    for (int l = 0; l + 1 < num_layers; ++l) {
        const int eb = layers[l].out_dtype == DGI_BF16 ? 2 : 4;
        hid_bytes = std::max<size_t>(hid_bytes, (size_t)round_up((int64_t)((size_t)N * (size_t)round_up(layers[l].out_dim, 16 / eb) * eb), 256));
    }
    const int n_hidden = std::min(2, num_layers - 1);
    if (n_hidden > 0 && g->hs_arena_bytes < (uint64_t)n_hidden * hid_bytes) {
        (void)hipFree(g->hs_arena); g->hs_arena = nullptr; g->hs_arena_bytes = 0;
        DGI_HIP(hipMalloc(reinterpret_cast<void**>(&g->hs_arena), (size_t)n_hidden * hid_bytes));
        g->hs_arena_bytes = (uint64_t)n_hidden * hid_bytes;
    }
    struct { void* p; } hid[2] = {{g->hs_arena}, {g->hs_arena ? g->hs_arena + hid_bytes : nullptr}};
    const void* cur = x;
    int64_t ld_cur = ld_x;
    // dgi_infer keeps its arena in the graph handle; the sampled graphs live for one layer each, so the arena is
    // handed from one to the next instead of being allocated per layer
    // ... and between calls it stays in the full graph's handle, where dgi_infer would keep its own.
    std::lock_guard<std::mutex> ws_lock(g->ws_mutex);
    struct Arena {
        const dgi_graph* home; char* p; uint64_t bytes;
        ~Arena() { home->ws_ptr = p; home->ws_bytes = bytes; }
    } arena{g, g->ws_ptr, g->ws_bytes};
    g->ws_ptr = nullptr; g->ws_bytes = 0;
    for (int l = 0; l < num_layers; ++l) {
        const bool last = l == num_layers - 1;
        const int eb = layers[l].out_dtype == DGI_BF16 ? 2 : 4;
        void* dst = last ? out : hid[l % 2].p;
        const int64_t ld_dst = last ? ld_out : round_up(layers[l].out_dim, 16 / eb);
        dgi_graph_t* gs = nullptr;
        // only GCN reads the sampled graph's out-degrees; counting them costs an integer atomic per sampled edge
        DGI_TRY(sample_graph(g, fanout, seed, l, true, layers[l].agg == DGI_AGG_GCN, s, &gs));
        gs->ws_ptr = arena.p; gs->ws_bytes = arena.bytes;
        arena.p = nullptr; arena.bytes = 0;
        const dgi_status_t st = dgi_infer(gs, &layers[l], 1, cur, ld_cur, dst, ld_dst, &o, s);  // waits for completion
        arena.p = gs->ws_ptr; arena.bytes = gs->ws_bytes;
        gs->ws_ptr = nullptr; gs->ws_bytes = 0;
        g->ss_ip = std::move(gs->h_indptr);  // the host vector goes back to the cache; the device arrays were borrowed
        dgi_graph_free(gs);
        DGI_TRY(st);
        cur = dst;
        ld_cur = ld_dst;
    }
    return DGI_OK;
}
