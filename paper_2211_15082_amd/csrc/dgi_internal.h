// Internal declarations shared by the translation units of libdgi (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>
#include <string>
#include <vector>

#include "dgi.h"

namespace dgi {

// ---- error reporting -------------------------------------------------------------------------
void set_error(const char* fmt, ...);
#define DGI_HIP(call)                                                                          \
    do {                                                                                       \
        hipError_t _e = (call);                                                                \
        if (_e != hipSuccess) {                                                                \
            ::dgi::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(_e), __FILE__,  \
                             __LINE__);                                                        \
            return (_e == hipErrorOutOfMemory) ? DGI_ERR_OOM : DGI_ERR_DEVICE;                 \
        }                                                                                      \
    } while (0)
#define DGI_TRY(expr)                       \
    do {                                    \
        dgi_status_t _s = (expr);           \
        if (_s != DGI_OK) return _s;        \
    } while (0)
#define DGI_REQUIRE(cond, status, ...)      \
    do {                                    \
        if (!(cond)) {                      \
            ::dgi::set_error(__VA_ARGS__);  \
            return (status);                \
        }                                   \
    } while (0)

// Rows with more in-edges than kHubDegree are split into chunks of kHubChunk edges, each reduced by
// its own wavefront into an fp32 partial row; a second kernel adds the partials in chunk order, so the
// result does not depend on scheduling.
constexpr int64_t kHubDegree = 1024;
constexpr int64_t kHubChunk = 512;

}  // namespace dgi

struct dgi_graph {
    int64_t N = 0, E = 0;
    int32_t itype = DGI_I32;
    const void* d_indptr = nullptr;     // device, itype entries
    const int32_t* d_indices = nullptr; // device
    bool own_csr = false;               // device CSR allocated by the handle
    bool own_vectors = true;            // d_deg_out / d_rs_in / d_rs_out allocated by the handle (else borrowed)
    bool has_out_degrees = true;        // d_deg_out / d_rs_out are filled (a sampled graph for a layer without GCN skips the count)
    int32_t* d_deg_out = nullptr;
    float* d_rs_in = nullptr;           // in-degree^-1/2, degree clamped to >= 1
    float* d_rs_out = nullptr;
    // hub rows (in-degree > kHubDegree), ascending row id
    int64_t* d_hub_rows = nullptr;      // [n_hubs]
    int64_t* d_hub_chunk_ptr = nullptr; // [n_hubs + 1] prefix of chunk counts
    std::vector<int64_t> h_indptr;      // host copy, always int64
    std::vector<int64_t> h_hub_rows;
    std::vector<int64_t> h_hub_chunk_ptr;
    int64_t max_in_degree = 0;
    uint64_t device_bytes = 0;
    int device = 0;
    // dgi_infer's arena (hidden layers + temporaries), kept between calls: allocating and freeing tens of
    // gigabytes costs far more than the inference itself.  Guarded by ws_mutex for the whole call.
    mutable std::mutex ws_mutex;
    mutable char* ws_ptr = nullptr;
    mutable uint64_t ws_bytes = 0;
    // dgi_infer_host's buffers, kept between calls for the same reason (page-locking gigabytes of host memory is
    // slow as well): the device memory of its two batch slots and the two host matrices of the hidden layers.
    // Guarded by hs_mutex for the whole call.
    mutable std::mutex hs_mutex;
    mutable char* hs_arena = nullptr;
    mutable uint64_t hs_arena_bytes = 0;
    mutable void* hs_hid[2] = {nullptr, nullptr};
    mutable uint64_t hs_hid_bytes = 0;
    mutable void* hs_z = nullptr;       // page-locked host buffer of a transform-first layer's transformed rows
    mutable uint64_t hs_z_bytes = 0;
    // dgi_infer_sampled builds one sampled graph per layer: its host indptr, device indptr and device indices
    // live here between layers and calls (the sampled handle borrows them).  Guarded by hs_mutex as well.
    mutable std::vector<int64_t> ss_ip;
    mutable int64_t* ss_d_ip = nullptr;
    mutable int32_t* ss_d_ix = nullptr;
    mutable uint64_t ss_ix_cap = 0;  // entries
    mutable void* ss_d_tmp = nullptr;   // the sampler's scan workspace and out-degree counters, kept between calls
    mutable uint64_t ss_tmp_cap = 0;    // bytes
    mutable int32_t* ss_d_deg = nullptr;
    mutable char* ss_d_vec = nullptr;   // 3 N-vectors lent to the sampled graph of a layer (degrees and normalisers)
    mutable int64_t ss_ip_fanout = -1;  // fan-out ss_ip (and ss_d_ip) were computed for: the sample's indptr depends on nothing else
};

namespace dgi {

// ---- kernel launch descriptors ------------------------------------------------------------------
// MODE_GCN_PRE: GCN whose source rows were already multiplied by d_out(u)^-1/2 by the kernel that produced
// them, so the gather needs no per-edge coefficient (only the destination scale d_in(v)^-1/2).
enum : int { MODE_SUM = 0, MODE_MEAN = 1, MODE_GCN = 2, MODE_GCN_PRE = 3 };

// Gather/aggregate of destination rows [row_begin,row_end):
//   out[v - out_row0, c] = act( scale_v * sum_{u in N(v)} coef_u * S[u, c] + self[v, c] + bias[c] )
// SUM: scale 1; MEAN: 1/deg (0 for empty rows); GCN: coef_u = rs_out[u], scale_v = rs_in[v].
struct AggArgs {
    const dgi_graph* g = nullptr;
    int mode = MODE_SUM;
    const void* S = nullptr;  // source rows, element (u, c) at S[u * ld_s + c]
    int64_t ld_s = 0;
    int s_dtype = DGI_F32;
    int width = 0;            // columns gathered
    void* out = nullptr;      // element (v, c) at out[(v - out_row0) * ld_out + c]
    void* out_lo = nullptr;   // bf16 output only, optional: a second matrix of the same shape and leading dimension that
                              // receives what the bf16 rounding dropped, so that out + out_lo carries 16 mantissa bits:
    int lo_bytes = 2;         // as bf16(value - float(bf16(value))) (2), or as one byte per element (1): the remainder in
                              // units of 2^-8 of the bf16 value's last place, plus 128
    int64_t ld_out = 0;
    int64_t out_row0 = 0;
    int out_dtype = DGI_F32;
    const void* self = nullptr; // optional addend rows, dtype s_dtype, element (v, c) at self[v * ld_self + c]
    int64_t ld_self = 0;
    const float* bias = nullptr;
    int act = DGI_ACT_NONE;
    float act_slope = 0.f;
    const float* out_scale = nullptr;  // optional per-row factor applied after the activation (indexed by node id)
    int64_t row_begin = 0, row_end = 0;
    float* hub_partials = nullptr;  // fp32 [chunks in range x width_padded], needed when the range holds hub rows
};
uint64_t agg_hub_partial_bytes(const dgi_graph* g, int64_t row_begin, int64_t row_end, int width);
// stage 0: the gather launch (row tiles + hub chunks); stage 1: the second-stage reduce of the hub rows
// in the range (a no-op when there are none).  Callers run stage 0 then stage 1.
dgi_status_t launch_aggregate(const AggArgs& a, int stage, hipStream_t stream);

// Aggregate-first layer in one launch: out[v,:] = act([h_v | m_v] Wt^T + bias) for rows [row_begin,row_end),
// m_v aggregated on the fly and kept in LDS (never written to HBM).
struct FusedArgs {
    const dgi_graph* g = nullptr;
    int mode = MODE_SUM;
    const void* H = nullptr; int64_t ld_h = 0; int dtype = DGI_F32; int K = 0;
    const void* Wt = nullptr; int64_t ldw = 0; int K1p = 0; bool has_self = false; int N = 0;
    const void* Wf = nullptr;  // the same weights in MFMA fragment order (launch_pack_fragments); what the kernel reads
    const float* bias = nullptr; int act = DGI_ACT_NONE; float act_slope = 0.f;
    const float* out_scale = nullptr;  // optional per-row factor applied after the activation (indexed by node id)
    void* out = nullptr; int64_t ld_out = 0; int64_t out_row0 = 0; int out_dtype = DGI_F32;
    int64_t row_begin = 0, row_end = 0;
    void* temp = nullptr;  // fused_temp_bytes() of scratch when the range holds hub rows
};
// elements of the fragment-order copy of an [N x ldw] packed weight
inline uint64_t fragment_weight_elems(int N, int64_t ldw) { return (uint64_t)((N + 31) / 32) * 32 * (uint64_t)ldw; }
bool fused_supported(const FusedArgs& a);
uint64_t fused_temp_bytes(const dgi_graph* g, int64_t row_begin, int64_t row_end, int K);
// stage 0: hub pre-pass (no-op without hub rows in the range); stage 1: the fused kernel.  Run 0 then 1.
dgi_status_t launch_fused(const FusedArgs& a, int stage, hipStream_t stream);

// GAT edge pass over rows [row_begin,row_end).  Zx row u = [ z (heads*F) | el (heads) | er (heads) | pad ].
struct GatArgs {
    const dgi_graph* g = nullptr;
    const float* Zx = nullptr;
    int64_t ld_z = 0;
    int heads = 1, head_dim = 0;
    float attn_slope = 0.2f;
    void* out = nullptr;
    int64_t ld_out = 0;
    int64_t out_row0 = 0;
    int out_dtype = DGI_F32;
    const float* bias = nullptr;
    int act = DGI_ACT_NONE;
    float act_slope = 0.f;
    int64_t row_begin = 0, row_end = 0;
};
dgi_status_t launch_gat(const GatArgs& a, hipStream_t stream);

// Y[r, n] = act( sum_k A1[r,k] Wt[n,k] + sum_k (A2[r,k] + A3[r,k]) Wt[n,K1p+k] + bias[n] ),  r in [0,M), n in [0,Nout).
// Wt is the packed transposed weight [Nout x ldw] (K contiguous); the A2 block starts at column K1p.  A3 (optional,
// needs A2; same shape and leading dimension) multiplies the same weight columns as A2: the low-order halves of an
// A2 that is kept as a pair of bf16 values.
struct GemmArgs {
    int dtype = DGI_F32;        // dtype of A1, A2 and Wt
    const void* A1 = nullptr; int64_t ld_a1 = 0; int K1 = 0;
    const void* A2 = nullptr; int64_t ld_a2 = 0; int K2 = 0;
    const void* A3 = nullptr;     // bf16 only, optional: the remainders of A2 as a second bf16 matrix (same shape and ld)
    const void* A_lo8 = nullptr;  // bf16 only, optional: the remainders of the last block (A2 if present, else A1) as one byte
                                  // per element, same shape, leading dimension in bytes = that block's in elements
                                  // (AggArgs.lo_bytes == 1); needs gemm_stationary_applies()
    const void* Wt = nullptr; int64_t ldw = 0; int K1p = 0;
    const float* bias = nullptr;
    int act = DGI_ACT_NONE; float act_slope = 0.f;
    void* Y = nullptr; int64_t ld_y = 0; int out_dtype = DGI_F32;
    int64_t M = 0; int Nout = 0;
    const float* out_scale = nullptr; int64_t row0 = 0;  // optional: Y[r,:] *= out_scale[row0 + r] after the activation
};
dgi_status_t launch_gemm(const GemmArgs& a, hipStream_t stream);
// Whether a bf16 GEMM of this shape runs on the weights-stationary kernel whatever the output's alignment (the weight
// fragments and an output stage fit in LDS, accumulators and row buffers in registers, A1 rows are 16-byte aligned; the
// other blocks live in the library's own aligned temporaries).  blocks: 1 = A1, 2 = A1 A2, 3 = A1 A2 A3; with_bytes: the
// last block comes with remainder bytes (A_lo8), which only this kernel reads.
bool gemm_stationary_applies(const void* A1, int64_t ld_a1, int K1, int blocks, int K2, int Nout, int out_dtype, bool with_bytes);

// Wt[n, koff + k] = W[k, n] for k < K, n < Nout (W row-major [K x Nout]); dtype preserved.
dgi_status_t launch_pack_weight(const void* W, int dtype, int K, int Nout, void* Wt, int64_t ldw, int koff,
                                hipStream_t stream);
// Wf[((cb * KS + ks) * 64 + lane) * VEC + i] = Wt[(cb*32 + lane%32) * ldw + ks*2*VEC + (lane/32)*VEC + i] (0 for rows >= N),
// VEC = elements per 16 bytes, KS = ldw / (2 VEC): the B operand of one 32-column block and K step is 1 KB of
// consecutive memory, one 16-byte piece per lane, instead of 32 pieces in 32 different rows.
dgi_status_t launch_pack_fragments(const void* Wt, int dtype, int N, int64_t ldw, void* Wf, hipStream_t stream);
// GAT: Wt rows [HF, HF+heads) = W a_src^h, rows [HF+heads, HF+2 heads) = W a_dst^h  (fp32 only).
dgi_status_t launch_pack_gat_attn(const float* W, int K, int heads, int F, const float* a_src, const float* a_dst,
                                  float* Wt, int64_t ldw, hipStream_t stream);
dgi_status_t launch_fill_zero(void* p, uint64_t bytes, hipStream_t stream);
// out[r, c] = in[r, c] * scale[r]  (rows x width, dtype fp32 or bf16)
dgi_status_t launch_scale_rows(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int width,
                               int elem_bytes, const float* scale, hipStream_t stream);
// rows of `width` elements between matrices with different leading dimensions: gather=false: out[perm[r]] = in[r];
// gather=true: out[r] = in[perm[r]]; perm == nullptr is the identity (a strided copy)
dgi_status_t launch_permute_rows(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int width,
                                 int elem_bytes, const int32_t* perm, bool gather, hipStream_t stream);

// BFS reordering enumerates at most this many connected components breadth-first; what is left after that is
// appended in (degree, id) order (a graph with very many tiny components gains nothing from more).
constexpr int kMaxBfsComponents = 256;

// permutation computed on the device (dgi_reorder_gpu.hip): DEGREE and BFS_RCM; d_perm is a DEVICE buffer of N ints.
// Returns DGI_ERR_UNSUPPORTED for graphs beyond its size limits (the caller then uses the host routine).
dgi_status_t reorder_permutation_device(const dgi_graph* g, int method, int32_t* d_perm, hipStream_t stream);

// host-side permutations (dgi_reorder.cpp)
dgi_status_t reorder_permutation(int64_t N, const int64_t* indptr, const int32_t* indices, int method, uint64_t seed,
                                 int32_t* perm_new_of_old);

// handle over device CSR arrays built by the library (int64 indptr); takes ownership of the arrays and of h_indptr
dgi_status_t graph_adopt(int64_t N, int64_t E, int64_t* d_indptr, int32_t* d_indices, std::vector<int64_t>&& h_indptr, int64_t max_degree,
                         bool own_arrays, bool count_out_degrees, hipStream_t stream, dgi_graph_t** out,
                         const int32_t* counted_out_degrees = nullptr /* DEVICE, N entries: used instead of counting */,
                         void* node_vectors = nullptr /* DEVICE, 3 x round_up(4 N, 256) bytes lent for the handle's N-vectors */);

// dgi_layer_forward with an output buffer whose first row is destination row out_base (0 = the whole matrix)
dgi_status_t layer_forward_rows(const dgi_graph* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in, void* h_out, int64_t ld_out,
                                int64_t out_base, int64_t dst_begin, int64_t dst_end, void* workspace, uint64_t workspace_bytes, hipStream_t s);

// The dense and the sparse half of a transform-first layer as separate calls (dgi_infer_host runs them as two passes
// when the transformed rows are narrower than the layer's input rows).
struct TransformInfo {
    bool transform_first;   // the layer's plan multiplies before it aggregates (always for GAT)
    int z_cols;             // columns of a transformed row: [z_self |] z_neigh, or [z | e_l | e_r] for GAT
    int64_t z_ld;
    int z_dtype;
    uint64_t weight_bytes;  // device scratch layer_transform_rows needs for the packed weights
    bool has_self;          // GraphSAGE: columns [0, z_neigh_col) hold z_self, the rest z_neigh
    int z_neigh_col;
};
dgi_status_t layer_transform_info(const dgi_graph* g, const dgi_layer_t* layer, TransformInfo* info);
// Z[0:rows) = H[0:rows) W  (h_in, Z, weights: DEVICE; weights 256-byte aligned, info.weight_bytes long)
dgi_status_t layer_transform_rows(const dgi_graph* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in, int64_t rows, void* Z,
                                  void* weights, hipStream_t s);
// destination rows [b, e) of g from transformed rows Z (one per node of g, leading dimension info.z_ld); temp as sized
// by layer_aggregate_temp_bytes; h_out's first row is destination row out_base
uint64_t layer_aggregate_temp_bytes(const dgi_graph* g, const dgi_layer_t* layer, int64_t b, int64_t e);
// The same for a GraphSAGE layer with the two blocks of Z in separate matrices: Zn holds z_neigh of every node of g
// (leading dimension ld_n), Zs holds z_self of the destination rows only, its first row being row b (ld_s).
dgi_status_t layer_aggregate_rows_split(const dgi_graph* g, const dgi_layer_t* layer, const void* Zn, int64_t ld_n, const void* Zs, int64_t ld_s,
                                        void* h_out, int64_t ld_out, int64_t out_base, int64_t b, int64_t e, void* temp, uint64_t temp_bytes,
                                        hipStream_t s);
dgi_status_t layer_aggregate_rows(const dgi_graph* g, const dgi_layer_t* layer, const void* Z, void* h_out, int64_t ld_out, int64_t out_base,
                                  int64_t b, int64_t e, void* temp, uint64_t temp_bytes, hipStream_t s);

// dgi_infer with an optional per-layer limit on the rows computed (row_limit[l] rows of layer l, NULL = all)
dgi_status_t infer_rows(const dgi_graph* g, const dgi_layer_t* layers, int32_t num_layers, const void* x, int64_t ld_x, void* out,
                        int64_t ld_out, const dgi_infer_opts_t* opts, const int64_t* row_limit, void* hip_stream);

// frees dgi_infer's cached arena (takes ws_mutex; dgi_infer_host calls it while holding hs_mutex)
dgi_status_t release_infer_arena(const dgi_graph* g);

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace dgi
