// C ABI entry points for one layer (dgi_layer_forward) and the whole layer-wise schedule (dgi_infer,
// Algorithm 2 of the DGI paper), plus the host-side batch planner of Section 4.1.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdlib>
#include <cstring>
#include <unordered_set>

#include "dgi_internal.h"

namespace dgi {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

namespace {

int elem_bytes(int dtype) { return dtype == DGI_BF16 ? 2 : 4; }

// A dispatch holds fewer than 2^32 threads; the widest kernels here spend 64 threads per row, so a launch
// never covers more than this many rows (dgi_infer splits batches and transforms accordingly).
constexpr int64_t kMaxRowsPerLaunch = (int64_t)1 << 25;

// Build-time switch for measurements: 1 takes the byte form of the aggregate's remainders wherever it is available, 0 only
// where the bf16 form does not fit the weights-stationary kernel (111 M rows, 128 -> 128: 20.4 ms against 21.5 per GEMM).
#ifndef DGI_PREFER_LO8
#define DGI_PREFER_LO8 1
#endif
constexpr bool kPreferRemainderBytes = DGI_PREFER_LO8 != 0;

// How one layer is laid out and executed.
struct LayerPlan {
    bool transform_first = false;
    bool gat = false;
    bool has_self = false;
    int E = 4;            // elements per 16 bytes of the feature dtype
    int eb = 4;           // bytes per feature element
    int K1p = 0;          // column of the packed weight where the second K block starts
    int64_t ldw = 0;      // packed weight leading dimension (elements)
    int w_rows = 0;       // packed weight rows (= GEMM output columns)
    uint64_t wt_bytes = 0;   // packed weights: row order, then (fused plans) the fragment-order copy at wf_off
    uint64_t wf_off = 0;
    int mode = MODE_SUM;
    // transform-first: Z = H Wt^T for all nodes
    int z_cols = 0;       // GEMM output columns
    int64_t z_ld = 0;
    int z_neigh_col = 0;  // first column of the neighbour block in Z
    int z_dtype = DGI_F32;
    // aggregate-first: AGG tile of the batch (unfused path only)
    int64_t agg_ld = 0;
    bool fused = false;   // aggregate-first with the transform fused into the gather kernel
    bool wide_agg = false;  // bf16 features: the aggregated tile carries 16 mantissa bits per element: a pair of bf16 values,
    bool lo8 = false;       // ... or (split path on the weights-stationary GEMM) a bf16 value and a remainder byte
    bool wide_sum = false;  // bf16 features under SUM: transformed rows (transform-first) stay fp32
};

// Fusing the transform into the gather kernel removes the aggregated matrix's HBM round trip and hides the MFMA
// work under other workgroups' gathers, but every 32-row tile re-reads the packed weight from L2 in a
// latency-bound sweep.  It pays when a row's gather (avg_degree * K elements) outweighs its share of that
// sweep (ldw * N / 32 elements).  Measured on MI355X (fused vs split, whole layer):
//   GCN fp32 256->256, degree 52 (ratio 6.5): 18.8 vs 22.0 ms;  GraphSAGE fp32 256->256, degree 20 (ratio 1.25):
//   99 vs 108 ms;  GraphSAGE bf16 128->128, degree 14 (ratio 1.8): 129-155 vs 87 ms.
// The split path's bf16 GEMM is cheap next to its fp32 GEMM, hence the two thresholds.
// The fp32 threshold comes from a 20 M-node graph sampled down to average degrees 4..16 (fused / split, ms per layer):
//   GraphSAGE 256->256 (threshold ratio 1 = degree 16): degree 4 61/52, 8 64/70, 12 76/80, 16 82/101;
//   GCN 256->256 (degree 8): 4 40/39, 8 48/54, 12 58/75;  GraphSAGE 128->128 (degree 8): 4 26/22, 8 28/26, 12 32/33;
//   GraphSAGE 128->256 (degree 16): 4 40/31, 8 42/37, 12 43/45.  The crossovers sit at ratios 0.4-1.4: 0.5 it is.
// dgi_layer_t.order = AGG_FIRST_FUSED / AGG_FIRST_SPLIT overrides this choice per layer.
bool want_fused(const dgi_graph* g, int dtype, int K, int64_t ldw, int N) {
    const double avg_deg = g && g->N > 0 ? (double)g->E / (double)g->N : 0.0;
    const double ratio = avg_deg * (double)K / ((double)ldw * (double)N / 32.0);
    return ratio >= (dtype == DGI_BF16 ? 3.0 : 0.5);
}

dgi_status_t validate_layer(const dgi_layer_t* L) {
    DGI_REQUIRE(L != nullptr, DGI_ERR_INVALID_ARG, "layer is NULL");
    DGI_REQUIRE(L->agg >= DGI_AGG_SUM && L->agg <= DGI_AGG_GAT, DGI_ERR_INVALID_ARG, "unknown aggregator %d", L->agg);
    DGI_REQUIRE(L->act >= DGI_ACT_NONE && L->act <= DGI_ACT_LEAKY_RELU, DGI_ERR_INVALID_ARG, "unknown activation %d", L->act);
    DGI_REQUIRE(L->in_dim > 0 && L->out_dim > 0, DGI_ERR_INVALID_ARG, "layer dims must be positive");
    DGI_REQUIRE(L->W_neigh != nullptr, DGI_ERR_INVALID_ARG, "W_neigh is NULL");
    DGI_REQUIRE((L->feat_dtype == DGI_F32 || L->feat_dtype == DGI_BF16) && (L->out_dtype == DGI_F32 || L->out_dtype == DGI_BF16),
                DGI_ERR_INVALID_ARG, "unknown dtype");
    DGI_REQUIRE(L->order >= DGI_ORDER_AUTO && L->order <= DGI_ORDER_AGG_FIRST_SPLIT, DGI_ERR_INVALID_ARG, "unknown order %d", L->order);
    if (L->agg == DGI_AGG_GAT) {
        DGI_REQUIRE(L->heads >= 1 && L->out_dim % L->heads == 0, DGI_ERR_INVALID_ARG, "GAT: out_dim must be heads*head_dim");
        DGI_REQUIRE(L->attn_src && L->attn_dst, DGI_ERR_INVALID_ARG, "GAT: attention vectors are NULL");
        DGI_REQUIRE(L->feat_dtype == DGI_F32, DGI_ERR_UNSUPPORTED, "GAT runs on fp32 features only");
        DGI_REQUIRE(L->order == DGI_ORDER_AUTO || L->order == DGI_ORDER_TRANSFORM_FIRST, DGI_ERR_UNSUPPORTED,
                    "GAT is transform-first by definition");
    }
    return DGI_OK;
}

// h_in / ld_in: the layer's input as it will be passed (its alignment decides which kernels can run).
dgi_status_t plan_layer(const dgi_graph* g, const dgi_layer_t* L, const void* h_in, int64_t ld_in, LayerPlan* P) {
    DGI_TRY(validate_layer(L));
    DGI_REQUIRE(L->agg != DGI_AGG_GCN || g->has_out_degrees, DGI_ERR_INVALID_ARG, "GCN layer on a graph handle built without out-degrees");
    LayerPlan p;
    p.eb = elem_bytes(L->feat_dtype);
    p.E = 16 / p.eb;
    p.gat = L->agg == DGI_AGG_GAT;
    p.has_self = (L->agg == DGI_AGG_SUM || L->agg == DGI_AGG_MEAN) && L->W_self != nullptr;
    p.mode = L->agg == DGI_AGG_MEAN ? MODE_MEAN : L->agg == DGI_AGG_GCN ? MODE_GCN : MODE_SUM;
    p.transform_first = p.gat || L->order == DGI_ORDER_TRANSFORM_FIRST ||
                        (L->order == DGI_ORDER_AUTO && L->out_dim < L->in_dim);
    // bf16 storage means: inputs, weights and stored layers are bf16, everything in between is accumulated in fp32.
    // An aggregated vector cut to 8 bits before the transform would be a second rounding per layer that the stored
    // data does not have (measured on a 1.7 M-node down-scale of the 111 M-node bf16 benchmark: 2.3e-2 against the
    // oracle instead of 1.1e-2), and under SUM, whose aggregate over a long neighbour list is far larger than its
    // terms, an absolute error that is large next to the other rows of the output.  So the aggregated tile is a pair
    // of bf16 values per element (the rounded value and the rounding remainder, together 16 mantissa bits) and both go
    // through the matrix cores; and a transform-first SUM layer keeps its transformed rows in fp32.
    p.wide_agg = L->feat_dtype == DGI_BF16 && !p.gat;
    p.wide_sum = L->feat_dtype == DGI_BF16 && L->agg == DGI_AGG_SUM;
    const int in_p = (int)round_up(L->in_dim, p.E);
    if (p.gat) {
        p.K1p = in_p; p.ldw = in_p;
        p.w_rows = L->out_dim + 2 * L->heads;
        p.z_cols = p.w_rows; p.z_ld = round_up(p.z_cols, 4); p.z_neigh_col = 0; p.z_dtype = DGI_F32;
    } else if (p.transform_first) {
        p.K1p = in_p; p.ldw = in_p;
        p.z_neigh_col = p.has_self ? (int)round_up(L->out_dim, p.E) : 0;
        p.w_rows = p.z_neigh_col + L->out_dim;
        p.z_cols = p.w_rows; p.z_ld = round_up(p.z_cols, p.E); p.z_dtype = p.wide_sum ? (int)DGI_F32 : L->feat_dtype;
    } else {
        const int in_p2 = (int)round_up(L->in_dim, 2 * p.E);  // MFMA k-step granularity of the fused kernel
        p.K1p = p.has_self ? in_p2 : 0;
        p.ldw = p.K1p + in_p2;
        p.w_rows = L->out_dim;
        p.agg_ld = in_p;
        FusedArgs fa;
        fa.H = h_in; fa.ld_h = ld_in; fa.dtype = L->feat_dtype; fa.K = L->in_dim;
        fa.Wt = nullptr; fa.ldw = p.ldw; fa.K1p = p.K1p;
        const bool want = L->order == DGI_ORDER_AGG_FIRST_FUSED ||
                          (L->order != DGI_ORDER_AGG_FIRST_SPLIT && want_fused(g, L->feat_dtype, L->in_dim, p.ldw, L->out_dim));
        p.fused = want && fused_supported(fa);
        // The split path's GEMM reads [own rows | aggregate] (GraphSAGE) or the aggregate alone, and the aggregate's
        // remainders as bytes that the weights-stationary kernel decodes (a quarter less to write, a sixth less to read, some
        // 7 instructions per element), or, where that kernel does not apply, as one more bf16 block.
        if (p.wide_agg && !p.fused) {
            const void* a1 = p.has_self ? h_in : nullptr;
            const int64_t ld1 = p.has_self ? ld_in : 8;
            const int nb = p.has_self ? 2 : 1;
            const bool pair_ok = gemm_stationary_applies(a1, ld1, L->in_dim, nb + 1, L->in_dim, L->out_dim, L->out_dtype, false);
            const bool bytes_ok = gemm_stationary_applies(a1, ld1, L->in_dim, nb, L->in_dim, L->out_dim, L->out_dtype, true);
            p.lo8 = bytes_ok && (kPreferRemainderBytes || !pair_ok);
        }
    }
    if (!p.fused) {
        // The GEMM reads 128-byte pieces of consecutive weight rows out of L2, every workgroup the same ones.  A row
        // pitch that is a multiple of 2 KB puts all of them on one of an L2's 16 channels (measured: a 256->256 fp32
        // GraphSAGE GEMM ran at a third of its speed); an odd number of 128-byte units walks through all channels.
        const int64_t units = (p.ldw * p.eb + 127) / 128;
        p.ldw = (units | 1) * 128 / p.eb;
    }
    p.wt_bytes = (uint64_t)round_up((int64_t)p.w_rows * p.ldw * p.eb, 256);
    if (p.fused) {
        p.wf_off = p.wt_bytes;
        p.wt_bytes += (uint64_t)round_up((int64_t)fragment_weight_elems(p.w_rows, p.ldw) * p.eb, 256);
    }
    *P = p;
    return DGI_OK;
}

// Packed, transposed weights for the layer's GEMM (zero padded).
dgi_status_t prepare_weights(const dgi_layer_t* L, const LayerPlan& P, void* Wt, hipStream_t s) {
    DGI_TRY(launch_fill_zero(Wt, P.wt_bytes, s));
    if (P.gat) {
        DGI_TRY(launch_pack_weight(L->W_neigh, L->feat_dtype, L->in_dim, L->out_dim, Wt, P.ldw, 0, s));
        return launch_pack_gat_attn((const float*)L->W_neigh, L->in_dim, L->heads, L->out_dim / L->heads, L->attn_src,
                                    L->attn_dst, (float*)Wt, P.ldw, s);
    }
    if (P.transform_first) {
        if (P.has_self) DGI_TRY(launch_pack_weight(L->W_self, L->feat_dtype, L->in_dim, L->out_dim, Wt, P.ldw, 0, s));
        char* neigh = (char*)Wt + (int64_t)P.z_neigh_col * P.ldw * P.eb;
        return launch_pack_weight(L->W_neigh, L->feat_dtype, L->in_dim, L->out_dim, neigh, P.ldw, 0, s);
    }
    if (P.has_self) DGI_TRY(launch_pack_weight(L->W_self, L->feat_dtype, L->in_dim, L->out_dim, Wt, P.ldw, 0, s));
    DGI_TRY(launch_pack_weight(L->W_neigh, L->feat_dtype, L->in_dim, L->out_dim, Wt, P.ldw, P.K1p, s));
    if (P.fused) DGI_TRY(launch_pack_fragments(Wt, L->feat_dtype, P.w_rows, P.ldw, (char*)Wt + P.wf_off, s));
    return DGI_OK;
}

// Transform-first: Z[r,:] = H[r,:] Wt^T for rows [r0,r1) of the graph.
dgi_status_t run_transform(const dgi_layer_t* L, const LayerPlan& P, const void* h_in, int64_t ld_in, const void* Wt,
                           void* Z, int64_t r0, int64_t r1, hipStream_t s) {
    // row chunks keep every launch far below the 2^32-thread limit of a dispatch
    for (int64_t c0 = r0; c0 < r1; c0 += kMaxRowsPerLaunch) {
        const int64_t c1 = std::min(r1, c0 + kMaxRowsPerLaunch);
        GemmArgs ga;
        ga.dtype = L->feat_dtype;
        ga.A1 = (const char*)h_in + c0 * ld_in * P.eb; ga.ld_a1 = ld_in; ga.K1 = L->in_dim;
        ga.Wt = Wt; ga.ldw = P.ldw; ga.K1p = P.K1p;
        ga.Y = (char*)Z + c0 * P.z_ld * elem_bytes(P.z_dtype); ga.ld_y = P.z_ld; ga.out_dtype = P.z_dtype;
        ga.M = c1 - c0; ga.Nout = P.z_cols;
        DGI_TRY(launch_gemm(ga, s));
    }
    return DGI_OK;
}

uint64_t batch_temp_bytes(const dgi_graph* g, const dgi_layer_t* L, const LayerPlan& P, int64_t b, int64_t e) {
    if (P.fused) return fused_temp_bytes(g, b, e, L->in_dim);
    uint64_t bytes = 0;
    if (!P.gat) bytes += round_up((int64_t)agg_hub_partial_bytes(g, b, e, P.transform_first ? L->out_dim : L->in_dim), 256);
    if (!P.transform_first) {
        bytes += (uint64_t)round_up((e - b) * P.agg_ld * P.eb, 256);
        if (P.wide_agg) bytes += (uint64_t)round_up((e - b) * P.agg_ld * (P.lo8 ? 1 : P.eb), 256);
    }
    return bytes;
}

struct KernelTimer;  // defined below

// One batch of destination rows [b,e): the body of the inner loop of Algorithm 2.
// in_prescaled: the rows of h_in already carry the GCN source factor d_out(u)^-1/2; out_scale: per-node factor
// to fold into this layer's output rows (the next GCN layer's source factor), or NULL.  h_out's first row is
// destination row out_base (0: the whole output matrix; b: a buffer that holds just this batch).
dgi_status_t run_batch(const dgi_graph* g, const dgi_layer_t* L, const LayerPlan& P, const void* h_in, int64_t ld_in,
                       void* h_out, int64_t ld_out, int64_t b, int64_t e, const void* Wt, const void* Z, void* temp,
                       hipStream_t s, KernelTimer* timer, bool in_prescaled, const float* out_scale, int64_t out_base = 0);

// HIP-event timing of kernel classes on the caller's stream.
struct KernelTimer {
    struct Span { hipEvent_t a, b; int layer; int kind; };
    std::vector<Span> spans;
    hipStream_t stream;
    int layer = 0;
    explicit KernelTimer(hipStream_t s) : stream(s) {}
    ~KernelTimer() { for (auto& sp : spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); } }
    dgi_status_t begin(int kind) {
        Span sp{nullptr, nullptr, layer, kind};
        DGI_HIP(hipEventCreate(&sp.a));
        DGI_HIP(hipEventCreate(&sp.b));
        spans.push_back(sp);
        DGI_HIP(hipEventRecord(sp.a, stream));
        return DGI_OK;
    }
    dgi_status_t end() { DGI_HIP(hipEventRecord(spans.back().b, stream)); return DGI_OK; }
};
enum { SPAN_AGG = 0, SPAN_GEMM = 1, SPAN_LAYER = 2, SPAN_TOTAL = 3, SPAN_HUB = 4 };

dgi_status_t run_batch(const dgi_graph* g, const dgi_layer_t* L, const LayerPlan& P, const void* h_in, int64_t ld_in,
                       void* h_out, int64_t ld_out, int64_t b, int64_t e, const void* Wt, const void* Z, void* temp,
                       hipStream_t s, KernelTimer* timer, bool in_prescaled, const float* out_scale, int64_t out_base) {
    if (e <= b) return DGI_OK;
    const int ob = elem_bytes(L->out_dtype);
    const int mode = (P.mode == MODE_GCN && in_prescaled) ? (int)MODE_GCN_PRE : P.mode;
    if (P.gat) {
        GatArgs a;
        a.g = g; a.Zx = (const float*)Z; a.ld_z = P.z_ld; a.heads = L->heads; a.head_dim = L->out_dim / L->heads;
        a.attn_slope = L->attn_slope;
        a.out = (char*)h_out + (b - out_base) * ld_out * ob; a.ld_out = ld_out; a.out_row0 = b; a.out_dtype = L->out_dtype;
        a.bias = L->bias; a.act = L->act; a.act_slope = L->act_slope; a.row_begin = b; a.row_end = e;
        if (timer) DGI_TRY(timer->begin(SPAN_AGG));
        DGI_TRY(launch_gat(a, s));
        if (timer) DGI_TRY(timer->end());
        return DGI_OK;
    }
    const uint64_t part_bytes = round_up((int64_t)agg_hub_partial_bytes(g, b, e, P.transform_first ? L->out_dim : L->in_dim), 256);
    AggArgs a;
    a.g = g; a.mode = mode; a.row_begin = b; a.row_end = e;
    a.hub_partials = part_bytes ? (float*)temp : nullptr;
    if (P.transform_first) {
        const int zb = elem_bytes(P.z_dtype);
        a.S = (const char*)Z + (int64_t)P.z_neigh_col * zb; a.ld_s = P.z_ld; a.s_dtype = P.z_dtype; a.width = L->out_dim;
        a.self = P.has_self ? Z : nullptr; a.ld_self = P.z_ld;
        a.out = (char*)h_out + (b - out_base) * ld_out * ob; a.ld_out = ld_out; a.out_row0 = b; a.out_dtype = L->out_dtype;
        a.bias = L->bias; a.act = L->act; a.act_slope = L->act_slope; a.out_scale = out_scale;
        if (timer) DGI_TRY(timer->begin(SPAN_AGG));
        DGI_TRY(launch_aggregate(a, 0, s));
        if (timer) DGI_TRY(timer->end());
        return launch_aggregate(a, 1, s);
    }
    if (P.fused) {
        FusedArgs fa;
        fa.g = g; fa.mode = mode; fa.H = h_in; fa.ld_h = ld_in; fa.dtype = L->feat_dtype; fa.K = L->in_dim;
        fa.Wt = Wt; fa.ldw = P.ldw; fa.K1p = P.K1p; fa.has_self = P.has_self; fa.N = L->out_dim;
        fa.Wf = (const char*)Wt + P.wf_off;
        fa.bias = L->bias; fa.act = L->act; fa.act_slope = L->act_slope; fa.out_scale = out_scale;
        fa.out = (char*)h_out + (b - out_base) * ld_out * ob; fa.ld_out = ld_out; fa.out_row0 = b; fa.out_dtype = L->out_dtype;
        fa.row_begin = b; fa.row_end = e;
        fa.temp = fused_temp_bytes(g, b, e, L->in_dim) ? temp : nullptr;
        if (fa.temp) {
            if (timer) DGI_TRY(timer->begin(SPAN_HUB));
            DGI_TRY(launch_fused(fa, 0, s));
            if (timer) DGI_TRY(timer->end());
        }
        if (timer) DGI_TRY(timer->begin(SPAN_AGG));
        DGI_TRY(launch_fused(fa, 1, s));
        if (timer) DGI_TRY(timer->end());
        return DGI_OK;
    }
    void* agg = (char*)temp + part_bytes;
    void* agg_lo = P.wide_agg ? (char*)agg + round_up((e - b) * P.agg_ld * P.eb, 256) : nullptr;
    a.S = h_in; a.ld_s = ld_in; a.s_dtype = L->feat_dtype; a.width = L->in_dim;
    a.out = agg; a.out_lo = agg_lo; a.lo_bytes = P.lo8 ? 1 : 2; a.ld_out = P.agg_ld; a.out_row0 = b; a.out_dtype = L->feat_dtype;
    if (timer) DGI_TRY(timer->begin(SPAN_AGG));
    DGI_TRY(launch_aggregate(a, 0, s));
    if (timer) DGI_TRY(timer->end());
    DGI_TRY(launch_aggregate(a, 1, s));
    GemmArgs ga;
    ga.dtype = L->feat_dtype;
    if (P.has_self) {
        ga.A1 = (const char*)h_in + b * ld_in * P.eb; ga.ld_a1 = ld_in; ga.K1 = L->in_dim;
        ga.A2 = agg; ga.ld_a2 = P.agg_ld; ga.K2 = L->in_dim;
        if (P.lo8) ga.A_lo8 = agg_lo; else ga.A3 = agg_lo;
    } else {
        ga.A1 = agg; ga.ld_a1 = P.agg_ld; ga.K1 = L->in_dim;
        if (P.lo8) ga.A_lo8 = agg_lo;
        else if (agg_lo) { ga.A2 = agg_lo; ga.ld_a2 = P.agg_ld; ga.K2 = L->in_dim; }  // K1p is 0: the same weight block again
    }
    ga.Wt = Wt; ga.ldw = P.ldw; ga.K1p = P.K1p;
    ga.bias = L->bias; ga.act = L->act; ga.act_slope = L->act_slope;
    ga.Y = (char*)h_out + (b - out_base) * ld_out * ob; ga.ld_y = ld_out; ga.out_dtype = L->out_dtype;
    ga.M = e - b; ga.Nout = L->out_dim;
    ga.out_scale = out_scale; ga.row0 = b;
    if (timer) DGI_TRY(timer->begin(SPAN_GEMM));
    DGI_TRY(launch_gemm(ga, s));
    if (timer) DGI_TRY(timer->end());
    return DGI_OK;
}

// Workspace of dgi_layer_forward: [ packed weights | Z (transform-first, all N rows) | batch temporaries ]
struct ForwardLayout { uint64_t wt_off, z_off, temp_off, total; };
ForwardLayout forward_layout(const dgi_graph* g, const dgi_layer_t* L, const LayerPlan& P, int64_t b, int64_t e) {
    ForwardLayout f{};
    f.wt_off = 0;
    f.z_off = P.wt_bytes;
    const uint64_t zbytes = P.transform_first ? (uint64_t)round_up(g->N * P.z_ld * elem_bytes(P.z_dtype), 256) : 0;
    f.temp_off = f.z_off + zbytes;
    f.total = f.temp_off + batch_temp_bytes(g, L, P, b, e) + 256;
    return f;
}

dgi_status_t check_matrix(const void* p, int64_t ld, int dim, const char* what) {
    DGI_REQUIRE(p != nullptr, DGI_ERR_INVALID_ARG, "%s is NULL", what);
    DGI_REQUIRE(ld >= dim, DGI_ERR_INVALID_ARG, "%s: leading dimension %lld < width %d", what, (long long)ld, dim);
    return DGI_OK;
}

}  // namespace
}  // namespace dgi

using namespace dgi;

extern "C" const char* dgi_last_error(void) { return dgi::g_error; }
extern "C" int32_t dgi_version(void) { return DGI_VERSION_MAJOR * 1000 + DGI_VERSION_MINOR; }
extern "C" const char* dgi_status_string(dgi_status_t s) {
    switch (s) {
        case DGI_OK: return "ok";
        case DGI_ERR_INVALID_ARG: return "invalid argument";
        case DGI_ERR_BAD_GRAPH: return "malformed graph";
        case DGI_ERR_UNSUPPORTED: return "unsupported combination";
        case DGI_ERR_OOM: return "out of device memory";
        case DGI_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

dgi_status_t dgi::release_infer_arena(const dgi_graph* g) {
    std::lock_guard<std::mutex> ws_lock(g->ws_mutex);
    if (g->ws_ptr) {
        DGI_HIP(hipDeviceSynchronize());
        (void)hipFree(g->ws_ptr);
        g->ws_ptr = nullptr;
        g->ws_bytes = 0;
    }
    return DGI_OK;
}

extern "C" dgi_status_t dgi_graph_release_workspace(dgi_graph_t* g) {
    if (!g) return DGI_OK;
    DGI_TRY(release_infer_arena(g));
    std::lock_guard<std::mutex> hs_lock(g->hs_mutex);
    if (g->hs_arena || g->hs_hid[0] || g->hs_hid[1] || g->hs_z || g->ss_d_ip || g->ss_d_ix || g->ss_d_tmp || g->ss_d_deg || g->ss_d_vec) {
        DGI_HIP(hipDeviceSynchronize());
        (void)hipFree(g->hs_arena);
        (void)hipHostFree(g->hs_hid[0]);
        (void)hipHostFree(g->hs_hid[1]);
        (void)hipHostFree(g->hs_z);
        g->hs_z = nullptr; g->hs_z_bytes = 0;
        (void)hipFree(g->ss_d_ip);
        (void)hipFree(g->ss_d_ix);
        (void)hipFree(g->ss_d_tmp);
        (void)hipFree(g->ss_d_deg);
        g->ss_d_tmp = nullptr; g->ss_tmp_cap = 0; g->ss_d_deg = nullptr;
        (void)hipFree(g->ss_d_vec);
        g->ss_d_vec = nullptr; g->ss_ip_fanout = -1;
        g->hs_arena = nullptr; g->hs_arena_bytes = 0;
        g->hs_hid[0] = g->hs_hid[1] = nullptr; g->hs_hid_bytes = 0;
        g->ss_d_ip = nullptr; g->ss_d_ix = nullptr; g->ss_ix_cap = 0;
    }
    std::vector<int64_t>().swap(g->ss_ip);
    g->ss_ip_fanout = -1;
    return DGI_OK;
}

extern "C" dgi_status_t dgi_layer_workspace_bytes(const dgi_graph_t* g, const dgi_layer_t* layer, int64_t dst_begin,
                                                  int64_t dst_end, uint64_t* bytes) {
    DGI_REQUIRE(g && bytes, DGI_ERR_INVALID_ARG, "layer_workspace_bytes: NULL argument");
    DGI_REQUIRE(dst_begin >= 0 && dst_end >= dst_begin && dst_end <= g->N, DGI_ERR_INVALID_ARG, "bad destination range");
    // sized for the unfused path as well, so that any input alignment given to dgi_layer_forward fits
    LayerPlan P, Q;
    DGI_TRY(plan_layer(g, layer, reinterpret_cast<const void*>(16), 0, &P));
    DGI_TRY(plan_layer(g, layer, reinterpret_cast<const void*>(1), 1, &Q));
    *bytes = std::max(forward_layout(g, layer, P, dst_begin, dst_end).total, forward_layout(g, layer, Q, dst_begin, dst_end).total);
    return DGI_OK;
}

dgi_status_t dgi::layer_forward_rows(const dgi_graph* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in, void* h_out, int64_t ld_out,
                                     int64_t out_base, int64_t dst_begin, int64_t dst_end, void* workspace, uint64_t workspace_bytes, hipStream_t s) {
    DGI_REQUIRE(g != nullptr, DGI_ERR_INVALID_ARG, "graph is NULL");
    LayerPlan P;
    DGI_TRY(plan_layer(g, layer, h_in, ld_in, &P));
    DGI_REQUIRE(dst_begin >= 0 && dst_end >= dst_begin && dst_end <= g->N, DGI_ERR_INVALID_ARG,
                "bad destination range [%lld,%lld) for %lld nodes", (long long)dst_begin, (long long)dst_end, (long long)g->N);
    if (g->N == 0 || dst_end == dst_begin) return DGI_OK;
    DGI_TRY(check_matrix(h_in, ld_in, layer->in_dim, "h_in"));
    DGI_TRY(check_matrix(h_out, ld_out, layer->out_dim, "h_out"));
    const ForwardLayout f = forward_layout(g, layer, P, dst_begin, dst_end);
    DGI_REQUIRE(workspace != nullptr && workspace_bytes >= f.total, DGI_ERR_INVALID_ARG,
                "workspace too small: %llu bytes given, %llu needed", (unsigned long long)workspace_bytes, (unsigned long long)f.total);
    DGI_REQUIRE((uintptr_t)workspace % 256 == 0, DGI_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    char* ws = static_cast<char*>(workspace);
    DGI_TRY(prepare_weights(layer, P, ws + f.wt_off, s));
    if (P.transform_first) DGI_TRY(run_transform(layer, P, h_in, ld_in, ws + f.wt_off, ws + f.z_off, 0, g->N, s));
    return run_batch(g, layer, P, h_in, ld_in, h_out, ld_out, dst_begin, dst_end, ws + f.wt_off, ws + f.z_off, ws + f.temp_off, s, nullptr, false, nullptr,
                     out_base);
}

dgi_status_t dgi::layer_transform_info(const dgi_graph* g, const dgi_layer_t* layer, TransformInfo* info) {
    LayerPlan P;
    DGI_TRY(plan_layer(g, layer, reinterpret_cast<const void*>(16), 0, &P));
    info->transform_first = P.transform_first;
    info->z_cols = P.z_cols; info->z_ld = P.z_ld; info->z_dtype = P.z_dtype;
    info->weight_bytes = P.wt_bytes;
    info->has_self = P.has_self && !P.gat;
    info->z_neigh_col = P.z_neigh_col;
    return DGI_OK;
}

dgi_status_t dgi::layer_transform_rows(const dgi_graph* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in, int64_t rows, void* Z,
                                       void* weights, hipStream_t s) {
    LayerPlan P;
    DGI_TRY(plan_layer(g, layer, reinterpret_cast<const void*>(16), 0, &P));
    DGI_REQUIRE(P.transform_first, DGI_ERR_INVALID_ARG, "layer_transform_rows: not a transform-first layer");
    DGI_REQUIRE(weights != nullptr && (uintptr_t)weights % 256 == 0, DGI_ERR_INVALID_ARG, "layer_transform_rows: weight scratch missing or misaligned");
    if (rows <= 0) return DGI_OK;
    DGI_TRY(check_matrix(h_in, ld_in, layer->in_dim, "h_in"));
    DGI_TRY(prepare_weights(layer, P, weights, s));
    return run_transform(layer, P, h_in, ld_in, weights, Z, 0, rows, s);
}

uint64_t dgi::layer_aggregate_temp_bytes(const dgi_graph* g, const dgi_layer_t* layer, int64_t b, int64_t e) {
    LayerPlan P;
    if (plan_layer(g, layer, reinterpret_cast<const void*>(16), 0, &P) != DGI_OK) return 0;
    return batch_temp_bytes(g, layer, P, b, e) + 256;
}

dgi_status_t dgi::layer_aggregate_rows(const dgi_graph* g, const dgi_layer_t* layer, const void* Z, void* h_out, int64_t ld_out, int64_t out_base,
                                       int64_t b, int64_t e, void* temp, uint64_t temp_bytes, hipStream_t s) {
    LayerPlan P;
    DGI_TRY(plan_layer(g, layer, reinterpret_cast<const void*>(16), 0, &P));
    DGI_REQUIRE(P.transform_first, DGI_ERR_INVALID_ARG, "layer_aggregate_rows: not a transform-first layer");
    DGI_REQUIRE(b >= 0 && e >= b && e <= g->N, DGI_ERR_INVALID_ARG, "layer_aggregate_rows: bad destination range");
    if (e == b) return DGI_OK;
    DGI_REQUIRE(Z != nullptr, DGI_ERR_INVALID_ARG, "layer_aggregate_rows: Z is NULL");
    DGI_TRY(check_matrix(h_out, ld_out, layer->out_dim, "h_out"));
    DGI_REQUIRE(temp != nullptr && (uintptr_t)temp % 256 == 0 && temp_bytes >= batch_temp_bytes(g, layer, P, b, e), DGI_ERR_INVALID_ARG,
                "layer_aggregate_rows: temporary buffer missing, misaligned or too small");
    return run_batch(g, layer, P, nullptr, 0, h_out, ld_out, b, e, nullptr, Z, temp, s, nullptr, false, nullptr, out_base);
}

dgi_status_t dgi::layer_aggregate_rows_split(const dgi_graph* g, const dgi_layer_t* layer, const void* Zn, int64_t ld_n, const void* Zs, int64_t ld_s,
                                             void* h_out, int64_t ld_out, int64_t out_base, int64_t b, int64_t e, void* temp, uint64_t temp_bytes,
                                             hipStream_t s) {
    LayerPlan P;
    DGI_TRY(plan_layer(g, layer, reinterpret_cast<const void*>(16), 0, &P));
    DGI_REQUIRE(P.transform_first && !P.gat && P.has_self, DGI_ERR_INVALID_ARG, "layer_aggregate_rows_split: not a transform-first GraphSAGE layer");
    DGI_REQUIRE(b >= 0 && e >= b && e <= g->N, DGI_ERR_INVALID_ARG, "layer_aggregate_rows_split: bad destination range");
    if (e == b) return DGI_OK;
    DGI_REQUIRE(Zn != nullptr && Zs != nullptr && ld_n >= layer->out_dim && ld_s >= layer->out_dim, DGI_ERR_INVALID_ARG,
                "layer_aggregate_rows_split: NULL matrix or leading dimension too small");
    DGI_TRY(check_matrix(h_out, ld_out, layer->out_dim, "h_out"));
    const uint64_t part_bytes = round_up((int64_t)agg_hub_partial_bytes(g, b, e, layer->out_dim), 256);
    DGI_REQUIRE(part_bytes == 0 || (temp != nullptr && (uintptr_t)temp % 256 == 0 && temp_bytes >= part_bytes), DGI_ERR_INVALID_ARG,
                "layer_aggregate_rows_split: temporary buffer missing, misaligned or too small");
    const int zb = elem_bytes(P.z_dtype), ob = elem_bytes(layer->out_dtype);
    AggArgs a;
    a.g = g; a.mode = P.mode; a.row_begin = b; a.row_end = e;
    a.hub_partials = part_bytes ? (float*)temp : nullptr;
    a.S = Zn; a.ld_s = ld_n; a.s_dtype = P.z_dtype; a.width = layer->out_dim;
    // the kernels address the own-feature addend by destination row: row v of `self` is row v - b of Zs
    a.self = (const char*)Zs - b * ld_s * zb; a.ld_self = ld_s;
    a.out = (char*)h_out + (b - out_base) * ld_out * ob; a.ld_out = ld_out; a.out_row0 = b; a.out_dtype = layer->out_dtype;
    a.bias = layer->bias; a.act = layer->act; a.act_slope = layer->act_slope; a.out_scale = nullptr;
    DGI_TRY(launch_aggregate(a, 0, s));
    return launch_aggregate(a, 1, s);
}

extern "C" dgi_status_t dgi_layer_forward(const dgi_graph_t* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in,
                                          void* h_out, int64_t ld_out, int64_t dst_begin, int64_t dst_end, void* workspace,
                                          uint64_t workspace_bytes, void* hip_stream) {
    return layer_forward_rows(g, layer, h_in, ld_in, h_out, ld_out, 0, dst_begin, dst_end, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

// ---- dgi_layer_forward without any allocation: the workspace is a static device array -----------------------
// One array per GPU (every device that loads the library's code object holds its own copy).  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels and fills get the address that call returns.
static __device__ __align__(256) unsigned char scratch[DGI_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on device i, looked up on first use there

// the calling thread's current device must be the one the lookup is for
dgi_status_t static_scratch(void** out) {
    int dev = -1;
    DGI_HIP(hipGetDevice(&dev));
    DGI_REQUIRE(dev >= 0 && dev < kMaxDevices, DGI_ERR_UNSUPPORTED, "static workspace: device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        DGI_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        DGI_REQUIRE(p != nullptr && (uintptr_t)p % 256 == 0, DGI_ERR_DEVICE, "static workspace: symbol address missing or misaligned");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DGI_OK;
}
}  // namespace

extern "C" dgi_status_t dgi_layer_forward_static(const dgi_graph_t* g, const dgi_layer_t* layer, const void* h_in, int64_t ld_in,
                                                 void* h_out, int64_t ld_out, int64_t dst_begin, int64_t dst_end, void* hip_stream) {
    DGI_REQUIRE(g != nullptr, DGI_ERR_INVALID_ARG, "graph is NULL");
    int dev = -1;
    DGI_HIP(hipGetDevice(&dev));
    DGI_REQUIRE(dev == g->device, DGI_ERR_INVALID_ARG, "layer_forward_static: current device %d is not the graph's device %d", dev, g->device);
    uint64_t need = 0;
    DGI_TRY(dgi_layer_workspace_bytes(g, layer, dst_begin, dst_end, &need));
    DGI_REQUIRE(need <= (uint64_t)DGI_STATIC_WORKSPACE_BYTES, DGI_ERR_UNSUPPORTED,
                "layer_forward_static: this layer and row range need %llu bytes of workspace, the static workspace holds %llu; "
                "use dgi_layer_forward with a caller-provided workspace",
                (unsigned long long)need, (unsigned long long)DGI_STATIC_WORKSPACE_BYTES);
    void* ws = nullptr;
    DGI_TRY(static_scratch(&ws));
    // every region of the workspace the kernels read is written first in the same call (packed weights are zero-filled
    // by a kernel, Z / partials / the aggregated tile are produced before they are consumed), so what the previous
    // call left behind is never observed
    return layer_forward_rows(g, layer, h_in, ld_in, h_out, ld_out, 0, dst_begin, dst_end, ws, DGI_STATIC_WORKSPACE_BYTES,
                              static_cast<hipStream_t>(hip_stream));
}

extern "C" dgi_status_t dgi_infer(const dgi_graph_t* g, const dgi_layer_t* layers, int32_t num_layers, const void* x,
                                  int64_t ld_x, void* out, int64_t ld_out, const dgi_infer_opts_t* opts, void* hip_stream) {
    return infer_rows(g, layers, num_layers, x, ld_x, out, ld_out, opts, nullptr, hip_stream);
}

// dgi_infer with an optional per-layer row limit: layer l computes destination rows [0, row_limit[l]) only and reads
// source rows [0, row_limit[l-1]) (all N rows of x for l = 0).  Partial inference numbers its sub-problem so that the
// per-layer target sets of Section 3.3 are such prefixes.  Rows beyond a limit are neither read nor written.
dgi_status_t dgi::infer_rows(const dgi_graph* g, const dgi_layer_t* layers, int32_t num_layers, const void* x, int64_t ld_x, void* out,
                             int64_t ld_out, const dgi_infer_opts_t* opts, const int64_t* row_limit, void* hip_stream) {
    DGI_REQUIRE(g != nullptr && layers != nullptr, DGI_ERR_INVALID_ARG, "infer: NULL argument");
    DGI_REQUIRE(num_layers >= 1 && num_layers <= DGI_MAX_LAYERS, DGI_ERR_INVALID_ARG, "infer: 1..%d layers supported", DGI_MAX_LAYERS);
    dgi_infer_opts_t o{};
    if (opts) o = *opts;
    // Jumping-knowledge stack (the paper's JKNet example): the last layer reads the concatenation of all earlier
    // layer outputs.  The hidden layers then live side by side in one [N x sum(out_dim)] matrix: layer l writes
    // its column block, layer l+1 reads that block, the last layer reads all of it (leading dimensions do the rest),
    // and no hidden layer is released before the last layer has run.
    const bool jk = o.jk_concat != 0;
    int64_t ld_cat = 0;
    std::vector<int64_t> cat_off((size_t)num_layers, 0);
    if (jk) {
        DGI_REQUIRE(num_layers >= 2, DGI_ERR_INVALID_ARG, "infer: a jumping-knowledge stack needs at least 2 layers");
        const int hd = layers[0].out_dtype, E = 16 / elem_bytes(hd);
        for (int l = 0; l + 1 < num_layers; ++l) {
            DGI_REQUIRE(layers[l].out_dtype == hd, DGI_ERR_INVALID_ARG, "infer: jumping-knowledge layers must share one hidden dtype");
            DGI_REQUIRE(layers[l].out_dim % E == 0, DGI_ERR_UNSUPPORTED, "infer: jumping-knowledge hidden widths must be multiples of 16 bytes");
            cat_off[l] = ld_cat;
            ld_cat += layers[l].out_dim;
        }
        DGI_REQUIRE(layers[num_layers - 1].in_dim == ld_cat && layers[num_layers - 1].feat_dtype == hd, DGI_ERR_INVALID_ARG,
                    "infer: the last jumping-knowledge layer must read the concatenation of all earlier outputs");
    }
    // A first GCN layer gathers rows that already carry d_out(u)^-1/2 from a scaled copy of x (one pass over x:
    // 2 N ld bytes) instead of fetching the factor per edge (a 128-byte line for 4 bytes on most edges).  With few
    // edges per node (a sampled graph) the copy costs more than the per-edge fetches; then the layer keeps them.
    const bool scale_x = layers[0].agg == DGI_AGG_GCN && !jk &&
                         (double)g->E * 128.0 >= 2.0 * (double)g->N * (double)round_up(layers[0].in_dim, 16 / elem_bytes(layers[0].feat_dtype)) *
                                                     elem_bytes(layers[0].feat_dtype);
    std::vector<LayerPlan> plans((size_t)num_layers);
    for (int l = 0; l < num_layers; ++l) {
        // layer 0 reads the caller's x; later layers read the library's own 16-byte aligned hidden buffers.  With a
        // permutation, layer 0 reads the library's permuted copy of x instead.
        const bool own_input = l > 0 || o.perm_new_of_old || scale_x;
        const int64_t own_ld = (jk && l > 0) ? ld_cat : round_up(layers[l].in_dim, 16 / elem_bytes(layers[l].feat_dtype));
        DGI_TRY(plan_layer(g, &layers[l], own_input ? reinterpret_cast<const void*>(256) : x, own_input ? own_ld : ld_x, &plans[l]));
        if (l > 0 && !(jk && l == num_layers - 1)) {
            DGI_REQUIRE(layers[l].in_dim == layers[l - 1].out_dim, DGI_ERR_INVALID_ARG, "layer %d: in_dim != previous out_dim", l);
            DGI_REQUIRE(layers[l].feat_dtype == layers[l - 1].out_dtype, DGI_ERR_INVALID_ARG, "layer %d: feat_dtype != previous out_dtype", l);
        }
    }
    DGI_REQUIRE(o.batch_size >= 0, DGI_ERR_INVALID_ARG, "infer: negative batch_size");
    if (o.stats) { std::memset(o.stats, 0, sizeof(dgi_stats_t)); o.stats->num_layers = num_layers; }
    const int64_t N = g->N;
    if (N == 0) return DGI_OK;
    const dgi_layer_t& L0 = layers[0];
    const dgi_layer_t& LL = layers[num_layers - 1];
    DGI_TRY(check_matrix(x, ld_x, L0.in_dim, "x"));
    DGI_TRY(check_matrix(out, ld_out, LL.out_dim, "out"));
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    // ---- memory plan -------------------------------------------------------------------------------
    std::lock_guard<std::mutex> ws_lock(g->ws_mutex);  // one dgi_infer at a time per graph handle
    uint64_t budget = o.mem_budget_bytes;
    if (budget == 0) {
        size_t free_b = 0, total_b = 0;
        DGI_HIP(hipMemGetInfo(&free_b, &total_b));
        budget = (uint64_t)(0.9 * (double)(free_b + g->ws_bytes));  // the cached arena counts as available
    }
    uint64_t hidden_bytes = 0;  // one ping-pong buffer
    for (int l = 0; l + 1 < num_layers; ++l) {
        const int eb = elem_bytes(layers[l].out_dtype);
        hidden_bytes = std::max<uint64_t>(hidden_bytes, (uint64_t)round_up(N * round_up(layers[l].out_dim, 16 / eb) * eb, 256));
    }
    int n_hidden = num_layers >= 3 ? 2 : (num_layers == 2 ? 1 : 0);
    if (jk) {  // one concatenated matrix instead of ping-pong buffers
        hidden_bytes = (uint64_t)round_up(N * ld_cat * elem_bytes(layers[0].out_dtype), 256);
        n_hidden = 1;
    }
    const bool permuted = o.perm_new_of_old != nullptr;
    const int xb = elem_bytes(L0.feat_dtype), yb = elem_bytes(LL.out_dtype);
    const int64_t ld_xp = round_up(L0.in_dim, 16 / xb), ld_yp = round_up(LL.out_dim, 16 / yb);
    // GCN layers gather rows already multiplied by d_out(u)^-1/2: every layer folds the next layer's factor into
    // its epilogue, and the input of a first GCN layer is scaled once into a library-owned copy.
    // (a jumping-knowledge output has several consumers: no folding of the factor, and no scaled copy of x)
    const uint64_t xp_bytes = (permuted || scale_x) ? (uint64_t)round_up(N * ld_xp * xb, 256) : 0;
    const uint64_t yp_bytes = permuted ? (uint64_t)round_up(N * ld_yp * yb, 256) : 0;
    uint64_t fixed_max = 0, temp_full_max = 0;
    for (int l = 0; l < num_layers; ++l) {
        const LayerPlan& P = plans[l];
        uint64_t fixed = P.wt_bytes;
        if (P.transform_first) fixed += (uint64_t)round_up(N * P.z_ld * elem_bytes(P.z_dtype), 256);
        fixed_max = std::max(fixed_max, fixed);
        temp_full_max = std::max(temp_full_max, batch_temp_bytes(g, &layers[l], P, 0, row_limit ? std::min(N, row_limit[l]) : N));
    }
    const uint64_t persistent = hidden_bytes * n_hidden + xp_bytes + yp_bytes + fixed_max;
    DGI_REQUIRE(budget > persistent + 4096, DGI_ERR_OOM,
                "memory budget %llu bytes cannot hold the hidden layers and per-layer buffers (%llu bytes)",
                (unsigned long long)budget, (unsigned long long)persistent);
    // Expected consumption M of Eq. 2 for the batch temporaries: what is left of the budget (the budget is
    // already 90 % of free memory when it was not given), but no more than one whole-graph batch needs.
    const uint64_t temp_cap = std::max<uint64_t>(std::min<uint64_t>(budget - persistent, temp_full_max), 256);

    const uint64_t arena_bytes = persistent + temp_cap + 1024;
    if (g->ws_bytes < arena_bytes || g->ws_bytes > std::max<uint64_t>(budget, arena_bytes)) {
        // (re)allocate: too small, or larger than this call's budget allows it to hold
        if (g->ws_ptr) { DGI_HIP(hipStreamSynchronize(s)); (void)hipFree(g->ws_ptr); g->ws_ptr = nullptr; g->ws_bytes = 0; }
        DGI_HIP(hipMalloc(reinterpret_cast<void**>(&g->ws_ptr), arena_bytes));
        g->ws_bytes = arena_bytes;
    }
    char* arena = g->ws_ptr;
    uint64_t off = 0;
    auto carve = [&](uint64_t bytes) { char* p = arena + off; off += (uint64_t)round_up((int64_t)bytes, 256); return p; };
    char* hid[2] = {nullptr, nullptr};
    for (int i = 0; i < n_hidden; ++i) hid[i] = carve(hidden_bytes);
    char* xp = (permuted || scale_x) ? carve(xp_bytes) : nullptr;
    char* yp = permuted ? carve(yp_bytes) : nullptr;
    char* fixed = carve(fixed_max);
    char* temp = carve(temp_cap);
    if (o.stats) o.stats->workspace_bytes = (int64_t)arena_bytes;

    KernelTimer timer(s);
    KernelTimer* tm = o.stats ? &timer : nullptr;
    if (tm) { tm->layer = -1; DGI_TRY(tm->begin(SPAN_TOTAL)); }

    const void* cur = x;
    int64_t ld_cur = ld_x;
    if (permuted) {  // rows to the reordered numbering: xp[perm[r]] = x[r]
        DGI_TRY(launch_permute_rows(x, ld_x, xp, ld_xp, N, L0.in_dim, xb, o.perm_new_of_old, false, s));
        cur = xp; ld_cur = ld_xp;
    }
    if (scale_x) {  // in place on the permuted copy, or from the caller's x into the copy
        DGI_TRY(launch_scale_rows(cur, ld_cur, xp, ld_xp, N, L0.in_dim, xb, g->d_rs_out, s));
        cur = xp; ld_cur = ld_xp;
    }
    const double avg_deg = N > 0 ? (double)g->E / (double)N : 0.0;
    for (int l = 0; l < num_layers; ++l) {
        const dgi_layer_t& L = layers[l];
        const LayerPlan& P = plans[l];
        const bool last = l == num_layers - 1;
        void* dst; int64_t ld_dst;
        if (last) { dst = permuted ? (void*)yp : out; ld_dst = permuted ? ld_yp : ld_out; }
        else if (jk) { dst = hid[0] + cat_off[l] * elem_bytes(L.out_dtype); ld_dst = ld_cat; }
        else { dst = hid[l % 2]; ld_dst = round_up(L.out_dim, 16 / elem_bytes(L.out_dtype)); }
        if (jk && last) { cur = hid[0]; ld_cur = ld_cat; }  // the whole concatenation
        const bool in_prescaled = !jk && L.agg == DGI_AGG_GCN && (l == 0 ? scale_x : layers[l - 1].agg != DGI_AGG_GAT);
        const float* out_scale = (!jk && !last && layers[l + 1].agg == DGI_AGG_GCN && L.agg != DGI_AGG_GAT) ? g->d_rs_out : nullptr;
        if (tm) { tm->layer = l; DGI_TRY(tm->begin(SPAN_LAYER)); }
        const size_t layer_span = tm ? tm->spans.size() - 1 : 0;
        char* Wt = fixed;
        char* Z = fixed + P.wt_bytes;
        DGI_TRY(prepare_weights(&L, P, Wt, s));
        if (P.transform_first) {
            if (tm) DGI_TRY(tm->begin(SPAN_GEMM));
            DGI_TRY(run_transform(&L, P, cur, ld_cur, Wt, Z, 0, (row_limit && l > 0) ? std::min(N, row_limit[l - 1]) : N, s));
            if (tm) DGI_TRY(tm->end());
        }
        // ---- batches of destination rows (Section 4.1) ----------------------------------------------
        int64_t n_t = o.batch_size > 0 ? o.batch_size : (o.init_node_threshold > 0 ? o.init_node_threshold : 65536);
        int64_t n_i = o.batch_size > 0 ? INT64_MAX / 4
                                       : (o.init_edge_threshold > 0 ? o.init_edge_threshold : (int64_t)std::max(1.0, (double)n_t * std::max(avg_deg, 1.0)));
        int64_t b = 0, batches = 0;
        const int64_t N_full = g->N;
        const int64_t N = row_limit ? std::min(N_full, row_limit[l]) : N_full;   // rows this layer computes
        while (b < N) {
            int64_t e = 0;
            DGI_TRY(dgi_plan_batch_end(g->h_indptr.data(), DGI_I64, N, b, std::min(std::max<int64_t>(n_t, 1), kMaxRowsPerLaunch * 4),
                                       std::max<int64_t>(n_i, 0), &e));
            // With everything resident the temporaries of a planned batch are known before it runs, so the first batch
            // of a layer applies Eq. 2 to its own plan (repeatedly: temporaries grow with the batch, but not in
            // proportion) instead of running an undersized batch just to learn r.
            if (o.batch_size == 0 && b == 0) {
                const int64_t row_cap = kMaxRowsPerLaunch * 4;
                for (int it = 0; it < 16 && e < N; ++it) {
                    const uint64_t nd = batch_temp_bytes(g, &L, P, b, e);
                    if (nd > temp_cap) break;  // the halving below takes over
                    int64_t t2 = n_t, i2 = n_i, e2 = 0;
                    if (nd == 0) { t2 = N; i2 = std::max<int64_t>(g->E, 1); }
                    else DGI_TRY(dgi_threshold_update((double)temp_cap, (double)nd, &t2, &i2));
                    if (t2 <= n_t && i2 <= n_i) break;
                    DGI_TRY(dgi_plan_batch_end(g->h_indptr.data(), DGI_I64, N, b, std::min(std::max<int64_t>(t2, 1), row_cap), std::max<int64_t>(i2, 0), &e2));
                    if (e2 <= e || batch_temp_bytes(g, &L, P, b, e2) > temp_cap) break;  // no growth, or growing overshoots
                    n_t = t2; n_i = i2; e = e2;
                }
            }
            const uint64_t need = batch_temp_bytes(g, &L, P, b, e);
            if (need > temp_cap) {  // the batch would not fit: the out-of-memory reaction of Section 4.1
                if (o.stats) o.stats->oom_retries += 1;
                dgi_status_t hs = dgi_threshold_halve(&n_t, &n_i);
                if (hs != DGI_OK || e - b <= 1) {
                    set_error("layer %d: a single destination row needs %llu bytes of temporaries, budget leaves %llu", l,
                              (unsigned long long)need, (unsigned long long)temp_cap);
                    return DGI_ERR_OOM;
                }
                n_t = std::min(n_t, std::max<int64_t>((e - b) / 2, 1));
                continue;
            }
            DGI_TRY(run_batch(g, &L, P, cur, ld_cur, dst, ld_dst, b, e, Wt, Z, temp, s, tm, in_prescaled, out_scale));
            ++batches;
            if (o.batch_size == 0) {
                if (need == 0) { n_t = N; n_i = std::max<int64_t>(g->E, 1); }  // nothing to bound
                else DGI_TRY(dgi_threshold_update((double)temp_cap, (double)need, &n_t, &n_i));
            }
            b = e;
        }
        if (tm) { DGI_HIP(hipEventRecord(tm->spans[layer_span].b, s)); }
        if (o.stats) {
            o.stats->batches[l] = batches;
            o.stats->edges[l] = g->h_indptr[(size_t)N] - g->h_indptr[0];
            o.stats->transform_first[l] = P.transform_first ? 1 : 0;
            o.stats->fused[l] = P.fused ? 1 : 0;
            o.stats->gather_width[l] = P.gat ? (int)P.z_ld : (P.transform_first ? L.out_dim : L.in_dim);
        }
        cur = dst; ld_cur = ld_dst;  // H^{l-1} is dead from here on: its buffer is the next layer's output
    }
    if (permuted)  // back to the caller's numbering: out[r] = yp[perm[r]]
        DGI_TRY(launch_permute_rows(yp, ld_yp, out, ld_out, N, LL.out_dim, yb, o.perm_new_of_old, true, s));
    if (tm) DGI_HIP(hipEventRecord(tm->spans[0].b, s));
    DGI_HIP(hipStreamSynchronize(s));
    if (o.stats) {
        for (const auto& sp : timer.spans) {
            float ms = 0.f;
            DGI_HIP(hipEventElapsedTime(&ms, sp.a, sp.b));
            if (sp.kind == SPAN_TOTAL) o.stats->total_ms = ms;
            else if (sp.kind == SPAN_LAYER) o.stats->layer_ms[sp.layer] = ms;
            else if (sp.kind == SPAN_AGG) { o.stats->agg_ms[sp.layer] += ms; o.stats->agg_launches[sp.layer] += 1; }
            else if (sp.kind == SPAN_HUB) o.stats->hub_ms[sp.layer] += ms;
            else if (sp.kind == SPAN_GEMM) { o.stats->gemm_ms[sp.layer] += ms; o.stats->gemm_launches[sp.layer] += 1; }
        }
    }
    return DGI_OK;
}

// ---- host-side planning helpers ---------------------------------------------------------------------
extern "C" dgi_status_t dgi_plan_batch_end(const void* indptr, int32_t indptr_type, int64_t row_limit, int64_t begin,
                                           int64_t n_t, int64_t n_i, int64_t* end) {
    DGI_REQUIRE(indptr && end, DGI_ERR_INVALID_ARG, "plan_batch_end: NULL argument");
    DGI_REQUIRE(begin >= 0 && begin < row_limit, DGI_ERR_INVALID_ARG, "plan_batch_end: begin outside [0,row_limit)");
    DGI_REQUIRE(n_t >= 1 && n_i >= 0, DGI_ERR_INVALID_ARG, "plan_batch_end: thresholds must be positive");
    auto at = [&](int64_t i) { return indptr_type == DGI_I64 ? ((const int64_t*)indptr)[i] : (int64_t)((const int32_t*)indptr)[i]; };
    const int64_t hi_lim = std::min(row_limit, begin + n_t);
    const int64_t cap = at(begin) + n_i;
    // binary search on the in-degree prefix sum: largest end in [begin+1, hi_lim] with at(end) <= cap
    int64_t lo = begin + 1, hi = hi_lim;
    if (at(lo) > cap) { *end = lo; return DGI_OK; }  // one row alone exceeds n_i: it forms a batch by itself
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo + 1) / 2;
        if (at(mid) <= cap) lo = mid; else hi = mid - 1;
    }
    *end = lo;
    return DGI_OK;
}

extern "C" dgi_status_t dgi_threshold_update(double M_expected, double M_k, int64_t* n_t, int64_t* n_i) {
    DGI_REQUIRE(n_t && n_i, DGI_ERR_INVALID_ARG, "threshold_update: NULL argument");
    if (!(M_k > 0.0) || !(M_expected > 0.0)) return DGI_OK;
    const double r = M_expected / M_k;
    auto scale = [&](int64_t v) {
        const double x = std::floor(r * (double)v);
        if (x < 1.0) return (int64_t)1;
        if (x > 4.0e18) return (int64_t)4000000000000000000ll;
        return (int64_t)x;
    };
    *n_t = scale(*n_t);
    *n_i = scale(*n_i);
    return DGI_OK;
}

extern "C" dgi_status_t dgi_threshold_halve(int64_t* n_t, int64_t* n_i) {
    DGI_REQUIRE(n_t && n_i, DGI_ERR_INVALID_ARG, "threshold_halve: NULL argument");
    if (*n_t <= 1 && *n_i <= 1) { set_error("thresholds cannot be halved below one"); return DGI_ERR_OOM; }
    *n_t = std::max<int64_t>(*n_t / 2, 1);
    *n_i = std::max<int64_t>(*n_i / 2, 1);
    return DGI_OK;
}

extern "C" dgi_status_t dgi_batch_input_set_size(int64_t num_nodes, const int64_t* indptr, const int32_t* indices,
                                                 int64_t begin, int64_t end, int64_t* count) {
    DGI_REQUIRE(indptr && count && (indices || indptr[num_nodes] == 0), DGI_ERR_INVALID_ARG, "batch_input_set_size: NULL argument");
    DGI_REQUIRE(begin >= 0 && end >= begin && end <= num_nodes, DGI_ERR_INVALID_ARG, "batch_input_set_size: bad range");
    std::unordered_set<int32_t> seen;
    for (int64_t e = indptr[begin]; e < indptr[end]; ++e) seen.insert(indices[e]);
    *count = (int64_t)seen.size();
    return DGI_OK;
}

extern "C" dgi_status_t dgi_reorder_permutation(int64_t num_nodes, const int64_t* indptr, const int32_t* indices,
                                                int32_t method, uint64_t seed, int32_t* perm_new_of_old) {
    return reorder_permutation(num_nodes, indptr, indices, method, seed, perm_new_of_old);
}
