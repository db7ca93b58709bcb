// GAT edge pass: per destination v and head h, e_u = LeakyReLU(el[u,h] + er[v,h]) over u in N(v), softmax
// over the neighbourhood, out[v,h,:] = sum_u alpha_u z[u,h,:]  (the attention instance of Eq. 1's AGGREGATE).
//
// Input rows come from the transform GEMM as  [ z (heads*F) | el (heads) | er (heads) | pad ], so the score
// terms of a source sit next to the features the same wavefront gathers.  One wavefront per destination
// row, G lanes per source row (16-byte loads), 64/G neighbours per load instruction.  The softmax is a
// single sweep: every lane group keeps a running maximum m, a running denominator l and the weighted
// sum rescaled by exp(m_old - m_new) per block of UNROLL neighbours; the lane groups are merged at the
// end with the same rule.  Scores are shifted by the running maximum before exp, so nothing overflows.
// Rows with more than kHubDegree in-edges get a whole workgroup (see gat_rows_kernel), merged in a fixed order,
// so the result of a row does not depend on scheduling or on the batch it falls in.
#include <algorithm>

#include "dgi_device.h"
#include "dgi_internal.h"

namespace dgi {
namespace {

constexpr int kWaves = 4;
constexpr int kRowsPerWg = 16;
constexpr float kNegBig = -1.0e30f;

struct GatParams {
    const void* indptr;
    const int32_t* indices;
    const float* Zx;
    int64_t ld_z;
    int heads, F, HF;
    float slope;
    void* out;
    int64_t ld_out;
    int64_t out_row0;
    int out_bf16;
    int out_vec_ok;  // output rows can be written in 16-byte (fp32) / 8-byte (bf16) pieces of 4 columns
    const float* bias;
    int act;
    float act_slope;
    int64_t row_begin, row_end;
    // rows with more than kHubDegree in-edges inside [row_begin,row_end): hub_rows[hub_begin..hub_end), one workgroup each
    const int64_t* hub_rows;
    int64_t hub_begin, hub_end;
};

__device__ __forceinline__ void store_out(const GatParams& p, int64_t v, int c, float val) {
    if (p.bias) val += p.bias[c];
    val = activate(val, p.act, p.act_slope);
    const int64_t o = (v - p.out_row0) * p.ld_out + c;
    if (p.out_bf16) static_cast<uint16_t*>(p.out)[o] = float_to_bf16(val);
    else static_cast<float*>(p.out)[o] = val;
}

// the 4 consecutive columns a lane owns, as one store where the layout allows it
__device__ __forceinline__ void store_out4(const GatParams& p, int64_t v, int col, const float* a, float inv) {
    if (!(p.out_vec_ok && col + 4 <= p.HF)) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (col + i < p.HF) store_out(p, v, col + i, a[i] * inv);
        return;
    }
    float val[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        val[i] = a[i] * inv;
        if (p.bias) val[i] += p.bias[col + i];
        val[i] = activate(val[i], p.act, p.act_slope);
    }
    const int64_t o = (v - p.out_row0) * p.ld_out + col;
    if (p.out_bf16)
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + o) =
            make_uint2((uint32_t)float_to_bf16(val[0]) | ((uint32_t)float_to_bf16(val[1]) << 16),
                       (uint32_t)float_to_bf16(val[2]) | ((uint32_t)float_to_bf16(val[3]) << 16));
    else
        *reinterpret_cast<float4*>(static_cast<float*>(p.out) + o) = make_float4(val[0], val[1], val[2], val[3]);
}

// Running softmax state of one lane: maximum score m, denominator l, weighted sum of its 4 columns.
struct Soft {
    float m, l, acc[4];
};

__device__ __forceinline__ void soft_merge(Soft& a, float m2, float l2, const float* acc2) {
    const float M = fmaxf(a.m, m2);
    const float x = __expf(a.m - M), y = __expf(m2 - M);
    a.l = a.l * x + l2 * y;
#pragma unroll
    for (int i = 0; i < 4; ++i) a.acc[i] = a.acc[i] * x + acc2[i] * y;
    a.m = M;
}

// Single sweep with a running maximum over the 64-edge blocks e0 = first, first + step, ... of the list [., ee),
// lane groups side by side on NSUB neighbours; ends with the lane groups merged (every lane holds the result).
template <int G>
__device__ __forceinline__ Soft gat_sweep(const GatParams& p, int64_t first, int64_t ee, int64_t step, int lane, float er, const float* zbase,
                                         const float* elbase, bool col_ok) {
    constexpr int NSUB = 64 / G;
    constexpr int UNROLL = (G == 64) ? 8 : 4;
    const int sub = lane / G;
    Soft st;
    st.m = kNegBig; st.l = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) st.acc[i] = 0.f;
    for (int64_t e0 = first; e0 < ee; e0 += step) {
        const int64_t left = ee - e0;
        const int cnt = left < 64 ? (int)left : 64;
        const int my = lane < cnt ? p.indices[e0 + lane] : 0;
        for (int j = 0; j < cnt; j += NSUB * UNROLL) {
            float4 z[UNROLL];
            float sc[UNROLL];
            bool ok[UNROLL];
            int64_t off[UNROLL];
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                const int k = j + t * NSUB + sub;
                ok[t] = k < cnt;
                const int ks = ok[t] ? k : 0;
                const int u = (G == 64) ? __builtin_amdgcn_readlane(my, ks) : __shfl(my, ks, 64);
                off[t] = (int64_t)u * p.ld_z;
            }
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                sc[t] = elbase[off[t]];
                z[t] = col_ok ? *reinterpret_cast<const float4*>(zbase + off[t]) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            float mx = st.m;
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                float s = sc[t] + er;
                s = s > 0.f ? s : p.slope * s;
                sc[t] = ok[t] ? s : kNegBig;
                mx = fmaxf(mx, sc[t]);
            }
            const float corr = __expf(st.m - mx);
            st.l *= corr;
#pragma unroll
            for (int i = 0; i < 4; ++i) st.acc[i] *= corr;
            st.m = mx;
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                const float w = ok[t] ? __expf(sc[t] - mx) : 0.f;
                st.l += w;
                st.acc[0] = fmaf(w, z[t].x, st.acc[0]);
                st.acc[1] = fmaf(w, z[t].y, st.acc[1]);
                st.acc[2] = fmaf(w, z[t].z, st.acc[2]);
                st.acc[3] = fmaf(w, z[t].w, st.acc[3]);
            }
        }
    }
#pragma unroll
    for (int o = G; o < 64; o <<= 1) {  // merge the lane groups
        float other[4];
        const float m2 = __shfl_xor(st.m, o, 64), l2 = __shfl_xor(st.l, o, 64);
#pragma unroll
        for (int i = 0; i < 4; ++i) other[i] = __shfl_xor(st.acc[i], o, 64);
        soft_merge(st, m2, l2, other);
    }
    return st;
}

// Requires: all 4 columns of a lane belong to one head (heads == 1 or F % 4 == 0), 16-byte aligned rows.
// The first hub_end - hub_begin workgroups take one hub row each (they are the longest work items, so they go
// first): its four wavefronts sweep interleaved 64-edge blocks of the list and their states are merged in
// wavefront order through LDS.  The other workgroups take kRowsPerWg consecutive rows, one wavefront per row.
template <typename IdxT, int G>
__global__ __launch_bounds__(kWaves * 64) void gat_rows_kernel(GatParams p) {
    __shared__ float part[kWaves][6][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane / G, gl = lane % G;
    const int col = gl * 4;
    const bool col_ok = col < p.HF;
    const int h = col_ok ? col / p.F : 0;
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const float* zbase = p.Zx + col;
    const float* elbase = p.Zx + p.HF + h;
    const int64_t n_hub = p.hub_end - p.hub_begin;
    if ((int64_t)blockIdx.x < n_hub) {
        const int64_t v = p.hub_rows[p.hub_begin + blockIdx.x];
        const int64_t eb = (int64_t)indptr[v], ee = (int64_t)indptr[v + 1];
        const float er = p.Zx[v * p.ld_z + p.HF + p.heads + h];
        Soft st = gat_sweep<G>(p, eb + 64 * wave, ee, 64 * kWaves, lane, er, zbase, elbase, col_ok);
        part[wave][0][lane] = st.m;
        part[wave][1][lane] = st.l;
#pragma unroll
        for (int i = 0; i < 4; ++i) part[wave][2 + i][lane] = st.acc[i];
        __syncthreads();
        if (wave == 0) {
            for (int w = 1; w < kWaves; ++w) {
                float other[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) other[i] = part[w][2 + i][lane];
                soft_merge(st, part[w][0][lane], part[w][1][lane], other);
            }
            if (sub == 0 && col_ok) store_out4(p, v, col, st.acc, st.l > 0.f ? 1.0f / st.l : 0.f);
        }
        return;
    }
    const int64_t v0 = p.row_begin + ((int64_t)blockIdx.x - n_hub) * kRowsPerWg;
    for (int r = wave; r < kRowsPerWg; r += kWaves) {
        const int64_t v = v0 + r;
        if (v >= p.row_end) break;
        const int64_t eb = (int64_t)indptr[v], ee = (int64_t)indptr[v + 1];
        if (n_hub > 0 && ee - eb > kHubDegree) continue;  // a hub workgroup has it
        const float er = p.Zx[v * p.ld_z + p.HF + p.heads + h];
        const Soft st = gat_sweep<G>(p, eb, ee, 64, lane, er, zbase, elbase, col_ok);
        if (sub == 0 && col_ok) store_out4(p, v, col, st.acc, st.l > 0.f ? 1.0f / st.l : 0.f);
    }
}

// Any layout: one wavefront per row, one output column per lane, two sweeps (maximum, then weights).
template <typename IdxT>
__global__ __launch_bounds__(kWaves * 64) void gat_rows_generic_kernel(GatParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t v = p.row_begin + (int64_t)blockIdx.x * kWaves + wave;
    if (v >= p.row_end) return;
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const int64_t eb = (int64_t)indptr[v], ee = (int64_t)indptr[v + 1];
    for (int c = lane; c < p.HF; c += 64) {
        const int h = c / p.F;
        const float er = p.Zx[v * p.ld_z + p.HF + p.heads + h];
        float m = kNegBig;
        for (int64_t e = eb; e < ee; ++e) {
            float s = p.Zx[(int64_t)p.indices[e] * p.ld_z + p.HF + h] + er;
            s = s > 0.f ? s : p.slope * s;
            m = fmaxf(m, s);
        }
        float l = 0.f, acc = 0.f;
        for (int64_t e = eb; e < ee; ++e) {
            const int64_t u = p.indices[e];
            float s = p.Zx[u * p.ld_z + p.HF + h] + er;
            s = s > 0.f ? s : p.slope * s;
            const float w = __expf(s - m);
            l += w;
            acc = fmaf(w, p.Zx[u * p.ld_z + c], acc);
        }
        store_out(p, v, c, l > 0.f ? acc / l : 0.f);
    }
}

template <typename IdxT, int G>
dgi_status_t launch_g(const GatParams& p, hipStream_t stream) {
    const int64_t rows = p.row_end - p.row_begin;
    const int64_t grid = (rows + kRowsPerWg - 1) / kRowsPerWg + (p.hub_end - p.hub_begin);
    DGI_REQUIRE(grid * kWaves * 64 < (int64_t)1 << 32, DGI_ERR_INVALID_ARG, "gat: row range too large for one launch");
    hipLaunchKernelGGL((gat_rows_kernel<IdxT, G>), dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

template <typename IdxT>
dgi_status_t dispatch(const GatParams& p, bool fast, hipStream_t stream) {
    if (!fast) {
        for (int64_t r0 = p.row_begin; r0 < p.row_end; r0 += (int64_t)1 << 25) {  // < 2^32 threads per launch
            GatParams q = p;
            q.row_begin = r0;
            q.row_end = p.row_end < r0 + ((int64_t)1 << 25) ? p.row_end : r0 + ((int64_t)1 << 25);
            const int64_t rows = q.row_end - q.row_begin;
            hipLaunchKernelGGL((gat_rows_generic_kernel<IdxT>), dim3((unsigned)((rows + kWaves - 1) / kWaves)), dim3(kWaves * 64), 0,
                               stream, q);
            DGI_HIP(hipGetLastError());
        }
        return DGI_OK;
    }
    const int lanes = (p.HF + 3) / 4;
    if (lanes <= 4) return launch_g<IdxT, 4>(p, stream);
    if (lanes <= 8) return launch_g<IdxT, 8>(p, stream);
    if (lanes <= 16) return launch_g<IdxT, 16>(p, stream);
    if (lanes <= 32) return launch_g<IdxT, 32>(p, stream);
    return launch_g<IdxT, 64>(p, stream);
}

}  // namespace

dgi_status_t launch_gat(const GatArgs& a, hipStream_t stream) {
    if (a.row_end <= a.row_begin) return DGI_OK;
    const dgi_graph* g = a.g;
    DGI_REQUIRE(a.row_begin >= 0 && a.row_end <= g->N, DGI_ERR_INVALID_ARG, "gat: row range outside the graph");
    GatParams p{};
    p.indptr = g->d_indptr;
    p.indices = g->d_indices;
    p.Zx = a.Zx; p.ld_z = a.ld_z;
    p.heads = a.heads; p.F = a.head_dim; p.HF = a.heads * a.head_dim;
    p.slope = a.attn_slope;
    p.out = a.out; p.ld_out = a.ld_out; p.out_row0 = a.out_row0; p.out_bf16 = a.out_dtype == DGI_BF16;
    p.out_vec_ok = ((uintptr_t)a.out % 16 == 0) && ((a.ld_out * (p.out_bf16 ? 2 : 4)) % 16 == 0);
    p.bias = a.bias; p.act = a.act; p.act_slope = a.act_slope;
    p.row_begin = a.row_begin; p.row_end = a.row_end;
    {
        const auto& hr = g->h_hub_rows;
        p.hub_rows = g->d_hub_rows;
        p.hub_begin = std::lower_bound(hr.begin(), hr.end(), a.row_begin) - hr.begin();
        p.hub_end = std::lower_bound(hr.begin(), hr.end(), a.row_end) - hr.begin();
    }
    DGI_REQUIRE(a.ld_z >= p.HF + 2 * a.heads, DGI_ERR_INVALID_ARG, "gat: ld_z too small for [z|el|er]");
    const bool fast = ((uintptr_t)a.Zx % 16 == 0) && (a.ld_z % 4 == 0) && (a.heads == 1 || a.head_dim % 4 == 0) && p.HF <= 256;
    return g->itype == DGI_I64 ? dispatch<int64_t>(p, fast, stream) : dispatch<int32_t>(p, fast, stream);
}

}  // namespace dgi
