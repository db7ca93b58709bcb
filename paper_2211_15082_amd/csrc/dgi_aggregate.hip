// One-hop CSR gather + aggregation (the per-batch "gather N_v and H^{l-1}(N_v), run layer l" steps of
// Algorithm 2, for the SUM / MEAN / GCN-normalised aggregators of Eq. 1).
//
// Mapping to CDNA4: one 64-lane wavefront per destination row.  A source row is fetched with 16-byte
// loads; G = lanes needed to cover one row (4..64), so one load instruction of the wavefront fetches
// 64/G different neighbours.  The row's neighbour ids are loaded 64 at a time, coalesced, one per lane,
// and handed to the lane groups with cross-lane reads; UNROLL independent row loads are in flight per
// lane before the first is consumed.  Each lane keeps fp32 partial sums of its 16-byte column slice;
// the 64/G groups are combined with xor-shuffles at the end of the row.  The summation order of a row
// depends only on (G, UNROLL), never on the batch the row is in.
//
// Power-law skew: rows longer than kHubDegree are skipped by the row kernel and cut into kHubChunk-edge
// chunks, one wavefront each (hub kernel), writing fp32 partial rows; a reduce kernel adds the partials
// of a row in chunk order and applies the epilogue.  No floating-point atomics anywhere.
#include <algorithm>
#include <cstdlib>

#include "dgi_device.h"
#include "dgi_internal.h"

namespace dgi {
namespace {

// Row loads in flight per lane.  Measured: 8 instead of 4 for 32-lane groups takes 10 % off the 400-byte-row gather
// of the 100 -> 256 GCN layer (16 costs a wavefront of occupancy and gives it back); 8 instead of 4 for the
// group-per-row gather costs two wavefronts of occupancy and 12 % on the 111 M-node bf16 graph.
#ifndef DGI_UNROLL_GROUPED
#define DGI_UNROLL_GROUPED 4
#endif
#ifndef DGI_UNROLL_G32
#define DGI_UNROLL_G32 8
#endif
#ifndef DGI_UNROLL_WIDE
#define DGI_UNROLL_WIDE 8        // row loads in flight per lane when a whole wavefront covers one source row
#endif
#ifndef DGI_FUSED_RING_STEPS
#define DGI_FUSED_RING_STEPS 2   // K steps per batch of weight fragments in the fused kernel's transform phase
#endif
constexpr int kWaves = 4;        // wavefronts per workgroup
constexpr int kRowsPerWg = 16;   // destination rows per workgroup (wide rows)
// Narrow rows (G <= 16 lanes per source row): every lane group owns its own destination row, so a wavefront
// works on 64/G rows at once and a workgroup on 4 times that.
template <int G> constexpr int rows_per_wave() { return (64 / G) > 4 ? (64 / G) : 4; }
template <int G> constexpr int rows_per_wg() { return kWaves * rows_per_wave<G>(); }
constexpr int kGroupRowMaxDegree = 64;  // longer rows are gathered by the whole wavefront instead
constexpr int kXcds = 8;         // XCDs of MI355X; workgroup i is dispatched to XCD i % 8
constexpr int kXcdRun = 8;       // consecutive tiles handed to one XCD, so that neighbouring rows share an L2

struct AggParams {
    const void* indptr;
    const int32_t* indices;
    const float* rs_out;
    const float* rs_in;
    const void* S;
    int64_t ld_s;
    int width;
    void* out;
    void* out_lo;          // bf16 output only: receives the part of each value its bf16 rounding dropped (or null)
    int lo_bytes;          // ... as a second bf16 value (2) or as a byte in units of 2^-8 of the value's last place (1)
    int64_t ld_out;
    int64_t out_row0;
    int out_bf16;
    int out_vec_ok;
    int self_vec_ok;       // self rows can be read in 16-byte pieces
    const void* self;
    int64_t ld_self;
    const float* bias;
    int act;
    float act_slope;
    const float* out_scale;
    int64_t row_begin, row_end;
    int64_t n_tiles;
    int skip_hubs;
    // hub pass
    const int64_t* hub_rows;
    const int64_t* hub_chunk_ptr;
    int64_t hub_begin, hub_end;
    int64_t chunk0;
    float* partials;
    int wpad;
    int64_t n_chunks;    // hub chunks in the range
    int64_t hub_blocks;  // leading workgroups of the launch that work on hub chunks (multiple of 64)
    int hub_compact;     // hub reduce writes row (h - hub_begin) of `out` instead of row (v - out_row0)
};

// The fused layer kernel: gather description + the dense transform that consumes the aggregated tile.
struct FusedParams {
    AggParams a;           // S = H^{l-1}, width = K; out/self/bias/act unused
    const void* Wf;        // packed weights in MFMA fragment order: [column block][K step][lane][16 bytes]; K steps run over
                           // the self block (columns [0, K1p) of the row-order matrix) and then the neighbour block
    int64_t ldw;
    int K1p;
    int has_self;
    int N;
    const float* bias;
    int act;
    float act_slope;
    const float* out_scale;
    void* out;
    int64_t ld_out;
    int64_t out_row0;
    int out_bf16;
    const float* hub_agg;  // aggregated and scaled hub rows of the range, in hub order, fp32 [n_hubs x hub_ld]
    int64_t hub_ld;
    int lds_ld;            // elements per row of the LDS tile
    int self_lds;          // 0: self rows from global memory; 1: in the tile, 4 wavefronts; 2: in the tile, 8 wavefronts
};

template <typename T> struct Row;
template <> struct Row<float> {
    static constexpr int VEC = 4;
    using Raw = float4;
    static __device__ __forceinline__ Raw zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ void unpack(const Raw& r, float* f) { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
    static __device__ __forceinline__ float one(const float* p) { return *p; }
    // acc += row chunk if ok.  A masked-out chunk was loaded from another neighbour of the same destination row,
    // so weighting it with 0 cannot bring in a NaN the true sum does not already have.
    static __device__ __forceinline__ void add_masked(const Raw& r, bool ok, float* acc) {
        const float w = ok ? 1.f : 0.f;
        acc[0] = fmaf(w, r.x, acc[0]); acc[1] = fmaf(w, r.y, acc[1]);
        acc[2] = fmaf(w, r.z, acc[2]); acc[3] = fmaf(w, r.w, acc[3]);
    }
};
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
template <> struct Row<uint16_t> {
    static constexpr int VEC = 8;
    using Raw = uint4;
    static __device__ __forceinline__ Raw zero() { return make_uint4(0u, 0u, 0u, 0u); }
    static __device__ __forceinline__ void unpack(const Raw& r, float* f) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
    }
    static __device__ __forceinline__ float one(const uint16_t* p) { return bf16_to_float(*p); }
    // acc += row chunk if ok, two fp32 accumulators per 32-bit word with v_dot2_f32_bf16 against (1,0) / (0,1):
    // no unpacking, and the mask costs two selects per chunk instead of one per element.
    // The selectors are kept in registers (the empty asm hides their value from the optimiser): folded into an
    // inline constant, the (1,0) pair did not select the low half on gfx950.
    static __device__ __forceinline__ void add_masked(const Raw& r, bool ok, float* acc) {
        uint32_t one_lo = 0x00003f80u, one_hi = 0x3f800000u;
        asm volatile("" : "+v"(one_lo), "+v"(one_hi));
        const uint32_t sel_lo = ok ? one_lo : 0u, sel_hi = ok ? one_hi : 0u;
        bf16x2_t lo, hi;
        __builtin_memcpy(&lo, &sel_lo, 4);
        __builtin_memcpy(&hi, &sel_hi, 4);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            bf16x2_t v;
            __builtin_memcpy(&v, &w[i], 4);
            acc[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(v, lo, acc[2 * i], false);
            acc[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(v, hi, acc[2 * i + 1], false);
        }
    }
};

// Tile handled by workgroup `bid`: runs of kXcdRun consecutive tiles go to the same XCD.
__device__ __forceinline__ int64_t xcd_tile(int64_t bid) {
    constexpr int64_t group = (int64_t)kXcds * kXcdRun;
    const int64_t base = bid / group * group;
    const int64_t r = bid - base;
    return base + (r % kXcds) * kXcdRun + r / kXcds;
}

// Adds  sum_{e in [eb,ee)} coef(indices[e]) * S[indices[e], col0 + gl*VEC .. +VEC)  into acc (per lane;
// the 64/G lane groups hold disjoint subsets of the edges).  When `preloaded` is set, `first_my` holds
// indices[eb + lane] (0 beyond the row) fetched earlier by the caller.
struct NoOp {
    __device__ __forceinline__ void operator()() const {}
};

// `between` is called once per block of UNROLL row loads, right after they have been issued and before their
// data is needed: independent work placed there overlaps the memory latency (wave-uniform control flow only).
template <typename T, int G, int MODE, int UNROLL, typename Between = NoOp>
__device__ __forceinline__ void gather_range(const AggParams& p, int64_t eb, int64_t ee, int lane, int col0,
                                             float (&acc)[Row<T>::VEC], bool preloaded = false, int first_my = 0,
                                             Between&& between = Between()) {
    constexpr int VEC = Row<T>::VEC;
    constexpr int NSUB = 64 / G;
    using Raw = typename Row<T>::Raw;
    const int sub = lane / G, gl = lane % G;
    const int col = col0 + gl * VEC;
    const bool col_ok = col < p.width;
    const T* sbase = static_cast<const T*>(p.S) + col;
    for (int64_t e0 = eb; e0 < ee; e0 += 64) {
        const int64_t left = ee - e0;
        const int cnt = left < 64 ? (int)left : 64;
        int my;
        if (preloaded && e0 == eb) my = first_my;
        else my = lane < cnt ? p.indices[e0 + lane] : 0;
        float myc = 1.f;
        if (MODE == MODE_GCN) myc = lane < cnt ? p.rs_out[my] : 0.f;
        for (int j = 0; j < cnt; j += NSUB * UNROLL) {
            Raw raw[UNROLL];
            float c[UNROLL];
            int64_t off[UNROLL];
            bool ok[UNROLL];
            int ks[UNROLL];
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                const int k = j + t * NSUB + sub;
                ok[t] = k < cnt;
                ks[t] = ok[t] ? k : 0;
                const int u = (G == 64) ? __builtin_amdgcn_readlane(my, ks[t]) : __shfl(my, ks[t], 64);
                off[t] = (int64_t)u * p.ld_s;
            }
            if (col_ok) {
#pragma unroll
                for (int t = 0; t < UNROLL; ++t) raw[t] = *reinterpret_cast<const Raw*>(sbase + off[t]);
            } else {
#pragma unroll
                for (int t = 0; t < UNROLL; ++t) raw[t] = Row<T>::zero();
            }
            between();
            // the per-source coefficients are handed out only now, so the row loads above do not wait for them
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                if (MODE == MODE_GCN)
                    c[t] = (G == 64) ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(myc), ks[t])) : __shfl(myc, ks[t], 64);
                else
                    c[t] = 1.f;
            }
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                if (MODE == MODE_GCN) {
                    float f[VEC];
                    Row<T>::unpack(raw[t], f);
                    const float w = ok[t] ? c[t] : 0.f;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, f[i], acc[i]);
                } else {
                    Row<T>::add_masked(raw[t], ok[t], acc);
                }
            }
        }
    }
}

template <int G, int VEC>
__device__ __forceinline__ void combine_groups(float (&acc)[VEC]) {
#pragma unroll
    for (int off = G; off < 64; off <<= 1) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
    }
}

// What rounding `val` to the bf16 value `hi` dropped, in units of 2^-8 of hi's last place, as a byte with offset 128:
// val = hi + (byte - 128) * 2^(e - 15) up to 2^(e - 16), e = hi's exponent (the remainder is at most half a last place
// = 128 units; 128 itself is stored as 127).  hi + byte carry 16 significant bits in 3 bytes.  Zero, denormal-range
// (e < -112) and non-finite hi get the byte of a zero remainder.
__device__ __forceinline__ uint32_t remainder_byte(float val, uint32_t hi) {
    const uint32_t eb = (hi >> 7) & 0xffu;
    if (eb < 15u || eb == 255u) return 128u;
    const float scale = __uint_as_float((269u - eb) << 23);   // 2^(15 - e)
    float q = rintf((val - bf16_to_float(hi)) * scale);
    q = fminf(fmaxf(q, -127.f), 127.f);
    return (uint32_t)((int)q + 128);
}

// scale, self addend, bias, activation, store of one output element
template <typename T>
__device__ __forceinline__ void finish_store(const AggParams& p, int64_t v, int64_t out_row, int c, float sum, float scale) {
    float val = sum * scale;
    if (p.self) val += Row<T>::one(static_cast<const T*>(p.self) + v * p.ld_self + c);
    if (p.bias) val += p.bias[c];
    val = activate(val, p.act, p.act_slope);
    if (p.out_scale) val *= p.out_scale[v];
    const int64_t o = out_row * p.ld_out + c;
    if (p.out_bf16) {
        const uint16_t hi = float_to_bf16(val);
        static_cast<uint16_t*>(p.out)[o] = hi;
        if (p.out_lo) {
            if (p.lo_bytes == 1) static_cast<uint8_t*>(p.out_lo)[o] = (uint8_t)remainder_byte(val, hi);
            else static_cast<uint16_t*>(p.out_lo)[o] = float_to_bf16(val - bf16_to_float(hi));
        }
    } else {
        static_cast<float*>(p.out)[o] = val;
    }
}

// The same epilogue for the VEC consecutive elements a lane owns (columns col .. col+VEC-1 of row v), stored as one
// 16-byte piece when the output layout allows it: element-wise 2- or 4-byte stores of a row reach HBM as partial
// lines (measured: three times the bytes of the output matrix).  Arithmetic per element is that of finish_store.
template <typename T>
__device__ __forceinline__ void store_chunk(const AggParams& p, int64_t v, int64_t out_row, int col, const float* sum, float scale) {
    constexpr int VEC = Row<T>::VEC;
    if (!(p.out_vec_ok && col + VEC <= p.width)) {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            if (col + i < p.width) finish_store<T>(p, v, out_row, col + i, sum[i], scale);
        return;
    }
    float val[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) val[i] = sum[i] * scale;
    if (p.self) {
        const T* srow = static_cast<const T*>(p.self) + v * p.ld_self + col;
        float f[VEC];
        if (p.self_vec_ok) {
            Row<T>::unpack(*reinterpret_cast<const typename Row<T>::Raw*>(srow), f);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) f[i] = Row<T>::one(srow + i);
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) val[i] += f[i];
    }
    if (p.bias) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) val[i] += p.bias[col + i];
    }
    const float os = p.out_scale ? p.out_scale[v] : 1.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        val[i] = activate(val[i], p.act, p.act_slope);
        if (p.out_scale) val[i] *= os;
    }
    const int64_t o = out_row * p.ld_out + col;
    if (p.out_bf16) {
        uint32_t w[(VEC + 1) / 2];
#pragma unroll
        for (int i = 0; i < VEC / 2; ++i) w[i] = (uint32_t)float_to_bf16(val[2 * i]) | ((uint32_t)float_to_bf16(val[2 * i + 1]) << 16);
        // VEC bf16 values are 8 bytes (fp32 sources) or 16 bytes (bf16 sources)
        if constexpr (VEC == 4) *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + o) = make_uint2(w[0], w[1]);
        else *reinterpret_cast<uint4*>(static_cast<uint16_t*>(p.out) + o) = make_uint4(w[0], w[1], w[(VEC > 4) ? 2 : 0], w[(VEC > 4) ? 3 : 0]);
        if (p.out_lo && p.lo_bytes == 1) {  // what the rounding above dropped, one byte per element
            uint32_t q[(VEC + 3) / 4];
#pragma unroll
            for (int i = 0; i < VEC / 4; ++i) {
                q[i] = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = 4 * i + j;
                    const uint32_t hi = (e & 1) ? (w[e / 2] >> 16) : (w[e / 2] & 0xffffu);
                    q[i] |= remainder_byte(val[e], hi) << (8 * j);
                }
            }
            if constexpr (VEC == 4) *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(p.out_lo) + o) = q[0];
            else *reinterpret_cast<uint2*>(static_cast<uint8_t*>(p.out_lo) + o) = make_uint2(q[0], q[(VEC > 4) ? 1 : 0]);
        } else if (p.out_lo) {  // ... or as a second bf16 value per element
            uint32_t l[(VEC + 1) / 2];
#pragma unroll
            for (int i = 0; i < VEC / 2; ++i) {
                const float r0 = val[2 * i] - __uint_as_float(w[i] << 16), r1 = val[2 * i + 1] - __uint_as_float(w[i] & 0xffff0000u);
                l[i] = (uint32_t)float_to_bf16(r0) | ((uint32_t)float_to_bf16(r1) << 16);
            }
            if constexpr (VEC == 4) *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out_lo) + o) = make_uint2(l[0], l[1]);
            else *reinterpret_cast<uint4*>(static_cast<uint16_t*>(p.out_lo) + o) = make_uint4(l[0], l[1], l[(VEC > 4) ? 2 : 0], l[(VEC > 4) ? 3 : 0]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) *reinterpret_cast<float4*>(static_cast<float*>(p.out) + o + i) = make_float4(val[i], val[i + 1], val[i + 2], val[i + 3]);
    }
}

template <int MODE, typename IdxT>
__device__ __forceinline__ float row_scale(const AggParams& p, int64_t v, IdxT deg) {
    if (MODE == MODE_MEAN) return deg > 0 ? 1.0f / (float)deg : 0.f;
    if (MODE == MODE_GCN || MODE == MODE_GCN_PRE) return p.rs_in[v];
    return 1.f;
}

template <typename IdxT>
__device__ __forceinline__ IdxT bcast_lane(IdxT x, int src) {
    if (sizeof(IdxT) == 8) {
        const uint64_t u = (uint64_t)x;
        const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)u, src, 64), hi = (uint32_t)__shfl((int)(uint32_t)(u >> 32), src, 64);
        return (IdxT)(((uint64_t)hi << 32) | lo);
    }
    return (IdxT)__shfl((int)x, src, 64);
}

// Narrow rows: one lane group per destination row.  The 64/G groups of a wavefront walk their own neighbour
// lists side by side (a group whose list is exhausted idles with its loads masked off), each lane keeps the
// whole sum of its column slice, and no cross-group reduction or per-row bookkeeping by all 64 lanes is
// needed: for low-degree graphs this kernel is bound by instruction issue, not by memory, and this mapping
// issues about a quarter of the vector instructions per row.  Rows longer than kGroupRowMaxDegree are left to
// the cooperative path below (whole wavefront per row), so one long list does not stall three short ones.
template <typename T, typename IdxT, int G, int MODE>
__device__ __forceinline__ void rows_tile_grouped(const AggParams& p, int64_t bid) {
    constexpr int VEC = Row<T>::VEC;
    constexpr int NSUB = 64 / G;
    constexpr int RPW = rows_per_wave<G>();
    constexpr int UNROLL = DGI_UNROLL_GROUPED;
    static_assert(RPW == NSUB, "one row per lane group");
    using Raw = typename Row<T>::Raw;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = xcd_tile(bid);
    if (tile >= p.n_tiles) return;
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const int sub = lane / G, gl = lane % G;
    const int64_t vw = p.row_begin + tile * rows_per_wg<G>() + wave * RPW;
    if (vw >= p.row_end) return;
    IdxT ipv = 0;
    if (lane <= RPW) {
        const int64_t i = vw + lane;
        ipv = indptr[i < p.row_end ? i : p.row_end];
    }
    // ---- phase A: every group gathers its own (short) row ----------------------------------------------------
    const int64_t eb = (int64_t)bcast_lane<IdxT>(ipv, sub), ee = (int64_t)bcast_lane<IdxT>(ipv, sub + 1);
    const int64_t v = vw + sub;
    const int64_t deg = ee - eb;  // 0 for rows past the range
    const bool mine = v < p.row_end && deg <= kGroupRowMaxDegree;
    const int dg = mine ? (int)deg : 0;
    const int col = gl * VEC;
    const bool col_ok = col < p.width;
    const T* sbase = static_cast<const T*>(p.S) + col;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    for (int base = 0; __any(base < dg); base += G) {
        const int left = dg - base;  // edges of this group's row still to do (may be <= 0)
        const int my = gl < left ? p.indices[eb + base + gl] : 0;
        float myc = 1.f;
        if (MODE == MODE_GCN) myc = gl < left ? p.rs_out[my] : 0.f;
        for (int j = 0; j < G && __any(j < left); j += UNROLL) {
            Raw raw[UNROLL];
            float c[UNROLL];
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                const int k = j + t;
                const bool ok = k < left && col_ok;
                const int u = __shfl(my, k, G);
                if (MODE == MODE_GCN) c[t] = __shfl(myc, k, G);
                raw[t] = ok ? *reinterpret_cast<const Raw*>(sbase + (int64_t)u * p.ld_s) : Row<T>::zero();
            }
#pragma unroll
            for (int t = 0; t < UNROLL; ++t) {
                if (MODE == MODE_GCN) {
                    float f[VEC];
                    Row<T>::unpack(raw[t], f);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[i] = fmaf(c[t], f[i], acc[i]);
                } else {
                    Row<T>::add_masked(raw[t], true, acc);  // masked-off chunks are zero already
                }
            }
        }
    }
    if (mine && col_ok) store_chunk<T>(p, v, v - p.out_row0, col, acc, row_scale<MODE, int64_t>(p, v, deg));
    // ---- phase B: the wavefront's long rows, all lane groups on one row at a time ------------------------------
    IdxT bound[RPW + 1];
#pragma unroll
    for (int i = 0; i <= RPW; ++i) bound[i] = bcast_lane<IdxT>(ipv, i);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int64_t vr = vw + r;
        if (vr >= p.row_end) break;
        const IdxT rb = bound[r], re = bound[r + 1];
        const IdxT rdeg = re - rb;
        if (rdeg <= (IdxT)kGroupRowMaxDegree) continue;
        if (p.skip_hubs && rdeg > (IdxT)kHubDegree) continue;
        const float scale = row_scale<MODE, IdxT>(p, vr, rdeg);
        float a2[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) a2[i] = 0.f;
        gather_range<T, G, MODE, UNROLL>(p, (int64_t)rb, (int64_t)re, lane, 0, a2);
        combine_groups<G, VEC>(a2);
        if (sub == 0 && col_ok) store_chunk<T>(p, vr, vr - p.out_row0, col, a2, scale);
    }
}

// Workgroup `bid` of the row part: kRowsPerWg destination rows; each wavefront owns kRowsPerWg / kWaves
// consecutive rows, reads their indptr entries with one load, and fetches the first 64 neighbour ids of the
// next row while it gathers the current one (a row costs one dependent memory latency instead of three).
template <typename T, typename IdxT, int G, int MODE>
__device__ __forceinline__ void rows_tile(const AggParams& p, int64_t bid) {
    constexpr int VEC = Row<T>::VEC;
    constexpr int UNROLL = (G == 64) ? DGI_UNROLL_WIDE : (G == 32 ? DGI_UNROLL_G32 : 4);
    constexpr int RPW = kRowsPerWg / kWaves;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = xcd_tile(bid);
    if (tile >= p.n_tiles) return;
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const int sub = lane / G, gl = lane % G;
    const int64_t vw = p.row_begin + tile * kRowsPerWg + wave * RPW;
    if (vw >= p.row_end) return;
    IdxT ipv = 0;
    if (lane <= RPW) {
        const int64_t i = vw + lane;
        ipv = indptr[i < p.row_end ? i : p.row_end];  // rows past the range read as empty
    }
    IdxT bound[RPW + 1];
#pragma unroll
    for (int i = 0; i <= RPW; ++i) bound[i] = bcast_lane<IdxT>(ipv, i);
    int nxt = (int64_t)lane < (int64_t)(bound[1] - bound[0]) ? p.indices[(int64_t)bound[0] + lane] : 0;
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int64_t v = vw + r;
        if (v >= p.row_end) break;
        const IdxT eb = bound[r], ee = bound[r + 1];
        const IdxT deg = ee - eb;
        const int cur = nxt;
        if (r + 1 < RPW) nxt = (int64_t)lane < (int64_t)(bound[r + 2 <= RPW ? r + 2 : RPW] - ee) ? p.indices[(int64_t)ee + lane] : 0;
        if (p.skip_hubs && deg > (IdxT)kHubDegree) continue;
        const float scale = row_scale<MODE, IdxT>(p, v, deg);
        for (int col0 = 0; col0 < p.width; col0 += G * VEC) {
            float acc[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
            gather_range<T, G, MODE, UNROLL>(p, (int64_t)eb, (int64_t)ee, lane, col0, acc, true, cur);
            combine_groups<G, VEC>(acc);
            const int c = col0 + gl * VEC;
            if (sub == 0 && c < p.width) store_chunk<T>(p, v, v - p.out_row0, c, acc, scale);
        }
    }
}

// One wavefront per kHubChunk-edge chunk of a hub row: fp32 partial row, no scale.
template <typename T, typename IdxT, int G, int MODE>
__device__ __forceinline__ void hub_chunk(const AggParams& p, int64_t block) {
    constexpr int VEC = Row<T>::VEC;
    constexpr int UNROLL = (G == 64) ? DGI_UNROLL_WIDE : (G == 32 ? DGI_UNROLL_G32 : 4);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t qi = block * kWaves + wave;
    if (qi >= p.n_chunks) return;
    const int64_t q = p.chunk0 + qi;
    int64_t lo = p.hub_begin, hi = p.hub_end;  // largest h in [lo,hi) with hub_chunk_ptr[h] <= q
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (p.hub_chunk_ptr[mid] <= q) lo = mid; else hi = mid;
    }
    const int64_t v = p.hub_rows[lo];
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const int64_t rb = (int64_t)indptr[v], re = (int64_t)indptr[v + 1];
    const int64_t eb = rb + (q - p.hub_chunk_ptr[lo]) * kHubChunk;
    const int64_t ee = eb + kHubChunk < re ? eb + kHubChunk : re;
    const int sub = lane / G, gl = lane % G;
    for (int col0 = 0; col0 < p.width; col0 += G * VEC) {
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
        gather_range<T, G, MODE, UNROLL>(p, eb, ee, lane, col0, acc);
        combine_groups<G, VEC>(acc);
        const int c = col0 + gl * VEC;
        if (sub == 0 && c < p.width) {
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (c + i < p.wpad) p.partials[qi * p.wpad + c + i] = acc[i];
        }
    }
}

// The aggregation launch: the first hub_blocks workgroups take the hub chunks (the longest work items go
// first), the rest take row tiles.
template <typename T, typename IdxT, int G, int MODE>
__global__ __launch_bounds__(kWaves * 64) void agg_kernel(AggParams p) {
    const int64_t bid = blockIdx.x;
    if (bid < p.hub_blocks) hub_chunk<T, IdxT, G, MODE>(p, bid);
    else if (G <= 16) rows_tile_grouped<T, IdxT, (G <= 16 ? G : 16), MODE>(p, bid - p.hub_blocks);
    else rows_tile<T, IdxT, G, MODE>(p, bid - p.hub_blocks);
}


typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
constexpr int kFusedRows = 32;  // destination rows per workgroup = one MFMA row block

template <typename T>
__device__ __forceinline__ uint4 pack_row_chunk(const float* f) {  // VEC floats -> 16 bytes of T
    if (sizeof(T) == 4) return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    return make_uint4((uint32_t)float_to_bf16(f[0]) | ((uint32_t)float_to_bf16(f[1]) << 16),
                      (uint32_t)float_to_bf16(f[2]) | ((uint32_t)float_to_bf16(f[3]) << 16),
                      (uint32_t)float_to_bf16(f[4 % Row<T>::VEC]) | ((uint32_t)float_to_bf16(f[5 % Row<T>::VEC]) << 16),
                      (uint32_t)float_to_bf16(f[6 % Row<T>::VEC]) | ((uint32_t)float_to_bf16(f[7 % Row<T>::VEC]) << 16));
}

// The part of a row chunk that its bf16 rounding dropped (bf16 tiles only): f - float(bf16(f)), again as bf16.
__device__ __forceinline__ uint4 pack_row_chunk_lo(const float* f) {
    float r[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = f[i] - bf16_to_float(float_to_bf16(f[i]));
    return pack_row_chunk<uint16_t>(r);
}

// Aggregation fused with the layer's dense transform (aggregate-first layers).  A workgroup of W wavefronts
// owns 32 destination rows.  Phase 1: the wavefronts gather and aggregate 32/W rows each exactly as the
// stand-alone kernel does, but deposit the scaled result in an LDS tile (32 x K).  Phase 2: the tile is the
// A operand of MFMA, B comes from the packed weight through L2, each wavefront owns every W-th 32-column
// block; bias, activation and the output conversion happen in registers.  The aggregated matrix never
// exists in HBM.  Hub rows arrive pre-aggregated (fp32) from the two-stage hub pass that runs before this
// launch.  The rows' own features (GraphSAGE) are a second A block: with SL they are copied into the tile
// (LDS row = [h_v | m_v]) by coalesced loads before the gather starts, so phase 2 reads both blocks from
// LDS; without SL they are read from global memory straight into fragment layout (smaller tile, but every
// column block re-reads them with 32 cache lines per load instruction).
// bf16 tiles hold m_v as two bf16 values per element, the rounded value and what the rounding dropped (LDS row =
// [h_v |] m_hi | m_lo), and both blocks are multiplied with the neighbour weights: the fp32 accumulation of the
// gather is not cut to 8 bits before the transform (two bf16 MFMAs cost a tenth of one fp32 MFMA pass).
template <typename T, typename IdxT, int G, int MODE, int W, bool SL>
__global__ __launch_bounds__(W * 64) __attribute__((amdgpu_waves_per_eu(W == 8 ? 4 : 1)))  // 8-wavefront form: two workgroups per CU
void fused_layer_kernel(FusedParams fp) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T* tile = reinterpret_cast<T*>(lds_raw);
    const AggParams& p = fp.a;
    constexpr int VEC = Row<T>::VEC;  // elements per 16 bytes
    constexpr int UNROLL = (G == 64) ? DGI_UNROLL_WIDE : (G == 32 ? DGI_UNROLL_G32 : 4);
    constexpr int RPW = kFusedRows / W;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile_id = xcd_tile(blockIdx.x);
    if (tile_id >= p.n_tiles) return;  // whole workgroup leaves together
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const int sub = lane / G, gl = lane % G;
    const int64_t vt = p.row_begin + tile_id * kFusedRows;
    const int64_t vw = vt + wave * RPW;
    const int K = p.width;
    const int Kp = (K + 2 * VEC - 1) / (2 * VEC) * (2 * VEC);
    const int chunks = Kp / VEC;
    const int acol = SL ? Kp : 0;  // column of the aggregated block inside an LDS row
    constexpr bool HL = sizeof(T) == 2;  // a second block of Kp columns right after it holds the rounding remainders

    if (SL) {  // the rows' own features: [0, Kp) of every LDS row, zero past K and past the row range
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            const int64_t v = vw + r;
            T* trow = tile + (wave * RPW + r) * fp.lds_ld;
            const T* srow = static_cast<const T*>(p.S) + (v < p.row_end ? v : p.row_begin) * p.ld_s;
            for (int ch = lane; ch < chunks; ch += 64)
                *reinterpret_cast<uint4*>(trow + ch * VEC) =
                    (v < p.row_end && ch * VEC < K) ? *reinterpret_cast<const uint4*>(srow + ch * VEC) : make_uint4(0u, 0u, 0u, 0u);
        }
    }

    // MFMA fragment layout: lane = (row or column lane % 32, K half lane / 32), 16 bytes of K per lane and step
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int nblk = (fp.N + 31) / 32;
    const int ksteps = Kp / (2 * VEC);
    const T* a_lds = tile + lrow * fp.lds_ld + lhalf * VEC;
    auto mma = [&](floatx16_t& acc, const uint4& a, const uint4& b) {
        if (sizeof(T) == 4) {
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
        } else {
            bf16x8_t av, bv;
            __builtin_memcpy(&av, &a, 16);
            __builtin_memcpy(&bv, &b, 16);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
        }
    };
    // Interleaving (8-wavefront form): the transform of the rows' own features does not depend on the gather, so
    // each wavefront works through it for its first column block in the shadow of its own row loads: a few MFMA
    // steps after every block of loads, with the weight fragments of the next steps fetched one block ahead (they
    // must be issued before the row loads that follow, or waiting for them would wait for those loads too).
    constexpr bool IL = SL && W == 8;
    constexpr int UQ = (sizeof(T) == 4 && sizeof(IdxT) == 4) ? 4 : 2;  // what the register budget of two workgroups per CU allows
    floatx16_t acc0;
    uint4 bq[UQ];
    int ksq = 0;
    const bool own_blk = IL && wave < nblk;
    // B operand of column block cb, K step ks: 64 consecutive 16-byte pieces, one per lane
    const int64_t ks_tot = fp.ldw / (2 * VEC);
    const T* wf_lane = static_cast<const T*>(fp.Wf) + lane * VEC;
    const T* w0 = wf_lane + (int64_t)wave * ks_tot * 64 * VEC;
    auto fetch_bq = [&]() {
#pragma unroll
        for (int u = 0; u < UQ; ++u)
            bq[u] = (own_blk && ksq + u < ksteps) ? *reinterpret_cast<const uint4*>(w0 + (int64_t)(ksq + u) * 64 * VEC) : make_uint4(0u, 0u, 0u, 0u);
    };
    auto self_step = [&]() {
        if (!own_blk || ksq >= ksteps) return;
        uint4 a[UQ];
#pragma unroll
        for (int u = 0; u < UQ; ++u)
            a[u] = ksq + u < ksteps ? *reinterpret_cast<const uint4*>(a_lds + (ksq + u) * 2 * VEC) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int u = 0; u < UQ; ++u) mma(acc0, a[u], bq[u]);
        ksq += UQ;
        fetch_bq();
    };
    if (IL) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc0[i] = 0.f;
        __syncthreads();  // every row's own features are in the tile
        fetch_bq();
    }

    // ---- phase 1: aggregate 32/W rows per wavefront into the tile -------------------------------------
    IdxT ipv = 0;
    if (lane <= RPW) {
        const int64_t i = vw + lane;
        ipv = indptr[i < p.row_end ? i : p.row_end];
    }
    IdxT bound[RPW + 1];
#pragma unroll
    for (int i = 0; i <= RPW; ++i) bound[i] = bcast_lane<IdxT>(ipv, i);
    int nxt = (int64_t)lane < (int64_t)(bound[1] - bound[0]) ? p.indices[(int64_t)bound[0] + lane] : 0;
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int64_t v = vw + r;
        T* trow = tile + (wave * RPW + r) * fp.lds_ld + acol;
        const IdxT eb = bound[r], ee = bound[r + 1];
        const IdxT deg = ee - eb;
        const int cur = nxt;
        if (r + 1 < RPW) nxt = (int64_t)lane < (int64_t)(bound[r + 2 <= RPW ? r + 2 : RPW] - ee) ? p.indices[(int64_t)ee + lane] : 0;
        if (v >= p.row_end) {  // rows past the range: an all-zero A row
            for (int ch = lane; ch < (HL ? 2 : 1) * chunks; ch += 64) *reinterpret_cast<uint4*>(trow + ch * VEC) = make_uint4(0u, 0u, 0u, 0u);
            continue;
        }
        T* arow = trow;
        if (p.skip_hubs && deg > (IdxT)kHubDegree) {  // pre-aggregated by the hub pass
            int64_t lo = p.hub_begin, hi = p.hub_end;
            while (hi - lo > 1) {
                const int64_t mid = (lo + hi) >> 1;
                if (p.hub_rows[mid] <= v) lo = mid; else hi = mid;
            }
            const float* src = fp.hub_agg + (lo - p.hub_begin) * fp.hub_ld;
            for (int ch = lane; ch < chunks; ch += 64) {
                float f[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) f[i] = ch * VEC + i < K ? src[ch * VEC + i] : 0.f;
                *reinterpret_cast<uint4*>(arow + ch * VEC) = pack_row_chunk<T>(f);
                if constexpr (HL) *reinterpret_cast<uint4*>(arow + Kp + ch * VEC) = pack_row_chunk_lo(f);
            }
            continue;
        }
        const float scale = row_scale<MODE, IdxT>(p, v, deg);
        for (int col0 = 0; col0 < Kp; col0 += G * VEC) {
            float acc[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
            if constexpr (IL) gather_range<T, G, MODE, UNROLL>(p, (int64_t)eb, (int64_t)ee, lane, col0, acc, true, cur, self_step);
            else gather_range<T, G, MODE, UNROLL>(p, (int64_t)eb, (int64_t)ee, lane, col0, acc, true, cur);
            combine_groups<G, VEC>(acc);
            const int c = col0 + gl * VEC;
            if (sub == 0 && c < Kp) {  // columns in [K, Kp) hold zeros (no lane gathered them)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] *= scale;
                *reinterpret_cast<uint4*>(arow + c) = pack_row_chunk<T>(acc);
                if constexpr (HL) *reinterpret_cast<uint4*>(arow + Kp + c) = pack_row_chunk_lo(acc);
            }
        }
    }
    if (IL) {
        while (own_blk && ksq < ksteps) self_step();  // what the gather did not cover
    }
    __syncthreads();

    // ---- phase 2: out[32 x N] = act([h_v | tile] . Wt^T + bias) on the matrix cores ------------------------
    // A operand in MFMA fragment layout (lane = row, 16 bytes of K) from the LDS tile (and from global memory
    // for the rows' own features without SL).  B operand: the packed weight through L2.  A wavefront owns
    // column blocks wave, wave+W, ... one at a time (two per sweep would halve the A reads but costs
    // registers, i.e. gather occupancy: measured slower).
    const int64_t vrow = vt + lrow;
    const T* a_self = static_cast<const T*>(p.S) + (vrow < p.row_end ? vrow : p.row_begin) * p.ld_s + lhalf * VEC;
    const bool self_row = fp.has_self && vrow < p.row_end;
    for (int cb = wave; cb < nblk; cb += W) {
        const int n = cb * 32 + lrow;
        const T* w = wf_lane + (int64_t)cb * ks_tot * 64 * VEC;
        floatx16_t acc;
        const bool resumed = IL && cb == wave;  // its own-feature half was accumulated during the gather
        if (resumed) {
            acc = acc0;
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        }
        // All loops below are free of branches around loads: a step past the end re-reads the last one (a valid address)
        // and multiplies an A fragment masked to zero.  A load inside a branch, even a wave-uniform one, makes the
        // compiler wait for every outstanding load at the next use (it can no longer count the younger ones), which
        // turned the three-batch rotation below into one L2 round trip per batch.
        auto masked = [](uint4 v, bool keep) {
            const uint32_t m = keep ? 0xffffffffu : 0u;
            return make_uint4(v.x & m, v.y & m, v.z & m, v.w & m);
        };
        constexpr int U = 4;
        if (!SL && fp.has_self) {  // K block of the rows' own features: columns [0, Kp) of the packed weight
            for (int ks = 0; ks < ksteps; ks += U) {
                uint4 a[U], b[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int kc = ks + u < ksteps ? ks + u : ksteps - 1;
                    const int k = kc * 2 * VEC;  // + lhalf * VEC is inside the base pointers
                    const bool in = ks + u < ksteps && self_row && k + lhalf * VEC < K;
                    a[u] = masked(*reinterpret_cast<const uint4*>(a_self + (k + lhalf * VEC < K ? k : 0)), in);
                    b[u] = *reinterpret_cast<const uint4*>(w + (int64_t)kc * 64 * VEC);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) mma(acc, a[u], b[u]);
            }
        }
        // K block of the aggregated neighbourhood: columns [K1p, K1p + Kp) of the packed weight; with SL one
        // loop over the whole LDS row [h_v | m_v] against columns [0, 2 Kp) (the host checks K1p == Kp)
        const int lsteps = SL ? 2 * ksteps : ksteps;
        const int wks = SL ? 0 : fp.K1p / (2 * VEC);  // first K step of the block in the fragment-order weight
        // The weight fragments come from L2 with a latency of a microsecond or more while other workgroups gather:
        // three batches of R steps rotate, two on their way while the third is in the matrix cores (R = 2 keeps the
        // registers of this phase below those of the gather phase, so the kernel's occupancy does not change).
        constexpr int R = DGI_FUSED_RING_STEPS;
        auto load_b = [&](uint4 (&b)[R], int ks) {
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int kc = ks + u < lsteps ? ks + u : lsteps - 1;
                b[u] = *reinterpret_cast<const uint4*>(w + (int64_t)(wks + kc) * 64 * VEC);
            }
        };
        auto batch = [&](const uint4 (&b)[R], int ks) {  // R steps from K step ks on
            uint4 a[R];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int kc = ks + u < lsteps ? ks + u : lsteps - 1;
                a[u] = masked(*reinterpret_cast<const uint4*>(a_lds + kc * 2 * VEC), ks + u < lsteps);
            }
#pragma unroll
            for (int u = 0; u < R; ++u) mma(acc, a[u], b[u]);
        };
        const int ks0 = resumed ? ksteps : 0;
        uint4 b0[R], b1[R], b2[R];
        // (the scheduling barriers keep the compiler from sinking each batch's loads down to their first use, which it
        // does to shorten register lifetimes and which would expose the whole latency again)
        load_b(b0, ks0);
        load_b(b1, ks0 + R);
        __builtin_amdgcn_sched_barrier(0);
        for (int ks = ks0; ks < lsteps; ks += 3 * R) {
            load_b(b2, ks + 2 * R);
            __builtin_amdgcn_sched_barrier(0);
            batch(b0, ks);
            __builtin_amdgcn_sched_barrier(0);
            load_b(b0, ks + 3 * R);
            __builtin_amdgcn_sched_barrier(0);
            batch(b1, ks + R);
            __builtin_amdgcn_sched_barrier(0);
            load_b(b1, ks + 4 * R);
            __builtin_amdgcn_sched_barrier(0);
            batch(b2, ks + 2 * R);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (HL) {  // the rounding remainders of m_v against the neighbour weights once more
            const T* a_lo = a_lds + acol + Kp;
            const int wn = fp.K1p / (2 * VEC);
            for (int ks = 0; ks < ksteps; ks += R) {
                uint4 a[R], b[R];
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const int kc = ks + u < ksteps ? ks + u : ksteps - 1;
                    b[u] = *reinterpret_cast<const uint4*>(w + (int64_t)(wn + kc) * 64 * VEC);
                    a[u] = masked(*reinterpret_cast<const uint4*>(a_lo + kc * 2 * VEC), ks + u < ksteps);
                }
#pragma unroll
                for (int u = 0; u < R; ++u) mma(acc, a[u], b[u]);
            }
        }
        if (n < fp.N) {
            const float bias = fp.bias ? fp.bias[n] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t v = vt + 8 * (r / 4) + 4 * lhalf + (r % 4);
                if (v >= p.row_end) continue;
                float val = activate(acc[r] + bias, fp.act, fp.act_slope);
                if (fp.out_scale) val *= fp.out_scale[v];
                store_element(fp.out, (v - fp.out_row0) * fp.ld_out + n, val, fp.out_bf16);
            }
        }
    }
}

// One wavefront per hub row: add its partial rows in chunk order, then the epilogue.
template <typename T, typename IdxT, int MODE>
__global__ __launch_bounds__(kWaves * 64) void agg_hub_reduce_kernel(AggParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t h = p.hub_begin + (int64_t)blockIdx.x * kWaves + wave;
    if (h >= p.hub_end) return;
    const int64_t v = p.hub_rows[h];
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const IdxT deg = indptr[v + 1] - indptr[v];
    const float scale = row_scale<MODE, IdxT>(p, v, deg);
    const int64_t q0 = p.hub_chunk_ptr[h] - p.chunk0, q1 = p.hub_chunk_ptr[h + 1] - p.chunk0;
    for (int c = lane; c < p.width; c += 64) {
        float s = 0.f;
        for (int64_t q = q0; q < q1; ++q) s += p.partials[q * p.wpad + c];
        finish_store<T>(p, v, p.hub_compact ? h - p.hub_begin : v - p.out_row0, c, s, scale);
    }
}

// Fallback for layouts without 16-byte aligned rows: one wavefront per row, one element per lane.
template <typename T, typename IdxT, int MODE>
__global__ __launch_bounds__(kWaves * 64) void agg_rows_generic_kernel(AggParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t v = p.row_begin + (int64_t)blockIdx.x * kWaves + wave;
    if (v >= p.row_end) return;
    const IdxT* indptr = static_cast<const IdxT*>(p.indptr);
    const int64_t eb = (int64_t)indptr[v], ee = (int64_t)indptr[v + 1];
    const float scale = row_scale<MODE, IdxT>(p, v, (IdxT)(ee - eb));
    const T* S = static_cast<const T*>(p.S);
    for (int c = lane; c < p.width; c += 64) {
        float s = 0.f;
        for (int64_t e = eb; e < ee; ++e) {
            const int64_t u = p.indices[e];
            const float w = (MODE == MODE_GCN) ? p.rs_out[u] : 1.f;
            s = fmaf(w, Row<T>::one(S + u * p.ld_s + c), s);
        }
        finish_store<T>(p, v, v - p.out_row0, c, s, scale);
    }
}

template <typename T, typename IdxT, int G, int MODE>
dgi_status_t launch_fast(const AggParams& p0, const dgi_graph* g, hipStream_t stream) {
    AggParams p = p0;
    const int64_t rows = p.row_end - p.row_begin;
    constexpr int kTileRows = G <= 16 ? rows_per_wg<(G <= 16 ? G : 16)>() : kRowsPerWg;
    p.n_tiles = (rows + kTileRows - 1) / kTileRows;
    constexpr int64_t kGroup = (int64_t)kXcds * kXcdRun;
    // hub rows inside the range
    const auto& hr = g->h_hub_rows;
    const int64_t hb = std::lower_bound(hr.begin(), hr.end(), p.row_begin) - hr.begin();
    const int64_t he = std::lower_bound(hr.begin(), hr.end(), p.row_end) - hr.begin();
    p.skip_hubs = (he > hb) ? 1 : 0;
    p.hub_begin = hb;
    p.hub_end = he;
    if (p.skip_hubs) {
        DGI_REQUIRE(p.partials != nullptr, DGI_ERR_INVALID_ARG, "hub rows in range but no partial buffer");
        p.chunk0 = g->h_hub_chunk_ptr[hb];
        p.n_chunks = g->h_hub_chunk_ptr[he] - p.chunk0;
        p.hub_blocks = round_up((p.n_chunks + kWaves - 1) / kWaves, kGroup);
    }
    const int64_t grid = p.hub_blocks + round_up(p.n_tiles, kGroup);
    DGI_REQUIRE(grid * kWaves * 64 < (int64_t)1 << 32, DGI_ERR_INVALID_ARG,
                "row range too large for one launch (2^32 threads): use smaller destination batches");
    hipLaunchKernelGGL((agg_kernel<T, IdxT, G, MODE>), dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

// Second stage for the hub rows of the range (no-op when there are none).
template <typename T, typename IdxT, int MODE>
dgi_status_t launch_hub_reduce(const AggParams& p0, const dgi_graph* g, hipStream_t stream) {
    AggParams p = p0;
    const auto& hr = g->h_hub_rows;
    const int64_t hb = std::lower_bound(hr.begin(), hr.end(), p.row_begin) - hr.begin();
    const int64_t he = std::lower_bound(hr.begin(), hr.end(), p.row_end) - hr.begin();
    if (he <= hb) return DGI_OK;
    p.hub_begin = hb;
    p.hub_end = he;
    p.chunk0 = g->h_hub_chunk_ptr[hb];
    hipLaunchKernelGGL((agg_hub_reduce_kernel<T, IdxT, MODE>), dim3((unsigned)((he - hb + kWaves - 1) / kWaves)),
                       dim3(kWaves * 64), 0, stream, p);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

template <typename T, typename IdxT, int MODE>
dgi_status_t dispatch_g(const AggParams& p, const dgi_graph* g, bool fast, int stage, hipStream_t stream) {
    if (stage == 1) return fast ? launch_hub_reduce<T, IdxT, MODE>(p, g, stream) : DGI_OK;
    if (!fast) {
        // 64 threads per row: keep each launch below 2^32 threads
        for (int64_t r0 = p.row_begin; r0 < p.row_end; r0 += (int64_t)1 << 25) {
            AggParams q = p;
            q.row_begin = r0;
            q.row_end = std::min(p.row_end, r0 + ((int64_t)1 << 25));
            const int64_t rows = q.row_end - q.row_begin;
            hipLaunchKernelGGL((agg_rows_generic_kernel<T, IdxT, MODE>), dim3((unsigned)((rows + kWaves - 1) / kWaves)),
                               dim3(kWaves * 64), 0, stream, q);
            DGI_HIP(hipGetLastError());
        }
        return DGI_OK;
    }
    const int lanes = (p.width + Row<T>::VEC - 1) / Row<T>::VEC;
    if (lanes <= 4) return launch_fast<T, IdxT, 4, MODE>(p, g, stream);
    if (lanes <= 8) return launch_fast<T, IdxT, 8, MODE>(p, g, stream);
    if (lanes <= 16) return launch_fast<T, IdxT, 16, MODE>(p, g, stream);
    if (lanes <= 32) return launch_fast<T, IdxT, 32, MODE>(p, g, stream);
    return launch_fast<T, IdxT, 64, MODE>(p, g, stream);
}

template <typename T, typename IdxT>
dgi_status_t dispatch_mode(const AggParams& p, const dgi_graph* g, int mode, bool fast, int stage, hipStream_t stream) {
    switch (mode) {
        case MODE_SUM: return dispatch_g<T, IdxT, MODE_SUM>(p, g, fast, stage, stream);
        case MODE_MEAN: return dispatch_g<T, IdxT, MODE_MEAN>(p, g, fast, stage, stream);
        case MODE_GCN: return dispatch_g<T, IdxT, MODE_GCN>(p, g, fast, stage, stream);
        case MODE_GCN_PRE: return dispatch_g<T, IdxT, MODE_GCN_PRE>(p, g, fast, stage, stream);
    }
    set_error("unknown aggregation mode %d", mode);
    return DGI_ERR_INVALID_ARG;
}

// ---- fused path: hub pre-pass (chunks + compact reduce into hub_agg), then the fused layer kernel -------
template <typename T, typename IdxT, int G, int MODE, int W, bool SL>
dgi_status_t launch_fused_g(FusedParams fp, const dgi_graph* g, float* partials, float* hub_agg, int stage, hipStream_t stream) {
    AggParams& p = fp.a;
    constexpr int64_t kGroup = (int64_t)kXcds * kXcdRun;
    const auto& hr = g->h_hub_rows;
    const int64_t hb = std::lower_bound(hr.begin(), hr.end(), p.row_begin) - hr.begin();
    const int64_t he = std::lower_bound(hr.begin(), hr.end(), p.row_end) - hr.begin();
    p.hub_begin = hb;
    p.hub_end = he;
    p.skip_hubs = he > hb ? 1 : 0;
    const int Kp = (int)round_up(p.width, 2 * Row<T>::VEC);
    if (p.skip_hubs) {
        DGI_REQUIRE(partials && hub_agg, DGI_ERR_INVALID_ARG, "fused: hub rows in range but no hub buffers");
        AggParams h = p;  // hubs only: no row tiles in this launch
        h.partials = partials;
        h.chunk0 = g->h_hub_chunk_ptr[hb];
        h.n_chunks = g->h_hub_chunk_ptr[he] - h.chunk0;
        h.hub_blocks = round_up((h.n_chunks + kWaves - 1) / kWaves, kGroup);
        h.n_tiles = 0;
        h.out = hub_agg; h.ld_out = Kp; h.out_row0 = 0; h.out_bf16 = 0; h.out_vec_ok = 0; h.hub_compact = 1;
        h.self = nullptr; h.bias = nullptr; h.act = DGI_ACT_NONE; h.out_scale = nullptr;
        DGI_REQUIRE(h.hub_blocks * kWaves * 64 < (int64_t)1 << 32, DGI_ERR_INVALID_ARG, "fused: too many hub chunks for one launch");
        if (stage == 0) {
            hipLaunchKernelGGL((agg_kernel<T, IdxT, G, MODE>), dim3((unsigned)h.hub_blocks), dim3(kWaves * 64), 0, stream, h);
            DGI_HIP(hipGetLastError());
            hipLaunchKernelGGL((agg_hub_reduce_kernel<T, IdxT, MODE>), dim3((unsigned)((he - hb + kWaves - 1) / kWaves)),
                               dim3(kWaves * 64), 0, stream, h);
            DGI_HIP(hipGetLastError());
        }
        fp.hub_agg = hub_agg;
        fp.hub_ld = Kp;
    }
    if (stage == 0) return DGI_OK;
    const int64_t rows = p.row_end - p.row_begin;
    p.n_tiles = (rows + kFusedRows - 1) / kFusedRows;
    const int64_t grid = round_up(p.n_tiles, kGroup);
    DGI_REQUIRE(grid * W * 64 < (int64_t)1 << 32, DGI_ERR_INVALID_ARG, "fused: row range too large for one launch");
    const size_t lds = (size_t)kFusedRows * fp.lds_ld * sizeof(T);
    auto kernel = fused_layer_kernel<T, IdxT, G, MODE, W, SL>;
    if (lds > 48 * 1024)
        DGI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(W * 64), lds, stream, fp);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

template <typename T, typename IdxT, int MODE>
dgi_status_t launch_fused_mode(const FusedParams& fp, const dgi_graph* g, float* partials, float* hub_agg, int stage, hipStream_t stream) {
    const int lanes = (fp.a.width + Row<T>::VEC - 1) / Row<T>::VEC;
    // self rows exist only with the GraphSAGE aggregations
    if constexpr (MODE == MODE_SUM || MODE == MODE_MEAN) {
        if (fp.self_lds == 2) {
            if (lanes <= 16) return launch_fused_g<T, IdxT, 16, MODE, 8, true>(fp, g, partials, hub_agg, stage, stream);
            if (lanes <= 32) return launch_fused_g<T, IdxT, 32, MODE, 8, true>(fp, g, partials, hub_agg, stage, stream);
            return launch_fused_g<T, IdxT, 64, MODE, 8, true>(fp, g, partials, hub_agg, stage, stream);
        }
        if (fp.self_lds == 1) {
            if (lanes <= 16) return launch_fused_g<T, IdxT, 16, MODE, 4, true>(fp, g, partials, hub_agg, stage, stream);
            if (lanes <= 32) return launch_fused_g<T, IdxT, 32, MODE, 4, true>(fp, g, partials, hub_agg, stage, stream);
            return launch_fused_g<T, IdxT, 64, MODE, 4, true>(fp, g, partials, hub_agg, stage, stream);
        }
    }
    if (lanes <= 16) return launch_fused_g<T, IdxT, 16, MODE, 4, false>(fp, g, partials, hub_agg, stage, stream);
    if (lanes <= 32) return launch_fused_g<T, IdxT, 32, MODE, 4, false>(fp, g, partials, hub_agg, stage, stream);
    return launch_fused_g<T, IdxT, 64, MODE, 4, false>(fp, g, partials, hub_agg, stage, stream);
}

template <typename T, typename IdxT>
dgi_status_t launch_fused_t(const FusedParams& fp, const dgi_graph* g, int mode, float* partials, float* hub_agg, int stage, hipStream_t stream) {
    switch (mode) {
        case MODE_SUM: return launch_fused_mode<T, IdxT, MODE_SUM>(fp, g, partials, hub_agg, stage, stream);
        case MODE_MEAN: return launch_fused_mode<T, IdxT, MODE_MEAN>(fp, g, partials, hub_agg, stage, stream);
        case MODE_GCN: return launch_fused_mode<T, IdxT, MODE_GCN>(fp, g, partials, hub_agg, stage, stream);
        case MODE_GCN_PRE: return launch_fused_mode<T, IdxT, MODE_GCN_PRE>(fp, g, partials, hub_agg, stage, stream);
    }
    set_error("unknown aggregation mode %d", mode);
    return DGI_ERR_INVALID_ARG;
}

}  // namespace

constexpr size_t kFusedMaxLds = 128 * 1024;

bool fused_supported(const FusedArgs& a) {
    const int eb = a.dtype == DGI_BF16 ? 2 : 4, E = 16 / eb;
    if ((uintptr_t)a.H % 16 || (a.ld_h * eb) % 16 || a.K % E || a.K / E <= 8) return false;
    if (a.ldw % (2 * E) || a.K1p % (2 * E)) return false;
    if (a.ldw != a.K1p + round_up(a.K, 2 * E)) return false;
    const int blocks = a.dtype == DGI_BF16 ? 2 : 1;  // bf16 tiles carry m_v as two blocks (value, rounding remainder)
    return (size_t)kFusedRows * (size_t)(blocks * round_up(a.K, 2 * E) + E) * eb <= kFusedMaxLds;
}

uint64_t fused_temp_bytes(const dgi_graph* g, int64_t row_begin, int64_t row_end, int K) {
    const auto& hr = g->h_hub_rows;
    const int64_t hb = std::lower_bound(hr.begin(), hr.end(), row_begin) - hr.begin();
    const int64_t he = std::lower_bound(hr.begin(), hr.end(), row_end) - hr.begin();
    if (he <= hb) return 0;
    return (uint64_t)round_up((int64_t)agg_hub_partial_bytes(g, row_begin, row_end, K), 256) +
           (uint64_t)round_up((he - hb) * round_up(K, 16) * 4, 256);
}

dgi_status_t launch_fused(const FusedArgs& a, int stage, hipStream_t stream) {
    if (a.row_end <= a.row_begin) return DGI_OK;
    const dgi_graph* g = a.g;
    DGI_REQUIRE(a.row_begin >= 0 && a.row_end <= g->N, DGI_ERR_INVALID_ARG, "fused: row range outside the graph");
    DGI_REQUIRE(fused_supported(a), DGI_ERR_UNSUPPORTED, "fused: layout not supported");
    const int eb = a.dtype == DGI_BF16 ? 2 : 4, E = 16 / eb;
    FusedParams fp{};
    AggParams& p = fp.a;
    p.indptr = g->d_indptr; p.indices = g->d_indices; p.rs_out = g->d_rs_out; p.rs_in = g->d_rs_in;
    p.S = a.H; p.ld_s = a.ld_h; p.width = a.K;
    p.row_begin = a.row_begin; p.row_end = a.row_end;
    p.hub_rows = g->d_hub_rows; p.hub_chunk_ptr = g->d_hub_chunk_ptr;
    p.wpad = (int)round_up(a.K, 8);
    DGI_REQUIRE(a.Wf != nullptr && (uintptr_t)a.Wf % 16 == 0, DGI_ERR_INVALID_ARG, "fused: fragment-order weights missing or misaligned");
    fp.Wf = a.Wf; fp.ldw = a.ldw; fp.K1p = a.K1p; fp.has_self = a.has_self ? 1 : 0; fp.N = a.N;
    fp.bias = a.bias; fp.act = a.act; fp.act_slope = a.act_slope; fp.out_scale = a.out_scale;
    fp.out = a.out; fp.ld_out = a.ld_out; fp.out_row0 = a.out_row0; fp.out_bf16 = a.out_dtype == DGI_BF16;
    const int mblocks = a.dtype == DGI_BF16 ? 2 : 1;
    fp.lds_ld = (int)(mblocks * round_up(a.K, 2 * E) + E);
    {
        // Variant 2 (self rows in the tile, 8 wavefronts) when every wavefront gets a column block: phase 2 then
        // reads nothing but the weight from outside the workgroup, and half of it runs inside the gather (measured on
        // 256 -> 256 fp32 GraphSAGE, 20 M nodes, degree 20: 104 ms with variant 0, 121 with 1, 99 with 2).  Narrow
        // outputs would leave wavefronts idle there.  With 4 wavefronts the staged tile (variant 1) measured within
        // the run-to-run spread of variant 0 for K <= 128 and clearly slower beyond (256 -> 128: 74 vs 92-97 ms), so
        // it is only reachable by compiling with -DDGI_FUSED_SELF_VARIANT=1.
        const int Kp = (int)round_up(a.K, 2 * E);
#ifdef DGI_FUSED_SELF_VARIANT
        const int forced = DGI_FUSED_SELF_VARIANT;
#else
        const int forced = -1;
#endif
        const bool can = a.has_self && a.K1p == Kp && (a.mode == MODE_SUM || a.mode == MODE_MEAN) &&
                         (size_t)kFusedRows * (size_t)((1 + mblocks) * Kp + E) * eb <= 80 * 1024;
        int variant = 0;
        if (can) variant = forced >= 0 ? forced : ((a.N + 31) / 32 >= 8 ? 2 : 0);
        fp.self_lds = variant;
        if (variant) fp.lds_ld = (1 + mblocks) * Kp + E;
    }
    float* partials = static_cast<float*>(a.temp);
    float* hub_agg = a.temp ? reinterpret_cast<float*>(static_cast<char*>(a.temp) + round_up((int64_t)agg_hub_partial_bytes(g, a.row_begin, a.row_end, a.K), 256)) : nullptr;
    const bool i64 = g->itype == DGI_I64;
    if (a.dtype == DGI_BF16)
        return i64 ? launch_fused_t<uint16_t, int64_t>(fp, g, a.mode, partials, hub_agg, stage, stream)
                   : launch_fused_t<uint16_t, int32_t>(fp, g, a.mode, partials, hub_agg, stage, stream);
    return i64 ? launch_fused_t<float, int64_t>(fp, g, a.mode, partials, hub_agg, stage, stream)
               : launch_fused_t<float, int32_t>(fp, g, a.mode, partials, hub_agg, stage, stream);
}

uint64_t agg_hub_partial_bytes(const dgi_graph* g, int64_t row_begin, int64_t row_end, int width) {
    const auto& hr = g->h_hub_rows;
    const int64_t hb = std::lower_bound(hr.begin(), hr.end(), row_begin) - hr.begin();
    const int64_t he = std::lower_bound(hr.begin(), hr.end(), row_end) - hr.begin();
    if (he <= hb) return 0;
    const int64_t chunks = g->h_hub_chunk_ptr[he] - g->h_hub_chunk_ptr[hb];
    return (uint64_t)chunks * (uint64_t)round_up(width, 8) * sizeof(float);
}

dgi_status_t launch_aggregate(const AggArgs& a, int stage, hipStream_t stream) {
    if (a.row_end <= a.row_begin) return DGI_OK;
    const dgi_graph* g = a.g;
    DGI_REQUIRE(a.row_begin >= 0 && a.row_end <= g->N, DGI_ERR_INVALID_ARG, "aggregate: row range outside the graph");
    DGI_REQUIRE(a.width > 0 && a.ld_s >= a.width && a.ld_out >= a.width, DGI_ERR_INVALID_ARG, "aggregate: bad width / ld");
    AggParams p{};
    p.indptr = g->d_indptr;
    p.indices = g->d_indices;
    p.rs_out = g->d_rs_out;
    p.rs_in = g->d_rs_in;
    p.S = a.S; p.ld_s = a.ld_s; p.width = a.width;
    p.out = a.out; p.ld_out = a.ld_out; p.out_row0 = a.out_row0;
    p.out_bf16 = a.out_dtype == DGI_BF16;
    DGI_REQUIRE(a.out_lo == nullptr || (p.out_bf16 && (uintptr_t)a.out_lo % 16 == (uintptr_t)a.out % 16 && (a.lo_bytes == 1 || a.lo_bytes == 2)),
                DGI_ERR_INVALID_ARG, "aggregate: a low-order output needs a bf16 output of the same alignment");
    p.out_lo = a.out_lo; p.lo_bytes = a.lo_bytes;
    p.self = a.self; p.ld_self = a.ld_self;
    p.bias = a.bias; p.act = a.act; p.act_slope = a.act_slope; p.out_scale = a.out_scale;
    p.row_begin = a.row_begin; p.row_end = a.row_end;
    p.partials = a.hub_partials;
    p.hub_rows = g->d_hub_rows;
    p.hub_chunk_ptr = g->d_hub_chunk_ptr;
    p.wpad = (int)round_up(a.width, 8);
    const int sbytes = a.s_dtype == DGI_BF16 ? 2 : 4, obytes = a.out_dtype == DGI_BF16 ? 2 : 4;
    // fast path: every 16-byte lane load stays inside its (aligned) row
    const bool fast = ((uintptr_t)a.S % 16 == 0) && ((a.ld_s * sbytes) % 16 == 0) &&
                      (round_up(a.width, 16 / sbytes) <= a.ld_s);
    p.out_vec_ok = ((uintptr_t)a.out % 16 == 0) && ((a.ld_out * obytes) % 16 == 0);
    p.self_vec_ok = a.self && ((uintptr_t)a.self % 16 == 0) && ((a.ld_self * sbytes) % 16 == 0);
    const bool i64 = g->itype == DGI_I64;
    if (a.s_dtype == DGI_BF16) {
        return i64 ? dispatch_mode<uint16_t, int64_t>(p, g, a.mode, fast, stage, stream)
                   : dispatch_mode<uint16_t, int32_t>(p, g, a.mode, fast, stage, stream);
    }
    return i64 ? dispatch_mode<float, int64_t>(p, g, a.mode, fast, stage, stream)
               : dispatch_mode<float, int32_t>(p, g, a.mode, fast, stage, stream);
}

}  // namespace dgi
