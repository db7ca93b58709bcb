// Dense transform of a layer (the w^l part of Eq. 1) on the MFMA matrix cores, with the bias and the
// activation fused into the epilogue so they run once per node in the producing layer.
//
//   Y[r, n] = act( sum_k A1[r,k] Wt[n,k] + sum_k (A2[r,k] + A3[r,k]) Wt[n,K1p+k] + bias[n] )
//
// A1|A2 is the row-wise concatenation [h_v | m_v] of GraphSAGE (A2 may be absent); A3, when present, is the
// low-order part of an m_v that is stored as a pair of bf16 values (it multiplies the same weight block); Wt is the weight
// packed transposed, [Nout x ldw] with K contiguous, so both MFMA operands are read from LDS rows of
// the same shape.  bf16 data uses v_mfma_f32_32x32x16_bf16 with fp32 accumulators.  fp32 data runs on the same
// instruction (gemm_split_kernel below): both operands are split exactly into three bf16 terms, x = x1 + x2 + x3,
// and the six products of combined order up to 2^-16 are accumulated in fp32 (what is dropped is of relative size
// 2^-24, an fp32 rounding) -- 6 bf16 MFMAs instead of 8 fp32 ones per 16 elements of K, each at a quarter of the time.
// A workgroup of 4 wavefronts owns a BM x BN output tile; each k-step stages a
// 128-byte slab of every tile row in LDS (global -> registers -> LDS, the next slab's global loads are
// in flight while the current one is multiplied).  LDS rows are padded by 16 bytes so that the 16-byte
// fragment reads of 8 consecutive lanes cover all banks.
#include <algorithm>

#include "dgi_device.h"
#include "dgi_internal.h"

namespace dgi {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Build-time switch for measurements: 1 runs fp32 GEMMs on v_mfma_f32_32x32x2_f32 instead of the three-term bf16 split.
#ifndef DGI_GEMM_F32_MFMA
#define DGI_GEMM_F32_MFMA 0
#endif
constexpr bool kF32OnF32Mfma = DGI_GEMM_F32_MFMA != 0;
// ... and 1 here keeps bf16 GEMMs on the tiled kernel where the weights-stationary one would run.
#ifndef DGI_GEMM_BF16_TILED
#define DGI_GEMM_BF16_TILED 0
#endif
constexpr bool kTiledBf16 = DGI_GEMM_BF16_TILED != 0;
// The weights-stationary kernel: wavefronts per workgroup.
#ifndef DGI_STATIONARY_WAVES
#define DGI_STATIONARY_WAVES 8
#endif

struct GemmParams {
    const void* A1; int64_t ld_a1; int K1; int a1_vec;
    const void* A2; int64_t ld_a2; int K2; int a2_vec;
    const void* A3;  // optional third block: same shape, leading dimension and weight columns as A2
    const uint8_t* Q; int64_t ld_q;  // or the last block's remainder bytes (weights-stationary kernel only)
    const void* Wt; int64_t ldw; int K1p;
    const float* bias;
    int act; float act_slope;
    void* Y; int64_t ld_y; int out_bf16; int y_vec;
    int64_t M; int Nout;
    int tiles_n;
    const float* out_scale; int64_t row0;
};

// 16 bytes of row `row` starting at element k of a [rows x K] matrix; zero outside [0,rows) x [0,K).
template <typename T>
__device__ __forceinline__ uint4 load_chunk(const T* base, int64_t ld, int64_t row, int64_t rows, int k, int K, bool vec_ok) {
    constexpr int E = 16 / sizeof(T);
    uint4 z = make_uint4(0u, 0u, 0u, 0u);
    if (row >= rows || k >= K) return z;
    const T* p = base + row * ld + k;
    if (vec_ok && k + E <= K) return *reinterpret_cast<const uint4*>(p);
    alignas(16) T tmp[E];
#pragma unroll
    for (int e = 0; e < E; ++e) tmp[e] = (k + e < K) ? p[e] : T(0);
    return *reinterpret_cast<uint4*>(tmp);
}

// Workgroups are handed to the 8 XCDs round-robin by their index, and each XCD has its own L2.  The logical tile of
// a workgroup is chosen so that one XCD walks a contiguous run of tiles: the column tiles of one row tile, which read
// the same rows of A, then meet in one L2.
__device__ __forceinline__ int64_t xcd_contiguous_tile() {
    const int64_t b = blockIdx.x, G = gridDim.x;
    const int64_t x = b % 8, j = b / 8, q = G / 8, r = G % 8;
    return x * q + (x < r ? x : r) + j;
}

// Epilogue shared by the two GEMM kernels: bias, activation, per-row factor, conversion, and the store of the
// workgroup's output tile (through LDS as whole 16-byte row pieces when the output layout allows it).  `smem` is the
// kernel's LDS, free for reuse once the last slab has been multiplied (the caller has synchronised).
template <int WGM, int WGN, int TM, int TN>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[TM][TN], const GemmParams& p, unsigned char* smem, int64_t m0, int n0) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int lrow = lane & 31, lhalf = lane >> 5;
    // epilogue: lane holds column (lane % 32) of rows 8*(r/4) + 4*(lane/32) + r%4 of each 32x32 block
    auto value = [&](int i, int j, int r, int64_t m, float b) {
        float v = activate(acc[i][j][r] + b, p.act, p.act_slope);
        if (p.out_scale && m < p.M) v *= p.out_scale[p.row0 + m];
        return v;
    };
    if (p.y_vec) {
        // transpose through LDS so that every lane stores 16 contiguous bytes of an output row: one store
        // instruction per 1 KB instead of one per 128 (bf16) or 256 (fp32) bytes
        auto staged = [&](auto tag) {
            using O = decltype(tag);
            constexpr int OB = (int)sizeof(O), EPC = 16 / OB;
            constexpr int RS = TN * 32 * OB + 16;   // staged row stride in bytes
            constexpr int CPR = TN * 32 * OB / 16;  // 16-byte chunks per staged row
            unsigned char* stage = smem + wave * 32 * RS;
            unsigned char* Yb = static_cast<unsigned char*>(p.Y);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int64_t mb = m0 + (wm * TM + i) * 32;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = n0 + (wn * TN + j) * 32 + lrow;
                    const float b = (p.bias && n < p.Nout) ? p.bias[n] : 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = 8 * (r / 4) + 4 * lhalf + (r % 4);
                        const float v = value(i, j, r, mb + row, b);
                        O* dst = reinterpret_cast<O*>(stage + row * RS) + j * 32 + lrow;
                        if constexpr (OB == 2) *dst = float_to_bf16(v);
                        else *dst = v;
                    }
                }
                __syncthreads();
#pragma unroll 2
                for (int c = lane; c < 32 * CPR; c += 64) {
                    const int row = c / CPR, cc = c % CPR;
                    const int64_t m = mb + row;
                    const int n = n0 + wn * TN * 32 + cc * EPC;
                    if (m < p.M && n < p.Nout) {
                        const unsigned char* src = stage + row * RS + cc * 16;
                        unsigned char* y = Yb + (m * p.ld_y + n) * OB;
                        if (n + EPC <= p.Nout) {
                            *reinterpret_cast<uint4*>(y) = *reinterpret_cast<const uint4*>(src);
                        } else {
                            for (int t = 0; t < p.Nout - n; ++t) reinterpret_cast<O*>(y)[t] = reinterpret_cast<const O*>(src)[t];
                        }
                    }
                }
                if (i + 1 < TM) __syncthreads();
            }
        };
        if (p.out_bf16) staged(uint16_t{});
        else staged(float{});
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + (wn * TN + j) * 32 + lrow;
            if (n >= p.Nout) continue;
            const float b = p.bias ? p.bias[n] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * lhalf + (r % 4);
                if (m >= p.M) continue;
                const float v = value(i, j, r, m, b);
                if (p.out_bf16) static_cast<uint16_t*>(p.Y)[m * p.ld_y + n] = float_to_bf16(v);
                else static_cast<float*>(p.Y)[m * p.ld_y + n] = v;
            }
        }
}

// The register budget is pinned to the occupancy the accumulators allow (16 registers per 32x32 block):
// the kernel hides memory latency with resident workgroups, and measured slower whenever one was lost.
template <typename T, int WGM, int WGN, int TM, int TN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(TM * TN >= 6 ? 2 : TM * TN >= 4 ? 3 : 4)))
void gemm_kernel(GemmParams p) {
    constexpr int E = 16 / sizeof(T);      // elements per 16-byte chunk
    constexpr int BK = 8 * E;              // 128 bytes of K per step
    constexpr int LDS_LD = BK + E;         // padded row, in elements
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    constexpr int A_CHUNKS = BM * 8 / 256, B_CHUNKS = BN * 8 / 256;
    static_assert(WGM * WGN == 4, "4 wavefronts per workgroup");
    // the epilogue stages each wavefront's 32-row strip (TN*32 columns, up to 4 bytes each, rows padded by
    // 16 bytes) in the same memory once the last slab has been multiplied
    constexpr int MAIN_BYTES = (BM + BN) * LDS_LD * (int)sizeof(T);
    constexpr int EPI_BYTES = 4 * 32 * (TN * 32 * 4 + 16);
    __shared__ __attribute__((aligned(16))) unsigned char smem[MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES];
    T* As = reinterpret_cast<T*>(smem);
    T* Bs = As + BM * LDS_LD;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int64_t tile = xcd_contiguous_tile();
    const int64_t tile_m = tile / p.tiles_n;
    const int tile_n = (int)(tile % p.tiles_n);
    const int64_t m0 = tile_m * BM;
    const int n0 = tile_n * BN;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int S1 = (p.K1 + BK - 1) / BK;
    const int S2 = p.A2 ? (p.K2 + BK - 1) / BK : 0;
    const int S = S1 + S2 + (p.A3 ? S2 : 0);
    // the next slab's global loads are in flight while the current one is multiplied
    uint4 ra[A_CHUNKS], rb[B_CHUNKS];

    auto block_of = [&](int s, const T*& A, int64_t& lda, int& K, bool& vec, int& k0, int& wcol) {
        const bool second = s >= S1;
        const bool third = s >= S1 + S2;
        A = static_cast<const T*>(third ? p.A3 : second ? p.A2 : p.A1);
        lda = second ? p.ld_a2 : p.ld_a1;
        K = second ? p.K2 : p.K1;
        vec = second ? p.a2_vec : p.a1_vec;
        k0 = (third ? s - S1 - S2 : second ? s - S1 : s) * BK;
        wcol = second ? p.K1p : 0;
    };
    auto load_a = [&](int s) {
        const T* A; int64_t lda; int K, k0, wcol; bool vec;
        block_of(s, A, lda, K, vec, k0, wcol);
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            ra[i] = load_chunk<T>(A, lda, m0 + c / 8, p.M, k0 + (c % 8) * E, K, vec);
        }
    };
    auto load_b = [&](int s) {
        const T* A; int64_t lda; int K, k0, wcol; bool vec;
        block_of(s, A, lda, K, vec, k0, wcol);
        const T* W = static_cast<const T*>(p.Wt) + wcol;
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            const int n = n0 + c / 8, k = k0 + (c % 8) * E;
            // the packed weight is zero-padded to a multiple of E after each block, so a chunk that starts
            // below K may be read whole
            rb[i] = (n < p.Nout && k < K) ? *reinterpret_cast<const uint4*>(W + (int64_t)n * p.ldw + k) : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto store_step = [&]() {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            *reinterpret_cast<uint4*>(&As[(c / 8) * LDS_LD + (c % 8) * E]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            *reinterpret_cast<uint4*>(&Bs[(c / 8) * LDS_LD + (c % 8) * E]) = rb[i];
        }
    };
    const int lrow = lane & 31, lhalf = lane >> 5;
    auto multiply = [&]() {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {  // BK = 4 sub-steps of 2E elements
            uint4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const uint4*>(&As[((wm * TM + i) * 32 + lrow) * LDS_LD + kk * 2 * E + lhalf * E]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const uint4*>(&Bs[((wn * TN + j) * 32 + lrow) * LDS_LD + kk * 2 * E + lhalf * E]);
            if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const float a = __uint_as_float(e == 0 ? fa[i].x : e == 1 ? fa[i].y : e == 2 ? fa[i].z : fa[i].w);
                            const float b = __uint_as_float(e == 0 ? fb[j].x : e == 1 ? fb[j].y : e == 2 ? fb[j].z : fb[j].w);
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i][j], 0, 0, 0);
                        }
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        bf16x8 a, b;
                        __builtin_memcpy(&a, &fa[i], 16);
                        __builtin_memcpy(&b, &fb[j], 16);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i][j], 0, 0, 0);
                    }
            }
        }
    };

    if (S > 0) {
        load_b(0);
        load_a(0);
        store_step();
    }
    __syncthreads();
    for (int s = 0; s < S; ++s) {
        if (s + 1 < S) {
            load_b(s + 1);
            load_a(s + 1);
        }
        multiply();
        __syncthreads();
        if (s + 1 < S) {
            store_step();
            __syncthreads();
        }
    }

    gemm_epilogue<WGM, WGN, TM, TN>(acc, p, smem, m0, n0);
}

// x = t[0] + t[1] + t[2] exactly, each term a bf16 value: the value rounded to nearest, then twice the same of what is left
// (the second remainder has at most 8 significant bits).  Non-finite x gives NaN terms.
__device__ __forceinline__ void split3(float x, uint16_t (&t)[3]) {
    t[0] = float_to_bf16(x);
    const float r1 = x - bf16_to_float(t[0]);
    t[1] = float_to_bf16(r1);
    const float r2 = r1 - bf16_to_float(t[1]);
    t[2] = float_to_bf16(r2);
}

// The fp32 GEMM on the bf16 matrix instruction.  Operands are fp32 in memory; the staging step splits every element
// into its three bf16 terms (split3) and writes them as three 64-byte planes of the tile row's LDS slab
// (32 elements of K per step; 16 bytes of padding make the row 52 words, so 8 lanes' 16-byte reads cover all banks).
// For every 16 elements of K the products t_a[i] * t_b[j] with i + j <= 2 are accumulated: the terms fall off by
// 2^-8 each, so what is left out is below 2^-23 of |a||b|, with random sign.
template <int WGM, int WGN, int TM, int TN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(TM * TN >= 6 ? 2 : TM * TN >= 4 ? 3 : 4)))
void gemm_split_kernel(GemmParams p) {
    constexpr int BK = 32;                 // fp32 elements of K per step: 128 bytes of every tile row
    constexpr int ROW_B = 3 * 2 * BK + 16; // LDS row: three bf16 planes and the padding, in bytes
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    constexpr int A_CHUNKS = BM * 8 / 256, B_CHUNKS = BN * 8 / 256;
    static_assert(WGM * WGN == 4, "4 wavefronts per workgroup");
    constexpr int MAIN_BYTES = (BM + BN) * ROW_B;
    constexpr int EPI_BYTES = 4 * 32 * (TN * 32 * 4 + 16);
    __shared__ __attribute__((aligned(16))) unsigned char smem[MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES];
    unsigned char* As = smem;
    unsigned char* Bs = smem + BM * ROW_B;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int64_t tile = xcd_contiguous_tile();
    const int64_t tile_m = tile / p.tiles_n;
    const int tile_n = (int)(tile % p.tiles_n);
    const int64_t m0 = tile_m * BM;
    const int n0 = tile_n * BN;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int S1 = (p.K1 + BK - 1) / BK;
    const int S2 = p.A2 ? (p.K2 + BK - 1) / BK : 0;
    const int S = S1 + S2;
    uint4 ra[A_CHUNKS], rb[B_CHUNKS];

    auto load_a = [&](int s) {
        const bool second = s >= S1;
        const float* A = static_cast<const float*>(second ? p.A2 : p.A1);
        const int64_t lda = second ? p.ld_a2 : p.ld_a1;
        const int K = second ? p.K2 : p.K1;
        const bool vec = second ? p.a2_vec : p.a1_vec;
        const int k0 = (second ? s - S1 : s) * BK;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            ra[i] = load_chunk<float>(A, lda, m0 + c / 8, p.M, k0 + (c % 8) * 4, K, vec);
        }
    };
    auto load_b = [&](int s) {
        const bool second = s >= S1;
        const int K = second ? p.K2 : p.K1;
        const int k0 = (second ? s - S1 : s) * BK;
        const float* W = static_cast<const float*>(p.Wt) + (second ? p.K1p : 0);
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            const int n = n0 + c / 8, k = k0 + (c % 8) * 4;
            // the packed weight is zero-padded to a multiple of 4 after each block
            rb[i] = (n < p.Nout && k < K) ? *reinterpret_cast<const uint4*>(W + (int64_t)n * p.ldw + k) : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto store_split = [&](unsigned char* row, int chunk, const uint4& v) {
        const float x[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
        uint16_t t[4][3];
#pragma unroll
        for (int e = 0; e < 4; ++e) split3(x[e], t[e]);
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            uint2 w;
            w.x = (uint32_t)t[0][q] | ((uint32_t)t[1][q] << 16);
            w.y = (uint32_t)t[2][q] | ((uint32_t)t[3][q] << 16);
            *reinterpret_cast<uint2*>(row + q * 2 * BK + chunk * 8) = w;
        }
    };
    auto store_step = [&]() {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            store_split(As + (c / 8) * ROW_B, c % 8, ra[i]);
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            store_split(Bs + (c / 8) * ROW_B, c % 8, rb[i]);
        }
    };
    const int lrow = lane & 31, lhalf = lane >> 5;
    auto multiply = [&]() {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {  // 16 elements of K per MFMA: lane half h holds elements 8h .. 8h+7
            bf16x8 fa[TM][3], fb[TN][3];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int q = 0; q < 3; ++q)
                    fa[i][q] = *reinterpret_cast<const bf16x8*>(As + ((wm * TM + i) * 32 + lrow) * ROW_B + q * 2 * BK + ks * 32 + lhalf * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 3; ++q)
                    fb[j][q] = *reinterpret_cast<const bf16x8*>(Bs + ((wn * TN + j) * 32 + lrow) * ROW_B + q * 2 * BK + ks * 32 + lhalf * 16);
            // smallest products first
#pragma unroll
            for (int order = 2; order >= 0; --order)
#pragma unroll
                for (int qa = 0; qa <= order; ++qa)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i][qa], fb[j][order - qa], acc[i][j], 0, 0, 0);
        }
    };

    if (S > 0) {
        load_b(0);
        load_a(0);
        store_step();
    }
    __syncthreads();
    for (int s = 0; s < S; ++s) {
        if (s + 1 < S) {
            load_b(s + 1);
            load_a(s + 1);
        }
        multiply();
        __syncthreads();
        if (s + 1 < S) {
            store_step();
            __syncthreads();
        }
    }

    gemm_epilogue<WGM, WGN, TM, TN>(acc, p, smem, m0, n0);
}

// LDS writes of some lanes are read by other lanes of the same wavefront: order them without a workgroup barrier and
// without waiting for global loads and stores in flight (a fence over all address spaces would).
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// The bf16 GEMM of tall matrices with a small weight: weights-stationary and persistent.  A layer's GEMM here has millions
// of rows and a weight of at most a few hundred rows and columns, so it is a stream of A through the matrix cores
// and its bound is HBM.  The tiled kernel above falls well short of that bound on such shapes (measured 4.5 TB/s of A, hi, lo
// and output traffic on 111 M rows, K = 3 x 128, N = 128): every tile stages the same weight slabs again, and its two
// workgroup barriers per slab leave loads in flight only while a slab is multiplied.  Here one workgroup per CU stays for
// the whole launch and holds the weight in LDS as the B fragments of v_mfma_f32_32x32x16_bf16 (loaded once); after that its
// wavefronts never meet again.  Each wavefront loops over its own tiles of 32 rows, reads A from global memory straight
// into fragment layout (lane l: row l % 32, 8 elements of K from 8 (l / 32) of each 16; the four loads that cover one
// 64-byte stretch of a row follow each other) in steps of 128 elements of K, each step into registers of its own that are
// refilled for the wavefront's next tile as soon as the step is multiplied, and sends the finished 32 x N tile through a
// private LDS stage so that it leaves as 16-byte pieces of whole rows.  The kernel is bound by the loads it keeps in
// flight (8, 6 and 4 wavefronts with one step in flight each: 23, 26 and 32 ms on the 111 M-row GEMM).
// NB = column blocks of 32, NS = steps per tile, of which the last NS - QS (those of the last K block) come with
// remainder bytes.
// The bf16 values (value - 128) * 2^(e - 15) that the bytes q stand for, e = exponent of the bf16 value they belong to
// (remainder_byte of the aggregation kernel): 8 elements, hi and the result packed two per word.  Each has at most 7
// significant bits, so cutting the fp32 product to its upper half is exact.
__device__ __forceinline__ uint4 remainder_values(const uint4& hi, const uint2& q) {
    const uint32_t h[4] = {hi.x, hi.y, hi.z, hi.w};
    uint32_t out[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t qw = i < 2 ? q.x : q.y;
        const float q0 = (float)((qw >> (16 * (i & 1))) & 0xffu) - 128.f, q1 = (float)((qw >> (16 * (i & 1) + 8)) & 0xffu) - 128.f;
        const float s0 = __uint_as_float((h[i] << 16) & 0x7f800000u) * 0x1p-15f, s1 = __uint_as_float(h[i] & 0x7f800000u) * 0x1p-15f;
        out[i] = (__float_as_uint(q0 * s0) >> 16) | (__float_as_uint(q1 * s1) & 0xffff0000u);
    }
    return make_uint4(out[0], out[1], out[2], out[3]);
}

template <int NB, int NS, int QS>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_stationary_kernel(GemmParams p, int stage_blocks, int stage_bytes) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    using T = uint16_t;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    // a step = 8 k-steps of 16 (128 elements of K) of one A block; a block's last step is padded with zero weights, so
    // that the loops below have no branches and the compiler can overlap fragment reads, decoding and products
    const int P1 = (p.K1 + 127) / 128, P2 = p.A2 ? (p.K2 + 127) / 128 : 0;
    const int KS1 = 8 * P1, KS2 = 8 * P2;
    const int kstot = KS1 + KS2;   // k-steps over the weight's two column blocks

    // the weight -> LDS in fragment order: piece (cb, kg, lane) = W^T[32 cb + lane % 32][8 elements from 16 kg' + 8 (lane / 32)]
    {
        const T* Wt = static_cast<const T*>(p.Wt);
        const int pieces = NB * kstot * 64;
        for (int i = threadIdx.x; i < pieces; i += blockDim.x) {
            const int l = i & 63, kg = (i >> 6) % kstot, cb = (i >> 6) / kstot;
            const int n = cb * 32 + (l & 31);
            const bool second = kg >= KS1;
            const int k = (second ? kg - KS1 : kg) * 16 + (l >> 5) * 8;
            uint4 w = make_uint4(0u, 0u, 0u, 0u);
            // the packed weight is zero-padded to a multiple of 8 after each block, so a piece that starts below K may be read whole
            if (n < p.Nout && k < (second ? p.K2 : p.K1)) w = *reinterpret_cast<const uint4*>(Wt + (int64_t)n * p.ldw + (second ? p.K1p : 0) + k);
            *reinterpret_cast<uint4*>(lds + (size_t)i * 16) = w;
        }
    }
    float* bias_lds = reinterpret_cast<float*>(lds + (size_t)NB * kstot * 1024);
    for (int i = threadIdx.x; i < NB * 32; i += blockDim.x) bias_lds[i] = (p.bias && i < p.Nout) ? p.bias[i] : 0.f;
    __syncthreads();  // the only workgroup barrier
    const unsigned char* wl = lds + lane * 16;
    unsigned char* stage = lds + (size_t)NB * kstot * 1024 + (size_t)NB * 128 + (size_t)wave * stage_bytes;

    constexpr bool Q = QS < NS;   // steps QS .. NS-1 (those of the last K block) come with remainder bytes
    const int64_t tiles = (p.M + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * waves;
    struct Buffers {
        uint4 a[NS][8];
        uint2 q[Q ? NS - QS : 1][8];   // the remainder bytes of the same 8 elements per k-step
    };
    auto load_step = [&](int64_t t, int i, Buffers& bf) {
        const bool second = i >= P1, third = i >= P1 + P2;   // the third block (A3) repeats the second one's shape and weights
        const T* A = static_cast<const T*>(third ? p.A3 : second ? p.A2 : p.A1);
        const int64_t lda = second ? p.ld_a2 : p.ld_a1;
        const int K = second ? p.K2 : p.K1;
        const int part = third ? i - P1 - P2 : second ? i - P1 : i;
        const int64_t row = t * 32 + lrow;
        // every lane issues every load (out-of-range ones read the block's first bytes and are zeroed on arrival): the
        // number of loads in flight is then known at compile time, and waiting for one step's registers does not have
        // to wait for the younger loads and stores as well
        const T* arow = A + (row < p.M ? row : 0) * lda;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const int k = (part * 8 + ks) * 16 + lhalf * 8;   // K is a multiple of 8 (host-checked): a piece is in or out as a whole
            bf.a[i][ks] = *reinterpret_cast<const uint4*>(arow + (k < K ? k : 0));
        }
        if constexpr (Q) {
            if (i >= QS) {
                const uint8_t* qrow = p.Q + (row < p.M ? row : 0) * p.ld_q;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const int k = (part * 8 + ks) * 16 + lhalf * 8;
                    bf.q[i >= QS ? i - QS : 0][ks] = *reinterpret_cast<const uint2*>(qrow + (k < K ? k : 0));   // out of range: meets zero values
                }
            }
        }
    };
    const int ob = p.out_bf16 ? 2 : 4, epc = 16 / ob;
    const int rs = stage_blocks * 32 * ob + 16;   // staged row pitch in bytes

    int64_t t = (int64_t)blockIdx.x * waves + wave;
    // One register buffer per step of a tile (NS = nsteps, checked by the host).  A buffer is refilled with the same step
    // of the wavefront's next tile as soon as its products are issued, so the loads of a whole tile are in flight behind
    // the multiplication (no buffer is ever copied: moving a register that a load is still to fill would wait for it).
    Buffers buf;
    if (t < tiles) {
#pragma unroll
        for (int i = 0; i < NS; ++i) load_step(t, i, buf);
    }
    const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (; t < tiles; t += stride) {
        // The products are taken as (W^T fragment) x (A fragment): the accumulator block is then the transposed output
        // block, lane l holds row l % 32 of the tile and, in register r, column 8 (r / 4) + 4 (l / 32) + r % 4 of the
        // block: four consecutive columns per group of four registers, which leave as one packed store.  A row's result
        // depends on that row of A alone, so rows past M and pieces past K need no masking: the former are never stored,
        // the latter meet zero weights (they re-read the row's first bytes, finite whenever the row is).
        floatx16 acc[NB];
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const bool second = i >= P1, third = i >= P1 + P2;
            const int part = third ? i - P1 - P2 : second ? i - P1 : i;
            const int kg0 = (second ? KS1 : 0) + part * 8;           // first k-step of the step in the weight's order
            const unsigned char* wk = wl + (size_t)kg0 * 1024;
            const bool with_q = Q && i >= QS;   // known at compile time: i is unrolled
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                bf16x8 w[NB];   // the fragments of all column blocks first, then the products: independent accumulators back to back
#pragma unroll
                for (int cb = 0; cb < NB; ++cb) w[cb] = *reinterpret_cast<const bf16x8*>(wk + ((size_t)cb * kstot + ks) * 1024);
                bf16x8 a, lo;
                __builtin_memcpy(&a, &buf.a[i][ks], 16);
                if (with_q) {
                    const uint4 l = remainder_values(buf.a[i][ks], buf.q[i >= QS ? i - QS : 0][ks]);
                    __builtin_memcpy(&lo, &l, 16);
                }
                // the tile's first product starts from zero
#pragma unroll
                for (int cb = 0; cb < NB; ++cb)
                    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[cb], a, (i == 0 && ks == 0) ? zero16 : acc[cb], 0, 0, 0);
                if (with_q) {
#pragma unroll
                    for (int cb = 0; cb < NB; ++cb) acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[cb], lo, acc[cb], 0, 0, 0);
                }
            }
            load_step(t + stride < tiles ? t + stride : t, i, buf);   // the last tile once more rather than a conditional load (see load_step)
        }
        // epilogue; the stage takes stage_blocks column blocks at a time
        const int64_t m0 = t * 32;
        const float osc = (p.out_scale && m0 + lrow < p.M) ? p.out_scale[p.row0 + m0 + lrow] : 1.f;
#pragma unroll
        for (int cb = 0; cb < NB; ++cb) {
            const int j = cb % stage_blocks;
            unsigned char* dst = stage + lrow * rs + (j * 32 + 4 * lhalf) * ob;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b = *reinterpret_cast<const float4*>(bias_lds + cb * 32 + 8 * g + 4 * lhalf);
                float v[4] = {acc[cb][4 * g] + b.x, acc[cb][4 * g + 1] + b.y, acc[cb][4 * g + 2] + b.z, acc[cb][4 * g + 3] + b.w};
                if (p.act == DGI_ACT_RELU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
                } else if (p.act != DGI_ACT_NONE) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = activate(v[e], p.act, p.act_slope);
                }
                if (p.out_scale) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] *= osc;
                }
                if (p.out_bf16) {
                    *reinterpret_cast<uint2*>(dst + 8 * g * ob) = make_uint2((uint32_t)float_to_bf16(v[0]) | ((uint32_t)float_to_bf16(v[1]) << 16),
                                                                            (uint32_t)float_to_bf16(v[2]) | ((uint32_t)float_to_bf16(v[3]) << 16));
                } else {
                    *reinterpret_cast<float4*>(dst + 8 * g * ob) = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
            if (j + 1 == stage_blocks || cb + 1 == NB) {  // wave-uniform: the stage is full
                wave_lds_fence();
                const int n_first = (cb - j) * 32;
                const int ncols = (p.Nout - n_first) < (j + 1) * 32 ? (p.Nout - n_first) : (j + 1) * 32;
                if (ncols > 0) {
                    // piece c of the stage is 16 bytes of staged row c / cpr; cpr is a power of two for the usual row
                    // lengths, and then the split is a shift (a division by a run-time value costs some twenty instructions)
                    const int cpr = (ncols * ob + 15) / 16;
                    const int shift = (cpr & (cpr - 1)) == 0 ? 31 - __clz(cpr) : -1;   // wave-uniform
                    unsigned char* Yb = static_cast<unsigned char*>(p.Y);
                    for (int c = lane; c < 32 * cpr; c += 64) {
                        const int row = shift >= 0 ? c >> shift : c / cpr, cc = c - row * cpr;
                        const int64_t m = m0 + row;
                        if (m >= p.M) continue;
                        const int n = cc * epc;   // column inside the staged stretch
                        const unsigned char* src = stage + row * rs + cc * 16;
                        unsigned char* y = Yb + (m * p.ld_y + n_first + n) * ob;
                        if (n + epc <= ncols && p.y_vec) {
                            *reinterpret_cast<uint4*>(y) = *reinterpret_cast<const uint4*>(src);
                        } else if (n + epc <= ncols) {  // output rows that are not 16-byte aligned
                            for (int e = 0; e < 16; e += 2) *reinterpret_cast<uint16_t*>(y + e) = *reinterpret_cast<const uint16_t*>(src + e);
                        } else {
                            for (int e = 0; e < (ncols - n) * ob; e += 2) *reinterpret_cast<uint16_t*>(y + e) = *reinterpret_cast<const uint16_t*>(src + e);
                        }
                    }
                }
                wave_lds_fence();  // the stage may be written again
            }
        }
    }
}

template <typename T>
__global__ void pack_weight_kernel(const T* W, int K, int Nout, T* Wt, int64_t ldw, int koff) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)K * Nout) return;
    const int k = (int)(i / Nout), n = (int)(i % Nout);
    Wt[(int64_t)n * ldw + koff + k] = W[i];
}

template <typename T>
__global__ void pack_fragments_kernel(const T* Wt, int64_t ldw, int N, int64_t total, T* Wf) {
    constexpr int VEC = 16 / (int)sizeof(T);
    const int64_t KS = ldw / (2 * VEC);
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int i = (int)(idx % VEC);
        const int lane = (int)((idx / VEC) % 64);
        const int64_t ks = (idx / (VEC * 64)) % KS;
        const int64_t cb = idx / (VEC * 64 * KS);
        const int64_t n = cb * 32 + (lane & 31);
        const int64_t k = ks * 2 * VEC + (lane >> 5) * VEC + i;
        Wf[idx] = n < N ? Wt[n * ldw + k] : T(0);
    }
}

__global__ void pack_gat_attn_kernel(const float* W, int K, int heads, int F, const float* a_src, const float* a_dst,
                                     float* Wt, int64_t ldw) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= K * heads * 2) return;
    const int k = i / (heads * 2), hh = i % (heads * 2);
    const int h = hh % heads;
    const float* a = (hh < heads ? a_src : a_dst) + h * F;
    float s = 0.f;
    for (int f = 0; f < F; ++f) s = fmaf(W[(int64_t)k * heads * F + h * F + f], a[f], s);
    Wt[(int64_t)(heads * F + hh) * ldw + k] = s;
}

__global__ void fill_zero_kernel(uint32_t* p, uint64_t words) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (uint64_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// rows of `width` elements; one thread per 4-byte (fp32) or 2-byte (bf16) element, coalesced along the row
template <typename T>
__global__ void permute_rows_kernel(const T* in, int64_t ld_in, T* out, int64_t ld_out, int64_t rows, int width,
                                    const int32_t* perm, int gather) {
    const int64_t total = rows * width;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / width;
        const int c = (int)(i % width);
        const int64_t pr = perm ? (int64_t)perm[r] : r;  // no permutation: a strided row copy
        if (gather) out[r * ld_out + c] = in[pr * ld_in + c];
        else out[pr * ld_out + c] = in[r * ld_in + c];
    }
}

// The same row move in 16-byte pieces (rows, leading dimensions and bases all multiples of 16 bytes): `chunks` pieces
// per row, consecutive lanes take consecutive pieces of a row, so a wavefront moves 1 KB of whole rows per instruction.
// This is the form that reads rows out of mapped host memory: large requests use the host link far better.
__global__ void permute_rows_vec_kernel(const uint4* in, int64_t ld_in, uint4* out, int64_t ld_out, int64_t rows, int chunks,
                                        const int32_t* perm, int gather) {
    const int64_t total = rows * chunks;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / chunks;
        const int c = (int)(i % chunks);
        const int64_t pr = perm ? (int64_t)perm[r] : r;
        if (gather) out[r * ld_out + c] = in[pr * ld_in + c];
        else out[pr * ld_out + c] = in[r * ld_in + c];
    }
}

// out[r, c] = in[r, c] * scale[r]
template <typename T>
__global__ void scale_rows_kernel(const T* in, int64_t ld_in, T* out, int64_t ld_out, int64_t rows, int width, const float* scale) {
    const int64_t total = rows * width;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / width;
        const int c = (int)(i % width);
        if (sizeof(T) == 4) {
            reinterpret_cast<float*>(out)[r * ld_out + c] = reinterpret_cast<const float*>(in)[r * ld_in + c] * scale[r];
        } else {
            const float f = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(in)[r * ld_in + c] << 16) * scale[r];
            reinterpret_cast<uint16_t*>(out)[r * ld_out + c] = float_to_bf16(f);
        }
    }
}

template <typename T, int WGM, int WGN, int TM, int TN>
dgi_status_t launch_cfg(GemmParams p, hipStream_t stream) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    const int64_t tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.Nout + BN - 1) / BN;
    const int64_t grid = tiles_m * p.tiles_n;
    DGI_REQUIRE(grid * 256 < (int64_t)1 << 32, DGI_ERR_INVALID_ARG, "gemm: too many tiles for one launch");
    if constexpr (sizeof(T) == 4 && !kF32OnF32Mfma) hipLaunchKernelGGL((gemm_split_kernel<WGM, WGN, TM, TN>), dim3((unsigned)grid), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((gemm_kernel<T, WGM, WGN, TM, TN>), dim3((unsigned)grid), dim3(256), 0, stream, p);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

constexpr int kStationaryWaves = DGI_STATIONARY_WAVES;

int device_cu_count() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        return v;
    }();
    return n;
}

// LDS one workgroup may have: all of a CU's 160 KB on gfx950 (the device says how much it grants)
size_t stationary_lds_bytes() {
    static const size_t n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || v <= 0) v = 64 * 1024;
        return std::min<size_t>((size_t)v, 160 * 1024);
    }();
    return n;
}

// LDS plan of the stationary kernel: weight fragments, bias, one output stage per wavefront that holds as many column
// blocks as fit (whole rows when it can).  Returns the column blocks per stage, 0 if the weight leaves no room.
// the kernel is built for 2, 4, 6 and 8 column blocks of 32
int stationary_blocks(int Nout) { return ((Nout + 63) / 64) * 2; }

// steps of 128 elements of K per tile
int stationary_steps(const GemmParams& p) { return (p.K1 + 127) / 128 + (p.A2 ? (p.K2 + 127) / 128 : 0) * (p.A3 ? 2 : 1); }

// steps (of the NS) without remainder bytes: all of them, or those of the first block when there are two
int stationary_plain_steps(const GemmParams& p, bool with_bytes) {
    return !with_bytes ? stationary_steps(p) : p.A2 ? (p.K1 + 127) / 128 : 0;
}

// registers of the accumulators and step buffers, in units the compiler's results were fitted to (176 builds without
// spilling at two wavefronts per SIMD, 192 does not)
constexpr int stationary_regs(int NB, int NS, int QS) { return 16 * NB + 32 * NS + 16 * (NS - QS); }

// LDS plan of the stationary kernel: weight fragments, bias, one output stage per wavefront that holds as many column
// blocks as fit (whole rows when it can).  Returns the column blocks per stage; 0 if the weight leaves no room, or if the
// accumulators and the steps' buffers (and their remainder bytes: with_bytes) would not fit the registers of a wavefront.
int stationary_stage_blocks(const GemmParams& p, bool with_bytes, size_t* weight_bytes) {
    const int NB = stationary_blocks(p.Nout), NS = stationary_steps(p);
    const int kstot = 8 * ((p.K1 + 127) / 128 + (p.A2 ? (p.K2 + 127) / 128 : 0));   // whole steps: see the kernel
    const size_t wb = (size_t)NB * kstot * 1024 + (size_t)NB * 128;
    if (weight_bytes) *weight_bytes = wb;
    const size_t kStationaryLds = stationary_lds_bytes();
    if (NB > 8 || NS > 3 || wb >= kStationaryLds || p.K1 % 8 != 0 || (p.A2 && p.K2 % 8 != 0)) return 0;
    if (stationary_regs(NB, NS, stationary_plain_steps(p, with_bytes)) > 176) return 0;
    const int ob = p.out_bf16 ? 2 : 4;
    const int64_t per_row = (int64_t)((kStationaryLds - wb) / kStationaryWaves / 32);   // bytes of one staged row
    const int64_t sb = (per_row - 16) / (32 * ob);
    return (int)std::min<int64_t>(NB, std::max<int64_t>(sb, 0));
}

template <int NB, int NS, int QS>
dgi_status_t launch_stationary_k(const GemmParams& p, int sb, size_t wb, hipStream_t stream) {
    if constexpr (QS < 0 || QS > NS || stationary_regs(NB, NS, QS) > 176) {
        set_error("gemm: the weights-stationary kernel is not built for this shape");
        return DGI_ERR_UNSUPPORTED;
    } else {
        const int ob = p.out_bf16 ? 2 : 4;
        const int stage_bytes = 32 * (sb * 32 * ob + 16);
        const size_t lds = wb + (size_t)kStationaryWaves * stage_bytes;
        const int64_t tiles = (p.M + 31) / 32;
        const int64_t grid = std::min<int64_t>(device_cu_count(), (tiles + kStationaryWaves - 1) / kStationaryWaves);
        auto kernel = gemm_stationary_kernel<NB, NS, QS>;
        if (lds > 48 * 1024)
            DGI_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kStationaryWaves * 64), lds, stream, p, sb, stage_bytes);
        DGI_HIP(hipGetLastError());
        return DGI_OK;
    }
}

template <int NB, int NS>
dgi_status_t launch_stationary_ns(const GemmParams& p, int sb, size_t wb, hipStream_t stream) {
    switch (stationary_plain_steps(p, p.Q != nullptr)) {
        case 0: return launch_stationary_k<NB, NS, 0>(p, sb, wb, stream);
        case 1: return launch_stationary_k<NB, NS, 1>(p, sb, wb, stream);
        case 2: return launch_stationary_k<NB, NS, 2>(p, sb, wb, stream);
        default: return launch_stationary_k<NB, NS, 3>(p, sb, wb, stream);
    }
}

template <int NB>
dgi_status_t launch_stationary_nb(const GemmParams& p, int sb, size_t wb, hipStream_t stream) {
    switch (stationary_steps(p)) {
        case 1: return launch_stationary_ns<NB, 1>(p, sb, wb, stream);
        case 2: return launch_stationary_ns<NB, 2>(p, sb, wb, stream);
        default: return launch_stationary_ns<NB, 3>(p, sb, wb, stream);
    }
}

dgi_status_t launch_stationary(const GemmParams& p, int sb, size_t wb, hipStream_t stream) {
    const int NB = stationary_blocks(p.Nout);
    if (NB <= 2) return launch_stationary_nb<2>(p, sb, wb, stream);
    if (NB <= 4) return launch_stationary_nb<4>(p, sb, wb, stream);
    if (NB <= 6) return launch_stationary_nb<6>(p, sb, wb, stream);
    return launch_stationary_nb<8>(p, sb, wb, stream);
}

}  // namespace

bool gemm_stationary_applies(const void* A1, int64_t ld_a1, int K1, int blocks, int K2, int Nout, int out_dtype, bool with_bytes) {
    if ((uintptr_t)A1 % 16 != 0 || (ld_a1 * 2) % 16 != 0) return false;
    GemmParams p{};
    const void* some = reinterpret_cast<const void*>(16);   // only the presence of a block matters to the plan
    p.K1 = K1; p.K2 = K2; p.A2 = blocks >= 2 ? some : nullptr; p.A3 = blocks >= 3 ? some : nullptr;
    p.Nout = Nout; p.out_bf16 = out_dtype == DGI_BF16;
    return stationary_stage_blocks(p, with_bytes, nullptr) > 0;
}

dgi_status_t launch_gemm(const GemmArgs& a, hipStream_t stream) {
    if (a.M <= 0 || a.Nout <= 0) return DGI_OK;
    const int eb = a.dtype == DGI_BF16 ? 2 : 4, E = 16 / eb;
    DGI_REQUIRE(a.A1 && a.Wt && a.Y, DGI_ERR_INVALID_ARG, "gemm: null operand");
    DGI_REQUIRE(a.dtype == DGI_BF16 || (!a.A3 && !a.A_lo8), DGI_ERR_INVALID_ARG, "gemm: the low-order block is a bf16 operand");
    DGI_REQUIRE(!(a.A3 && a.A_lo8), DGI_ERR_INVALID_ARG, "gemm: one form of low-order block at a time");
    DGI_REQUIRE(!a.A_lo8 || (uintptr_t)a.A_lo8 % 8 == 0, DGI_ERR_INVALID_ARG, "gemm: remainder bytes misaligned");
    DGI_REQUIRE((uintptr_t)a.Wt % 16 == 0 && a.ldw % E == 0 && a.K1p % E == 0, DGI_ERR_INVALID_ARG, "gemm: packed weight misaligned");
    GemmParams p{};
    p.A1 = a.A1; p.ld_a1 = a.ld_a1; p.K1 = a.K1;
    p.a1_vec = ((uintptr_t)a.A1 % 16 == 0) && (a.ld_a1 % E == 0);
    p.A2 = a.K2 > 0 ? a.A2 : nullptr; p.ld_a2 = a.ld_a2; p.K2 = a.K2;
    p.A3 = p.A2 ? a.A3 : nullptr;
    p.a2_vec = p.A2 && ((uintptr_t)a.A2 % 16 == 0) && (a.ld_a2 % E == 0) && ((uintptr_t)p.A3 % 16 == 0);
    p.Wt = a.Wt; p.ldw = a.ldw; p.K1p = a.K1p;
    p.bias = a.bias; p.act = a.act; p.act_slope = a.act_slope;
    p.Y = a.Y; p.ld_y = a.ld_y; p.out_bf16 = a.out_dtype == DGI_BF16;
    p.M = a.M; p.Nout = a.Nout;
    {
        const int ob = p.out_bf16 ? 2 : 4;
        p.y_vec = ((uintptr_t)a.Y % 16 == 0) && ((a.ld_y * ob) % 16 == 0);
    }
    p.out_scale = a.out_scale; p.row0 = a.row0;
    // 128-wide column tiles: a 256-wide tile would read A once but leaves one wavefront per SIMD and measured slower
    if (a.dtype == DGI_BF16) {
        // the weights-stationary kernel where it applies
        if (p.a1_vec && (!p.A2 || p.a2_vec) && (!kTiledBf16 || a.A_lo8)) {
            size_t wb = 0;
            const int sb = stationary_stage_blocks(p, a.A_lo8 != nullptr, &wb);
            if (sb > 0) {
                p.Q = static_cast<const uint8_t*>(a.A_lo8); p.ld_q = p.A2 ? a.ld_a2 : a.ld_a1;
                return launch_stationary(p, sb, wb, stream);
            }
        }
        DGI_REQUIRE(!a.A_lo8, DGI_ERR_UNSUPPORTED, "gemm: remainder bytes need the weights-stationary kernel (ask gemm_stationary_applies first)");
        if (a.Nout <= 64) return launch_cfg<uint16_t, 4, 1, 1, 2>(p, stream);
        if (a.Nout > 128 && a.Nout <= 192) return launch_cfg<uint16_t, 2, 2, 2, 3>(p, stream);
        return launch_cfg<uint16_t, 2, 2, 2, 2>(p, stream);
    }
    if (a.Nout <= 64) return launch_cfg<float, 4, 1, 1, 2>(p, stream);
    if (a.Nout > 128 && a.Nout <= 192) return launch_cfg<float, 2, 2, 2, 3>(p, stream);
    return launch_cfg<float, 2, 2, 2, 2>(p, stream);
}

dgi_status_t launch_pack_weight(const void* W, int dtype, int K, int Nout, void* Wt, int64_t ldw, int koff, hipStream_t stream) {
    const int64_t n = (int64_t)K * Nout;
    if (n == 0) return DGI_OK;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (dtype == DGI_BF16)
        hipLaunchKernelGGL(pack_weight_kernel<uint16_t>, dim3(grid), dim3(256), 0, stream, (const uint16_t*)W, K, Nout, (uint16_t*)Wt, ldw, koff);
    else
        hipLaunchKernelGGL(pack_weight_kernel<float>, dim3(grid), dim3(256), 0, stream, (const float*)W, K, Nout, (float*)Wt, ldw, koff);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

dgi_status_t launch_pack_fragments(const void* Wt, int dtype, int N, int64_t ldw, void* Wf, hipStream_t stream) {
    const int64_t total = (int64_t)fragment_weight_elems(N, ldw);
    if (total == 0) return DGI_OK;
    const int E = dtype == DGI_BF16 ? 8 : 4;
    DGI_REQUIRE(ldw % (2 * E) == 0, DGI_ERR_INVALID_ARG, "pack_fragments: leading dimension must be a multiple of the K step");
    const unsigned grid = (unsigned)std::min<int64_t>((total + 255) / 256, 65536);
    if (dtype == DGI_BF16)
        hipLaunchKernelGGL(pack_fragments_kernel<uint16_t>, dim3(grid), dim3(256), 0, stream, (const uint16_t*)Wt, ldw, N, total, (uint16_t*)Wf);
    else
        hipLaunchKernelGGL(pack_fragments_kernel<float>, dim3(grid), dim3(256), 0, stream, (const float*)Wt, ldw, N, total, (float*)Wf);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

dgi_status_t launch_pack_gat_attn(const float* W, int K, int heads, int F, const float* a_src, const float* a_dst,
                                  float* Wt, int64_t ldw, hipStream_t stream) {
    const int n = K * heads * 2;
    hipLaunchKernelGGL(pack_gat_attn_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, W, K, heads, F, a_src, a_dst, Wt, ldw);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

dgi_status_t launch_fill_zero(void* ptr, uint64_t bytes, hipStream_t stream) {
    if (bytes == 0) return DGI_OK;
    DGI_REQUIRE((uintptr_t)ptr % 4 == 0 && bytes % 4 == 0, DGI_ERR_INVALID_ARG, "fill_zero: needs 4-byte granularity");
    const uint64_t words = bytes / 4;
    uint64_t grid = (words + 255) / 256;
    if (grid > 65536) grid = 65536;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)grid), dim3(256), 0, stream, (uint32_t*)ptr, words);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

dgi_status_t launch_scale_rows(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int width,
                               int elem_bytes, const float* scale, hipStream_t stream) {
    const int64_t n = rows * width;
    if (n == 0) return DGI_OK;
    const int64_t grid = std::min<int64_t>((n + 255) / 256, (int64_t)1 << 22);
    if (elem_bytes == 2)
        hipLaunchKernelGGL(scale_rows_kernel<uint16_t>, dim3((unsigned)grid), dim3(256), 0, stream, (const uint16_t*)in, ld_in,
                           (uint16_t*)out, ld_out, rows, width, scale);
    else
        hipLaunchKernelGGL(scale_rows_kernel<float>, dim3((unsigned)grid), dim3(256), 0, stream, (const float*)in, ld_in,
                           (float*)out, ld_out, rows, width, scale);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

dgi_status_t launch_permute_rows(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int width,
                                 int elem_bytes, const int32_t* perm, bool gather, hipStream_t stream) {
    const int64_t n = rows * width;
    if (n == 0) return DGI_OK;
    if ((width * elem_bytes) % 16 == 0 && (ld_in * elem_bytes) % 16 == 0 && (ld_out * elem_bytes) % 16 == 0 &&
        (uintptr_t)in % 16 == 0 && (uintptr_t)out % 16 == 0) {
        const int chunks = width * elem_bytes / 16;
        const int64_t grid = std::min<int64_t>((rows * chunks + 255) / 256, (int64_t)1 << 22);
        hipLaunchKernelGGL(permute_rows_vec_kernel, dim3((unsigned)grid), dim3(256), 0, stream, (const uint4*)in, ld_in * elem_bytes / 16,
                           (uint4*)out, ld_out * elem_bytes / 16, rows, chunks, perm, gather ? 1 : 0);
        DGI_HIP(hipGetLastError());
        return DGI_OK;
    }
    // a launch may not exceed 2^32 threads in total: cap the grid and stride
    const int64_t grid = std::min<int64_t>((n + 255) / 256, (int64_t)1 << 22);
    if (elem_bytes == 2)
        hipLaunchKernelGGL(permute_rows_kernel<uint16_t>, dim3((unsigned)grid), dim3(256), 0, stream, (const uint16_t*)in, ld_in,
                           (uint16_t*)out, ld_out, rows, width, perm, gather ? 1 : 0);
    else
        hipLaunchKernelGGL(permute_rows_kernel<float>, dim3((unsigned)grid), dim3(256), 0, stream, (const float*)in, ld_in,
                           (float*)out, ld_out, rows, width, perm, gather ? 1 : 0);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

}  // namespace dgi
