// Dense transform of a layer (the w^l part of Eq. 1) on the MFMA matrix cores, with the bias and the
// activation fused into the epilogue so they run once per node in the producing layer.
//
//   Y[r, n] = act( sum_k A1[r,k] Wt[n,k] + sum_k (A2[r,k] + A3[r,k]) Wt[n,K1p+k] + bias[n] )
//
// A1|A2 is the row-wise concatenation [h_v | m_v] of GraphSAGE (A2 may be absent); A3, when present, is the
// low-order part of an m_v that is stored as a pair of bf16 values (it multiplies the same weight block); Wt is the weight
// packed transposed, [Nout x ldw] with K contiguous, so both MFMA operands are read from LDS rows of
// the same shape.  fp32 data uses v_mfma_f32_32x32x2_f32, bf16 data v_mfma_f32_32x32x16_bf16, both with
// fp32 accumulators.  A workgroup of 4 wavefronts owns a BM x BN output tile; each k-step stages a
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

struct GemmParams {
    const void* A1; int64_t ld_a1; int K1; int a1_vec;
    const void* A2; int64_t ld_a2; int K2; int a2_vec;
    const void* A3;  // optional third block: same shape, leading dimension and weight columns as A2
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
    const int64_t tile_m = blockIdx.x / p.tiles_n;
    const int tile_n = blockIdx.x % p.tiles_n;
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
    uint4 ra[A_CHUNKS], rb[B_CHUNKS];

    auto load_step = [&](int s) {
        const bool second = s >= S1;
        const bool third = s >= S1 + S2;
        const T* A = static_cast<const T*>(third ? p.A3 : second ? p.A2 : p.A1);
        const int64_t lda = second ? p.ld_a2 : p.ld_a1;
        const int K = second ? p.K2 : p.K1;
        const bool vec = second ? p.a2_vec : p.a1_vec;
        const int k0 = (third ? s - S1 - S2 : second ? s - S1 : s) * BK;
        const int wcol = second ? p.K1p : 0;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + 256 * i;
            ra[i] = load_chunk<T>(A, lda, m0 + c / 8, p.M, k0 + (c % 8) * E, K, vec);
        }
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

    if (S > 0) {
        load_step(0);
        store_step();
    }
    __syncthreads();
    const int lrow = lane & 31, lhalf = lane >> 5;
    for (int s = 0; s < S; ++s) {
        if (s + 1 < S) load_step(s + 1);
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
        __syncthreads();
        if (s + 1 < S) {
            store_step();
            __syncthreads();
        }
    }

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
    hipLaunchKernelGGL((gemm_kernel<T, WGM, WGN, TM, TN>), dim3((unsigned)grid), dim3(256), 0, stream, p);
    DGI_HIP(hipGetLastError());
    return DGI_OK;
}

}  // namespace

dgi_status_t launch_gemm(const GemmArgs& a, hipStream_t stream) {
    if (a.M <= 0 || a.Nout <= 0) return DGI_OK;
    const int eb = a.dtype == DGI_BF16 ? 2 : 4, E = 16 / eb;
    DGI_REQUIRE(a.A1 && a.Wt && a.Y, DGI_ERR_INVALID_ARG, "gemm: null operand");
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
