// Dense fp32 matmul C = A.B on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32),
// for the X.W products of the two-layer GCN (Eq. (1)).  A is tall (one row per
// graph node), B is a small weight matrix.
//
// Block = 4 waves = 128 rows of C by BN = 32*NT columns; each wave owns 32 rows
// and NT 32x32 accumulator tiles.  K is walked in slabs of 32 through two LDS
// buffers; the next slab is fetched into registers while the current one is
// multiplied.  One 32x32x2 MFMA contracts two k indices; a lane in wave-half hh
// takes the four consecutive k = k0+4hh .. k0+4hh+3 and feeds element j to MFMA
// j, so MFMA j contracts {k0+j, k0+4+j} -- A and B use the same pairing, and a
// sum over k does not care about the order.  The A slab is stored [row][k]
// (one 128-bit LDS read per lane and k-group), the B slab [k][n] as it lies in
// memory (four 32-bit reads, conflict-free: a half-wave reads 32 consecutive n).
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "cbm_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;
constexpr int BK = 32;
constexpr int LDA_S = BK + 4;  // padded k-stride of the A slab (floats)

// VEC: K, N, lda, ldb are multiples of 4 and A, B are 16-byte aligned (128-bit global loads);
// otherwise the same slabs are fetched element by element.
template <int NT, bool VEC>
__global__ __launch_bounds__(256) void cbm_gemm_kernel(int64_t M, int N, int K, const float* __restrict__ A,
                                                       int64_t lda, const float* __restrict__ B, int64_t ldb,
                                                       float* __restrict__ C, int64_t ldc) {
    constexpr int BN = 32 * NT;
    constexpr int LDB_S = BN + 4;                       // padded n-stride of the B slab
    constexpr int BUF = BM * LDA_S + BK * LDB_S;        // one buffer: A slab [BM][LDA_S], then B slab [BK][LDB_S]
    constexpr int BV = BK * BN / 4 / 256;               // float4 of the B slab per thread (= NT)
    extern __shared__ float smem[];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int hh = lane >> 5;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    const int col0 = blockIdx.y * BN;

    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    // global -> register staging: A slab 128 x 32 (4 float4 per thread), B slab 32 x BN (NT float4 per thread).
    // Loads are unconditional: addresses are clamped into the matrix; only what would reach a stored
    // output wrongly (k >= K) is zeroed.  Rows >= M and columns >= N feed outputs that are never stored.
    float4 ra[4];
    float4 rb[BV];
    const int a_r = tid >> 3;  // + 32*i
    const int a_k = (tid & 7) * 4;
    // keep[..] = all-ones where the fetched elements lie inside K, else 0: applied with a bitwise AND when the
    // slab is stored, so the loads themselves stay unconditional and all in flight together
    uint32_t keep_a[4][4], keep_b[BV];
    auto load4 = [&](const float* base, int64_t stride, int64_t r, int c, int cmax) -> float4 {
        float4 v;  // four consecutive elements c..c+3 of row r, from clamped (always valid) addresses
        if (VEC) {
            v = *reinterpret_cast<const float4*>(base + r * stride + min(c, cmax - 4));
        } else {
            const float* p = base + r * stride;
            v.x = p[min(c + 0, cmax - 1)];
            v.y = p[min(c + 1, cmax - 1)];
            v.z = p[min(c + 2, cmax - 1)];
            v.w = p[min(c + 3, cmax - 1)];
        }
        return v;
    };
    auto load_slab = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ra[i] = load4(A, lda, min(row0 + a_r + 32 * i, M - 1), k0 + a_k, K);
#pragma unroll
            for (int j = 0; j < 4; ++j) keep_a[i][j] = (k0 + a_k + j < K) ? 0xffffffffu : 0u;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int idx = tid + 256 * i;  // float4 index over 32 x (BN/4), n fastest
            const int kk = k0 + idx / (BN / 4);
            rb[i] = load4(B, ldb, min(kk, K - 1), col0 + (idx % (BN / 4)) * 4, N);
            keep_b[i] = kk < K ? 0xffffffffu : 0u;
        }
    };
    auto masked = [](float v, uint32_t keep) { return __uint_as_float(__float_as_uint(v) & keep); };
    auto store_slab = [&](int buf) {
        float* as = smem + buf * BUF;
        float* bs = as + BM * LDA_S;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 v = make_float4(masked(ra[i].x, keep_a[i][0]), masked(ra[i].y, keep_a[i][1]),
                                         masked(ra[i].z, keep_a[i][2]), masked(ra[i].w, keep_a[i][3]));
            *reinterpret_cast<float4*>(as + (a_r + 32 * i) * LDA_S + a_k) = v;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int idx = tid + 256 * i;
            const float4 v = make_float4(masked(rb[i].x, keep_b[i]), masked(rb[i].y, keep_b[i]),
                                         masked(rb[i].z, keep_b[i]), masked(rb[i].w, keep_b[i]));
            *reinterpret_cast<float4*>(bs + (idx / (BN / 4)) * LDB_S + (idx % (BN / 4)) * 4) = v;
        }
    };

    struct Frag {
        float4 a;
        float b[NT][4];
    };
    const int nslab = (K + BK - 1) / BK;
    load_slab(0);
    store_slab(0);
    __syncthreads();
    for (int s = 0; s < nslab; ++s) {
        const int buf = s & 1;
        if (s + 1 < nslab) load_slab((s + 1) * BK);
        const float* as = smem + buf * BUF + (wave * 32 + l32) * LDA_S + 4 * hh;
        const float* bs = smem + buf * BUF + BM * LDA_S + (4 * hh) * LDB_S + l32;
        auto read_frag = [&](Frag& f, int k8) {
            f.a = *reinterpret_cast<const float4*>(as + k8);
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) f.b[t][j] = bs[(k8 + j) * LDB_S + t * 32];
        };
        auto mma = [&](const Frag& f) {
            // consecutive MFMAs go to different accumulator tiles: no back-to-back dependency
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a.x, f.b[t][0], acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a.y, f.b[t][1], acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a.z, f.b[t][2], acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a.w, f.b[t][3], acc[t], 0, 0, 0);
        };
        // LDS operands of k-group i+1 are fetched while the MFMAs of k-group i run
        Frag f0, f1;
        read_frag(f0, 0);
#pragma unroll
        for (int k8 = 0; k8 < BK; k8 += 16) {
            read_frag(f1, k8 + 8);
            __builtin_amdgcn_sched_barrier(0);
            mma(f0);
            __builtin_amdgcn_sched_barrier(0);
            if (k8 + 16 < BK) read_frag(f0, k8 + 16);
            __builtin_amdgcn_sched_barrier(0);
            mma(f1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (s + 1 < nslab) store_slab(buf ^ 1);
        __syncthreads();
    }

    // accumulator layout of the 32x32 tile: register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int c = col0 + t * 32 + l32;
        if (c >= N) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t r = row0 + wave * 32 + 8 * (v / 4) + 4 * hh + (v % 4);
            if (r < M) C[r * ldc + c] = acc[t][v];
        }
    }
}

// The same product on 16x16 tiles (v_mfma_f32_16x16x4_f32) for weight matrices whose width leaves more than half of
// the last 32-column tile empty (N mod 32 in 1..16; the GCN's 256 x 112 layer: 7 tiles of 16 columns instead of 4 of 32,
// of which the last is half padding).  Block = 4 waves = 128 rows by 16 NT16 columns; a wave owns 32 rows = two
// 16-row halves and 2 NT16 accumulator tiles.  One 16x16x4 MFMA contracts four k: lane l feeds A[row l%16][k l/16] and
// B[k l/16][column l%16].  The slabs lie in LDS as in the kernel above; with an odd NT16 the B slab needs no padding
// (its row stride is 16 mod 32 banks, so the four k rows a wave reads fall on disjoint halves of the banks).
typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int NT16, int H, bool VEC>
__global__ __launch_bounds__(256) void cbm_gemm16_kernel(int64_t M, int N, int K, const float* __restrict__ A, int64_t lda,
                                                         const float* __restrict__ B, int64_t ldb, float* __restrict__ C,
                                                         int64_t ldc) {
    constexpr int BN = 16 * NT16;
    constexpr int BM = 64 * H;                           // a wave owns H halves of 16 rows
    constexpr int LDB_S = BN + ((NT16 & 1) ? 0 : 16);   // row stride = 16 mod 32 words
    constexpr int BUF = BM * LDA_S + BK * LDB_S;
    constexpr int BQ = BK * BN / 4;                      // float4 of the B slab
    constexpr int BV = (BQ + 255) / 256;
    extern __shared__ float smem[];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l16 = lane & 15;
    const int kq = lane >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * BM;
    const int col0 = blockIdx.y * BN;

    floatx4 acc[H][NT16];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int t = 0; t < NT16; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[h][t][v] = 0.0f;

    float4 ra[2 * H];
    float4 rb[BV];
    const int a_r = tid >> 3;
    const int a_k = (tid & 7) * 4;
    uint32_t keep_a[2 * H][4], keep_b[BV];
    auto load4 = [&](const float* base, int64_t stride, int64_t r, int c, int cmax) -> float4 {
        float4 v;  // four consecutive elements c..c+3 of row r, from clamped (always valid) addresses
        if (VEC) {
            v = *reinterpret_cast<const float4*>(base + r * stride + min(c, cmax - 4));
        } else {
            const float* p = base + r * stride;
            v.x = p[min(c + 0, cmax - 1)];
            v.y = p[min(c + 1, cmax - 1)];
            v.z = p[min(c + 2, cmax - 1)];
            v.w = p[min(c + 3, cmax - 1)];
        }
        return v;
    };
    auto load_slab = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2 * H; ++i) {
            ra[i] = load4(A, lda, min(row0 + a_r + 32 * i, M - 1), k0 + a_k, K);
#pragma unroll
            for (int j = 0; j < 4; ++j) keep_a[i][j] = (k0 + a_k + j < K) ? 0xffffffffu : 0u;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int idx = min(tid + 256 * i, BQ - 1);  // float4 index over 32 x (BN/4), n fastest (the last pass is partly idle)
            const int kk = k0 + idx / (BN / 4);
            rb[i] = load4(B, ldb, min(kk, K - 1), col0 + (idx % (BN / 4)) * 4, N);
            keep_b[i] = kk < K ? 0xffffffffu : 0u;
        }
    };
    auto masked = [](float v, uint32_t keep) { return __uint_as_float(__float_as_uint(v) & keep); };
    auto store_slab = [&](int buf) {
        float* as = smem + buf * BUF;
        float* bs = as + BM * LDA_S;
#pragma unroll
        for (int i = 0; i < 2 * H; ++i) {
            const float4 v = make_float4(masked(ra[i].x, keep_a[i][0]), masked(ra[i].y, keep_a[i][1]),
                                         masked(ra[i].z, keep_a[i][2]), masked(ra[i].w, keep_a[i][3]));
            *reinterpret_cast<float4*>(as + (a_r + 32 * i) * LDA_S + a_k) = v;
        }
#pragma unroll
        for (int i = 0; i < BV; ++i) {
            const int idx = tid + 256 * i;
            if (idx < BQ) {
                const float4 v = make_float4(masked(rb[i].x, keep_b[i]), masked(rb[i].y, keep_b[i]),
                                             masked(rb[i].z, keep_b[i]), masked(rb[i].w, keep_b[i]));
                *reinterpret_cast<float4*>(bs + (idx / (BN / 4)) * LDB_S + (idx % (BN / 4)) * 4) = v;
            }
        }
    };

    struct Frag {
        float a[H];
        float b[NT16];
    };
    const int nslab = (K + BK - 1) / BK;
    load_slab(0);
    store_slab(0);
    __syncthreads();
    for (int s = 0; s < nslab; ++s) {
        const int buf = s & 1;
        if (s + 1 < nslab) load_slab((s + 1) * BK);
        const float* as = smem + buf * BUF + (wave * 16 * H + l16) * LDA_S + kq;
        const float* bs = smem + buf * BUF + BM * LDA_S + kq * LDB_S + l16;
        auto read_frag = [&](Frag& f, int k4) {
#pragma unroll
            for (int h = 0; h < H; ++h) f.a[h] = as[h * 16 * LDA_S + k4];
#pragma unroll
            for (int t = 0; t < NT16; ++t) f.b[t] = bs[k4 * LDB_S + t * 16];
        };
        auto mma = [&](const Frag& f) {
#pragma unroll
            for (int t = 0; t < NT16; ++t)  // neighbouring MFMAs write different accumulators
#pragma unroll
                for (int h = 0; h < H; ++h) acc[h][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(f.a[h], f.b[t], acc[h][t], 0, 0, 0);
        };
        Frag f0, f1;
        read_frag(f0, 0);
#pragma unroll
        for (int k4 = 0; k4 < BK; k4 += 8) {
            read_frag(f1, k4 + 4);
            __builtin_amdgcn_sched_barrier(0);
            mma(f0);
            __builtin_amdgcn_sched_barrier(0);
            if (k4 + 8 < BK) read_frag(f0, k4 + 8);
            __builtin_amdgcn_sched_barrier(0);
            mma(f1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (s + 1 < nslab) store_slab(buf ^ 1);
        __syncthreads();
    }

    // accumulator layout of the 16x16 tile: register v of lane l is row 4*(l/16) + v, column l%16
#pragma unroll
    for (int t = 0; t < NT16; ++t) {
        const int c = col0 + t * 16 + l16;
        if (c >= N) continue;
#pragma unroll
        for (int h = 0; h < H; ++h)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t r = row0 + wave * 16 * H + h * 16 + 4 * kq + v;
                if (r < M) C[r * ldc + c] = acc[h][t][v];
            }
    }
}

template <int NT16, int H, bool VEC>
cbm_status launch16(int64_t M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                    hipStream_t stream) {
    constexpr int BN = 16 * NT16;
    constexpr int BMH = 64 * H;
    constexpr int LDB_S = BN + ((NT16 & 1) ? 0 : 16);
    const size_t smem = 2 * (size_t)(BMH * LDA_S + BK * LDB_S) * sizeof(float);  // 64 KiB at NT16 = 7, H = 2
    static bool lds_opt_in = false;
    if (smem > 64 * 1024 && !lds_opt_in) {
        hipError_t e = hipFuncSetAttribute((const void*)cbm_gemm16_kernel<NT16, H, VEC>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) {
            cbm_set_error_detail("hipFuncSetAttribute(MaxDynamicSharedMemorySize)", hipGetErrorString(e));
            return CBM_ERR_HIP;
        }
        lds_opt_in = true;
    }
    dim3 grid((unsigned)((M + BMH - 1) / BMH), (unsigned)((N + BN - 1) / BN));
    hipLaunchKernelGGL((cbm_gemm16_kernel<NT16, H, VEC>), grid, dim3(256), smem, stream, M, N, K, A, lda, B, ldb, C, ldc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        cbm_set_error_detail("cbm_gemm16_kernel launch", hipGetErrorString(e));
        return CBM_ERR_HIP;
    }
    return CBM_OK;
}

// Share of the busiest compute unit's time that is work, if nblocks equal blocks are dealt evenly over the 256 units.
inline double cu_balance(int64_t nblocks) {
    const int64_t per_cu = (nblocks + 255) / 256;
    return (double)nblocks / (256.0 * (double)per_cu);
}

template <int NT16>
cbm_status launch16_nt(int64_t M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, float* C,
                       int64_t ldc, hipStream_t stream) {
    const bool vec = K % 4 == 0 && N % 4 == 0 && lda % 4 == 0 && ldb % 4 == 0 && ((uintptr_t)A & 15) == 0 &&
                     ((uintptr_t)B & 15) == 0 && K >= 4 && N >= 4;
    // blocks of 64 rows where blocks of 128 would leave the compute units unevenly loaded (a few blocks each)
    static const char* env = std::getenv("CBM_GEMM16_ROWS");
    const bool half = env ? std::atoi(env) == 64 : cu_balance((M + 63) / 64) > 1.05 * cu_balance((M + 127) / 128);
    if (half)
        return vec ? launch16<NT16, 1, true>(M, N, K, A, lda, B, ldb, C, ldc, stream)
                   : launch16<NT16, 1, false>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    return vec ? launch16<NT16, 2, true>(M, N, K, A, lda, B, ldb, C, ldc, stream)
               : launch16<NT16, 2, false>(M, N, K, A, lda, B, ldb, C, ldc, stream);
}

template <int NT, bool VEC>
cbm_status launch(int64_t M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                  hipStream_t stream) {
    constexpr int BN = 32 * NT;
    const size_t smem = 2 * (size_t)(BM * LDA_S + BK * (BN + 4)) * sizeof(float);
    static bool lds_opt_in = false;  // buffers above 64 KiB need the per-kernel opt-in, once
    if (smem > 64 * 1024 && !lds_opt_in) {
        hipError_t e = hipFuncSetAttribute((const void*)cbm_gemm_kernel<NT, VEC>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) {
            cbm_set_error_detail("hipFuncSetAttribute(MaxDynamicSharedMemorySize)", hipGetErrorString(e));
            return CBM_ERR_HIP;
        }
        lds_opt_in = true;
    }
    dim3 grid((unsigned)((M + BM - 1) / BM), (unsigned)((N + BN - 1) / BN));
    hipLaunchKernelGGL((cbm_gemm_kernel<NT, VEC>), grid, dim3(256), smem, stream, M, N, K, A, lda, B, ldb, C, ldc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        cbm_set_error_detail("cbm_gemm_kernel launch", hipGetErrorString(e));
        return CBM_ERR_HIP;
    }
    return CBM_OK;
}

template <int NT>
cbm_status launch_nt(int64_t M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, float* C,
                     int64_t ldc, hipStream_t stream) {
    const bool vec = K % 4 == 0 && N % 4 == 0 && lda % 4 == 0 && ldb % 4 == 0 && ((uintptr_t)A & 15) == 0 &&
                     ((uintptr_t)B & 15) == 0 && K >= 4 && N >= 4;
    return vec ? launch<NT, true>(M, N, K, A, lda, B, ldb, C, ldc, stream)
               : launch<NT, false>(M, N, K, A, lda, B, ldb, C, ldc, stream);
}

}  // namespace

cbm_status cbm_launch_gemm(int64_t M, int32_t N, int32_t K, const float* A, int64_t lda, const float* B, int64_t ldb,
                           float* C, int64_t ldc, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (M == 0 || N == 0) return CBM_OK;
    if (K == 0) {  // empty sum: C = 0
        if (hipMemset2DAsync(C, (size_t)ldc * sizeof(float), 0, (size_t)N * sizeof(float), (size_t)M, stream) != hipSuccess)
            return CBM_ERR_HIP;
        return CBM_OK;
    }
    // widths that would leave more than half of the last 32-column tile empty go to the 16-column tiles
    if (N > 32 && N <= 48) return launch16_nt<3>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N > 64 && N <= 80) return launch16_nt<5>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N > 96 && N <= 112) return launch16_nt<7>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N <= 32) return launch_nt<1>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N <= 64) return launch_nt<2>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    return launch_nt<4>(M, N, K, A, lda, B, ldb, C, ldc, stream);
}
