// Dense fp32 matmul C = A.B on the gfx950 matrix cores, for the X.W products of
// the two-layer GCN (Eq. (1)).  A is tall (one row per graph node), B is a small
// weight matrix.  Three kernels: tall products whose weight panel fits in LDS take
// the panel-resident kernel further down (cbm_gemm_panel_kernel); the rest are
// staged through LDS slabs, on 32x32x2 tiles (first kernel) or 16x16x4 tiles.
//
// First kernel (v_mfma_f32_32x32x2_f32):
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

#include <algorithm>
#include <cstdlib>
#include <type_traits>

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

// Third form, for tall A against a weight panel that fits in LDS (K rows by up to 128 columns, 160 KiB): the panel is loaded
// once per block and stays; the waves then run free of one another, each streaming its own rows of A straight from memory
// into MFMA operand registers (no LDS staging of A, no barrier in the loop).  One block of 8 waves per compute unit
// (twelve were measured slower: fewer whole groups per wave, more of the work in narrow chunks).
// Work comes in groups of 32 rows.  Every wave takes the same number of whole groups (a contiguous run of rows, all
// column tiles of the panel); the groups left over, fewer than there are waves, are cut into chunks of column tiles and
// spread over the waves, at most one chunk each, so the waves end (nearly) together whatever M is.
// One 16x16x4 MFMA contracts four k: lane (c = l%16, q = l/16) holds A[row c][k0 + 4q .. 4q+3] of a group of 16 k as one
// 128-bit load and feeds element e to MFMA e, which therefore contracts k0 + 4q + e over q; the B operand of MFMA e is
// panel[k0 + 4q + e][16t + c].  The panel's row stride (16 NT16 + 4 floats) puts q and q+1 on disjoint halves of the banks.
// Loads of A run four groups of 16 k ahead through a ring of registers and are unconditional (addresses clamped into the
// matrix; what lies beyond K is zeroed when used, rows beyond M are never stored).
constexpr int WPB = 8;  // waves per block of the panel kernel

template <int NT16>
__global__ __launch_bounds__(64 * WPB) void cbm_gemm_panel_kernel(int64_t M, int N, int K, int Kp, const float* __restrict__ A, int64_t lda,
                                                             const float* __restrict__ B, int64_t ldb, float* __restrict__ C,
                                                             int64_t ldc) {
    constexpr int BN = 16 * NT16;
    constexpr int LDB = BN + 4;
    extern __shared__ float smem[];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: what follows from it stays in scalar registers
    const int lane = tid & 63;
    const int c = lane & 15;
    const int q = lane >> 4;
    const int nkg = Kp / 16;  // groups of 16 k; Kp is a multiple of 64
    const int64_t G = (M + 31) / 32;
    const int64_t nwaves = (int64_t)gridDim.x * WPB;
    const int64_t gw = (int64_t)blockIdx.x * WPB + wave;
    const int npanels = (N + BN - 1) / BN;

    // groups [g_begin, g_end) of 32 rows, NTL column tiles from tile0 on, of the panel at column col0
    // RING groups of 16 k are in flight per wave (nkg is a multiple of RING)
    auto groups = [&](auto ntl_tag, auto ring_tag, int64_t g_begin, int64_t g_end, int tile0, int col0) {
        constexpr int NTL = decltype(ntl_tag)::value;
        constexpr int RING = decltype(ring_tag)::value;
        float4 ring[RING][2];
        const float* arow[2];  // this lane's two rows of the group being loaded from
        auto set_rows = [&](int64_t g) {
#pragma unroll
            for (int h = 0; h < 2; ++h) arow[h] = A + min(32 * g + 16 * h + c, M - 1) * lda;
        };
        auto issue = [&](int j, int kg) {
            const int k = min(16 * kg + 4 * q, K - 4);
#pragma unroll
            for (int h = 0; h < 2; ++h) ring[j][h] = *reinterpret_cast<const float4*>(arow[h] + k);
        };
        set_rows(g_begin);
#pragma unroll
        for (int j = 0; j < RING; ++j) {
            issue(j, j);
            __builtin_amdgcn_sched_barrier(0);  // in this order: the loop waits for the slots oldest first
        }
        const float* bcol = smem + 4 * q * LDB + 16 * tile0 + c;

        for (int64_t g = g_begin; g < g_end; ++g) {
            floatx4 acc[2][NTL];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int t = 0; t < NTL; ++t)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[h][t][v] = 0.0f;

            for (int kg0 = 0; kg0 < nkg; kg0 += RING) {
                const bool last = kg0 + RING == nkg;
                if (last) set_rows(min(g + 1, G - 1));  // the refills of the last pass belong to the next group
#pragma unroll
                for (int j = 0; j < RING; ++j) {
                    const int kg = kg0 + j;
                    const uint32_t keep = (16 * kg + 4 * q < K) ? 0xffffffffu : 0u;
                    float a[2][4];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        a[h][0] = __uint_as_float(__float_as_uint(ring[j][h].x) & keep);
                        a[h][1] = __uint_as_float(__float_as_uint(ring[j][h].y) & keep);
                        a[h][2] = __uint_as_float(__float_as_uint(ring[j][h].z) & keep);
                        a[h][3] = __uint_as_float(__float_as_uint(ring[j][h].w) & keep);
                    }
                    issue(j, last ? j : kg + RING);  // refill the slot: RING groups of k ahead
                    const float* bb = bcol + 16 * kg * LDB;
                    float bf[2][NTL];
#pragma unroll
                    for (int t = 0; t < NTL; ++t) bf[0][t] = bb[16 * t];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (e < 3) {
#pragma unroll
                            for (int t = 0; t < NTL; ++t) bf[(e + 1) & 1][t] = bb[(e + 1) * LDB + 16 * t];
                        }
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int t = 0; t < NTL; ++t) {
                            acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0][e], bf[e & 1][t], acc[0][t], 0, 0, 0);
                            acc[1][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1][e], bf[e & 1][t], acc[1][t], 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }

            // accumulator layout of the 16x16 tile: register v of lane l is row 4*(l/16) + v, column l%16
            const bool rows_inside = 32 * g + 32 <= M;  // wave-uniform: only the last group of the matrix can be ragged
#pragma unroll
            for (int t = 0; t < NTL; ++t) {
                const int col = col0 + 16 * (tile0 + t) + c;
                if (col >= N) continue;
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int64_t r = 32 * g + 16 * h + 4 * q + v;
                        if (rows_inside || r < M) C[r * ldc + col] = acc[h][t][v];
                    }
            }
        }
    };

    // Two panels: the blocks split into two sets that work side by side, one panel each, on all rows (sets alternate every
    // 8 blocks, so the two blocks that stream the same rows of A at the same time share an XCD and its L2).  One panel, or
    // more than two: every block takes the panels one after the other.
    const bool side_by_side = npanels == 2 && gridDim.x % 16 == 0;
    const int64_t nw = side_by_side ? nwaves / 2 : nwaves;  // waves that share a panel's rows
    const int64_t gwp = side_by_side ? ((int64_t)(blockIdx.x / 16) * 8 + blockIdx.x % 8) * WPB + wave : gw;
    const int p_begin = side_by_side ? (int)(blockIdx.x / 8) % 2 : 0;
    const int p_end = side_by_side ? p_begin + 1 : npanels;
    for (int p = p_begin; p < p_end; ++p) {
        const int col0 = p * BN;
        const int ntp = min(NT16, (N - col0 + 15) / 16);  // column tiles of this panel that hold columns of C
        if (p > p_begin) __syncthreads();                  // every wave is done with the previous panel
        // the panel: eight 128-bit loads per thread in flight at a time, from clamped addresses; what lies outside B is zeroed
        constexpr int FILL = 8;
        const int total = Kp * (BN / 4);
        for (int base = tid; base < total; base += 64 * WPB * FILL) {
            float4 v[FILL];
#pragma unroll
            for (int u = 0; u < FILL; ++u) {
                const int idx = min(base + 64 * WPB * u, total - 1);
                const int k = idx / (BN / 4), col = col0 + (idx % (BN / 4)) * 4;
                v[u] = *reinterpret_cast<const float4*>(B + (int64_t)min(k, K - 1) * ldb + min(col, N - 4));  // N % 4 == 0
                if (k >= K || col >= N) v[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
#pragma unroll
            for (int u = 0; u < FILL; ++u) {
                const int idx = base + 64 * WPB * u;
                if (idx < total) *reinterpret_cast<float4*>(smem + (idx / (BN / 4)) * LDB + (idx % (BN / 4)) * 4) = v[u];
            }
        }
        __syncthreads();

        const int64_t each = G / nw;  // whole groups per wave
        const int64_t left0 = each * nw;
        // The groups left over (fewer than there are waves) are cut into chunks of 1, 2, 4 or all column tiles: the
        // smallest chunk that still gives no wave more than one.  They go first: a narrow chunk waits on memory more
        // than it computes (so it keeps more of K in flight), and the wave it shares its SIMD with has whole groups to
        // fill the matrix pipe meanwhile.  The chunks are spread evenly over the blocks (every stride-th wave takes one).
        int chunk = NT16;
        if ((G - left0) * ntp <= nw) chunk = 1;
        else if (NT16 > 2 && (G - left0) * ((ntp + 1) / 2) <= nw) chunk = 2;
        else if (NT16 > 4 && (G - left0) * ((ntp + 3) / 4) <= nw) chunk = 4;
        const int nchunks = (ntp + chunk - 1) / chunk;
        const int64_t ntasks = (G - left0) * nchunks;
        const int64_t stride = ntasks > 0 ? nw / ntasks : 1;
        if (gwp % stride == 0 && gwp / stride < ntasks) {
            const int64_t task = gwp / stride;
            const int64_t g = left0 + task / nchunks;
            const int t = min((int)(task % nchunks) * chunk, NT16 - chunk);  // (a last chunk that would overhang moves left)
            if (chunk == 1) {
                if (nkg % 16 == 0)
                    groups(std::integral_constant<int, 1>{}, std::integral_constant<int, 16>{}, g, g + 1, t, col0);
                else if (nkg % 8 == 0)
                    groups(std::integral_constant<int, 1>{}, std::integral_constant<int, 8>{}, g, g + 1, t, col0);
                else
                    groups(std::integral_constant<int, 1>{}, std::integral_constant<int, 4>{}, g, g + 1, t, col0);
            } else if (NT16 > 2 && chunk == 2) {
                if (nkg % 8 == 0)
                    groups(std::integral_constant<int, (NT16 > 2 ? 2 : 1)>{}, std::integral_constant<int, 8>{}, g, g + 1, t, col0);
                else
                    groups(std::integral_constant<int, (NT16 > 2 ? 2 : 1)>{}, std::integral_constant<int, 4>{}, g, g + 1, t, col0);
            } else if (NT16 > 4 && chunk == 4) {
                groups(std::integral_constant<int, (NT16 > 4 ? 4 : 1)>{}, std::integral_constant<int, 4>{}, g, g + 1, t, col0);
            } else {
                groups(std::integral_constant<int, NT16>{}, std::integral_constant<int, 4>{}, g, g + 1, 0, col0);
            }
        }
        if (each > 0)
            groups(std::integral_constant<int, NT16>{}, std::integral_constant<int, 4>{}, gwp * each, (gwp + 1) * each, 0, col0);
    }
}

// LDS bytes of the resident panel, or 0 if this product cannot take the panel kernel.
inline size_t panel_lds_bytes(int64_t M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, int* nt16) {
    const bool vec = K % 4 == 0 && N % 4 == 0 && lda % 4 == 0 && ldb % 4 == 0 && ((uintptr_t)A & 15) == 0 &&
                     ((uintptr_t)B & 15) == 0 && K >= 4 && N >= 4;
    if (!vec || N < 16) return 0;
    const int tiles = (N + 15) / 16, npanels = (tiles + 7) / 8;
    *nt16 = (tiles + npanels - 1) / npanels;  // panels of equal width, at most 128 columns
    const int64_t Kp = ((int64_t)K + 63) / 64 * 64;
    const size_t bytes = (size_t)Kp * (16 * *nt16 + 4) * sizeof(float);
    return bytes <= 160 * 1024 ? bytes : 0;
}

template <int NT16>
cbm_status launch_panel(int64_t M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                        size_t smem, hipStream_t stream) {
    static size_t lds_opt_in = 0;  // buffers above 64 KiB need the per-kernel opt-in; raised when a larger one comes
    if (smem > 64 * 1024 && smem > lds_opt_in) {
        hipError_t e = hipFuncSetAttribute((const void*)cbm_gemm_panel_kernel<NT16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) {
            cbm_set_error_detail("hipFuncSetAttribute(MaxDynamicSharedMemorySize)", hipGetErrorString(e));
            return CBM_ERR_HIP;
        }
        lds_opt_in = smem;
    }
    const int Kp = (K + 63) / 64 * 64;
    hipLaunchKernelGGL((cbm_gemm_panel_kernel<NT16>), dim3(256), dim3(64 * WPB), smem, stream, M, N, K, Kp, A, lda, B, ldb, C, ldc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        cbm_set_error_detail("cbm_gemm_panel_kernel launch", hipGetErrorString(e));
        return CBM_ERR_HIP;
    }
    return CBM_OK;
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
    {   // tall A, a weight panel that fits in LDS: the panel-resident kernel
        static const char* env = std::getenv("CBM_GEMM_PANEL_MIN_ROWS");
        const int64_t min_rows = env ? std::atoll(env) : 8192;
        int nt16 = 0;
        const size_t smem = M >= min_rows ? panel_lds_bytes(M, N, K, A, lda, B, ldb, &nt16) : 0;
        if (smem) {
            switch (nt16) {
                case 1: return launch_panel<1>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
                case 2: return launch_panel<2>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
                case 3: return launch_panel<3>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
                case 4: return launch_panel<4>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
                case 5: return launch_panel<5>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
                case 6: return launch_panel<6>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
                case 7: return launch_panel<7>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
                default: return launch_panel<8>(M, N, K, A, lda, B, ldb, C, ldc, smem, stream);
            }
        }
    }
    // widths that would leave more than half of the last 32-column tile empty go to the 16-column tiles
    if (N > 32 && N <= 48) return launch16_nt<3>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N > 64 && N <= 80) return launch16_nt<5>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N > 96 && N <= 112) return launch16_nt<7>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N <= 32) return launch_nt<1>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N <= 64) return launch_nt<2>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    return launch_nt<4>(M, N, K, A, lda, B, ldb, C, ldc, stream);
}
