// Dense fp32 matmul C = A.B on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32),
// for the X.W products of the two-layer GCN (Eq. (1)).  A is tall (one row per
// graph node), B is a small weight matrix.
//
// Block = 4 waves = 128 rows of C by BN = 32*NT columns; each wave owns 32 rows
// and NT 32x32 accumulator tiles.  K is walked in slabs of 32 through two LDS
// buffers.  One 32x32x2 MFMA contracts two k indices; a lane in wave-half hh
// reads four consecutive k (one 128-bit LDS read) and feeds element j to MFMA j,
// so MFMA j contracts {k0+j, k0+4+j} -- A and B use the same pairing, and a sum
// over k does not care about the order.
#include <hip/hip_runtime.h>

#include "cbm_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;
constexpr int BK = 32;
constexpr int LDT = BK + 4;  // padded k-stride of both LDS tiles (floats)

template <int NT>
__global__ __launch_bounds__(256) void cbm_gemm_kernel(int64_t M, int N, int K, const float* __restrict__ A,
                                                       int64_t lda, const float* __restrict__ B, int64_t ldb,
                                                       float* __restrict__ C, int64_t ldc, int vecA) {
    constexpr int BN = 32 * NT;
    extern __shared__ float smem[];
    constexpr int BUF = (BM + BN) * LDT;  // one buffer: A slab [BM][LDT], then B slab transposed [BN][LDT]

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

    // global -> register staging: A slab 128 x 32 (4 float4 per thread), B slab 32 x BN (NT*4 floats per thread)
    float4 ra[4];
    float rb[NT * 4];
    const int a_r = tid >> 3;        // + 32*i
    const int a_k = (tid & 7) * 4;
    auto load_slab = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t r = row0 + a_r + 32 * i;
            const int kk = k0 + a_k;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < M) {
                const float* p = A + r * lda + kk;
                if (vecA && kk + 3 < K) {
                    v = *reinterpret_cast<const float4*>(p);
                } else {
                    if (kk + 0 < K) v.x = p[0];
                    if (kk + 1 < K) v.y = p[1];
                    if (kk + 2 < K) v.z = p[2];
                    if (kk + 3 < K) v.w = p[3];
                }
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < NT * 4; ++i) {
            const int idx = tid + 256 * i;  // over 32 x BN, n fastest
            const int kk = k0 + idx / BN;
            const int n = col0 + idx % BN;
            rb[i] = (kk < K && n < N) ? B[(int64_t)kk * ldb + n] : 0.0f;
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<float4*>(smem + buf * BUF + (a_r + 32 * i) * LDT + a_k) = ra[i];
#pragma unroll
        for (int i = 0; i < NT * 4; ++i) {
            const int idx = tid + 256 * i;
            smem[buf * BUF + BM * LDT + (idx % BN) * LDT + idx / BN] = rb[i];
        }
    };

    const int nslab = (K + BK - 1) / BK;
    load_slab(0);
    store_slab(0);
    __syncthreads();
    for (int s = 0; s < nslab; ++s) {
        const int buf = s & 1;
        if (s + 1 < nslab) load_slab((s + 1) * BK);
        const float* as = smem + buf * BUF + (wave * 32 + l32) * LDT + 4 * hh;
        const float* bs = smem + buf * BUF + BM * LDT + l32 * LDT + 4 * hh;
#pragma unroll
        for (int k8 = 0; k8 < BK; k8 += 8) {
            const float4 a = *reinterpret_cast<const float4*>(as + k8);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float4 b = *reinterpret_cast<const float4*>(bs + t * 32 * LDT + k8);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc[t], 0, 0, 0);
            }
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

template <int NT>
cbm_status launch(int64_t M, int N, int K, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
            hipStream_t stream) {
    constexpr int BN = 32 * NT;
    const size_t smem = 2 * (size_t)(BM + BN) * LDT * sizeof(float);
    const int vecA = (K % 4 == 0 && lda % 4 == 0 && ((uintptr_t)A & 15) == 0) ? 1 : 0;
    static bool lds_opt_in = false;  // buffers above 64 KiB need the per-kernel opt-in, once
    if (smem > 64 * 1024 && !lds_opt_in) {
        hipError_t e = hipFuncSetAttribute((const void*)cbm_gemm_kernel<NT>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) {
            cbm_set_error_detail("hipFuncSetAttribute(MaxDynamicSharedMemorySize)", hipGetErrorString(e));
            return CBM_ERR_HIP;
        }
        lds_opt_in = true;
    }
    dim3 grid((unsigned)((M + BM - 1) / BM), (unsigned)((N + BN - 1) / BN));
    hipLaunchKernelGGL(cbm_gemm_kernel<NT>, grid, dim3(256), smem, stream, M, N, K, A, lda, B, ldb, C, ldc, vecA);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        cbm_set_error_detail("cbm_gemm_kernel launch", hipGetErrorString(e));
        return CBM_ERR_HIP;
    }
    return CBM_OK;
}

}  // namespace

cbm_status cbm_launch_gemm(int64_t M, int32_t N, int32_t K, const float* A, int64_t lda, const float* B, int64_t ldb,
                           float* C, int64_t ldc, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (M == 0 || N == 0) return CBM_OK;
    if (N <= 32) return launch<1>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    if (N <= 64) return launch<2>(M, N, K, A, lda, B, ldb, C, ldc, stream);
    return launch<4>(M, N, K, A, lda, B, ldb, C, ldc, stream);
}
