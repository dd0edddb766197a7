// fp32 path of the output layer: a plain LDS-tiled FMA GEMM with arbitrary operand strides.
// It serves the fp32 configuration, where the products must be true fp32 contractions
// (no bf16 operands), and doubles as the simple reference shape of the three products of
// section 4.2:  Y = X W^T,  dX += D W,  dW = D^T X.
//
// C[m, n] (+)= sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk]
// 64x64 output tile per 256-thread workgroup, 4x4 outputs per thread, K step 16.
#include "vp_internal.h"

namespace vp {

constexpr int FT = 64, FK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t sam, int64_t sak,
                                                       const float* __restrict__ B, int64_t sbn, int64_t sbk,
                                                       float* __restrict__ C, int64_t ldc, int M, int N, int K,
                                                       int accumulate) {
    __shared__ float sA[FK][FT + 1];
    __shared__ float sB[FK][FT + 1];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += FK) {
        // 64 x 16 elements per operand, 4 per thread; pick the index order that walks the
        // contiguous dimension of the operand with consecutive threads
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + 256 * i;
            int r, k;
            if (sak == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
            const int gm = m0 + r, gk = k0 + k;
            sA[k][r] = (gm < M && gk < K) ? A[(int64_t)gm * sam + (int64_t)gk * sak] : 0.f;
            if (sbk == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
            const int gn = n0 + r;
            const int gk2 = k0 + k;
            sB[k][r] = (gn < N && gk2 < K) ? B[(int64_t)gn * sbn + (int64_t)gk2 * sbk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < FK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sA[k][ty + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = sB[k][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty + 16 * i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx + 16 * j;
            if (gn < N) {
                float* c = C + (int64_t)gm * ldc + gn;
                *c = accumulate ? (*c + acc[i][j]) : acc[i][j];
            }
        }
    }
}

hipError_t launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* B, int64_t sbn, int64_t sbk,
                           float* C, int64_t ldc, int M, int N, int K, bool accumulate, hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
    dim3 grid((unsigned)ceil_div(N, FT), (unsigned)ceil_div(M, FT));
    if (grid.y > 65535u) return hipErrorInvalidValue;
    ProfScope prof(K_GEMM_F32, st);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, A, sam, sak, B, sbn, sbk, C, ldc, M, N, K,
                       accumulate ? 1 : 0);
    return hipGetLastError();
}

}  // namespace vp
