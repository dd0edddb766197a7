// fp32 path of the output layer: a plain LDS-tiled FMA GEMM with arbitrary operand strides.
// It serves the fp32 configuration, where the products must be true fp32 contractions
// (no bf16 operands), and doubles as the simple reference shape of the three products of
// section 4.2:  Y = X W^T,  dX += D W,  dW = D^T X.
//
// C[m, n] (+)= sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk]
// 64x64 output tile per 256-thread workgroup, 4x4 outputs per thread, K step 16.
//
// Small outputs with a long K (dX of the tiny configuration: 128 x 256 outputs, K = 4096) would
// occupy a handful of compute units.  With scratch memory the K range is cut into S slices
// (grid.z); every slice writes its partial tile to scratch[z], and a second kernel adds the S
// partials in ascending z (a fixed order: results repeat bit for bit).
#include "vp_internal.h"

namespace vp {

constexpr int FT = 64, FK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t sam, int64_t sak,
                                                       const float* __restrict__ B, int64_t sbn, int64_t sbk,
                                                       float* __restrict__ C, int64_t ldc, int M, int N, int K,
                                                       int accumulate, int k_per_slice, int64_t slice_stride) {
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

    // slice z of the K range; with one slice this is all of K and C is the real output
    const int k_begin = blockIdx.z * k_per_slice;
    const int k_end = min(K, k_begin + k_per_slice);
    C += (int64_t)blockIdx.z * slice_stride;
    for (int k0 = k_begin; k0 < k_end; k0 += FK) {
        // 64 x 16 elements per operand, 4 per thread; pick the index order that walks the
        // contiguous dimension of the operand with consecutive threads
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + 256 * i;
            int r, k;
            if (sak == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
            const int gm = m0 + r, gk = k0 + k;
            sA[k][r] = (gm < M && gk < k_end) ? A[(int64_t)gm * sam + (int64_t)gk * sak] : 0.f;
            if (sbk == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
            const int gn = n0 + r;
            const int gk2 = k0 + k;
            sB[k][r] = (gn < N && gk2 < k_end) ? B[(int64_t)gn * sbn + (int64_t)gk2 * sbk] : 0.f;
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

// C (+)= sum over the S partial matrices [M, N] in scratch, ascending slice index
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int S, int64_t MN, int N,
                                                            float* __restrict__ C, int64_t ldc, int accumulate) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= MN) return;
    float acc = part[t];
    for (int z = 1; z < S; ++z) acc += part[(int64_t)z * MN + t];
    float* c = C + (t / N) * ldc + (t % N);
    *c = accumulate ? (*c + acc) : acc;
}

// K slices for an [M, N] output: enough workgroups to cover the chip, slices of at least 64.
static int splitk_slices(int M, int N, int K) {
    const int64_t tiles = ceil_div(M, FT) * ceil_div(N, FT);
    int64_t S = 256 / tiles;
    if (S > 32) S = 32;
    if (S > K / 64) S = K / 64;
    return S < 2 ? 1 : (int)S;
}

size_t gemm_f32_scratch_floats(int64_t M, int64_t N, int64_t K) {
    const int S = splitk_slices((int)M, (int)N, (int)K);
    return S > 1 ? (size_t)S * (size_t)M * (size_t)N : 0;
}

hipError_t launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* B, int64_t sbn, int64_t sbk,
                           float* C, int64_t ldc, int M, int N, int K, bool accumulate, float* scratch,
                           hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
    dim3 grid((unsigned)ceil_div(N, FT), (unsigned)ceil_div(M, FT));
    if (grid.y > 65535u) return hipErrorInvalidValue;
    ProfScope prof(K_GEMM_F32, st);
    const int S = scratch ? splitk_slices(M, N, K) : 1;
    if (S > 1) {
        const int kps = (int)(ceil_div(ceil_div(K, S), FK) * FK);     // multiple of the K step
        grid.z = (unsigned)ceil_div(K, kps);
        const int64_t MN = (int64_t)M * N;
        hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, A, sam, sak, B, sbn, sbk, scratch, (int64_t)N, M, N, K,
                           0, kps, MN);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)ceil_div(MN, 256)), dim3(256), 0, st, scratch,
                           (int)grid.z, MN, N, C, ldc, accumulate ? 1 : 0);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, A, sam, sak, B, sbn, sbk, C, ldc, M, N, K,
                       accumulate ? 1 : 0, K, (int64_t)0);
    return hipGetLastError();
}

}  // namespace vp
