// Small bandwidth/latency-bound kernels around the GEMMs: softmax statistics, their folds
// (barrier C1 of Algorithm 1), and the D = softmax - G matrix of pass T from stored logits.
#include "vp_internal.h"

namespace vp {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Block-wide reductions over 256 threads with a fixed tree (deterministic).
__device__ __forceinline__ float block_max256(float v, float* sh) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}
__device__ __forceinline__ float block_sum256(float v, float* sh) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// fp32 path, pass S statistics of one shard from its stored logits: one workgroup per row.
__global__ __launch_bounds__(256) void row_stats_f32_kernel(const float* __restrict__ Y, int64_t ldy,
                                                            const int64_t* __restrict__ labels, int64_t off,
                                                            int Vs, float* lmax, float* lsum, float* ltgt) {
    __shared__ float sh[4];
    const int i = blockIdx.x;
    const float* y = Y + (int64_t)i * ldy;
    float m = -INFINITY;
    for (int j = threadIdx.x; j < Vs; j += 256) m = fmaxf(m, y[j]);
    m = block_max256(m, sh);
    float s = 0.f;
    for (int j = threadIdx.x; j < Vs; j += 256) s += expf(y[j] - m);
    s = block_sum256(s, sh);
    if (threadIdx.x == 0) {
        lmax[i] = m;
        lsum[i] = s;
        const int64_t loc = labels[i] - off;
        ltgt[i] = (loc >= 0 && loc < Vs) ? y[loc] : 0.f;
    }
}

hipError_t launch_row_stats_f32(const float* Y, int64_t ldy, const int64_t* labels, int64_t off, int N, int Vs,
                                float* lmax, float* lsum, float* ltgt, hipStream_t st) {
    ProfScope prof(K_ROWSTATS_F32, st);
    hipLaunchKernelGGL(row_stats_f32_kernel, dim3(N), dim3(256), 0, st, Y, ldy, labels, off, Vs, lmax, lsum, ltgt);
    return hipGetLastError();
}

// Fold of the per-column-tile partial (max, sum-exp) pairs of one shard with the same online
// rescaling as the cross-shard fold.  A workgroup folds 64 token rows; wavefront g takes the
// tiles congruent to g mod 4 (independent loads, several in flight), and the four partial
// results meet in LDS in the fixed order g = 0..3.
__global__ __launch_bounds__(256) void fold_partials_kernel(const float* __restrict__ pm, const float* __restrict__ ps,
                                                            const float* __restrict__ pt, int tiles, int N,
                                                            const int64_t* __restrict__ labels, int64_t off, int Vs,
                                                            float* lmax, float* lsum, float* ltgt) {
    __shared__ float xm[4][64], xs[4][64];
    const int g = threadIdx.x >> 6, r = threadIdx.x & 63;
    const int i = blockIdx.x * 64 + r;
    const int ic = i < N ? i : N - 1;
    float m = -INFINITY, s = 0.f;
    int t = g;
    for (; t + 12 < tiles; t += 16) {
        float a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a[u] = pm[(size_t)(t + 4 * u) * N + ic];
            b[u] = ps[(size_t)(t + 4 * u) * N + ic];
        }
        const float mn = fmaxf(fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3])), m);
        s *= __expf(m - mn);          // m = -inf only while s = 0: exp(-inf) = 0
#pragma unroll
        for (int u = 0; u < 4; ++u) s += b[u] * __expf(a[u] - mn);
        m = mn;
    }
    for (; t < tiles; t += 4) {
        const float a = pm[(size_t)t * N + ic], b = ps[(size_t)t * N + ic];
        const float mn = fmaxf(a, m);
        s = s * __expf(m - mn) + b * __expf(a - mn);
        m = mn;
    }
    xm[g][r] = m;
    xs[g][r] = s;
    __syncthreads();
    if (g == 0 && i < N) {
        float mm = fmaxf(fmaxf(xm[0][r], xm[1][r]), fmaxf(xm[2][r], xm[3][r]));
        float ss = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (xm[q][r] > -INFINITY) ss += xs[q][r] * __expf(xm[q][r] - mm);
        lmax[i] = mm;
        lsum[i] = ss;
        const int64_t loc = labels[i] - off;
        ltgt[i] = (loc >= 0 && loc < Vs) ? pt[i] : 0.f;
    }
}

hipError_t launch_fold_partials(const float* pm, const float* ps, const float* pt, int tiles, int N,
                                const int64_t* labels, int64_t off, int Vs, float* lmax, float* lsum, float* ltgt,
                                hipStream_t st) {
    ProfScope prof(K_FOLD, st);
    hipLaunchKernelGGL(fold_partials_kernel, dim3((unsigned)ceil_div(N, 64)), dim3(256), 0, st, pm, ps, pt, tiles, N,
                       labels, off, Vs, lmax, lsum, ltgt);
    return hipGetLastError();
}

// Barrier C1: global max, rescaled sum, per-row loss.  One thread per token row; the mean
// loss is reduced by a second single-workgroup kernel with a fixed tree.
__global__ __launch_bounds__(256) void combine_rows_kernel(const float* __restrict__ lmax, const float* __restrict__ lsum,
                                                           const float* __restrict__ ltgt, int p, int N, float* gmax,
                                                           float* gsum, float* loss_row) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    float m = -INFINITY;
    for (int r = 0; r < p; ++r) m = fmaxf(m, lmax[(size_t)r * N + i]);
    float s = 0.f, t = 0.f;
    for (int r = 0; r < p; ++r) {
        s += lsum[(size_t)r * N + i] * expf(lmax[(size_t)r * N + i] - m);
        t += ltgt[(size_t)r * N + i];
    }
    gmax[i] = m;
    gsum[i] = s;
    if (loss_row) loss_row[i] = m + logf(s) - t;
}

// Mean loss over the N rows by one workgroup: thread t sums rows t, t+1024, ... in order, then
// a fixed tree over the 1024 threads.  Rows are recomputed from the global statistics so that
// the per-row output stays optional.
__global__ __launch_bounds__(1024) void mean_loss_kernel(const float* __restrict__ gmax, const float* __restrict__ gsum,
                                                         const float* __restrict__ ltgt, int p, int N, float* out) {
    __shared__ float sh[16];
    float acc = 0.f;
    for (int i = threadIdx.x; i < N; i += 1024) {
        float t = 0.f;
        for (int r = 0; r < p; ++r) t += ltgt[(size_t)r * N + i];
        acc += gmax[i] + logf(gsum[i]) - t;
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int w = 0; w < 16; ++w) s += sh[w];
        out[0] = s / (float)N;
    }
}

hipError_t launch_combine(const float* lmax, const float* lsum, const float* ltgt, int p, int N, float* gmax,
                          float* gsum, float* loss_row, float* loss_mean, hipStream_t st) {
    ProfScope prof(K_COMBINE, st);
    hipLaunchKernelGGL(combine_rows_kernel, dim3((unsigned)ceil_div(N, 256)), dim3(256), 0, st, lmax, lsum, ltgt, p, N,
                       gmax, gsum, loss_row);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(1024), 0, st, gmax, gsum, ltgt, p, N, loss_mean);
    return hipGetLastError();
}

// D = (exp(Y - m)/sum - G) * scale from stored logits (pass T of Algorithm 1 written with
// the rescale identity of section 4.3 folded in: softmax' * sum' e^{m'-m} / sum = e^{Y-m}/sum).
template <typename T>
__device__ __forceinline__ float ld_as_f32(const T* p);
template <>
__device__ __forceinline__ float ld_as_f32<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ld_as_f32<u16>(const u16* p) { return __uint_as_float((unsigned)(*p) << 16); }

__device__ __forceinline__ void st_from_f32(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_from_f32(u16* p, float v) {
    __bf16 b = (__bf16)v;
    *p = __builtin_bit_cast(u16, b);
}

template <typename T, bool PRECISE>
__global__ __launch_bounds__(256) void dlogits_kernel(const T* Y, T* D,   // may alias (in place)
                                                      const int64_t* __restrict__ labels, int64_t off,
                                                      const float* __restrict__ gmax, const float* __restrict__ gsum,
                                                      float scale, int Vs, int64_t ldy, int64_t ldd) {
    const int i = blockIdx.y;
    const float m = gmax[i];
    const float inv = 1.0f / gsum[i];
    const int64_t loc = labels ? labels[i] - off : (int64_t)-1;
    const T* y = Y + (int64_t)i * ldy;
    T* d = D + (int64_t)i * ldd;
    for (int j = blockIdx.x * 256 + threadIdx.x; j < ldd; j += gridDim.x * 256) {
        if (j >= Vs) {   // padding of the row: zero, because the dH product multiplies it by zero
            st_from_f32(d + j, 0.f);
            continue;
        }
        const float v = ld_as_f32<T>(y + j) - m;
        float pr = (PRECISE ? expf(v) : __expf(v)) * inv;
        if ((int64_t)j == loc) pr -= 1.0f;
        st_from_f32(d + j, pr * scale);
    }
}

// Vector form: one thread per 16 bytes of a row (8 bf16 or 4 fp32); needs Vs % (16/sizeof(T)) == 0.
// Workgroup (x, y): row x, chunks 256 y .. 256 y + 255 of it: no division per thread, and the row's
// statistics and label are the same for the whole workgroup.
template <typename T, bool PRECISE>
__global__ __launch_bounds__(256) void dlogits_vec_kernel(const T* Y, T* D,   // may alias (in place)
                                                          const int64_t* __restrict__ labels, int64_t off,
                                                          const float* __restrict__ gmax, const float* __restrict__ gsum,
                                                          float scale, int chunks_per_row, int Vs, int64_t ldy,
                                                          int64_t ldd) {
    constexpr int E = 16 / (int)sizeof(T);
    const int i = blockIdx.x;
    const int c = blockIdx.y * 256 + threadIdx.x;      // chunk of the row of D: chunks_per_row = ldd / E
    if (c >= chunks_per_row) return;
    const int j0 = c * E;
    if (j0 >= Vs) {   // padding of the row: zero, because the dH product multiplies it by zero
        *reinterpret_cast<uint4*>(D + (int64_t)i * ldd + j0) = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
    const float m = gmax[i];
    const float inv = 1.0f / gsum[i];
    // position of the label inside this chunk, if 0 <= loc < E
    const int64_t loc = labels ? labels[i] - off - j0 : (int64_t)-1;
    const uint4 raw = *reinterpret_cast<const uint4*>(Y + (int64_t)i * ldy + j0);
    const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
    float v[E];
    if (sizeof(T) == 2) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(w[e] << 16);
            v[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = __uint_as_float(w[e]);
    }
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const float x = v[e] - m;
        float pr = (PRECISE ? expf(x) : __expf(x)) * inv;
        if (loc == (int64_t)e) pr -= 1.0f;
        v[e] = pr * scale;
    }
    uint4 o;
    if (sizeof(T) == 2) {
        unsigned q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const __bf16 a = (__bf16)v[2 * e], b = (__bf16)v[2 * e + 1];
            q[e] = (unsigned)__builtin_bit_cast(u16, a) | ((unsigned)__builtin_bit_cast(u16, b) << 16);
        }
        o = make_uint4(q[0], q[1], q[2], q[3]);
    } else {
        o = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[E > 2 ? 2 : 0]),
                       __float_as_uint(v[E > 3 ? 3 : 0]));
    }
    *reinterpret_cast<uint4*>(D + (int64_t)i * ldd + j0) = o;
}

// Zeroes columns Vs .. ldd-1 of every row of the bf16 matrix D (recompute mode: the GEMM
// epilogue that writes D stops at column Vs).
__global__ __launch_bounds__(256) void zero_pad_columns_kernel(u16* D, int N, int Vs, int64_t ldd) {
    const int pad = (int)(ldd - Vs);
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (int64_t)N * pad) return;
    const int i = (int)(t / pad), j = (int)(t - (int64_t)i * pad);
    D[(int64_t)i * ldd + Vs + j] = 0;
}

hipError_t launch_zero_pad_columns(void* D, int N, int Vs, int64_t ldd, hipStream_t st) {
    if (ldd <= Vs) return hipSuccess;
    hipLaunchKernelGGL(zero_pad_columns_kernel, dim3((unsigned)ceil_div((int64_t)N * (ldd - Vs), 256)), dim3(256), 0, st,
                       (u16*)D, N, Vs, ldd);
    return hipGetLastError();
}

hipError_t launch_dlogits(const void* Y, int64_t ldy, void* D, int64_t ldd, int is_bf16, const int64_t* labels,
                          int64_t off, const float* gmax, const float* gsum, float scale, int N, int Vs,
                          hipStream_t st) {
    ProfScope prof(K_DLOGITS_EW, st);
    const int E = is_bf16 ? 8 : 4;
    if (Vs % E == 0 && ldd % E == 0 && ldy % E == 0 && ((((uintptr_t)Y) | ((uintptr_t)D)) & 15u) == 0) {
        const int cpr = (int)(ldd / E);
        const dim3 grid((unsigned)N, (unsigned)ceil_div(cpr, 256));     // rows in x: no 65535 limit on them
        if (is_bf16) {
            hipLaunchKernelGGL((dlogits_vec_kernel<u16, false>), grid, dim3(256), 0, st, (const u16*)Y, (u16*)D, labels,
                               off, gmax, gsum, scale, cpr, Vs, ldy, ldd);
        } else {
            hipLaunchKernelGGL((dlogits_vec_kernel<float, true>), grid, dim3(256), 0, st, (const float*)Y, (float*)D,
                               labels, off, gmax, gsum, scale, cpr, Vs, ldy, ldd);
        }
        return hipGetLastError();
    }
    unsigned gx = (unsigned)ceil_div(ldd, 256);
    if (gx > 64) gx = 64;
    // grid.y carries the row; rows beyond 65535 are covered by launching in slabs
    for (int r0 = 0; r0 < N; r0 += 65535) {
        const int rows = (N - r0 < 65535) ? (N - r0) : 65535;
        const int64_t* lab = labels ? labels + r0 : nullptr;
        if (is_bf16) {
            hipLaunchKernelGGL((dlogits_kernel<u16, false>), dim3(gx, rows), dim3(256), 0, st,
                               (const u16*)Y + (int64_t)r0 * ldy, (u16*)D + (int64_t)r0 * ldd, lab, off,
                               gmax + r0, gsum + r0, scale, Vs, ldy, ldd);
        } else {
            hipLaunchKernelGGL((dlogits_kernel<float, true>), dim3(gx, rows), dim3(256), 0, st,
                               (const float*)Y + (int64_t)r0 * ldy, (float*)D + (int64_t)r0 * ldd, lab, off,
                               gmax + r0, gsum + r0, scale, Vs, ldy, ldd);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Input gradient of Algorithm 2 (section 4.4): dH += (A c - B) scale (OVERWRITE: dH = ...), one thread per
// 4 columns.
template <typename TB, bool OVERWRITE>
__global__ __launch_bounds__(256) void dx_alg2_kernel(const float* __restrict__ A, const TB* __restrict__ Bm,
                                                      const float* __restrict__ lmax, const float* __restrict__ lsum,
                                                      const float* __restrict__ gmax, const float* __restrict__ gsum,
                                                      int h, int64_t total, float scale, float* dH, int vec) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (vec) {
        const int q = h / 4;
        if (t >= total) return;
        const int i = (int)(t / q);
        const int64_t e0 = (int64_t)i * h + (t - (int64_t)i * q) * 4;
        const float ml = lmax[i];
        const float c = (ml > -INFINITY) ? lsum[i] * expf(ml - gmax[i]) / gsum[i] : 0.f;
        const float4 a = *reinterpret_cast<const float4*>(A + e0);
        float b[4];
        if (sizeof(TB) == 2) {
            const uint2 w = *reinterpret_cast<const uint2*>(Bm + e0);
            b[0] = __uint_as_float(w.x << 16); b[1] = __uint_as_float(w.x & 0xFFFF0000u);
            b[2] = __uint_as_float(w.y << 16); b[3] = __uint_as_float(w.y & 0xFFFF0000u);
        } else {
            const float4 w = *reinterpret_cast<const float4*>(Bm + e0);
            b[0] = w.x; b[1] = w.y; b[2] = w.z; b[3] = w.w;
        }
        float4 d = OVERWRITE ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4*>(dH + e0);
        d.x += (a.x * c - b[0]) * scale;
        d.y += (a.y * c - b[1]) * scale;
        d.z += (a.z * c - b[2]) * scale;
        d.w += (a.w * c - b[3]) * scale;
        *reinterpret_cast<float4*>(dH + e0) = d;
    } else {
        if (t >= total) return;
        const int i = (int)(t / h);
        const float ml = lmax[i];
        const float c = (ml > -INFINITY) ? lsum[i] * expf(ml - gmax[i]) / gsum[i] : 0.f;
        dH[t] = (OVERWRITE ? 0.f : dH[t]) + (A[t] * c - ld_as_f32<TB>(Bm + t)) * scale;
    }
}

template <typename TB>
static void launch_dx_alg2_t(const float* A, const TB* B, const float* lmax, const float* lsum, const float* gmax,
                             const float* gsum, int h, int64_t total, float scale, bool overwrite, float* dH, int vec,
                             unsigned blocks, hipStream_t st) {
    if (overwrite)
        hipLaunchKernelGGL((dx_alg2_kernel<TB, true>), dim3(blocks), dim3(256), 0, st, A, B, lmax, lsum, gmax, gsum, h,
                           total, scale, dH, vec);
    else
        hipLaunchKernelGGL((dx_alg2_kernel<TB, false>), dim3(blocks), dim3(256), 0, st, A, B, lmax, lsum, gmax, gsum, h,
                           total, scale, dH, vec);
}

hipError_t launch_dx_alg2(const float* A, const void* B, int b_is_bf16, const float* lmax, const float* lsum,
                          const float* gmax, const float* gsum, int N, int h, float scale, bool overwrite, float* dH,
                          hipStream_t st) {
    ProfScope prof(K_DX_ALG2, st);
    const int vec = (h % 4 == 0) ? 1 : 0;
    const int64_t total = vec ? (int64_t)N * (h / 4) : (int64_t)N * h;
    const unsigned blocks = (unsigned)ceil_div(total, 256);
    if (b_is_bf16)
        launch_dx_alg2_t<u16>(A, (const u16*)B, lmax, lsum, gmax, gsum, h, total, scale, overwrite, dH, vec, blocks, st);
    else
        launch_dx_alg2_t<float>(A, (const float*)B, lmax, lsum, gmax, gsum, h, total, scale, overwrite, dH, vec, blocks, st);
    return hipGetLastError();
}

}  // namespace vp
