// Input (embedding) layer of one vocabulary shard (appendix C of the paper): the gather that
// builds the full-size [N, h] output with zero rows for ids the shard does not own, and the
// scatter-add of the output gradient into the shard's fp32 table gradient.
//
// The scatter-add uses no atomics.  Tokens are keyed by (local row, token position), the keys
// are sorted (bitonic network; keys are unique so the order is total), and every run of equal
// rows is summed by one workgroup in increasing token position, starting from the value
// already in the table gradient.  The result does not depend on scheduling.
#include "vp_internal.h"

namespace vp {

typedef unsigned long long u64;
constexpr u64 KEY_NONE = ~0ull;          // sorts after every real key
constexpr int SORT_CHUNK = 16384;        // keys sorted inside one workgroup's LDS (128 KB)
constexpr int SORT_THREADS = 1024;

// ------------------------------------------------------------------------- forward
// One workgroup per token row; VEC bytes per thread per step.
template <typename V>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const V* __restrict__ table, const int64_t* __restrict__ ids,
                                                        int row_vecs, int Vs, int64_t off, V* __restrict__ out) {
    const int i = blockIdx.x;
    const int64_t loc = ids[i] - off;
    V* o = out + (size_t)i * row_vecs;
    if (loc >= 0 && loc < Vs) {
        const V* t = table + (size_t)loc * row_vecs;
        for (int c = threadIdx.x; c < row_vecs; c += 256) o[c] = t[c];
    } else {
        V z;
        __builtin_memset(&z, 0, sizeof(V));
        for (int c = threadIdx.x; c < row_vecs; c += 256) o[c] = z;
    }
}

hipError_t launch_embed_fwd(const void* table, const int64_t* ids, int N, int h, int Vs, int64_t off, int elem_bytes,
                            void* out, hipStream_t st) {
    const int64_t row_bytes = (int64_t)h * elem_bytes;
    ProfScope prof(K_EMBED_FWD, st);
    if (row_bytes % 16 == 0) {
        hipLaunchKernelGGL((embed_fwd_kernel<uint4>), dim3(N), dim3(256), 0, st, (const uint4*)table, ids,
                           (int)(row_bytes / 16), Vs, off, (uint4*)out);
    } else if (elem_bytes == 4) {
        hipLaunchKernelGGL((embed_fwd_kernel<unsigned>), dim3(N), dim3(256), 0, st, (const unsigned*)table, ids, h, Vs,
                           off, (unsigned*)out);
    } else {
        hipLaunchKernelGGL((embed_fwd_kernel<u16>), dim3(N), dim3(256), 0, st, (const u16*)table, ids, h, Vs, off,
                           (u16*)out);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------- backward: keys + sort
__global__ __launch_bounds__(256) void embed_keys_kernel(const int64_t* __restrict__ ids, int N, int n_pad, int Vs,
                                                         int64_t off, u64* __restrict__ keys) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_pad) return;
    u64 k = KEY_NONE;
    if (i < N) {
        const int64_t loc = ids[i] - off;
        if (loc >= 0 && loc < Vs) k = ((u64)loc << 32) | (u64)(unsigned)i;
    }
    keys[i] = k;
}

// compare-exchange of the bitonic network on LDS-resident keys; gbase = global index of sh[0]
__device__ __forceinline__ void bitonic_pass_lds(u64* sh, int ch, int j, int k, int gbase) {
    for (int t = threadIdx.x; t < ch / 2; t += SORT_THREADS) {
        const int a = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int b = a | j;
        const bool asc = (((gbase + a) & k) == 0);
        const u64 x = sh[a], y = sh[b];
        if ((x > y) == asc) { sh[a] = y; sh[b] = x; }
    }
    __syncthreads();
}

// Sorts every chunk of `ch` keys (ch = power of two <= SORT_CHUNK): all stages k = 2..ch.
__global__ __launch_bounds__(SORT_THREADS) void bitonic_sort_chunks_kernel(u64* __restrict__ keys, int ch) {
    __shared__ u64 sh[SORT_CHUNK];
    const int gbase = blockIdx.x * ch;
    for (int t = threadIdx.x; t < ch; t += SORT_THREADS) sh[t] = keys[gbase + t];
    __syncthreads();
    for (int k = 2; k <= ch; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) bitonic_pass_lds(sh, ch, j, k, gbase);
    for (int t = threadIdx.x; t < ch; t += SORT_THREADS) keys[gbase + t] = sh[t];
}

// One global compare-exchange pass (distance j >= chunk size) of stage k.
__global__ __launch_bounds__(256) void bitonic_global_step_kernel(u64* __restrict__ keys, int half_n, int j, int k) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= half_n) return;
    const int a = ((t & ~(j - 1)) << 1) | (t & (j - 1));
    const int b = a | j;
    const bool asc = ((a & k) == 0);
    const u64 x = keys[a], y = keys[b];
    if ((x > y) == asc) { keys[a] = y; keys[b] = x; }
}

// Finishes stage k inside each chunk: passes j = ch/2 .. 1.
__global__ __launch_bounds__(SORT_THREADS) void bitonic_merge_chunks_kernel(u64* __restrict__ keys, int ch, int k) {
    __shared__ u64 sh[SORT_CHUNK];
    const int gbase = blockIdx.x * ch;
    for (int t = threadIdx.x; t < ch; t += SORT_THREADS) sh[t] = keys[gbase + t];
    __syncthreads();
    for (int j = ch >> 1; j > 0; j >>= 1) bitonic_pass_lds(sh, ch, j, k, gbase);
    for (int t = threadIdx.x; t < ch; t += SORT_THREADS) keys[gbase + t] = sh[t];
}

// ------------------------------------------------------------------------- backward: segmented sum
// Workgroup (x, s): sorted position s, column slab x.  Only the first position of a run of
// equal rows does work: it walks the run and adds the gradient rows in key order.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void embed_bwd_accum_kernel(const u64* __restrict__ keys, int n_pad, int s0,
                                                              const T* __restrict__ gout, int h,
                                                              float* __restrict__ dtable) {
    const int s = s0 + blockIdx.y;
    const u64 key = keys[s];
    if (key == KEY_NONE) return;
    const unsigned row = (unsigned)(key >> 32);
    if (s > 0 && (unsigned)(keys[s - 1] >> 32) == row) return;
    const int c0 = (blockIdx.x * 256 + threadIdx.x) * VEC;
    if (c0 >= h) return;

    float acc[VEC];
    float* d = dtable + (size_t)row * h + c0;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = d[e];

    for (int q = s; q < n_pad; ++q) {
        const u64 kq = keys[q];
        if ((unsigned)(kq >> 32) != row || kq == KEY_NONE) break;
        const unsigned tok = (unsigned)kq;
        const T* g = gout + (size_t)tok * h + c0;
        if (sizeof(T) == 2) {
            if (VEC == 8) {
                const uint4 v = *reinterpret_cast<const uint4*>(g);
                const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[2 * e] += __uint_as_float(w[e] << 16);
                    acc[2 * e + 1] += __uint_as_float(w[e] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] += __uint_as_float((unsigned)((const u16*)g)[e] << 16);
            }
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += ((const float*)g)[e];
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) d[e] = acc[e];
}

static int next_pow2(int64_t n) {
    int p = 2;
    while (p < n) p <<= 1;
    return p;
}

size_t embed_bwd_workspace(int64_t N) { return (size_t)next_pow2(N) * sizeof(u64); }

static hipError_t sort_keys(u64* keys, int n_pad, hipStream_t st) {
    ProfScope prof(K_EMBED_SORT, st);
    hipError_t e;
    const int ch = n_pad < SORT_CHUNK ? n_pad : SORT_CHUNK;
    const int chunks = n_pad / ch;
    hipLaunchKernelGGL(bitonic_sort_chunks_kernel, dim3(chunks), dim3(SORT_THREADS), 0, st, keys, ch);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    for (int64_t k = 2 * (int64_t)ch; k <= n_pad; k <<= 1) {
        for (int64_t j = k >> 1; j >= ch; j >>= 1) {
            hipLaunchKernelGGL(bitonic_global_step_kernel, dim3((unsigned)ceil_div(n_pad / 2, 256)), dim3(256), 0, st,
                               keys, n_pad / 2, (int)j, (int)k);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(bitonic_merge_chunks_kernel, dim3(chunks), dim3(SORT_THREADS), 0, st, keys, ch, (int)k);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

static hipError_t accumulate_runs(const u64* keys, int n_pad, const void* gout, int N, int h, int is_bf16,
                                  float* dtable, hipStream_t st) {
    ProfScope prof(K_EMBED_ACCUM, st);
    hipError_t e;
    // grid.y = sorted position (the first N positions hold every real key), in slabs of 65535
    for (int s0 = 0; s0 < N; s0 += 65535) {
        const int rows = (N - s0 < 65535) ? (N - s0) : 65535;
        if (is_bf16 && h % 8 == 0) {
            hipLaunchKernelGGL((embed_bwd_accum_kernel<u16, 8>), dim3((unsigned)ceil_div(h, 256 * 8), rows), dim3(256),
                               0, st, keys, n_pad, s0, (const u16*)gout, h, dtable);
        } else if (is_bf16) {
            hipLaunchKernelGGL((embed_bwd_accum_kernel<u16, 1>), dim3((unsigned)ceil_div(h, 256), rows), dim3(256), 0,
                               st, keys, n_pad, s0, (const u16*)gout, h, dtable);
        } else if (h % 4 == 0) {
            hipLaunchKernelGGL((embed_bwd_accum_kernel<float, 4>), dim3((unsigned)ceil_div(h, 256 * 4), rows),
                               dim3(256), 0, st, keys, n_pad, s0, (const float*)gout, h, dtable);
        } else {
            hipLaunchKernelGGL((embed_bwd_accum_kernel<float, 1>), dim3((unsigned)ceil_div(h, 256), rows), dim3(256),
                               0, st, keys, n_pad, s0, (const float*)gout, h, dtable);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_embed_bwd(const void* gout, const int64_t* ids, int N, int h, int Vs, int64_t off, int is_bf16,
                            float* dtable, void* ws, hipStream_t st) {
    u64* keys = (u64*)ws;
    const int n_pad = next_pow2(N);
    hipError_t e;
    {
        ProfScope prof(K_EMBED_KEYS, st);
        hipLaunchKernelGGL(embed_keys_kernel, dim3((unsigned)ceil_div(n_pad, 256)), dim3(256), 0, st, ids, N, n_pad,
                           Vs, off, keys);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if ((e = sort_keys(keys, n_pad, st)) != hipSuccess) return e;
    return accumulate_runs(keys, n_pad, gout, N, h, is_bf16, dtable, st);
}

}  // namespace vp
