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
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
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
    // the output is written once and read much later (by the reduce over shards): streaming stores
    if (loc >= 0 && loc < Vs) {
        const V* t = table + (size_t)loc * row_vecs;
        for (int c = threadIdx.x; c < row_vecs; c += 256) __builtin_nontemporal_store(t[c], o + c);
    } else {
        V z = V(0);
        for (int c = threadIdx.x; c < row_vecs; c += 256) __builtin_nontemporal_store(z, o + c);
    }
}

hipError_t launch_embed_fwd(const void* table, const int64_t* ids, int N, int h, int Vs, int64_t off, int elem_bytes,
                            void* out, hipStream_t st) {
    const int64_t row_bytes = (int64_t)h * elem_bytes;
    ProfScope prof(K_EMBED_FWD, st);
    if (row_bytes % 16 == 0) {
        hipLaunchKernelGGL((embed_fwd_kernel<uintx4>), dim3(N), dim3(256), 0, st, (const uintx4*)table, ids,
                           (int)(row_bytes / 16), Vs, off, (uintx4*)out);
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
__device__ __forceinline__ u64 token_key(const int64_t* __restrict__ ids, int i, int N, int Vs, int64_t off) {
    if (i < N) {
        const int64_t loc = ids[i] - off;
        if (loc >= 0 && loc < Vs) return ((u64)loc << 32) | (u64)(unsigned)i;
    }
    return KEY_NONE;
}

__device__ __forceinline__ void cmp_swap(u64& x, u64& y, bool asc) {
    if ((x > y) == asc) { const u64 t = x; x = y; y = t; }
}

// LEVELS consecutive passes (distances j, j/2, ...) of stage k of the bitonic network on
// LDS-resident keys, done in registers on groups of 2^LEVELS keys: one LDS round trip and one
// barrier instead of LEVELS.  gbase = global index of sh[0]; k > j, so the direction is the
// same for all keys of a group.
template <int LEVELS>
__device__ __forceinline__ void bitonic_levels_lds(u64* sh, int ch, int j, int k, int gbase) {
    constexpr int G = 1 << LEVELS;
    const int low = j >> (LEVELS - 1);          // smallest distance of this group of passes
    for (int t = threadIdx.x; t < ch / G; t += SORT_THREADS) {
        // spread t around the LEVELS index bits low .. j, which enumerate the group
        const int base = ((t & ~(low - 1)) << LEVELS) | (t & (low - 1));
        const bool asc = (((gbase + base) & k) == 0);
        u64 v[G];
#pragma unroll
        for (int e = 0; e < G; ++e) v[e] = sh[base + e * low];
#pragma unroll
        for (int d = G >> 1; d > 0; d >>= 1)
#pragma unroll
            for (int e = 0; e < G; ++e)
                if ((e & d) == 0) cmp_swap(v[e], v[e | d], asc);
#pragma unroll
        for (int e = 0; e < G; ++e) sh[base + e * low] = v[e];
    }
    __syncthreads();
}

// passes j_first, j_first/2, ..., 1 of stage k, three at a time
__device__ __forceinline__ void bitonic_stage_tail_lds(u64* sh, int ch, int j_first, int k, int gbase) {
    int j = j_first;
    for (; j >= 4; j >>= 3) bitonic_levels_lds<3>(sh, ch, j, k, gbase);
    if (j == 2) bitonic_levels_lds<2>(sh, ch, 2, k, gbase);
    else if (j == 1) bitonic_levels_lds<1>(sh, ch, 1, k, gbase);
}

// Workspace after the keys: the positions (in the sorted key array) where a run of equal rows
// starts, in no particular order, and their number.
struct RunList {
    unsigned* starts;   // [n_pad]
    unsigned* count;    // [1]
};

__device__ __forceinline__ bool starts_run(const u64* keys, int s) {
    const u64 k = keys[s];
    return k != KEY_NONE && (s == 0 || (unsigned)(keys[s - 1] >> 32) != (unsigned)(k >> 32));
}

// N <= SORT_CHUNK tokens, one workgroup: the keys of the tokens this shard owns are gathered
// into LDS (only those are sorted: m = next power of two of their number), sorted, written
// back followed by KEY_NONE up to n_pad, and the run starts are listed.
__global__ __launch_bounds__(SORT_THREADS) void embed_sort_single_kernel(const int64_t* __restrict__ ids, int N, int Vs,
                                                                         int64_t off, u64* __restrict__ keys,
                                                                         int n_pad, RunList runs) {
    __shared__ u64 sh[SORT_CHUNK];
    __shared__ int s_owned, s_runs;
    if (threadIdx.x == 0) { s_owned = 0; s_runs = 0; }
    __syncthreads();
    for (int i = threadIdx.x; i < N; i += SORT_THREADS) {
        const u64 k = token_key(ids, i, N, Vs, off);
        if (k != KEY_NONE) sh[atomicAdd(&s_owned, 1)] = k;    // any order: the keys are unique and get sorted
    }
    __syncthreads();
    const int owned = s_owned;
    int m = 2;
    while (m < owned) m <<= 1;
    for (int t = owned + threadIdx.x; t < m; t += SORT_THREADS) sh[t] = KEY_NONE;
    __syncthreads();
    for (int k = 2; k <= m; k <<= 1) bitonic_stage_tail_lds(sh, m, k >> 1, k, 0);
    for (int t = threadIdx.x; t < n_pad; t += SORT_THREADS) keys[t] = t < owned ? sh[t] : KEY_NONE;
    for (int t = threadIdx.x; t < owned; t += SORT_THREADS)
        if (starts_run(sh, t)) runs.starts[atomicAdd(&s_runs, 1)] = (unsigned)t;
    __syncthreads();
    if (threadIdx.x == 0) *runs.count = (unsigned)s_runs;
}

// More tokens than one workgroup sorts: builds the keys of every chunk of `ch` tokens from the
// ids and sorts the chunk (all stages k = 2..ch).  Also clears the run counter.
__global__ __launch_bounds__(SORT_THREADS) void embed_keys_sort_chunks_kernel(const int64_t* __restrict__ ids, int N,
                                                                              int Vs, int64_t off,
                                                                              u64* __restrict__ keys, int ch,
                                                                              RunList runs) {
    __shared__ u64 sh[SORT_CHUNK];
    const int gbase = blockIdx.x * ch;
    if (blockIdx.x == 0 && threadIdx.x == 0) *runs.count = 0u;
    for (int t = threadIdx.x; t < ch; t += SORT_THREADS) sh[t] = token_key(ids, gbase + t, N, Vs, off);
    __syncthreads();
    for (int k = 2; k <= ch; k <<= 1) bitonic_stage_tail_lds(sh, ch, k >> 1, k, gbase);
    for (int t = threadIdx.x; t < ch; t += SORT_THREADS) keys[gbase + t] = sh[t];
}

// Lists the run starts of a fully sorted key array (multi-chunk case).
__global__ __launch_bounds__(256) void embed_find_runs_kernel(const u64* __restrict__ keys, int N, RunList runs) {
    const int s = blockIdx.x * 256 + threadIdx.x;
    if (s < N && starts_run(keys, s)) runs.starts[atomicAdd(runs.count, 1u)] = (unsigned)s;
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
    bitonic_stage_tail_lds(sh, ch, ch >> 1, k, gbase);
    for (int t = threadIdx.x; t < ch; t += SORT_THREADS) keys[gbase + t] = sh[t];
}

// ------------------------------------------------------------------------- backward: segmented sum
// Workgroup (x, y): column slab x, runs y, y + gridDim.y, ... of the run list.  It walks a run
// and adds the gradient rows in key order (increasing token position), starting from the value
// already in the table gradient.  Runs are independent, so their order in the list does not
// matter.  The adds of a column form one serial chain, so the speed comes from the loads: a
// wavefront reads 64 keys of the run at once and keeps DEPTH gradient-row loads in flight
// ahead of the adds.
template <typename T, int VEC>
struct GradVec;
template <> struct GradVec<u16, 4> { typedef uint2 type; };
template <> struct GradVec<u16, 1> { typedef u16 type; };
template <> struct GradVec<float, 4> { typedef float4 type; };
template <> struct GradVec<float, 1> { typedef float type; };

// acc += gradient values; `on` false adds -0.0f instead, which leaves every float (either zero
// included) bit for bit unchanged.
__device__ __forceinline__ float gate(float x, bool on) { return on ? x : -0.0f; }
__device__ __forceinline__ void add_grad(float (&acc)[4], const uint2& v, bool on) {
    acc[0] += gate(__uint_as_float(v.x << 16), on);
    acc[1] += gate(__uint_as_float(v.x & 0xFFFF0000u), on);
    acc[2] += gate(__uint_as_float(v.y << 16), on);
    acc[3] += gate(__uint_as_float(v.y & 0xFFFF0000u), on);
}
__device__ __forceinline__ void add_grad(float (&acc)[1], const u16& v, bool on) {
    acc[0] += gate(__uint_as_float((unsigned)v << 16), on);
}
__device__ __forceinline__ void add_grad(float (&acc)[4], const float4& v, bool on) {
    acc[0] += gate(v.x, on); acc[1] += gate(v.y, on); acc[2] += gate(v.z, on); acc[3] += gate(v.w, on);
}
__device__ __forceinline__ void add_grad(float (&acc)[1], const float& v, bool on) { acc[0] += gate(v, on); }

// Loads of tokens u0 .. u0 + D - 1 of the 64 whose positions sit in the lanes of `tok`, issued
// back to back.  No branches: positions past cnt re-read the last valid row.
template <int D, typename GV, typename T>
__device__ __forceinline__ void load_batch(GV (&v)[D], const T* gcol, int h, unsigned tok, int u0, int cnt) {
#pragma unroll
    for (int u = 0; u < D; ++u) {
        const int idx = (u0 + u < cnt) ? (u0 + u) : (cnt - 1);
        const unsigned t = __builtin_amdgcn_readlane(tok, idx);
        v[u] = *reinterpret_cast<const GV*>(gcol + (size_t)t * h);
    }
}
// The adds of those tokens in order; positions past cnt add -0.0f.
template <int D, int VEC, typename GV>
__device__ __forceinline__ void add_batch(float (&acc)[VEC], const GV (&v)[D], int u0, int cnt) {
#pragma unroll
    for (int u = 0; u < D; ++u) add_grad(acc, v[u], u0 + u < cnt);
}
template <int D, int VEC, typename GV, typename T>
__device__ __forceinline__ void accum_batch(float (&acc)[VEC], const T* gcol, int h, unsigned tok, int u0, int cnt) {
    GV v[D];
    load_batch<D>(v, gcol, h, tok, u0, cnt);
    add_batch<D, VEC>(acc, v, u0, cnt);
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void embed_bwd_accum_kernel(const u64* __restrict__ keys, int n_pad, RunList runs,
                                                              const T* __restrict__ gout, int h,
                                                              float* __restrict__ dtable) {
    typedef typename GradVec<T, VEC>::type GV;
    constexpr int DEPTH = 32;
    const int c0 = (blockIdx.x * 256 + threadIdx.x) * VEC;
    const bool active = c0 < h;
    const int lane = threadIdx.x & 63;
    const int n_runs = (int)*runs.count;
    for (int r = blockIdx.y; r < n_runs; r += gridDim.y) {
    const int s = (int)runs.starts[r];
    const unsigned row = (unsigned)(keys[s] >> 32);

    float acc[VEC];
    float* d = dtable + (size_t)row * h + c0;
    if (active) {
        if (VEC == 4) {
            const float4 v = *reinterpret_cast<const float4*>(d);
            acc[0] = v.x; acc[1 % VEC] = v.y; acc[2 % VEC] = v.z; acc[3 % VEC] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = d[e];
        }
    }
    const T* gcol = gout + (active ? c0 : 0);

    // 64 keys of the run per wavefront-wide load; the keys of the next 64 positions are fetched
    // before this chunk is worked on, so a long run pays one memory latency per 64 tokens (its
    // 64 row loads, all in flight together) instead of three (keys, then two batches of 32)
    u64 kq = (s + lane < n_pad) ? keys[s + lane] : KEY_NONE;
    for (int q0 = s; q0 < n_pad; q0 += 64) {
        const u64 kq_next = (q0 + 64 + lane < n_pad) ? keys[q0 + 64 + lane] : KEY_NONE;
        const bool same = (kq != KEY_NONE) && ((unsigned)(kq >> 32) == row);
        const u64 m = __builtin_amdgcn_ballot_w64(same);
        const int cnt = (m == ~0ull) ? 64 : __builtin_ctzll(~m);   // how many of them continue the run
        const unsigned tok = (unsigned)kq;
        if (active) {
            if (cnt == 64) {
                GV v0[DEPTH], v1[DEPTH];
                load_batch<DEPTH>(v0, gcol, h, tok, 0, 64);
                load_batch<DEPTH>(v1, gcol, h, tok, DEPTH, 64);
                add_batch<DEPTH, VEC>(acc, v0, 0, 64);
                add_batch<DEPTH, VEC>(acc, v1, DEPTH, 64);
            } else {
                int u0 = 0;
                for (; u0 + DEPTH <= cnt; u0 += DEPTH) accum_batch<DEPTH, VEC, GV>(acc, gcol, h, tok, u0, cnt);
                for (; u0 < cnt; u0 += 4) accum_batch<4, VEC, GV>(acc, gcol, h, tok, u0, cnt);
            }
        }
        if (cnt < 64) break;
        kq = kq_next;
    }
    if (active) {
        if (VEC == 4) {
            *reinterpret_cast<float4*>(d) = make_float4(acc[0], acc[1 % VEC], acc[2 % VEC], acc[3 % VEC]);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) d[e] = acc[e];
        }
    }
    }   // runs of this workgroup
}

static int next_pow2(int64_t n) {
    int p = 2;
    while (p < n) p <<= 1;
    return p;
}

size_t embed_bwd_workspace(int64_t N) {
    const size_t n_pad = (size_t)next_pow2(N);
    return n_pad * sizeof(u64) + n_pad * sizeof(unsigned) + 256;
}

static RunList run_list_of(void* ws, int n_pad) {
    RunList r;
    r.starts = (unsigned*)((char*)ws + (size_t)n_pad * sizeof(u64));
    r.count = r.starts + n_pad;
    return r;
}

static hipError_t sort_keys(const int64_t* ids, int N, int Vs, int64_t off, u64* keys, int n_pad, RunList runs,
                            hipStream_t st) {
    ProfScope prof(K_EMBED_SORT, st);
    hipError_t e;
    if (n_pad <= SORT_CHUNK) {
        hipLaunchKernelGGL(embed_sort_single_kernel, dim3(1), dim3(SORT_THREADS), 0, st, ids, N, Vs, off, keys, n_pad,
                           runs);
        return hipGetLastError();
    }
    const int ch = SORT_CHUNK;
    const int chunks = n_pad / ch;
    hipLaunchKernelGGL(embed_keys_sort_chunks_kernel, dim3(chunks), dim3(SORT_THREADS), 0, st, ids, N, Vs, off, keys,
                       ch, runs);
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
    hipLaunchKernelGGL(embed_find_runs_kernel, dim3((unsigned)ceil_div(N, 256)), dim3(256), 0, st, keys, N, runs);
    return hipGetLastError();
}

static hipError_t accumulate_runs(const u64* keys, int n_pad, RunList runs, const void* gout, int N, int h,
                                  int is_bf16, float* dtable, hipStream_t st) {
    ProfScope prof(K_EMBED_ACCUM, st);
    // grid.y workgroups share the runs of the list; enough of them to fill the chip twice over
    const unsigned gy = (unsigned)(N < 1024 ? N : 1024);
    if (is_bf16 && h % 4 == 0) {
        hipLaunchKernelGGL((embed_bwd_accum_kernel<u16, 4>), dim3((unsigned)ceil_div(h, 256 * 4), gy), dim3(256), 0, st,
                           keys, n_pad, runs, (const u16*)gout, h, dtable);
    } else if (is_bf16) {
        hipLaunchKernelGGL((embed_bwd_accum_kernel<u16, 1>), dim3((unsigned)ceil_div(h, 256), gy), dim3(256), 0, st,
                           keys, n_pad, runs, (const u16*)gout, h, dtable);
    } else if (h % 4 == 0) {
        hipLaunchKernelGGL((embed_bwd_accum_kernel<float, 4>), dim3((unsigned)ceil_div(h, 256 * 4), gy), dim3(256), 0,
                           st, keys, n_pad, runs, (const float*)gout, h, dtable);
    } else {
        hipLaunchKernelGGL((embed_bwd_accum_kernel<float, 1>), dim3((unsigned)ceil_div(h, 256), gy), dim3(256), 0, st,
                           keys, n_pad, runs, (const float*)gout, h, dtable);
    }
    return hipGetLastError();
}

hipError_t launch_embed_bwd(const void* gout, const int64_t* ids, int N, int h, int Vs, int64_t off, int is_bf16,
                            float* dtable, void* ws, hipStream_t st) {
    u64* keys = (u64*)ws;
    const int n_pad = next_pow2(N);
    const RunList runs = run_list_of(ws, n_pad);
    hipError_t e;
    if ((e = sort_keys(ids, N, Vs, off, keys, n_pad, runs, st)) != hipSuccess) return e;
    return accumulate_runs(keys, n_pad, runs, gout, N, h, is_bf16, dtable, st);
}

}  // namespace vp
