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

template <int VEC>
__device__ __forceinline__ void load_acc(float (&acc)[VEC], const float* d) {
    if (VEC == 2) {
        const float2 v = *reinterpret_cast<const float2*>(d);
        acc[0] = v.x; acc[1 % VEC] = v.y;
    } else {
        acc[0] = d[0];
    }
}
template <int VEC>
__device__ __forceinline__ void store_acc(float* d, const float (&acc)[VEC]) {
    if (VEC == 2) *reinterpret_cast<float2*>(d) = make_float2(acc[0], acc[1 % VEC]);
    else d[0] = acc[0];
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
__device__ __forceinline__ void add_grad(float (&acc)[2], const unsigned& v, bool on) {
    acc[0] += gate(__uint_as_float(v << 16), on);
    acc[1] += gate(__uint_as_float(v & 0xFFFF0000u), on);
}
__device__ __forceinline__ void add_grad(float (&acc)[2], const float2& v, bool on) {
    acc[0] += gate(v.x, on); acc[1] += gate(v.y, on);
}

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


// ------------------------------------------------------------------------- backward: one kernel for N <= 8192
// Up to FUSED_MAX_N tokens and FUSED_MAX_VS rows: one launch does everything.  EVERY workgroup (1024 threads, one per
// compute unit) builds and sorts the shard's keys in its own LDS - the same few microseconds in all of them, instead
// of a sort kernel, a round trip of the keys through memory and a second launch - numbers the runs of equal rows,
// and then takes its share of the sums: workgroup (slab, group) covers 64 * VEC columns; its 16 wavefronts take the
// short runs group * 16 + w, + groups * 16, ... (four at a time while they have at most four tokens; all row loads
// in flight before the first add), and together the long runs of the group: wavefront w fetches the rows of tokens
// B w .. B w + B - 1 of a chunk of 16 B, and the running sum passes from wavefront 0 to 15 through LDS, so the adds of
// a column still happen in token order and the result equals the in-order loop bit for bit.
constexpr int FUSED_MAX_N = 8192;
constexpr int TOKEN_BITS = 13;                       // a key: local row << 13 | token position
constexpr int FUSED_MAX_VS = (1 << (32 - TOKEN_BITS)) - 1;   // so that no key equals KEY32_NONE
constexpr unsigned KEY32_NONE = 0xFFFFFFFFu;
constexpr int FUSED_THREADS = 1024;
constexpr int FUSED_WAVES = FUSED_THREADS / 64;
constexpr int WAVE_KEYS = 512;                       // eight consecutive keys per lane

__device__ __forceinline__ unsigned token_key32(const int64_t* __restrict__ ids, int i, int N, int Vs, int64_t off) {
    if (i < N) {
        const int64_t loc = ids[i] - off;
        if (loc >= 0 && loc < Vs) return ((unsigned)loc << TOKEN_BITS) | (unsigned)i;
    }
    return KEY32_NONE;
}
__device__ __forceinline__ unsigned key_row(unsigned k) { return k >> TOKEN_BITS; }
__device__ __forceinline__ unsigned key_token(unsigned k) { return k & ((1u << TOKEN_BITS) - 1u); }

__device__ __forceinline__ void order(unsigned& x, unsigned& y, bool asc) {
    const unsigned lo = x < y ? x : y, hi = x < y ? y : x;
    x = asc ? lo : hi;
    y = asc ? hi : lo;
}

// The value lane ^ X holds.  X = 1, 2, 8: one DPP move (quad_perm [1,0,3,2], [2,3,0,1], row_ror:8); X = 4: row_shl:4
// for the lanes with bit 2 clear and row_shr:4 for the others (bank masks 0x5 / 0xA); across rows of 16: ds_bpermute.
template <int X>
__device__ __forceinline__ unsigned lane_xor(unsigned x) {
    const int v = (int)x;
    if (X == 1) return (unsigned)__builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false);
    if (X == 2) return (unsigned)__builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false);
    if (X == 4) {
        const int a = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xF, 0x5, false);
        return (unsigned)__builtin_amdgcn_update_dpp(a, v, 0x114, 0xF, 0xA, false);
    }
    if (X == 8) return (unsigned)__builtin_amdgcn_update_dpp(v, v, 0x128, 0xF, 0xF, false);
    return (unsigned)__shfl_xor(v, X, 64);
}

// One pass of distance 8 X of stage k: the partner holds the same e in lane ^ X; k > 8 X >= 8, so the direction is
// the same for the whole lane.
template <int X>
__device__ __forceinline__ void exchange_pass(unsigned (&v)[8], int i0, int k) {
    const bool keep_min = ((i0 & (8 * X)) == 0) == ((i0 & k) == 0);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const unsigned o = lane_xor<X>(v[e]);
        const unsigned lo = v[e] < o ? v[e] : o, hi = v[e] < o ? o : v[e];
        v[e] = keep_min ? lo : hi;
    }
}

// Passes j_first, j_first / 2, ..., 1 (j_first <= 256) of stage k of the bitonic network on the 512 keys a wavefront
// holds, v[e] = key i0 + e with i0 a multiple of 8: distances of 8 and more exchange between lanes, 4, 2, 1 inside
// the lane.  No LDS traffic and no barrier.
__device__ __forceinline__ void bitonic_inwave(unsigned (&v)[8], int i0, int j_first, int k) {
    if (j_first >= 256) exchange_pass<32>(v, i0, k);
    if (j_first >= 128) exchange_pass<16>(v, i0, k);
    if (j_first >= 64) exchange_pass<8>(v, i0, k);
    if (j_first >= 32) exchange_pass<4>(v, i0, k);
    if (j_first >= 16) exchange_pass<2>(v, i0, k);
    if (j_first >= 8) exchange_pass<1>(v, i0, k);
    if (j_first >= 4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) order(v[e], v[e + 4], ((i0 + e) & k) == 0);
    }
    if (j_first >= 2) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if ((e & 2) == 0) order(v[e], v[e + 2], ((i0 + e) & k) == 0);
    }
#pragma unroll
    for (int e = 0; e < 8; e += 2) order(v[e], v[e + 1], ((i0 + e) & k) == 0);
}

// LEVELS consecutive passes (distances j, j / 2, ..., j >> (LEVELS - 1)) of stage k on LDS-resident keys, by the
// whole workgroup, in registers on groups of 2^LEVELS keys; ends with a barrier.
template <int LEVELS>
__device__ __forceinline__ void bitonic_levels_lds32(unsigned* sh, int m, int j, int k) {
    constexpr int G = 1 << LEVELS;
    const int low = j >> (LEVELS - 1);
    for (int t = threadIdx.x; t < m / G; t += FUSED_THREADS) {
        const int base = ((t & ~(low - 1)) << LEVELS) | (t & (low - 1));
        const bool asc = (base & k) == 0;
        unsigned v[G];
#pragma unroll
        for (int e = 0; e < G; ++e) v[e] = sh[base + e * low];
#pragma unroll
        for (int d = G >> 1; d > 0; d >>= 1)
#pragma unroll
            for (int e = 0; e < G; ++e)
                if ((e & d) == 0) order(v[e], v[e | d], asc);
#pragma unroll
        for (int e = 0; e < G; ++e) sh[base + e * low] = v[e];
    }
    __syncthreads();
}

__device__ __forceinline__ void load_keys8(unsigned (&v)[8], const unsigned* sh, int i0) {
    const uintx4 a = *reinterpret_cast<const uintx4*>(sh + i0), b = *reinterpret_cast<const uintx4*>(sh + i0 + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void store_keys8(unsigned* sh, int i0, const unsigned (&v)[8]) {
    uintx4 a, b;
    a.x = v[0]; a.y = v[1]; a.z = v[2]; a.w = v[3]; b.x = v[4]; b.y = v[5]; b.z = v[6]; b.w = v[7];
    *reinterpret_cast<uintx4*>(sh + i0) = a;
    *reinterpret_cast<uintx4*>(sh + i0 + 4) = b;
}

// Ascending bitonic sort of sh[0 .. m), m a power of two between 512 and 8192, by a workgroup of 16 wavefronts.
// Wavefront w owns keys 512 w .. 512 w + 511: it sorts them alone (stages 2 .. 512, 45 passes, no barrier), and in
// each later stage k the workgroup does the passes of distance >= 512 on LDS (one round trip) and the wavefronts the
// remaining nine.  Barriers: 1 + 2 log2(m / 512).
__device__ __forceinline__ void bitonic_sort_lds32(unsigned* sh, int m, int lane, int wave) {
    const bool on = wave * WAVE_KEYS < m;
    const int i0 = wave * WAVE_KEYS + lane * 8;
    unsigned v[8];
    if (on) {
        load_keys8(v, sh, i0);
        for (int k = 2; k <= WAVE_KEYS; k <<= 1) bitonic_inwave(v, i0, k >> 1, k);
        store_keys8(sh, i0, v);
    }
    __syncthreads();
    for (int k = 2 * WAVE_KEYS; k <= m; k <<= 1) {
        switch (k / WAVE_KEYS) {       // passes k / 2 .. 512
            case 2: bitonic_levels_lds32<1>(sh, m, k >> 1, k); break;
            case 4: bitonic_levels_lds32<2>(sh, m, k >> 1, k); break;
            case 8: bitonic_levels_lds32<3>(sh, m, k >> 1, k); break;
            default: bitonic_levels_lds32<4>(sh, m, k >> 1, k); break;
        }
        if (on) {
            load_keys8(v, sh, i0);
            bitonic_inwave(v, i0, WAVE_KEYS >> 1, k);
            store_keys8(sh, i0, v);
        }
        __syncthreads();
    }
}

typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
template <typename GV>
__device__ __forceinline__ GV buf_load(__amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned soff);
template <> __device__ __forceinline__ unsigned buf_load<unsigned>(__amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned soff) {
    return __builtin_amdgcn_raw_buffer_load_b32(rs, (int)voff, (int)soff, 0);
}
template <> __device__ __forceinline__ u16 buf_load<u16>(__amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned soff) {
    return __builtin_amdgcn_raw_buffer_load_b16(rs, (int)voff, (int)soff, 0);
}
template <> __device__ __forceinline__ float2 buf_load<float2>(__amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned soff) {
    const uintx2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)voff, (int)soff, 0);
    return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
}
template <> __device__ __forceinline__ float buf_load<float>(__amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned soff) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, (int)voff, (int)soff, 0));
}

// B: tokens a wavefront fetches before it adds (data registers: 1024 threads leave 128 per lane)
template <typename T, int VEC> struct FusedVec;
template <> struct FusedVec<u16, 2> { typedef unsigned type; static constexpr int BATCH = 32; };
template <> struct FusedVec<u16, 1> { typedef u16 type; static constexpr int BATCH = 32; };
template <> struct FusedVec<float, 2> { typedef float2 type; static constexpr int BATCH = 16; };
template <> struct FusedVec<float, 1> { typedef float type; static constexpr int BATCH = 32; };

// Row loads through a raw buffer descriptor over the whole gradient matrix (below 4 GB: checked on the host):
// the lane's column offset is one loop-invariant VGPR, the token's row offset a scalar, so a load in flight
// costs its data registers only.  Positions past cnt re-read the last valid row; their adds are gated to -0.0f.
template <int D, typename GV>
__device__ __forceinline__ void fused_load_batch(GV (&v)[D], __amdgpu_buffer_rsrc_t rs, unsigned voff, unsigned row_bytes,
                                                 unsigned tok, int cnt) {
#pragma unroll
    for (int u = 0; u < D; ++u) {
        const int idx = u < cnt ? u : cnt - 1;
        const unsigned t = __builtin_amdgcn_readlane(tok, idx);
        v[u] = buf_load<GV>(rs, voff, t * row_bytes);
    }
}

template <typename T, int VEC>
__global__ __launch_bounds__(FUSED_THREADS) void embed_bwd_fused_kernel(const int64_t* __restrict__ ids, int N, int Vs,
                                                                        int64_t off, const T* __restrict__ gout,
                                                                        unsigned grad_bytes, int h,
                                                                        float* __restrict__ dtable, int n_slabs,
                                                                        int n_groups) {
    typedef typename FusedVec<T, VEC>::type GV;
    constexpr int B = FusedVec<T, VEC>::BATCH;
    constexpr int Q = 4, TINY = 4;                          // runs of up to TINY tokens go Q at a time
    __shared__ __align__(16) unsigned sh[FUSED_MAX_N];      // the keys
    __shared__ unsigned short run_start[FUSED_MAX_N + 2];   // position of the first key of run r; [n_runs] = owned
    __shared__ int wave_cnt[FUSED_MAX_N / 64];
    __shared__ float xchg[64 * VEC];
    __shared__ int s_owned, s_runs;
    if (threadIdx.x == 0) { s_owned = 0; s_runs = 0; }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const u64 below = (1ull << lane) - 1ull;

    // keys of the tokens this shard owns (all ids requested before the first is used), packed into sh in any
    // order - they are unique and get sorted: one LDS atomic per wavefront
    constexpr int ROUNDS = FUSED_MAX_N / FUSED_THREADS;
    unsigned mine[ROUNDS];
    u64 have[ROUNDS];
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) mine[q] = token_key32(ids, q * FUSED_THREADS + threadIdx.x, N, Vs, off);
    int total = 0;
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
        have[q] = __builtin_amdgcn_ballot_w64(mine[q] != KEY32_NONE);
        total += __builtin_popcountll(have[q]);
    }
    int at = 0;
    if (lane == 0 && total) at = atomicAdd(&s_owned, total);
    at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
        if (mine[q] != KEY32_NONE) sh[at + __builtin_popcountll(have[q] & below)] = mine[q];
        at += __builtin_popcountll(have[q]);
    }
    __syncthreads();
    const int owned = s_owned;
    if (owned == 0) return;
    int m = WAVE_KEYS;
    while (m < owned) m <<= 1;
    for (int t = owned + threadIdx.x; t < m; t += FUSED_THREADS) sh[t] = KEY32_NONE;
    __syncthreads();
    bitonic_sort_lds32(sh, m, lane, wave);

    // Runs of equal rows, numbered by position: every workgroup must arrive at the SAME numbering, because the
    // groups of a slab share the runs out by number.  Run number = how many runs start before the position:
    // ballot per wavefront and round, then an exclusive scan of the ROUNDS * 16 counts by wavefront 0.
    u64 starts[ROUNDS];
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
        const int t = q * FUSED_THREADS + (int)threadIdx.x;
        bool st = false;
        if (t < owned) st = t == 0 || key_row(sh[t - 1]) != key_row(sh[t]);
        starts[q] = __builtin_amdgcn_ballot_w64(st);
        if (lane == 0) wave_cnt[q * FUSED_WAVES + wave] = __builtin_popcountll(starts[q]);
    }
    __syncthreads();
    if (wave == 0) {
        static_assert(ROUNDS * FUSED_WAVES == 128, "two counts per lane");
        const int a = wave_cnt[2 * lane], b2 = wave_cnt[2 * lane + 1];
        int incl = a + b2;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        wave_cnt[2 * lane] = incl - a - b2;
        wave_cnt[2 * lane + 1] = incl - b2;
        if (lane == 63) {
            s_runs = incl;
            run_start[incl] = (unsigned short)owned;
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q)
        if ((starts[q] >> lane) & 1ull)
            run_start[wave_cnt[q * FUSED_WAVES + wave] + __builtin_popcountll(starts[q] & below)] =
                (unsigned short)(q * FUSED_THREADS + (int)threadIdx.x);
    __syncthreads();
    const int n_runs = s_runs;

    const int slab = blockIdx.x % n_slabs, group = blockIdx.x / n_slabs;
    const int c0 = (slab * 64 + lane) * VEC;
    const bool active = c0 < h;
    const unsigned row_bytes = (unsigned)h * (unsigned)sizeof(T);
    const unsigned voff = (unsigned)c0 * (unsigned)sizeof(T);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)gout, 0, (int)grad_bytes, 0x00020000);
    float* const dcol = dtable + c0;

    // short runs: one wavefront each, Q of them per turn
    const int stride = n_groups * FUSED_WAVES;
    for (int r0 = group * FUSED_WAVES + wave; r0 < n_runs; r0 += Q * stride) {
        int len[Q];
        unsigned tok[Q], row[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int r = r0 + q * stride;
            int s = 0;
            len[q] = 0;
            if (r < n_runs) {
                s = run_start[r];
                len[q] = (int)run_start[r + 1] - s;
            }
            s = __builtin_amdgcn_readfirstlane(s);
            len[q] = __builtin_amdgcn_readfirstlane(len[q]);
            if (len[q] > B) len[q] = 0;                     // a long run: not here
            // (every lane fetches its token, also one whose columns lie past h: readlane takes it from there)
            tok[q] = lane < len[q] ? key_token(sh[s + lane]) : 0u;
            row[q] = key_row(sh[s]);
        }
        // the first run of 5 .. B tokens of this turn (seldom more than one) goes along with the small ones
        int mid = -1;
#pragma unroll
        for (int q = Q - 1; q >= 0; --q)
            if (len[q] > TINY) mid = q;
        unsigned tok_mid = 0, row_mid = 0;
        int len_mid = 0;
#pragma unroll
        for (int q = 0; q < Q; ++q)
            if (q == mid) { tok_mid = tok[q]; row_mid = row[q]; len_mid = len[q]; }
        if (active) {
            float acc[Q][VEC], acc_mid[VEC];
            GV few[Q][TINY], v[B];
#pragma unroll
            for (int q = 0; q < Q; ++q)
                if (len[q] >= 1 && len[q] <= TINY) {
                    load_acc<VEC>(acc[q], dcol + (size_t)row[q] * h);
                    fused_load_batch<TINY>(few[q], rs, voff, row_bytes, tok[q], len[q]);
                }
            if (mid >= 0) {
                load_acc<VEC>(acc_mid, dcol + (size_t)row_mid * h);
                fused_load_batch<B>(v, rs, voff, row_bytes, tok_mid, len_mid);
            }
#pragma unroll
            for (int q = 0; q < Q; ++q)
                if (len[q] >= 1 && len[q] <= TINY) {
                    add_batch<TINY, VEC>(acc[q], few[q], 0, len[q]);
                    store_acc<VEC>(dcol + (size_t)row[q] * h, acc[q]);
                }
            if (mid >= 0) {
                add_batch<B, VEC>(acc_mid, v, 0, len_mid);
                store_acc<VEC>(dcol + (size_t)row_mid * h, acc_mid);
            }
#pragma unroll
            for (int q = 1; q < Q; ++q)
                if (len[q] > TINY && q != mid) {
                    load_acc<VEC>(acc_mid, dcol + (size_t)row[q] * h);
                    fused_load_batch<B>(v, rs, voff, row_bytes, tok[q], len[q]);
                    add_batch<B, VEC>(acc_mid, v, 0, len[q]);
                    store_acc<VEC>(dcol + (size_t)row[q] * h, acc_mid);
                }
        }
    }
    // long runs: run r belongs to group r % n_groups, all 16 wavefronts of it.  Each wavefront looks through that
    // group's run numbers 64 at a time; LDS holds the same in all of them, so they agree on which runs are long
    // and meet at the same barriers.
    for (int base = 0; base < n_runs; base += 64 * n_groups) {
        const int cand = base + lane * n_groups + group;
        bool is_long = false;
        if (cand < n_runs) is_long = (int)run_start[cand + 1] - (int)run_start[cand] > B;
        u64 todo = __builtin_amdgcn_ballot_w64(is_long);
        while (todo) {
            const int r = base + __builtin_ctzll(todo) * n_groups + group;
            todo &= todo - 1;
            const int s = run_start[r], len = (int)run_start[r + 1] - s;
            float* const d = dcol + (size_t)key_row(sh[s]) * h;
            // Chunks of 16 B tokens; in a chunk wavefront w has tokens B w .. B w + B - 1 and turn w in the chain.
            // The rows of a chunk are requested by all wavefronts at once (one compute unit alone draws little from
            // memory: the requests, not the chain, take most of the time), the accumulator's load is in flight with the
            // first of them, and every wavefront turns its rows into floats (-0.0f past cnt) before the chain starts,
            // so that a turn is nothing but dependent adds.
            float acc[VEC];
            GV v[B];
            float f[B][VEC];
            __syncthreads();                   // xchg is free again (previous long run)
            if (wave == 0 && active) load_acc<VEC>(acc, d);
            for (int c = 0; c < len; c += FUSED_WAVES * B) {
                const int first = c + wave * B;
                const int cnt = len - first < 0 ? 0 : (len - first > B ? B : len - first);
                const int turns = len - c > FUSED_WAVES * B ? FUSED_WAVES : (len - c + B - 1) / B;
                const unsigned tok = lane < cnt ? key_token(sh[s + first + lane]) : 0u;
                if (active && cnt > 0) fused_load_batch<B>(v, rs, voff, row_bytes, tok, cnt);
                if (c == 0 && wave == 0 && active) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) xchg[e * 64 + lane] = acc[e];
                }
                if (active && cnt > 0) {
#pragma unroll
                    for (int u = 0; u < B; ++u) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) f[u][e] = -0.0f;
                        add_grad(f[u], v[u], u < cnt);          // -0.0f + x = x for every x
#pragma unroll
                        for (int e = 0; e < VEC; ++e) asm volatile("" : "+v"(f[u][e]));   // here, not inside the turn
                    }
                }
                __syncthreads();
#pragma unroll 1
                for (int p = 0; p < turns; ++p) {
                    if (wave == p && active) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[e] = xchg[e * 64 + lane];
#pragma unroll
                        for (int u = 0; u < B; ++u)
#pragma unroll
                            for (int e = 0; e < VEC; ++e) acc[e] += f[u][e];
#pragma unroll
                        for (int e = 0; e < VEC; ++e) xchg[e * 64 + lane] = acc[e];
                    }
                    __syncthreads();
                }
            }
            if (wave == 0 && active) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = xchg[e * 64 + lane];
                store_acc<VEC>(d, acc);
            }
        }
    }
}

template <typename T, int VEC>
static hipError_t launch_fused(const int64_t* ids, int N, int Vs, int64_t off, const T* gout, int h, float* dtable,
                               hipStream_t st) {
    ProfScope prof(K_EMBED_ACCUM, st);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
    }
    const int n_slabs = (int)ceil_div(h, 64 * VEC);
    int n_groups = cus / n_slabs;
    const int want = (int)ceil_div(N, 64);          // no more groups than there could be work for
    if (n_groups > want) n_groups = want;
    if (n_groups < 1) n_groups = 1;
    const unsigned grad_bytes = (unsigned)((size_t)N * h * sizeof(T));
    hipLaunchKernelGGL((embed_bwd_fused_kernel<T, VEC>), dim3((unsigned)(n_slabs * n_groups)), dim3(FUSED_THREADS), 0, st, ids,
                       N, Vs, off, gout, grad_bytes, h, dtable, n_slabs, n_groups);
    return hipGetLastError();
}

hipError_t launch_embed_bwd(const void* gout, const int64_t* ids, int N, int h, int Vs, int64_t off, int is_bf16,
                            float* dtable, void* ws, hipStream_t st) {
    // the one-kernel path: up to 8192 tokens and 2^19 - 1 rows (32-bit keys), gradient matrix addressable with
    // 32-bit byte offsets
    if (N <= FUSED_MAX_N && Vs <= FUSED_MAX_VS && (uint64_t)N * (uint64_t)h * (is_bf16 ? 2u : 4u) < ((uint64_t)1 << 32)) {
        if (is_bf16) return h % 2 == 0 ? launch_fused<u16, 2>(ids, N, Vs, off, (const u16*)gout, h, dtable, st)
                                       : launch_fused<u16, 1>(ids, N, Vs, off, (const u16*)gout, h, dtable, st);
        return h % 2 == 0 ? launch_fused<float, 2>(ids, N, Vs, off, (const float*)gout, h, dtable, st)
                          : launch_fused<float, 1>(ids, N, Vs, off, (const float*)gout, h, dtable, st);
    }
    u64* keys = (u64*)ws;
    const int n_pad = next_pow2(N);
    const RunList runs = run_list_of(ws, n_pad);
    hipError_t e;
    if ((e = sort_keys(ids, N, Vs, off, keys, n_pad, runs, st)) != hipSuccess) return e;
    return accumulate_runs(keys, n_pad, runs, gout, N, h, is_bf16, dtable, st);
}

}  // namespace vp
