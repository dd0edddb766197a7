// Shared pieces of the bf16 MFMA GEMM kernels: accumulator layout, workgroup -> tile map and
// the four epilogues (softmax statistics of pass S, the D matrix of pass T, fp32 store and
// fp32 accumulate).
//
// Accumulator layout (both kernels): 256x256 output tile per workgroup; the wavefronts form a
// 2 x WN grid (WN = 2: four wavefronts of 128x128, WN = 4: eight wavefronts of 128x64), each
// owning 4 x NJ tiles of the 32x32x16 bf16 MFMA (NJ = 128 / (32 WN) ... 4 or 2).  The MFMA is issued with
// the B operand first, i.e. it produces the transposed 32x32 tile, so that register r of lane l
// of tile (i, j) holds
//        C[ i*32 + l%32 ][ j*32 + 8*(r/4) + 4*(l/32) + r%4 ]
// of the wavefront's block: a lane owns ONE output row per i (a token in the forward pass) and,
// per j, four runs of four consecutive columns.  Row reductions (max / sum-exp over the
// vocabulary) are therefore almost entirely in-register, and stores are 16 bytes (fp32) or
// 8 bytes (bf16) per lane.
#pragma once
#include "vp_internal.h"

namespace vp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int BM = GEMM_BM, BN = GEMM_BN, BK = 64;
constexpr int NT = 256;   // threads per workgroup

__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;   // round to nearest even
    return (unsigned)__builtin_bit_cast(u16, a) | ((unsigned)__builtin_bit_cast(u16, b) << 16);
}
__device__ __forceinline__ u16 f32_to_bf16(float f) {
    const __bf16 b = (__bf16)f;
    return __builtin_bit_cast(u16, b);
}

// acc[i][j] += A-rows(i) x B-rows(j), stored transposed (see the layout above)
__device__ __forceinline__ void mfma_tile(floatx16& c, const bf16x8& a, const bf16x8& b) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c, 0, 0, 0);
}

// Workgroup id -> output tile.  Workgroups are handed to the 8 XCDs round-robin, so ids
// congruent mod 8 share an L2: give each XCD one contiguous run of logical tiles, and walk
// the tiles in panels of 8 tile-rows, so the 32 workgroups resident on an XCD cover a
// compact patch and re-use each other's operand panels from that L2.
__device__ __forceinline__ void tile_of_block(int b, int nb, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int x = b & 7, per = nb >> 3, rem = nb & 7;
    const int logical = x * per + (x < rem ? x : rem) + (b >> 3);
    constexpr int GM = 8;
    const int panel = logical / (GM * tiles_n);
    const int first_m = panel * GM;
    const int rows = (tiles_m - first_m < GM) ? (tiles_m - first_m) : GM;
    const int in_panel = logical - panel * GM * tiles_n;
    tm = first_m + in_panel % rows;
    tn = in_panel / rows;
}

// Stores four consecutive values of a row at column `col` (a multiple of 4), clipped to n_cols.
// vec: row start and leading dimension allow an aligned 16-byte (fp32) / 8-byte (bf16) access.
template <bool ACCUM>
__device__ __forceinline__ void store4_f32(float* row, int col, int n_cols, bool vec, float v0, float v1, float v2,
                                           float v3) {
    if (vec && col + 4 <= n_cols) {
        floatx4* p = reinterpret_cast<floatx4*>(row + col);
        floatx4 v = {v0, v1, v2, v3};
        if (ACCUM) v += *p;
        *p = v;
    } else {
        const float vals[4] = {v0, v1, v2, v3};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < n_cols) row[col + e] = ACCUM ? row[col + e] + vals[e] : vals[e];
    }
}
__device__ __forceinline__ void store4_bf16(u16* row, int col, int n_cols, bool vec, float v0, float v1, float v2,
                                            float v3) {
    if (vec && col + 4 <= n_cols) {
        *reinterpret_cast<uint2*>(row + col) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
    } else {
        const float vals[4] = {v0, v1, v2, v3};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < n_cols) row[col + e] = f32_to_bf16(vals[e]);
    }
}

// The LDS staging buffers are free when the epilogue runs; `smem` (>= 8 KB) carries the
// exchange between the WN wavefronts that share a row.
template <Epi EPI, int NJ, int WN>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[4][NJ], const GemmBf16Params& g, int tile_m, int tile_n,
                                              char* smem) {
    constexpr int WCOLS = NJ * 32;            // columns owned by one wavefront
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, hf = lane >> 5;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    // element (i, j, r) of this lane: row = rbase + i*32, col = cbase + j*32 + 8*(r/4) + (r%4)
    const int rbase = m0 + wm * 128 + l32;
    const int cbase = n0 + wn * WCOLS + 4 * hf;

    if (EPI == Epi::StoreF32 || EPI == Epi::AccumF32) {
        const bool vec = (g.ldc % 4 == 0) && (((uintptr_t)g.C & 15u) == 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = rbase + i * 32;
            if (row < g.M) {
                float* crow = g.C + (size_t)row * g.ldc;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        store4_f32<EPI == Epi::AccumF32>(crow, cbase + j * 32 + 8 * q, g.N, vec, acc[i][j][4 * q],
                                                         acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                                                         acc[i][j][4 * q + 3]);
            }
        }
    }

    if (EPI == Epi::DLogits) {
        // D = (softmax - G) * scale with the global statistics (pass T of Algorithm 1, with
        // the logits taken from the accumulators instead of memory)
        const bool vec = (g.ldy % 4 == 0) && (((uintptr_t)g.Y & 7u) == 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = rbase + i * 32;
            if (row < g.M) {
                const float m = g.gmax[row];
                const float inv = 1.0f / g.gsum[row];
                const int64_t lab64 = g.labels[row] - g.shard_offset - cbase;
                // column of the label relative to cbase, or -1 when it is not in this lane's range
                const int lab = (lab64 >= 0 && lab64 < WCOLS) ? (int)lab64 : -1;
                u16* drow = g.Y + (size_t)row * g.ldy;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float d[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            d[e] = __expf(acc[i][j][4 * q + e] - m) * inv;
                            if (lab == j * 32 + 8 * q + e) d[e] -= 1.0f;
                            d[e] *= g.scale;
                        }
                        store4_bf16(drow, cbase + j * 32 + 8 * q, g.N, vec, d[0], d[1], d[2], d[3]);
                    }
            }
        }
    }

    if (EPI == Epi::FwdStats) {
        // shard-local m' and sum' of Algorithm 1's pass S, restricted to this tile's 256
        // columns; the per-tile pairs are folded afterwards exactly like shards are (online
        // softmax rescaling).  A lane reduces its 64 columns of a row in registers, one
        // exchange with lane ^ 32 completes the wavefront's 128 columns, and the two wavefronts
        // that share the row meet in LDS.
        float* xm = reinterpret_cast<float*>(smem);          // [WN][256]
        float* xs = xm + WN * 256;                             // [WN][256]
        const bool vec = g.Y && (g.ldy % 4 == 0) && (((uintptr_t)g.Y & 7u) == 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = rbase + i * 32;
            float v = -INFINITY;
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (cbase + j * 32 + 8 * (r >> 2) + (r & 3) < g.N) v = fmaxf(v, acc[i][j][r]);
            const float m = fmaxf(v, __shfl_xor(v, 32, 64));
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (cbase + j * 32 + 8 * (r >> 2) + (r & 3) < g.N) s += __expf(acc[i][j][r] - m);
            s += __shfl_xor(s, 32, 64);
            if (hf == 0) {
                const int lr = wm * 128 + i * 32 + l32;
                xm[wn * 256 + lr] = m;
                xs[wn * 256 + lr] = s;
            }
            if (row < g.M) {
                const int64_t lab64 = g.labels[row] - g.shard_offset - cbase;
                if (lab64 >= 0 && lab64 < WCOLS && (lab64 & 4) == 0 && lab64 + cbase < g.N) {
                    const int lab = (int)lab64;
                    float t = 0.f;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (lab == j * 32 + 8 * (r >> 2) + (r & 3)) t = acc[i][j][r];
                    g.part_tgt[row] = t;
                }
                if (g.Y) {
                    u16* yrow = g.Y + (size_t)row * g.ldy;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            store4_bf16(yrow, cbase + j * 32 + 8 * q, g.N, vec, acc[i][j][4 * q], acc[i][j][4 * q + 1],
                                        acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                }
            }
        }
        __syncthreads();
        if (tid < 256) {
            const int row = m0 + tid;
            if (row < g.M) {
                float m = -INFINITY;
#pragma unroll
                for (int w = 0; w < WN; ++w) m = fmaxf(m, xm[w * 256 + tid]);
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < WN; ++w) {
                    const float mw = xm[w * 256 + tid];
                    if (mw > -INFINITY) s += xs[w * 256 + tid] * __expf(mw - m);
                }
                g.part_max[(size_t)tile_n * g.M + row] = m;
                g.part_sum[(size_t)tile_n * g.M + row] = s;
            }
        }
    }
}

}  // namespace vp
