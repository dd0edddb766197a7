// Shared pieces of the bf16 MFMA GEMM kernels: accumulator layout, workgroup -> tile map and
// the four epilogues (softmax statistics of pass S, the D matrix of pass T, fp32 store and
// fp32 accumulate).
//
// Accumulator layout (both kernels): 256x256 output tile per workgroup of 4 wavefronts (2x2),
// each wavefront owns 128x128 = 4x4 tiles of the 32x32x16 bf16 MFMA.  Register r of lane l of
// tile (i, j) holds C[i*32 + 8*(r/4) + 4*(l/32) + r%4][j*32 + l%32] of the wavefront's block.
#pragma once
#include "vp_internal.h"

namespace vp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = GEMM_BM, BN = GEMM_BN, BK = 64;
constexpr int NT = 256;   // threads per workgroup

__device__ __forceinline__ float xor_max32(float v) {
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float xor_sum32(float v) {
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ u16 f32_to_bf16(float f) {
    __bf16 b = (__bf16)f;   // round to nearest even
    return __builtin_bit_cast(u16, b);
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

// The LDS staging buffers are free when the epilogue runs; `smem` (>= 4 KB) carries the
// exchange between the two wavefronts that share a row.
template <Epi EPI>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[4][4], const GemmBf16Params& g, int tile_m, int tile_n,
                                              char* smem) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hf = lane >> 5;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    // element (i, j, r) of this lane: row = rbase + i*32 + 8*(r/4) + (r%4), col = cbase + j*32
    const int rbase = m0 + wm * 128 + 4 * hf;
    const int cbase = n0 + wn * 128 + l32;

    if (EPI == Epi::StoreF32 || EPI == Epi::AccumF32) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = rbase + i * 32 + 8 * (r >> 2) + (r & 3);
                if (row < g.M) {
                    float* crow = g.C + (size_t)row * g.ldc;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int col = cbase + j * 32;
                        if (col < g.N) {
                            if (EPI == Epi::AccumF32) crow[col] += acc[i][j][r];
                            else crow[col] = acc[i][j][r];
                        }
                    }
                }
            }
    }

    if (EPI == Epi::DLogits) {
        // D = (softmax - G) * scale with the global statistics (pass T of Algorithm 1, with
        // the logits taken from the accumulators instead of memory)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = rbase + i * 32 + 8 * (r >> 2) + (r & 3);
                if (row < g.M) {
                    const float m = g.gmax[row];
                    const float inv = 1.0f / g.gsum[row];
                    const int64_t lab = g.labels[row] - g.shard_offset;
                    u16* drow = g.Y + (size_t)row * g.ldy;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int col = cbase + j * 32;
                        if (col < g.N) {
                            float d = __expf(acc[i][j][r] - m) * inv;
                            if (lab == (int64_t)col) d -= 1.0f;
                            drow[col] = f32_to_bf16(d * g.scale);
                        }
                    }
                }
            }
    }

    if (EPI == Epi::FwdStats) {
        // shard-local m' and sum' of Algorithm 1's pass S, restricted to this tile's 256
        // columns; the per-tile pairs are folded afterwards exactly like shards are (online
        // softmax rescaling).  The LDS stages are free now and carry the 2-wave exchange.
        float* xm = reinterpret_cast<float*>(smem);          // [2][256]
        float* xs = xm + 512;                                  // [2][256]
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = rbase + i * 32 + 8 * (r >> 2) + (r & 3);
                float v = -INFINITY;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (cbase + j * 32 < g.N) v = fmaxf(v, acc[i][j][r]);
                const float m = xor_max32(v);
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (cbase + j * 32 < g.N) s += __expf(acc[i][j][r] - m);
                s = xor_sum32(s);
                if (l32 == 0) {
                    const int lr = row - m0;
                    xm[wn * 256 + lr] = m;
                    xs[wn * 256 + lr] = s;
                }
                if (row < g.M) {
                    const int64_t lab = g.labels[row] - g.shard_offset;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int col = cbase + j * 32;
                        if (lab == (int64_t)col && col < g.N) g.part_tgt[row] = acc[i][j][r];
                    }
                    if (g.Y) {
                        u16* yrow = g.Y + (size_t)row * g.ldy;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int col = cbase + j * 32;
                            if (col < g.N) yrow[col] = f32_to_bf16(acc[i][j][r]);
                        }
                    }
                }
            }
        __syncthreads();
        {
            const int row = m0 + tid;
            if (row < g.M) {
                const float ma = xm[tid], mb = xm[256 + tid];
                const float m = fmaxf(ma, mb);
                float s = 0.f;
                if (ma > -INFINITY) s += xs[tid] * __expf(ma - m);
                if (mb > -INFINITY) s += xs[256 + tid] * __expf(mb - m);
                g.part_max[(size_t)tile_n * g.M + row] = m;
                g.part_sum[(size_t)tile_n * g.M + row] = s;
            }
        }
    }
}

}  // namespace vp
