// Shared pieces of the bf16 MFMA GEMM kernels: accumulator layout, workgroup -> tile map and
// the four epilogues (softmax statistics of pass S, the D matrix of pass T, fp32 store and
// fp32 accumulate).
//
// Accumulator layout (both kernels): 256x256 output tile per workgroup of four wavefronts in a
// 2 x 2 grid, each owning 128x128 = 4 x 4 tiles of the 32x32x16 bf16 MFMA.  (The epilogue is
// written for a 2 x WN grid with 4 x NJ MFMA tiles per wavefront, NJ = 128 / (32 WN); the
// kernels use WN = 2, NJ = 4.)  The MFMA is issued with the B operand first, i.e. it produces
// the transposed 32x32 tile, so that register r of lane l of tile (i, j) holds
//        C[ i*32 + l%32 ][ j*32 + 8*(r/4) + 4*(l/32) + r%4 ]
// of the wavefront's block: a lane owns ONE output row per i (a token in the forward pass) and,
// per j, four runs of four consecutive columns.  Row reductions (max / sum-exp over the
// vocabulary) are therefore almost entirely in-register; outputs leave through an LDS staging
// block that turns this layout into row-contiguous 16-byte stores (see gemm_epilogue).
#pragma once
#include "vp_internal.h"

namespace vp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

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

constexpr float LOG2E = 1.44269504088896340736f;
// 2^x with the hardware instruction (1 ulp, flushes results below 2^-126 to zero)
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// acc[i][j] += A-rows(i) x B-rows(j), stored transposed (see the layout above)
template <Epi EPI>
__device__ __forceinline__ void mfma_tile(floatx16& c, const bf16x8& a, const bf16x8& b) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c, 0, 0, 0);
}

// Virtual workgroup id -> output tile.  v = round * nb + b with nb workgroups per round (one
// tile each; the last round may be short), total = tiles_m * tiles_n.  Workgroups are handed to
// the 8 XCDs round-robin, so ids congruent mod 8 share an L2; in both orders below the 32
// workgroups of an XCD cover a patch of 8 x 4 tiles at a time and re-use each other's operand
// panels from that L2 (12 panels for 32 tiles).
//
//  * Up to 16 tile rows (forward and dH products: the token dimension is short): every XCD gets
//    one contiguous run of tiles, walked in panels of 8 tile rows, column by column.
//  * More than 16 tile rows (dW products: the vocabulary dimension is long): tiles are ranked
//    hierarchically - blocks of 16 x 16 tiles (row-block major), inside a block groups of 4
//    columns, inside a group the upper and the lower 8 rows, column by column, all clipped at
//    the edges of the grid so that the rank is a bijection - and in every round the 8 XCDs
//    take the 8 sub-blocks of one block.  What misses the L2s is then shared in the
//    memory-side cache: 32 distinct panels per 256 tiles instead of 68 (measured on dW: -5 %
//    at 63 x 32 tiles, -1.5 % at 63 x 16; the other products lose 1-3 % with it).
__device__ __forceinline__ void tile_of_block(int v, int nb, int total, int tiles_m, int tiles_n, int& tm, int& tn) {
    if (tiles_m <= 16) {
        // all rounds laid end to end: XCD x owns ranks [x * per + min(x, rem), ...)
        const int round = v / nb, b = v - round * nb;
        const int x = b & 7, per = total >> 3, rem = total & 7;
        // (a workgroup count that is not a multiple of 8 with several rounds: plain order)
        const int logical = ((nb & 7) != 0 && total > nb) ? v
                                                          : x * per + (x < rem ? x : rem) + round * (nb >> 3) + (b >> 3);
        constexpr int GM = 8;
        const int panel = logical / (GM * tiles_n);
        const int first_m = panel * GM;
        const int rows = (tiles_m - first_m < GM) ? (tiles_m - first_m) : GM;
        const int in_panel = logical - panel * GM * tiles_n;
        tm = first_m + in_panel % rows;
        tn = in_panel / rows;
        return;
    }
    int logical = v;
    {
        const int round = v / nb, b = v - round * nb;
        const int here = min(nb, total - round * nb);      // workgroups active in this round
        if ((here & 7) == 0) logical = round * nb + (b & 7) * (here >> 3) + (b >> 3);
    }
    const int rb = logical / (16 * tiles_n);               // row-block of 16 tile rows
    int rem = logical - rb * 16 * tiles_n;
    const int hR = min(16, tiles_m - 16 * rb);
    const int cb = rem / (hR * 16);                        // column-block of 16 tile columns
    rem -= cb * hR * 16;
    const int wC = min(16, tiles_n - 16 * cb);
    const int sc = rem / (hR * 4);                         // group of 4 tile columns
    rem -= sc * hR * 4;
    const int w = min(4, wC - 4 * sc);
    const int h0 = min(8, hR);
    const int sr = rem >= h0 * w ? 1 : 0;                  // upper / lower 8 tile rows
    rem -= sr * h0 * w;
    const int hs = sr ? hR - h0 : h0;
    tm = 16 * rb + 8 * sr + rem % hs;
    tn = 16 * cb + 4 * sc + rem / hs;
}

// Stores four consecutive fp32 values of a row at column `col` (a multiple of 4), clipped to
// n_cols.  vec: row start and leading dimension allow an aligned 16-byte access.
template <bool ACCUM>
__device__ __forceinline__ void store4_f32(float* row, int col, int n_cols, bool vec, const floatx4& v) {
    if (vec && col + 4 <= n_cols) {
        floatx4* p = reinterpret_cast<floatx4*>(row + col);
        *p = ACCUM ? v + *p : v;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < n_cols) row[col + e] = ACCUM ? row[col + e] + v[e] : v[e];
    }
}
// Stores eight consecutive bf16 values (bit patterns packed in a uint4) of a row at column `col`
// (a multiple of 8), clipped to n_cols.
__device__ __forceinline__ void store8_bf16(u16* row, int col, int n_cols, bool vec, const uint4& v) {
    if (vec && col + 8 <= n_cols) {
        *reinterpret_cast<uint4*>(row + col) = v;
    } else {
        const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (col + e < n_cols) row[col + e] = (u16)(w[e >> 1] >> (16 * (e & 1)));
    }
}

// Orders a wavefront's own LDS writes before its following LDS reads (and the reverse).  The
// LDS executes one wavefront's accesses in program order; this only pins the program order.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Output staging.  In the accumulator layout one store instruction would touch 32 different
// rows with 32 (fp32) or 16 (bf16) bytes each, which the memory pipeline handles as 32 partial
// cache-line writes.  Each wavefront therefore passes its results through a private LDS block
// of 32 rows x WCOLS columns (rows padded by 16 bytes: conflict-free both ways) and stores
// them row-contiguously: 16 bytes per lane, 512 (fp32) or 256 (bf16) contiguous bytes per row.
constexpr int EPI_XCHG_BYTES = 8192;   // statistics exchange between wavefronts comes first

template <int WCOLS>
struct StageF32 {
    static constexpr int RS = WCOLS * 4 + 16;     // row stride in bytes
    static constexpr int BYTES = 32 * RS;
    static constexpr int LPR = WCOLS / 4;         // lanes per row on the way out
    static constexpr int RPI = 64 / LPR;          // rows per store instruction
    static constexpr int STEPS = 32 / RPI;
};
template <int WCOLS>
struct StageBf16 {
    static constexpr int RS = WCOLS * 2 + 16;
    static constexpr int BYTES = 32 * RS;
    static constexpr int LPR = WCOLS / 8;
    static constexpr int RPI = 64 / LPR;
    static constexpr int STEPS = 32 / RPI;
};

// Wavefront-private staging block -> global memory, bf16: 16 bytes per lane, row-contiguous.
template <typename St, bool STREAM>
__device__ __forceinline__ void flush_stage_bf16(const char* region, u16* Y, int ldy, int row_first, int M, int ocol,
                                                 int N, bool vec, bool interior, int orow, int ochunk) {
    if (interior) {
        uintx4 v[St::STEPS];
#pragma unroll
        for (int s = 0; s < St::STEPS; ++s)
            v[s] = *reinterpret_cast<const uintx4*>(region + (s * St::RPI + orow) * St::RS + ochunk * 16);
#pragma unroll
        for (int s = 0; s < St::STEPS; ++s) asm volatile("" : "+v"(v[s]));
#pragma unroll
        for (int s = 0; s < St::STEPS; ++s)
        {
            uintx4* dst = reinterpret_cast<uintx4*>(Y + (size_t)(row_first + s * St::RPI + orow) * ldy + ocol);
            if (STREAM) __builtin_nontemporal_store(v[s], dst);
            else *dst = v[s];
        }
    } else {
#pragma unroll
        for (int s = 0; s < St::STEPS; ++s) {
            const int rr = s * St::RPI + orow;
            const uint4 v = *reinterpret_cast<const uint4*>(region + rr * St::RS + ochunk * 16);
            if (row_first + rr < M) store8_bf16(Y + (size_t)(row_first + rr) * ldy, ocol, N, vec, v);
        }
    }
}

// The LDS buffers of the main loop are free when the epilogue runs: `xchg` (EPI_XCHG_BYTES, shared
// by the workgroup) carries the statistics exchange between the WN wavefronts that share a row,
// `region` (StageF32<WCOLS>::BYTES, private to the calling wavefront) is its staging block.
// STREAM: the output is written with non-temporal stores, so that it does not push the operand
// panels the workgroup's next tile re-reads out of the L2 (measured: +6..10 % per launch with
// four tiles per workgroup, -1.6 % with one; the launcher picks by tiles per workgroup).  A
// compile-time choice: two stores that differ only in that hint get merged into a plain one.
template <Epi EPI, int NJ, int WN, bool STREAM>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[4][NJ], const GemmBf16Params& g, int tile_m, int tile_n,
                                              char* xchg, char* region) {
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
        typedef StageF32<WCOLS> St;
        constexpr bool ACCUM = (EPI == Epi::AccumF32);
        const bool vec = (g.ldc % 4 == 0) && (((uintptr_t)g.C & 15u) == 0);
        const int orow = lane / St::LPR, ochunk = lane % St::LPR;
        const int col = n0 + wn * WCOLS + ochunk * 4;
        const bool fullc = vec && (col + 4 <= g.N);
        const bool interior = vec && (m0 + BM <= g.M) && (n0 + BN <= g.N);   // uniform over the workgroup
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row0 = m0 + wm * 128 + i * 32 + orow;
            // the old values of C start their way from memory before the staging round trip
            floatx4 cv[St::STEPS];
            if (ACCUM) {
#pragma unroll
                for (int s = 0; s < St::STEPS; ++s) {
                    const int row = row0 + s * St::RPI;
                    cv[s] = floatx4{0.f, 0.f, 0.f, 0.f};
                    if (fullc && row < g.M) {
                        const floatx4* src = reinterpret_cast<const floatx4*>(g.C + (size_t)row * g.ldc + col);
                        cv[s] = STREAM ? __builtin_nontemporal_load(src) : *src;
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    *reinterpret_cast<floatx4*>(region + l32 * St::RS + (j * 32 + 8 * q + 4 * hf) * 4) = v;
                }
            wave_lds_fence();
            if (interior) {
                // whole tile inside the matrix: all staged rows are fetched first, then stored
                floatx4 v[St::STEPS];
#pragma unroll
                for (int s = 0; s < St::STEPS; ++s)
                    v[s] = *reinterpret_cast<const floatx4*>(region + (s * St::RPI + orow) * St::RS + ochunk * 16);
#pragma unroll
                for (int s = 0; s < St::STEPS; ++s) asm volatile("" : "+v"(v[s]));
#pragma unroll
                for (int s = 0; s < St::STEPS; ++s) {
                    if (ACCUM) v[s] += cv[s];
                    floatx4* dst = reinterpret_cast<floatx4*>(g.C + (size_t)(row0 + s * St::RPI) * g.ldc + col);
                    if (STREAM) __builtin_nontemporal_store(v[s], dst);
                    else *dst = v[s];
                }
            } else {
#pragma unroll
                for (int s = 0; s < St::STEPS; ++s) {
                    const int rr = s * St::RPI + orow;
                    const int row = row0 + s * St::RPI;
                    floatx4 v = *reinterpret_cast<const floatx4*>(region + rr * St::RS + ochunk * 16);
                    if (row < g.M) {
                        float* crow = g.C + (size_t)row * g.ldc;
                        if (fullc) {
                            if (ACCUM) v += cv[s];
                            *reinterpret_cast<floatx4*>(crow + col) = v;
                        } else {
                            store4_f32<ACCUM>(crow, col, g.N, false, v);
                        }
                    }
                }
            }
            wave_lds_fence();
        }
    }

    if (EPI == Epi::DLogits) {
        // D = (softmax - G) * scale with the global statistics (pass T of Algorithm 1, with
        // the logits taken from the accumulators instead of memory)
        typedef StageBf16<WCOLS> St;
        const bool vec = (g.ldy % 8 == 0) && (((uintptr_t)g.Y & 15u) == 0);
        const bool interior = vec && (m0 + BM <= g.M) && (n0 + BN <= g.N);   // uniform over the workgroup
        const int orow = lane / St::LPR, ochunk = lane % St::LPR;
        const int ocol = n0 + wn * WCOLS + ochunk * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = rbase + i * 32;
            const int rowc = row < g.M ? row : g.M - 1;      // rows past the end compute on a copy, store nothing
            const float m = g.gmax[rowc];
            const float inv = 1.0f / g.gsum[rowc];
            const int64_t lab64 = g.labels[rowc] - g.shard_offset - cbase;
            // column of the label relative to cbase, or -1 when it is not in this lane's range
            const int lab = (lab64 >= 0 && lab64 < WCOLS) ? (int)lab64 : -1;
            const float ml2 = m * LOG2E;
            const float f = inv * g.scale;
            // the one-hot term touches at most one element per row: a wavefront-uniform branch
            // keeps the 64 compares out of the common case
            const bool any_label = __builtin_amdgcn_ballot_w64(lab >= 0) != 0;
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float d[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) d[e] = exp2_fast(fmaf(acc[i][j][4 * q + e], LOG2E, -ml2)) * f;
                    if (any_label) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (lab == j * 32 + 8 * q + e) d[e] -= g.scale;
                    }
                    *reinterpret_cast<uint2*>(region + l32 * St::RS + (j * 32 + 8 * q + 4 * hf) * 2) =
                        make_uint2(pack_bf16x2(d[0], d[1]), pack_bf16x2(d[2], d[3]));
                }
            wave_lds_fence();
            flush_stage_bf16<St, STREAM>(region, g.Y, g.ldy, m0 + wm * 128 + i * 32, g.M, ocol, g.N, vec, interior, orow, ochunk);
            wave_lds_fence();
        }
    }

    if (EPI == Epi::FwdStats) {
        // shard-local m' and sum' of Algorithm 1's pass S, restricted to this tile's 256
        // columns; the per-tile pairs are folded afterwards exactly like shards are (online
        // softmax rescaling).  A lane reduces its 64 columns of a row in registers, one
        // exchange with lane ^ 32 completes the wavefront's 128 columns, and the two wavefronts
        // that share the row meet in LDS.
        typedef StageBf16<WCOLS> St;
        float* xm = reinterpret_cast<float*>(xchg);          // [WN][256]
        float* xs = xm + WN * 256;                             // [WN][256]
        const bool vec = g.Y && (g.ldy % 8 == 0) && (((uintptr_t)g.Y & 15u) == 0);
        const bool interior = vec && (m0 + BM <= g.M) && (n0 + BN <= g.N);   // uniform over the workgroup
        const int orow = lane / St::LPR, ochunk = lane % St::LPR;
        const int ocol = n0 + wn * WCOLS + ochunk * 8;
        if (n0 + BN > g.N) {
            // ragged last column tile: columns past the shard take -inf, which leaves the
            // maximum alone and adds exp(-inf) = 0 to the sum
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (cbase + j * 32 + 8 * (r >> 2) + (r & 3) >= g.N) acc[i][j][r] = -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = rbase + i * 32;
            float v = acc[i][0][0];
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) v = fmaxf(v, acc[i][j][r]);
            const float m = fmaxf(v, __shfl_xor(v, 32, 64));
            // a wavefront whose 128 columns all lie past the shard has m = -inf; its sum is
            // never used (the fold below skips it)
            const float ml2 = m * LOG2E;
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) s += exp2_fast(fmaf(acc[i][j][r], LOG2E, -ml2));
            s += __shfl_xor(s, 32, 64);
            if (hf == 0) {
                const int lr = wm * 128 + i * 32 + l32;
                xm[wn * 256 + lr] = m;
                xs[wn * 256 + lr] = s;
            }
            {
                const int64_t lab64 = (row < g.M ? g.labels[row] : (int64_t)-1) - g.shard_offset - cbase;
                const bool mine = row < g.M && lab64 >= 0 && lab64 < WCOLS && (lab64 & 4) == 0 && lab64 + cbase < g.N;
                // at most one element per row is a target logit: wavefront-uniform branch
                if (__builtin_amdgcn_ballot_w64(mine) != 0) {
                    const int lab = mine ? (int)lab64 : -1;
                    float t = 0.f;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (lab == j * 32 + 8 * (r >> 2) + (r & 3)) t = acc[i][j][r];
                    if (mine) g.part_tgt[row] = t;
                }
            }
            if (g.Y) {
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<uint2*>(region + l32 * St::RS + (j * 32 + 8 * q + 4 * hf) * 2) =
                            make_uint2(pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]),
                                       pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]));
                wave_lds_fence();
                flush_stage_bf16<St, STREAM>(region, g.Y, g.ldy, m0 + wm * 128 + i * 32, g.M, ocol, g.N, vec, interior, orow, ochunk);
                wave_lds_fence();
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
