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

#include <type_traits>
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

// Pass S, ragged last column tile: the accumulators of the columns past the end of the shard are
// set to -inf before the main loop (the others hold zero).  Their products are exactly zero (rows of
// W past the end are read as zeros), so they stay -inf: they leave the row maximum alone and add
// exp(-inf) = 0 to the sum, with no masking pass over the accumulators in the epilogue.  Written
// straight into the AGPR half of the register file, like the zeros.
template <int NJ, int WN>
__device__ __forceinline__ void init_acc_ragged(floatx16 (&acc)[4][NJ], int n_cols, int tile_n) {
    const int lane = threadIdx.x & 63;
    const int wn = (threadIdx.x >> 6) % WN;
    // this lane holds columns cbase + j*32 + 8*(r/4) + r%4; those below nvalid exist
    const int nvalid = n_cols - (tile_n * BN + wn * (NJ * 32) + 4 * (lane >> 5));
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float z = (j * 32 + 8 * (r >> 2) + (r & 3) < nvalid) ? 0.f : -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i) { float t; asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(t) : "v"(z)); acc[i][j][r] = t; }
        }
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

// Output tiles are stored through a raw buffer descriptor that covers exactly the tile's rows
// (all columns): a lane whose row lies past the end of the matrix then has an offset beyond the
// buffer and the hardware drops its store (a load returns zero), and a lane whose 16-byte chunk
// lies past the last column is given the offset OOB_OFFSET, beyond any such buffer.  This keeps
// the epilogue free of branches: with a branch per store, every store would be followed by a
// full wait on the memory counter (which counts stores as well) and the stores would go out one
// acknowledgement at a time.  The host checks that 256 rows of the output stay below 2 GB.
constexpr unsigned OOB_OFFSET = 0x80000000u;
constexpr long long EPI_MAX_ROW_BYTES = (1ll << 31) / 256;   // limit on ld * sizeof(element) of an output

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rows_rsrc(void* first_row, int rows, unsigned row_bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(first_row, 0, (int)((unsigned)rows * row_bytes), 0x00020000);
}

// Wavefront-private staging block -> global memory, bf16: 16 bytes per lane, row-contiguous.
// `off` is the lane's byte offset of staged row `orow` (or beyond the buffer, see above).
template <typename St, bool STREAM>
__device__ __forceinline__ void flush_stage_bf16(const char* region, __amdgpu_buffer_rsrc_t rs, unsigned off,
                                                 unsigned row_bytes, int orow, int ochunk) {
    // the staged rows are all fetched first, then stored back to back
    uintx4 v[St::STEPS];
#pragma unroll
    for (int s = 0; s < St::STEPS; ++s)
        v[s] = *reinterpret_cast<const uintx4*>(region + (s * St::RPI + orow) * St::RS + ochunk * 16);
#pragma unroll
    for (int s = 0; s < St::STEPS; ++s) asm volatile("" : "+v"(v[s]));
#pragma unroll
    for (int s = 0; s < St::STEPS; ++s)
        __builtin_amdgcn_raw_buffer_store_b128(v[s], rs, (int)(off + (unsigned)(s * St::RPI) * row_bytes), 0, STREAM ? 2 : 0);
}

// The same for outputs whose rows are not 16-byte aligned (or whose last column cuts a chunk).
template <typename St>
__device__ __forceinline__ void flush_stage_bf16_unaligned(const char* region, u16* Y, int ldy, int row_first, int M,
                                                           int ocol, int N, bool aligned, int orow, int ochunk) {
#pragma unroll
    for (int s = 0; s < St::STEPS; ++s) {
        const int rr = s * St::RPI + orow;
        const uint4 v = *reinterpret_cast<const uint4*>(region + rr * St::RS + ochunk * 16);
        if (row_first + rr < M) store8_bf16(Y + (size_t)(row_first + rr) * ldy, ocol, N, aligned, v);
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
__device__ __forceinline__ void gemm_epilogue_f32(floatx16 (&acc)[4][NJ], const GemmBf16Params& g, int tile_m, int tile_n,
                                                  char* region) {
    constexpr int WCOLS = NJ * 32;            // columns owned by one wavefront
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, hf = lane >> 5;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    typedef StageF32<WCOLS> St;
    constexpr bool ACCUM = (EPI == Epi::AccumF32);
    const bool vec = (g.ldc % 4 == 0) && (((uintptr_t)g.C & 15u) == 0);
    const int orow = lane / St::LPR, ochunk = lane % St::LPR;
    const int col = n0 + wn * WCOLS + ochunk * 4;
    const bool interior = vec && (m0 + BM <= g.M) && (n0 + BN <= g.N);   // uniform over the workgroup
    // accumulators of row block i -> the wavefront's staging block
    auto stage = [&](int i) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const floatx4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                *reinterpret_cast<floatx4*>(region + l32 * St::RS + (j * 32 + 8 * q + 4 * hf) * 4) = v;
            }
    };
    if (interior) {
        // Whole tile inside the matrix: straight-line code.  The old values of C are fetched one row
        // block ahead, before the previous block's stores: the memory counter a load is waited on also
        // counts the stores issued before it, so waiting for loads issued after a block's stores would
        // mean waiting for those stores to be acknowledged.
        float* c0 = g.C + (size_t)(m0 + wm * 128 + orow) * g.ldc + col;
        auto c_at = [&](int i, int s) { return reinterpret_cast<floatx4*>(c0 + (size_t)(i * 32 + s * St::RPI) * g.ldc); };
        floatx4 cv[St::STEPS];
        if (ACCUM) {
#pragma unroll
            for (int s = 0; s < St::STEPS; ++s) cv[s] = STREAM ? __builtin_nontemporal_load(c_at(0, s)) : *c_at(0, s);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            stage(i);
            wave_lds_fence();
            // all staged rows are fetched first, then stored
            floatx4 v[St::STEPS];
#pragma unroll
            for (int s = 0; s < St::STEPS; ++s)
                v[s] = *reinterpret_cast<const floatx4*>(region + (s * St::RPI + orow) * St::RS + ochunk * 16);
#pragma unroll
            for (int s = 0; s < St::STEPS; ++s) asm volatile("" : "+v"(v[s]));
            if (ACCUM) {
#pragma unroll
                for (int s = 0; s < St::STEPS; ++s) v[s] += cv[s];
                if (i < 3) {
#pragma unroll
                    for (int s = 0; s < St::STEPS; ++s)
                        cv[s] = STREAM ? __builtin_nontemporal_load(c_at(i + 1, s)) : *c_at(i + 1, s);
                }
            }
#pragma unroll
            for (int s = 0; s < St::STEPS; ++s) {
                if (STREAM) __builtin_nontemporal_store(v[s], c_at(i, s));
                else *c_at(i, s) = v[s];
            }
            wave_lds_fence();
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row0 = m0 + wm * 128 + i * 32 + orow;
            stage(i);
            wave_lds_fence();
#pragma unroll
            for (int s = 0; s < St::STEPS; ++s) {
                const int rr = s * St::RPI + orow;
                const int row = row0 + s * St::RPI;
                const floatx4 v = *reinterpret_cast<const floatx4*>(region + rr * St::RS + ochunk * 16);
                if (row < g.M) store4_f32<ACCUM>(g.C + (size_t)row * g.ldc, col, g.N, vec, v);
            }
            wave_lds_fence();
        }
    }
}

// The epilogues of pass S (FwdStats) and of the fused pass T (DLogits): bf16 outputs.
template <Epi EPI, int NJ, int WN, bool STREAM>
__device__ __forceinline__ void gemm_epilogue_bf16(floatx16 (&acc)[4][NJ], const GemmBf16Params& g, int tile_m, int tile_n,
                                                   char* xchg, char* region) {
    constexpr int WCOLS = NJ * 32;            // columns owned by one wavefront
    // Arithmetic on threadIdx does not depend on the tile, so it is hoisted above the caller's tile
    // loop and main loop, where it occupies (and spills) registers; a reload from the spill area after
    // the first output stores would moreover wait for those stores to be acknowledged (a reload is a
    // load).  These epilogues are short of registers, so they take the lane index from the hardware's
    // lane count and make it opaque: what follows is computed here, per tile.
    int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(lane));
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tid = wave * 64 + lane;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, hf = lane >> 5;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    // element (i, j, r) of this lane: row = rbase + i*32, col = cbase + j*32 + 8*(r/4) + (r%4)
    const int rbase = m0 + wm * 128 + l32;
    const int cbase = n0 + wn * WCOLS + 4 * hf;

    if (EPI == Epi::DLogits) {
        // D = (softmax - G) * scale with the global statistics (pass T of Algorithm 1, with
        // the logits taken from the accumulators instead of memory)
        typedef StageBf16<WCOLS> St;
        // uniform over the grid: rows are 16-byte aligned and chunks are never cut by the last column
        const bool aligned = (g.ldy % 8 == 0) && (((uintptr_t)g.Y & 15u) == 0);
        const bool vec = aligned && (g.N % 8 == 0);
        const int orow = lane / St::LPR, ochunk = lane % St::LPR;
        const int ocol = n0 + wn * WCOLS + ochunk * 8;
        const unsigned row_bytes = (unsigned)g.ldy * 2u;
        const __amdgpu_buffer_rsrc_t rs =
            tile_rows_rsrc(g.Y + (size_t)m0 * g.ldy, g.M - m0 < BM ? g.M - m0 : BM, row_bytes);
        const unsigned off0 =
            (ocol + 8 <= g.N) ? (unsigned)(wm * 128 + orow) * row_bytes + (unsigned)ocol * 2u : OOB_OFFSET;
        // all loads come before the first store (see the note on the labels in the FwdStats branch)
        float ml2_[4], f_[4];
        int lab_[4];
        {
            float gm[4], gs[4];
            int64_t lraw[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = rbase + i * 32;
                const int rowc = row < g.M ? row : g.M - 1;      // rows past the end compute on a copy, store nothing
                gm[i] = g.gmax[rowc];
                gs[i] = g.gsum[rowc];
                lraw[i] = g.labels[rowc];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t lab64 = lraw[i] - g.shard_offset - cbase;
                // column of the label relative to cbase, or -1 when it is not in this lane's range
                lab_[i] = (lab64 >= 0 && lab64 < WCOLS) ? (int)lab64 : -1;
                ml2_[i] = gm[i] * LOG2E;
                f_[i] = (1.0f / gs[i]) * g.scale;
            }
            // keep the derived values, not the inputs
            asm volatile("" : "+v"(lab_[0]), "+v"(lab_[1]), "+v"(lab_[2]), "+v"(lab_[3]));
            asm volatile("" : "+v"(ml2_[0]), "+v"(ml2_[1]), "+v"(ml2_[2]), "+v"(ml2_[3]));
            asm volatile("" : "+v"(f_[0]), "+v"(f_[1]), "+v"(f_[2]), "+v"(f_[3]));
        }
        auto blocks = [&](auto vec_c) {
            constexpr bool VEC = decltype(vec_c)::value;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // One row block at a time: left alone, the scheduler uses every free register to overlap the
                // blocks and then spills, and a reload after the first stores waits for them (a reload is a load).
                __builtin_amdgcn_sched_barrier(0);
                const int lab = lab_[i];
                const float ml2 = ml2_[i];
                const float f = f_[i];
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
                if (VEC) flush_stage_bf16<St, STREAM>(region, rs, off0 + (unsigned)(i * 32) * row_bytes, row_bytes, orow, ochunk);
                else flush_stage_bf16_unaligned<St>(region, g.Y, g.ldy, m0 + wm * 128 + i * 32, g.M, ocol, g.N, aligned, orow, ochunk);
                wave_lds_fence();
            }
        };
        // (chosen once, outside the loop: see the fp32 branch above)
        if (vec) blocks(std::true_type{});
        else blocks(std::false_type{});
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
        // uniform over the grid: rows are 16-byte aligned and chunks are never cut by the last column
        const bool aligned = g.Y && (g.ldy % 8 == 0) && (((uintptr_t)g.Y & 15u) == 0);
        const bool vec = aligned && (g.N % 8 == 0);
        const int orow = lane / St::LPR, ochunk = lane % St::LPR;
        const int ocol = n0 + wn * WCOLS + ochunk * 8;
        const unsigned row_bytes = (unsigned)g.ldy * 2u;
        const __amdgpu_buffer_rsrc_t rs =
            tile_rows_rsrc(g.Y ? g.Y + (size_t)m0 * g.ldy : nullptr, g.Y ? (g.M - m0 < BM ? g.M - m0 : BM) : 0, row_bytes);
        const unsigned off0 =
            (ocol + 8 <= g.N) ? (unsigned)(wm * 128 + orow) * row_bytes + (unsigned)ocol * 2u : OOB_OFFSET;
        // The labels of the wavefront's four row blocks are fetched before the first store of
        // logits: the memory counter a load is waited on also counts the stores issued before it,
        // so a load inside the loop below would wait for the previous block's stores to be
        // acknowledged and serialise the epilogue.
        int64_t lraw[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) lraw[i] = (rbase + i * 32 < g.M) ? g.labels[rbase + i * 32] : (int64_t)-1;
        // lab[i]: column of row block i's label relative to cbase if this lane holds it, else -1
        int lab[4];
        // (columns past the shard in the ragged last column tile hold -inf: see init_acc)
        // MODE 0: the logits are not kept; 1: stored through the tile's buffer descriptor; 2: unaligned rows
        auto blocks = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __builtin_amdgcn_sched_barrier(0);          // one row block at a time (see the DLogits branch)
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
            if (i == 0) {
                // the four loads have had the first block's arithmetic to arrive
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int64_t lab64 = lraw[k] - g.shard_offset - cbase;
                    const bool mine = lraw[k] >= 0 && lab64 >= 0 && lab64 < WCOLS && (lab64 & 4) == 0 && lab64 + cbase < g.N;
                    lab[k] = mine ? (int)lab64 : -1;
                }
                asm volatile("" : "+v"(lab[0]), "+v"(lab[1]), "+v"(lab[2]), "+v"(lab[3]));   // narrowed here, not at the use
            }
            // at most one element per row is a target logit: wavefront-uniform branch
            if (__builtin_amdgcn_ballot_w64(lab[i] >= 0) != 0) {
                float t = 0.f;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (lab[i] == j * 32 + 8 * (r >> 2) + (r & 3)) t = acc[i][j][r];
                if (lab[i] >= 0) g.part_tgt[rbase + i * 32] = t;
            }
            if (MODE != 0) {
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<uint2*>(region + l32 * St::RS + (j * 32 + 8 * q + 4 * hf) * 2) =
                            make_uint2(pack_bf16x2(acc[i][j][4 * q], acc[i][j][4 * q + 1]),
                                       pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]));
                wave_lds_fence();
                if (MODE == 1) flush_stage_bf16<St, STREAM>(region, rs, off0 + (unsigned)(i * 32) * row_bytes, row_bytes, orow, ochunk);
                else flush_stage_bf16_unaligned<St>(region, g.Y, g.ldy, m0 + wm * 128 + i * 32, g.M, ocol, g.N, aligned, orow, ochunk);
                wave_lds_fence();
            }
        }
        };
        // (chosen once, outside the loop: see the fp32 branch above)
        if (!g.Y) blocks(std::integral_constant<int, 0>{});
        else if (vec) blocks(std::integral_constant<int, 1>{});
        else blocks(std::integral_constant<int, 2>{});
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

template <Epi EPI, int NJ, int WN, bool STREAM>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[4][NJ], const GemmBf16Params& g, int tile_m, int tile_n,
                                              char* xchg, char* region) {
    if constexpr (EPI == Epi::StoreF32 || EPI == Epi::AccumF32)
        gemm_epilogue_f32<EPI, NJ, WN, STREAM>(acc, g, tile_m, tile_n, region);
    else
        gemm_epilogue_bf16<EPI, NJ, WN, STREAM>(acc, g, tile_m, tile_n, xchg, region);
}

}  // namespace vp
