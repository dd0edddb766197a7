// Fast path of the bf16 MFMA GEMM (gfx950): operands go from global memory straight into LDS
// (buffer loads with the LDS bit, 16 bytes per lane), two 64 KB LDS stages, MFMA operands
// prefetched one 16-wide k sub-step ahead, one workgroup barrier per 64-wide k step.
//
// Preconditions (checked by gemm_bf16_fast_ok on the host; anything else takes the generic
// kernel): rows of both operands 16-byte aligned, operands smaller than 4 GB with slack for
// the offsets of the zero-filled tile overhang, and K a multiple of 64 when both operands
// are K-contiguous.
//
// Out-of-range handling relies on the buffer descriptor: every operand is described by a raw
// buffer of exactly its size, so a lane whose 16 bytes start at or beyond the end of the
// matrix receives zeros.  Rows past the end of a K-contiguous operand and k-rows past the
// end of a K-strided operand are therefore zero.  What is NOT zero is the overhang inside
// the matrix (the k tail of a K-contiguous row runs into the next row, the column tail of a
// K-strided row runs into the next k-row): that data is finite and either meets zeros of the
// other operand (k tails; this is why K % 64 == 0 is required when no operand is K-strided)
// or lands in output rows / columns that the epilogue never stores.
//
// LDS layouts (each operand tile is 32 KB, written by 32 wave-wide loads of 1 KB; a load
// writes lane i's 16 bytes at byte 16*i of its 1 KB slot, so the swizzles below are applied to
// the global address each lane fetches):
//   K-contiguous tile  [256 rows][64 k]: 128 B rows; 16-byte chunk c of row r sits at chunk
//       position c ^ (r & 7).  One ds_read_b128 per MFMA operand, conflict free.
//   K-strided tile [64 k][256 rows]: 512 B k-rows of 16 segments of 32 B (16 rows); segment s of
//       k-row k sits at segment position s ^ f(k & 3), f = {0,5,2,7}.  MFMA operands are read
//       with the transposing LDS load (ds_read_b64_tr_b16): in a group of 16 lanes, lane s
//       points at k-row kb + s/4, rows nb + 4*(s%4)..+3, and lane i receives rows nb + i for
//       the four k-rows kb..kb+3.  f makes the 4 k-rows of a group, and the 8 of two groups,
//       fall into different banks.
#include "vp_gemm_bf16_common.h"

namespace vp {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int TILE_BYTES = 32768;             // one operand tile
constexpr int STAGE_BYTES_F = 2 * TILE_BYTES; // A tile then B tile

__shared__ __attribute__((aligned(1024))) char g_stage0[STAGE_BYTES_F];
__shared__ __attribute__((aligned(1024))) char g_stage1[STAGE_BYTES_F];

__device__ __forceinline__ int seg_swizzle(int k_low2) { return k_low2 ^ ((k_low2 & 1) << 2); }

// Byte offsets (within the operand's buffer, before the k advance) of the 8 chunks this lane
// fetches for one operand tile: wave w fills 1 KB slots 8w .. 8w+7 of the tile.
template <bool KC>
__device__ __forceinline__ void tile_voffsets(unsigned (&voff)[8], int r0, int ld, int wave, int lane) {
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
        const int slot = wave * 8 + jj;
        if (KC) {
            const int row = slot * 8 + (lane >> 3);          // row & 7 == lane >> 3
            const int c = (lane & 7) ^ (lane >> 3);
            voff[jj] = ((unsigned)(r0 + row) * (unsigned)ld + (unsigned)(c * 8)) * 2u;
        } else {
            const int krow = slot * 2 + (lane >> 5);
            const int cpos = lane & 31;
            const int seg = (cpos >> 1) ^ seg_swizzle(krow & 3);
            const int c = seg * 2 + (cpos & 1);
            voff[jj] = ((unsigned)krow * (unsigned)ld + (unsigned)(r0 + c * 8)) * 2u;
        }
    }
}

// The k advance is applied to the descriptor (base += kadv, size -= kadv) rather than to the
// per-lane offsets: the offsets stay loop invariant, the advance costs two scalar ops, and the
// range check still sees the true distance to the end of the operand.
__device__ __forceinline__ void issue_tile_loads(const u16* base, unsigned bytes, unsigned kadv,
                                                 const unsigned (&voff)[8], char* tile, int wave) {
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)base + kadv), 0, (int)(bytes - kadv), 0x00020000);
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(tile + (wave * 8 + jj) * 1024), 16, (int)voff[jj], 0, 0,
                                                 0);
    }
}

// Per-lane LDS byte offsets for operand reads of the wavefront's 128 rows (4 MFMA tiles).
//  KC: base[kk] = address of (row = wt*128 + l32, chunk (2kk + hf) ^ (l32 & 7)); tile t adds t*4096
//  KS: base[t]  = address of (k = 8*(b>>1) + s/4, segment of tile t and lane group b, 8*(s&3));
//                 sub-step kk / half rd adds (16kk + 4rd) * 512
template <bool KC>
__device__ __forceinline__ void frag_offsets(int (&base)[4], int wt, int lane) {
    if (KC) {
        const int l32 = lane & 31, hf = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            base[kk] = (wt * 128 + l32) * 128 + ((((kk << 1) | hf) ^ (l32 & 7)) << 4);
    } else {
        const int b = lane >> 4, s = lane & 15;
        const int f = seg_swizzle(s >> 2);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int seg = (wt * 8 + t * 2 + (b & 1)) ^ f;
            base[t] = (8 * (b >> 1) + (s >> 2)) * 512 + seg * 32 + 8 * (s & 3);
        }
    }
}

template <bool KC>
__device__ __forceinline__ bf16x8 read_operand(const char* tile, const int (&base)[4], int t, int kk) {
    if (KC) {
        return *reinterpret_cast<const bf16x8*>(tile + base[kk] + t * 4096);
    } else {
        union { short4v h[2]; bf16x8 v; } u;
        const char* p = tile + base[t] + kk * 8192;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(p));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(p + 2048));
        return u.v;
    }
}

template <bool A_KC, bool B_KC>
__device__ __forceinline__ void read_frags(bf16x8 (&af)[4], bf16x8 (&bf)[4], const char* stage, const int (&abase)[4],
                                           const int (&bbase)[4], int kk) {
#pragma unroll
    for (int t = 0; t < 4; ++t) af[t] = read_operand<A_KC>(stage, abase, t, kk);
#pragma unroll
    for (int t = 0; t < 4; ++t) bf[t] = read_operand<B_KC>(stage + TILE_BYTES, bbase, t, kk);
}

__device__ __forceinline__ void mfma_step(floatx16 (&acc)[4][4], const bf16x8 (&af)[4], const bf16x8 (&bf)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
}

template <bool A_KC, bool B_KC, Epi EPI>
__global__ __launch_bounds__(NT) void gemm_bf16_fast_kernel(GemmBf16Params g) {
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { float z; asm volatile("v_accvgpr_write_b32 %0, 0" : "=a"(z)); acc[i][j][r] = z; }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS bases in SGPRs
    const int wm = wave >> 1, wn = wave & 1;

    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    int tile_m, tile_n;
    tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // raw buffer descriptors sized exactly to the operands: reads beyond return zero
    const unsigned a_bytes = (unsigned)(A_KC ? g.M : g.K) * (unsigned)g.lda * 2u;
    const unsigned b_bytes = (unsigned)(B_KC ? g.N : g.K) * (unsigned)g.ldb * 2u;
    const unsigned a_kstep = A_KC ? (unsigned)BK * 2u : (unsigned)BK * (unsigned)g.lda * 2u;
    const unsigned b_kstep = B_KC ? (unsigned)BK * 2u : (unsigned)BK * (unsigned)g.ldb * 2u;

    unsigned avoff[8], bvoff[8];
    tile_voffsets<A_KC>(avoff, m0, g.lda, wave, lane);
    tile_voffsets<B_KC>(bvoff, n0, g.ldb, wave, lane);
    int abase[4], bbase[4];
    frag_offsets<A_KC>(abase, wm, lane);
    frag_offsets<B_KC>(bbase, wn, lane);

    const int nkt = (g.K + BK - 1) / BK;

    // prologue: tile 0 -> stage 0, wait, then tile 1 -> stage 1 in flight
    issue_tile_loads(g.A, a_bytes, 0u, avoff, g_stage0, wave);
    issue_tile_loads(g.B, b_bytes, 0u, bvoff, g_stage0 + TILE_BYTES, wave);
    __syncthreads();
    if (nkt > 1) {
        issue_tile_loads(g.A, a_bytes, a_kstep, avoff, g_stage1, wave);
        issue_tile_loads(g.B, b_bytes, b_kstep, bvoff, g_stage1 + TILE_BYTES, wave);
    }
    bf16x8 af0[4], bf0[4], af1[4], bf1[4];
    read_frags<A_KC, B_KC>(af0, bf0, g_stage0, abase, bbase, 0);

    // One 64-wide k step on stage `cur` while tile kt+1 lands in `nxt`.  Entry: sub-step 0 operands
    // of tile kt in (af0, bf0).  The barrier sits before the last sub-step's MFMAs: by then every
    // wavefront has read all it needs from `cur`, so tile kt+2 can start streaming into it, and the
    // first operands of tile kt+1 are fetched while the last MFMAs run.
#define VP_K_STEP(cur, nxt, kt)                                                                     \
    {                                                                                               \
        read_frags<A_KC, B_KC>(af1, bf1, cur, abase, bbase, 1);                                      \
        mfma_step(acc, af0, bf0);                                                                   \
        read_frags<A_KC, B_KC>(af0, bf0, cur, abase, bbase, 2);                                      \
        mfma_step(acc, af1, bf1);                                                                   \
        read_frags<A_KC, B_KC>(af1, bf1, cur, abase, bbase, 3);                                      \
        mfma_step(acc, af0, bf0);                                                                   \
        __syncthreads();                                                                            \
        if ((kt) + 2 < nkt) {                                                                       \
            issue_tile_loads(g.A, a_bytes, (unsigned)((kt) + 2) * a_kstep, avoff, cur, wave);           \
            issue_tile_loads(g.B, b_bytes, (unsigned)((kt) + 2) * b_kstep, bvoff, cur + TILE_BYTES, wave); \
        }                                                                                           \
        if ((kt) + 1 < nkt) read_frags<A_KC, B_KC>(af0, bf0, nxt, abase, bbase, 0);                  \
        mfma_step(acc, af1, bf1);                                                                   \
    }

    for (int kt = 0; kt < nkt; kt += 2) {
        VP_K_STEP(g_stage0, g_stage1, kt)
        if (kt + 1 < nkt) VP_K_STEP(g_stage1, g_stage0, kt + 1)
    }
#undef VP_K_STEP
    __syncthreads();   // every wavefront is done with the stages before the epilogue reuses them

    // keep the epilogue's address arithmetic from being hoisted above the main loop, where it
    // would occupy registers (and spill) for the whole kernel
    asm volatile("" : "+s"(tile_m), "+s"(tile_n));
    gemm_epilogue<EPI>(acc, g, tile_m, tile_n, g_stage0);
}

template <bool A_KC, bool B_KC, Epi EPI>
static hipError_t launch_fast_t(const GemmBf16Params& p, hipStream_t st) {
    const int tiles = (int)(ceil_div(p.M, BM) * ceil_div(p.N, BN));
    hipLaunchKernelGGL((gemm_bf16_fast_kernel<A_KC, B_KC, EPI>), dim3(tiles), dim3(NT), 0, st, p);
    return hipGetLastError();
}

bool gemm_bf16_fast_ok(const GemmBf16Params& p) {
    if (!p.vec_ok) return false;
    if (((uintptr_t)p.A | (uintptr_t)p.B) & 15u) return false;
    if ((p.lda % 8) || (p.ldb % 8)) return false;
    if (p.a_kcontig && p.b_kcontig && (p.K % BK)) return false;
    // byte offsets are 32-bit: the furthest lane of the zero-filled overhang must still not wrap
    const uint64_t lim = ((uint64_t)1 << 32) - ((uint64_t)1 << 20);
    const uint64_t a_ext = p.a_kcontig ? ((uint64_t)p.M + BM) * p.lda * 2 + 2 * (uint64_t)p.K + 256
                                       : ((uint64_t)p.K + BK) * p.lda * 2 + 2 * ((uint64_t)p.M + BM);
    const uint64_t b_ext = p.b_kcontig ? ((uint64_t)p.N + BN) * p.ldb * 2 + 2 * (uint64_t)p.K + 256
                                       : ((uint64_t)p.K + BK) * p.ldb * 2 + 2 * ((uint64_t)p.N + BN);
    return a_ext < lim && b_ext < lim;
}

hipError_t launch_gemm_bf16_fast(const GemmBf16Params& p, hipStream_t st) {
    if (p.a_kcontig && p.b_kcontig && p.epi == Epi::FwdStats) return launch_fast_t<true, true, Epi::FwdStats>(p, st);
    if (p.a_kcontig && p.b_kcontig && p.epi == Epi::DLogits) return launch_fast_t<true, true, Epi::DLogits>(p, st);
    if (p.a_kcontig && !p.b_kcontig && p.epi == Epi::AccumF32) return launch_fast_t<true, false, Epi::AccumF32>(p, st);
    if (!p.a_kcontig && !p.b_kcontig && p.epi == Epi::StoreF32) return launch_fast_t<false, false, Epi::StoreF32>(p, st);
    return hipErrorInvalidValue;
}

}  // namespace vp
