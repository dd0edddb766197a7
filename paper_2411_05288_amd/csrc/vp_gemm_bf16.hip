// bf16 x bf16 -> fp32 MFMA GEMM for gfx950 with the vocabulary-layer epilogues.
//
// One kernel template serves the three dense products of the output layer (section 4.2 of
// the paper: Y = X W^T, dX = D W, dW = D^T X).  C[M,N] = A[M,K] * B[N,K]^T where each operand
// is stored either with K contiguous ("kcontig", read from LDS with one 16-byte load per
// MFMA operand) or with K strided (stored as [K][rows]).
//
// Work decomposition: 256x256 output tile per workgroup of 4 wavefronts (2x2), each
// wavefront owns 128x128 = 4x4 tiles of the 32x32x16 bf16 MFMA (256 fp32 accumulators per
// lane).  K advances in steps of 64 through two LDS stages; the global loads of step k+1 are
// issued before the MFMAs of step k and written to the other stage afterwards.
//
// MFMA 32x32x16 operand layout (wave64): lane l supplies row (l % 32) of its operand and the
// 8 consecutive k values starting at 8 * (l / 32).  The accumulator layout and the epilogues
// are shared with the fast kernel.
#include <atomic>

#include "vp_gemm_bf16_common.h"

namespace vp {

constexpr int KC_ROW_BYTES = BK * 2;          // 128 B per row of a kcontig tile
constexpr int KC_TILE_BYTES = 256 * KC_ROW_BYTES;           // 32 KB
constexpr int KS_ROW_BYTES = 256 * 2 + 16;    // k-strided tile: [BK][256] bf16 + pad
constexpr int KS_TILE_BYTES = BK * KS_ROW_BYTES;            // 33 KB
constexpr int OPERAND_BYTES = KS_TILE_BYTES;  // slot size that fits either layout
constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;
constexpr int LDS_BYTES = 2 * STAGE_BYTES;    // two stages: ~132 KB of the 160 KB per CU

// 16-byte chunk of 8 bf16 from a [rows][cols] row-major matrix at (row, col), zero-filled
// outside the matrix.  vec_ok: rows start 16-byte aligned and col is a multiple of 8.
__device__ __forceinline__ uint4 load_chunk(const u16* __restrict__ p, int row, int col, int rows, int cols,
                                            int ld, int vec_ok) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (row < rows) {
        const u16* q = p + (size_t)row * ld + col;
        if (vec_ok && col + 8 <= cols) {
            v = *reinterpret_cast<const uint4*>(q);
        } else {
            u16 e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = (col + j < cols) ? q[j] : (u16)0;
            v.x = e[0] | ((unsigned)e[1] << 16);
            v.y = e[2] | ((unsigned)e[3] << 16);
            v.z = e[4] | ((unsigned)e[5] << 16);
            v.w = e[6] | ((unsigned)e[7] << 16);
        }
    }
    return v;
}

// Global -> registers for one 256 x 64 operand tile (8 chunks of 16 B per thread).
//  kcontig : matrix stored [R][K]; chunk q -> row q/8, k-chunk q%8 (8 lanes read 128 B of a row)
//  kstrided: matrix stored [K][R]; chunk q -> k-row q/32, row-chunk q%32 (32 lanes read 512 B)
template <bool KC>
__device__ __forceinline__ void load_tile(uint4 (&r)[8], const u16* __restrict__ p, int r0, int k0, int R, int K,
                                          int ld, int vec_ok, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int q = tid + NT * i;
        if (KC) {
            r[i] = load_chunk(p, r0 + (q >> 3), k0 + (q & 7) * 8, R, K, ld, vec_ok);
        } else {
            r[i] = load_chunk(p, k0 + (q >> 5), r0 + (q & 31) * 8, K, R, ld, vec_ok);
        }
    }
}

// Registers -> LDS.  kcontig tiles are [256][64] bf16 with the 16-byte chunk index XOR-ed
// with (row >> 1) & 7, which makes both these stores and the operand reads bank-conflict free.
template <bool KC>
__device__ __forceinline__ void store_tile(const uint4 (&r)[8], char* s, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int q = tid + NT * i;
        if (KC) {
            const int row = q >> 3, c = q & 7;
            *reinterpret_cast<uint4*>(s + row * KC_ROW_BYTES + ((c ^ ((row >> 1) & 7)) << 4)) = r[i];
        } else {
            const int krow = q >> 5, c = q & 31;
            *reinterpret_cast<uint4*>(s + krow * KS_ROW_BYTES + (c << 4)) = r[i];
        }
    }
}

// MFMA operand for tile row `row` (0..255 within the block tile), k sub-step kk (0..3), lane half hf.
template <bool KC>
__device__ __forceinline__ bf16x8 read_frag(const char* s, int row, int kk, int hf) {
    if (KC) {
        const int chunk = kk * 2 + hf;
        return *reinterpret_cast<const bf16x8*>(s + row * KC_ROW_BYTES + ((chunk ^ ((row >> 1) & 7)) << 4));
    } else {
        union { u16 e[8]; bf16x8 v; } u;
        const int kbase = kk * 16 + hf * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            u.e[j] = *reinterpret_cast<const u16*>(s + (kbase + j) * KS_ROW_BYTES + row * 2);
        return u.v;
    }
}

template <bool A_KC, bool B_KC, Epi EPI>
__global__ __launch_bounds__(NT) void gemm_bf16_kernel(GemmBf16Params g) {
    __shared__ __attribute__((aligned(16))) char smem[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hf = lane >> 5;

    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    int tile_m, tile_n;
    tile_of_block(blockIdx.x, gridDim.x, tiles_m * tiles_n, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    if (EPI == Epi::FwdStats && n0 + BN > g.N) init_acc_ragged<4, 2>(acc, g.N, tile_n);

    uint4 ra[8], rb[8];
    const int nkt = (g.K + BK - 1) / BK;

    load_tile<A_KC>(ra, g.A, m0, 0, g.M, g.K, g.lda, g.vec_ok, tid);
    load_tile<B_KC>(rb, g.B, n0, 0, g.N, g.K, g.ldb, g.vec_ok, tid);
    store_tile<A_KC>(ra, smem, tid);
    store_tile<B_KC>(rb, smem + OPERAND_BYTES, tid);
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const char* sA = smem + (kt & 1) * STAGE_BYTES;
        const char* sB = sA + OPERAND_BYTES;
        const bool more = (kt + 1 < nkt);
        if (more) {
            load_tile<A_KC>(ra, g.A, m0, (kt + 1) * BK, g.M, g.K, g.lda, g.vec_ok, tid);
            load_tile<B_KC>(rb, g.B, n0, (kt + 1) * BK, g.N, g.K, g.ldb, g.vec_ok, tid);
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 af[4], bfr[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) af[t] = read_frag<A_KC>(sA, wm * 128 + t * 32 + l32, kk, hf);
#pragma unroll
            for (int t = 0; t < 4; ++t) bfr[t] = read_frag<B_KC>(sB, wn * 128 + t * 32 + l32, kk, hf);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    mfma_tile<EPI>(acc[i][j], af[i], bfr[j]);
        }
        if (more) {
            char* dA = smem + ((kt + 1) & 1) * STAGE_BYTES;
            store_tile<A_KC>(ra, dA, tid);
            store_tile<B_KC>(rb, dA + OPERAND_BYTES, tid);
        }
        __syncthreads();
    }

    gemm_epilogue<EPI, 4, 2, false>(acc, g, tile_m, tile_n, smem, smem + EPI_XCHG_BYTES + wave * StageF32<128>::BYTES);
}

template <bool A_KC, bool B_KC, Epi EPI>
static hipError_t launch_t(const GemmBf16Params& p, hipStream_t st) {
    const int tiles = (int)(ceil_div(p.M, BM) * ceil_div(p.N, BN));
    hipLaunchKernelGGL((gemm_bf16_kernel<A_KC, B_KC, EPI>), dim3(tiles), dim3(NT), 0, st, p);
    return hipGetLastError();
}

// Test switch: route every product through the generic kernel.
static std::atomic<bool> g_force_generic{false};
void gemm_bf16_force_generic(bool on) { g_force_generic.store(on, std::memory_order_relaxed); }

hipError_t launch_gemm_bf16(const GemmBf16Params& p, hipStream_t st) {
    if (p.M <= 0 || p.N <= 0 || p.K <= 0) return hipErrorInvalidValue;
    // the epilogue addresses the 256 rows of an output tile with 32-bit byte offsets
    const bool f32_out = p.epi == Epi::StoreF32 || p.epi == Epi::AccumF32;
    if (f32_out ? (long long)p.ldc * 4 > EPI_MAX_ROW_BYTES : (p.Y && (long long)p.ldy * 2 > EPI_MAX_ROW_BYTES))
        return hipErrorInvalidValue;
    const int kid = p.kernel_id ? p.kernel_id
                  : p.epi == Epi::FwdStats ? K_GEMM_FWD_STATS
                  : p.epi == Epi::DLogits  ? K_GEMM_DLOGITS
                  : p.epi == Epi::AccumF32 ? K_GEMM_DH : K_GEMM_DW;
    ProfScope prof(kid, st);
    if (!g_force_generic.load(std::memory_order_relaxed) && gemm_bf16_fast_ok(p)) {
        GemmBf16Params q = p;
        q.kernel_id = kid;
        return launch_gemm_bf16_fast(q, st);
    }
    // only the operand-layout / epilogue combinations the output layer uses are instantiated
    if (p.a_kcontig && p.b_kcontig && p.epi == Epi::FwdStats) return launch_t<true, true, Epi::FwdStats>(p, st);
    if (p.a_kcontig && p.b_kcontig && p.epi == Epi::DLogits) return launch_t<true, true, Epi::DLogits>(p, st);
    if (p.a_kcontig && !p.b_kcontig && p.epi == Epi::AccumF32) return launch_t<true, false, Epi::AccumF32>(p, st);
    if (p.a_kcontig && !p.b_kcontig && p.epi == Epi::StoreF32) return launch_t<true, false, Epi::StoreF32>(p, st);
    if (!p.a_kcontig && !p.b_kcontig && p.epi == Epi::StoreF32) return launch_t<false, false, Epi::StoreF32>(p, st);
    return hipErrorInvalidValue;
}

}  // namespace vp
