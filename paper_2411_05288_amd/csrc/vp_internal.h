// Internal declarations shared by the libvp translation units (host side only; device
// code does not call across files).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "vp.h"

namespace vp {

typedef unsigned short u16;  // bf16 bit pattern

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Kernel ids for the optional per-kernel timing (names in vp_profile.hip, same order).
enum KernelId : int {
    K_GEMM_FWD_STATS = 0, K_GEMM_DLOGITS, K_GEMM_DH, K_GEMM_DW, K_FOLD, K_COMBINE, K_DLOGITS_EW, K_GEMM_F32,
    K_ROWSTATS_F32, K_EMBED_FWD, K_EMBED_SORT, K_EMBED_ACCUM, K_GEMM_A_ALG2, K_DX_ALG2, K_COUNT
};

// Brackets the launches made during its lifetime with two events when timing is enabled;
// does nothing (and touches no HIP API) otherwise.
class ProfScope {
public:
    ProfScope(int id, hipStream_t st);
    ~ProfScope();
    ProfScope(const ProfScope&) = delete;
    ProfScope& operator=(const ProfScope&) = delete;
private:
    int id_;
    hipStream_t st_;
    void* a_;
};

// Macro tile of the bf16 MFMA kernels (rows x cols of the output per workgroup).
constexpr int GEMM_BM = 256;
constexpr int GEMM_BN = 256;

// What the bf16 GEMM does with its accumulators.
enum class Epi : int {
    FwdStats = 0,   // per-row partial max / sum-exp / target logit (+ optional bf16 store of Y)
    DLogits = 1,    // D = (exp(Y - m)/sum - onehot) * scale, stored as bf16
    StoreF32 = 2,   // C = acc
    AccumF32 = 3    // C += acc
};

struct GemmBf16Params {
    // operands: A is logically [M, K], B is logically [N, K]
    const u16* A;
    const u16* B;
    int M, N, K;
    int lda, ldb;        // leading dimension in elements of the matrices as stored
    int a_kcontig;       // 1: A stored [M][K]; 0: stored [K][M]
    int b_kcontig;       // 1: B stored [N][K]; 0: stored [K][N]
    int vec_ok;          // 1: all rows of A and B start 16-byte aligned (16-byte loads allowed)
    // epilogue
    Epi epi;
    float* C;            // StoreF32 / AccumF32: [M, N] fp32, ldc
    int ldc;
    u16* Y;              // FwdStats: optional bf16 [M, N] store (ldy); DLogits: D output
    int ldy;
    const int64_t* labels;   // [M]
    int64_t shard_offset;
    float* part_max;     // FwdStats: [tiles_n, M]
    float* part_sum;     // FwdStats: [tiles_n, M]
    float* part_tgt;     // FwdStats: [M], written only for rows whose label is in this shard
    const float* gmax;   // DLogits: [M]
    const float* gsum;   // DLogits: [M]
    float scale;         // DLogits
    int kernel_id;       // timing slot; 0 = chosen from the epilogue (resolved by launch_gemm_bf16)
    unsigned long long* trace;   // measurement aid: phase stamps per workgroup and tile (nullptr: none)
    int trace_cap;               // tiles per workgroup the trace buffer holds
};

// Dispatches to the fast kernel when its preconditions hold (and the generic kernel has not been
// forced through vp_profile_force_generic_gemm), else to the generic kernel.
hipError_t launch_gemm_bf16(const GemmBf16Params& p, hipStream_t st);
void gemm_bf16_force_generic(bool on);
// Measurement aid: device buffer into which the fast kernel's next launches write their phase stamps
// (nullptr: off); kernel_id >= 0 restricts it to the launches timed under that kernel id.
void gemm_bf16_set_trace(void* buf, size_t bytes, int kernel_id);
bool gemm_bf16_fast_ok(const GemmBf16Params& p);
hipError_t launch_gemm_bf16_fast(const GemmBf16Params& p, hipStream_t st);

// Generic strided fp32 GEMM: C[m,n] (+)= sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk].  scratch: nullptr or at
// least gemm_f32_scratch_floats(M, N, K) floats (then small outputs with a long K are computed in K slices).
hipError_t launch_gemm_f32(const float* A, int64_t sam, int64_t sak,
                           const float* B, int64_t sbn, int64_t sbk,
                           float* C, int64_t ldc, int M, int N, int K, bool accumulate, float* scratch,
                           hipStream_t st);
// Floats of scratch with which launch_gemm_f32 cuts K into slices for this shape (0: it would not).
size_t gemm_f32_scratch_floats(int64_t M, int64_t N, int64_t K);

// Row statistics of stored fp32 logits (fp32 path): m', sum', t'
hipError_t launch_row_stats_f32(const float* Y, int64_t ldy, const int64_t* labels, int64_t off,
                                int N, int Vs, float* lmax, float* lsum, float* ltgt, hipStream_t st);

// Fold the per-column-tile partial statistics written by the FwdStats epilogue.
hipError_t launch_fold_partials(const float* part_max, const float* part_sum, const float* part_tgt,
                                int tiles, int N, const int64_t* labels, int64_t off, int Vs,
                                float* lmax, float* lsum, float* ltgt, hipStream_t st);

hipError_t launch_combine(const float* lmax, const float* lsum, const float* ltgt, int p, int N,
                          float* gmax, float* gsum, float* loss_row, float* loss_mean, hipStream_t st);

// D = (exp(Y - m)/sum - onehot) * scale from stored logits; is_bf16 selects the type of Y and D.
// Y has row stride ldy, D row stride ldd (elements); columns Vs..ldd-1 of D are zeroed.
// labels == nullptr: no one-hot term (softmax' of Algorithm 2 with the local statistics).
hipError_t launch_dlogits(const void* Y, int64_t ldy, void* D, int64_t ldd, int is_bf16, const int64_t* labels,
                          int64_t off, const float* gmax, const float* gsum, float scale, int N, int Vs,
                          hipStream_t st);

// dH += (A * c - B) * scale with c_i = lsum_i exp(lmax_i - gmax_i) / gsum_i  (Algorithm 2)
// (overwrite: dH = ... instead of +=)
hipError_t launch_dx_alg2(const float* A, const void* B, int b_is_bf16, const float* lmax, const float* lsum,
                          const float* gmax, const float* gsum, int N, int h, float scale, bool overwrite, float* dH,
                          hipStream_t st);

// Zeroes the padding columns Vs .. ldd-1 of the bf16 matrix D [N, ldd].
hipError_t launch_zero_pad_columns(void* D, int N, int Vs, int64_t ldd, hipStream_t st);

hipError_t launch_embed_fwd(const void* table, const int64_t* ids, int N, int h, int Vs, int64_t off,
                            int elem_bytes, void* out, hipStream_t st);

size_t embed_bwd_workspace(int64_t N);
hipError_t launch_embed_bwd(const void* gout, const int64_t* ids, int N, int h, int Vs, int64_t off,
                            int is_bf16, float* dtable, void* ws, hipStream_t st);

}  // namespace vp
