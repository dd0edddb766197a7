// Optional per-kernel timing: when switched on, every kernel launch of the library is
// bracketed by a pair of HIP events on the launch stream; vp_profile_read() sums the elapsed
// times per kernel.  Off by default, in which case the library creates no events and keeps
// no state.  This is a measurement aid for the benchmark, not part of the method.
#include <atomic>
#include <mutex>
#include <vector>

#include "vp_internal.h"

namespace vp {

namespace {
struct Rec { hipEvent_t a, b; int id; };
std::mutex g_mu;
std::atomic<bool> g_on{false};   // read without the lock: a launch made while timing is off touches nothing else
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;

hipEvent_t take_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

ProfScope::ProfScope(int id, hipStream_t st) : id_(id), st_(st), a_(nullptr) {
    if (!g_on.load(std::memory_order_acquire)) return;
    std::lock_guard<std::mutex> lk(g_mu);
    a_ = take_event();
    if (a_) (void)hipEventRecord((hipEvent_t)a_, st_);
}

ProfScope::~ProfScope() {
    if (!a_) return;
    std::lock_guard<std::mutex> lk(g_mu);
    hipEvent_t b = take_event();
    if (!b) { g_pool.push_back((hipEvent_t)a_); return; }
    (void)hipEventRecord(b, st_);
    g_recs.push_back(Rec{(hipEvent_t)a_, b, id_});
}

static const char* const kNames[K_COUNT] = {
    "gemm_bf16_fwd_stats", "gemm_bf16_dlogits", "gemm_bf16_dH", "gemm_bf16_dW", "fold_partials",
    "combine_stats", "dlogits_elementwise", "gemm_f32", "row_stats_f32", "embed_fwd",
    "embed_bwd_sort", "embed_bwd_accum", "gemm_bf16_A_alg2", "dx_alg2"};

}  // namespace vp

namespace vp {
// Back-to-back MFMAs on register operands, no memory traffic in the loop: what the matrix cores
// sustain for the VALUES they are given (the chip is power limited and the rate depends on the
// bit patterns: zeros run near the nominal peak, normally distributed operands far below it).
// Each wavefront owns a 128 x 128 block of accumulators, like the GEMM kernels; the variants
// differ in instruction shape and issue order:
//   0  32x32x16, 4 x 4 tiles, column by column                 (16 MFMAs per iteration)
//   1  32x32x16, 4 x 4 tiles, column by column in a snake      (16)
//   2  32x32x16, two k sub-steps chained on each accumulator   (32)
//   3  32x32x16, four k sub-steps chained on each accumulator  (64)
//   4  16x16x32, 8 x 8 tiles, column by column                 (64, half the flops each)
//   5  16x16x32, 8 x 8 tiles, snake                            (64)
typedef __bf16 prof_bf16x8 __attribute__((ext_vector_type(8)));
typedef float prof_floatx16 __attribute__((ext_vector_type(16)));
typedef float prof_floatx4 __attribute__((ext_vector_type(4)));

constexpr int MFMA_VARIANTS = 6;
constexpr int MFMA_OPERAND_FRAGS = 32;   // fragments of 16 bytes per lane in the operand buffer

static double mfma_variant_flops_per_iter(int variant) {
    const double f32 = 2.0 * 32 * 32 * 16, f16 = 2.0 * 16 * 16 * 32;
    switch (variant) {
        case 0: case 1: return 16 * f32;
        case 2: return 32 * f32;
        case 3: return 64 * f32;
        case 4: case 5: return 64 * f16;
    }
    return 0.0;
}

template <int VARIANT>
__global__ __launch_bounds__(256) void mfma_rate_kernel(const prof_bf16x8* __restrict__ src, float* __restrict__ out,
                                                        int iters) {
    float s = 0.f;
    if constexpr (VARIANT <= 3) {
        constexpr int KD = VARIANT == 2 ? 2 : (VARIANT == 3 ? 4 : 1);   // k sub-steps held in registers
        prof_bf16x8 a[KD][4], b[KD][4];
        for (int k = 0; k < KD; ++k)
            for (int t = 0; t < 4; ++t) {
                a[k][t] = src[(k * 8 + t) * 256 + threadIdx.x];
                b[k][t] = src[(k * 8 + 4 + t) * 256 + threadIdx.x];
            }
        prof_floatx16 acc[4][4];
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 4; ++j)
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    const int i = (VARIANT == 1 && (j & 1)) ? 3 - ii : ii;
#pragma unroll
                    for (int k = 0; k < KD; ++k)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[k][j], a[k][i], acc[i][j], 0, 0, 0);
                    if (KD > 1) __builtin_amdgcn_sched_barrier(0);   // keep the chain on one accumulator together
                }
            asm volatile("" : "+v"(a[0][0]), "+v"(b[0][0]));   // keeps the loop from being collapsed
        }
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 4; ++j)
                for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    } else {
        prof_bf16x8 a[8], b[8];
        for (int t = 0; t < 8; ++t) {
            a[t] = src[t * 256 + threadIdx.x];
            b[t] = src[(8 + t) * 256 + threadIdx.x];
        }
        prof_floatx4 acc[8][8];
        for (int i = 0; i < 8; ++i)
            for (int j = 0; j < 8; ++j)
                for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int ii = 0; ii < 8; ++ii) {
                    const int i = (VARIANT == 5 && (j & 1)) ? 7 - ii : ii;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
                }
            asm volatile("" : "+v"(a[0]), "+v"(b[0]));
        }
        for (int i = 0; i < 8; ++i)
            for (int j = 0; j < 8; ++j)
                for (int r = 0; r < 4; ++r) s += acc[i][j][r];
    }
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace vp

extern "C" {

vp_status vp_profile_mfma_variant(const void* operands, float* out, int32_t iters, int32_t blocks, int32_t variant,
                                  void* stream) {
    if (!operands || !out || iters < 1 || blocks < 1 || blocks > 65535) return VP_ERR_INVALID_ARG;
    if (variant < 0 || variant >= vp::MFMA_VARIANTS) return VP_ERR_INVALID_ARG;
    if (((uintptr_t)operands & 15u) != 0) return VP_ERR_INVALID_ARG;
    const vp::prof_bf16x8* src = (const vp::prof_bf16x8*)operands;
    const dim3 grid((unsigned)blocks), block(256);
    hipStream_t st = (hipStream_t)stream;
    switch (variant) {
        case 0: hipLaunchKernelGGL(vp::mfma_rate_kernel<0>, grid, block, 0, st, src, out, (int)iters); break;
        case 1: hipLaunchKernelGGL(vp::mfma_rate_kernel<1>, grid, block, 0, st, src, out, (int)iters); break;
        case 2: hipLaunchKernelGGL(vp::mfma_rate_kernel<2>, grid, block, 0, st, src, out, (int)iters); break;
        case 3: hipLaunchKernelGGL(vp::mfma_rate_kernel<3>, grid, block, 0, st, src, out, (int)iters); break;
        case 4: hipLaunchKernelGGL(vp::mfma_rate_kernel<4>, grid, block, 0, st, src, out, (int)iters); break;
        default: hipLaunchKernelGGL(vp::mfma_rate_kernel<5>, grid, block, 0, st, src, out, (int)iters); break;
    }
    return hipGetLastError() == hipSuccess ? VP_OK : VP_ERR_DEVICE;
}

int vp_profile_mfma_variant_count(void) { return vp::MFMA_VARIANTS; }

double vp_profile_mfma_variant_flops(int32_t variant) { return vp::mfma_variant_flops_per_iter(variant); }

vp_status vp_profile_mfma_loop(const void* operands, float* out, int32_t iters, int32_t blocks, void* stream) {
    return vp_profile_mfma_variant(operands, out, iters, blocks, 0, stream);
}

int vp_profile_kernel_count(void) { return vp::K_COUNT; }

const char* vp_profile_kernel_name(int id) { return (id >= 0 && id < vp::K_COUNT) ? vp::kNames[id] : ""; }

vp_status vp_profile_enable(int on) {
    vp::g_on.store(on != 0, std::memory_order_release);
    return VP_OK;
}

vp_status vp_profile_force_generic_gemm(int on) {
    vp::gemm_bf16_force_generic(on != 0);
    return VP_OK;
}

vp_status vp_profile_gemm_trace(void* buffer, size_t bytes, int kernel_id) {
    if (buffer && (((uintptr_t)buffer & 7u) != 0 || bytes < 64)) return VP_ERR_INVALID_ARG;
    if (kernel_id >= vp::K_COUNT) return VP_ERR_INVALID_ARG;
    vp::gemm_bf16_set_trace(buffer, buffer ? bytes : 0, kernel_id);
    return VP_OK;
}

vp_status vp_profile_read(double* ms_total, int64_t* launches, int n) {
    if (!ms_total || !launches || n < vp::K_COUNT) return VP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(vp::g_mu);
    for (int i = 0; i < n; ++i) { ms_total[i] = 0.0; launches[i] = 0; }
    vp_status rc = VP_OK;
    for (const vp::Rec& r : vp::g_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) {
            rc = VP_ERR_DEVICE;
        } else {
            ms_total[r.id] += (double)ms;
            launches[r.id] += 1;
        }
        vp::g_pool.push_back(r.a);
        vp::g_pool.push_back(r.b);
    }
    vp::g_recs.clear();
    return rc;
}

}  // extern "C"
