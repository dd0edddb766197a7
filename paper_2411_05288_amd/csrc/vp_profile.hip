// Optional per-kernel timing: when switched on, every kernel launch of the library is
// bracketed by a pair of HIP events on the launch stream; vp_profile_read() sums the elapsed
// times per kernel.  Off by default, in which case the library creates no events and keeps
// no state.  This is a measurement aid for the benchmark, not part of the method.
#include <mutex>
#include <vector>

#include "vp_internal.h"

namespace vp {

namespace {
struct Rec { hipEvent_t a, b; int id; };
std::mutex g_mu;
bool g_on = false;
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
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_on) return;
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
// Same instruction and the same 4 x 4 accumulator blocking as the GEMM kernels.
typedef __bf16 prof_bf16x8 __attribute__((ext_vector_type(8)));
typedef float prof_floatx16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void mfma_rate_kernel(const prof_bf16x8* __restrict__ src, float* __restrict__ out,
                                                        int iters) {
    prof_bf16x8 a[4], b[4];
    for (int t = 0; t < 4; ++t) {
        a[t] = src[t * 256 + threadIdx.x];
        b[t] = src[(4 + t) * 256 + threadIdx.x];
    }
    prof_floatx16 acc[4][4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        asm volatile("" : "+v"(a[0]), "+v"(b[0]));   // keeps the loop from being collapsed
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace vp

extern "C" {

vp_status vp_profile_mfma_loop(const void* operands, float* out, int32_t iters, int32_t blocks, void* stream) {
    if (!operands || !out || iters < 1 || blocks < 1 || blocks > 65535) return VP_ERR_INVALID_ARG;
    if (((uintptr_t)operands & 15u) != 0) return VP_ERR_INVALID_ARG;
    hipLaunchKernelGGL(vp::mfma_rate_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const vp::prof_bf16x8*)operands, out, (int)iters);
    return hipGetLastError() == hipSuccess ? VP_OK : VP_ERR_DEVICE;
}

int vp_profile_kernel_count(void) { return vp::K_COUNT; }

const char* vp_profile_kernel_name(int id) { return (id >= 0 && id < vp::K_COUNT) ? vp::kNames[id] : ""; }

vp_status vp_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(vp::g_mu);
    vp::g_on = (on != 0);
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
