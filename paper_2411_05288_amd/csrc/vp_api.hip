// extern "C" entry points of libvp: argument validation, workspace carving and the order of
// kernel launches for each pass.  No allocation, no synchronisation, no state.
#include <mutex>

#include "vp_internal.h"

using namespace vp;

namespace {

constexpr int64_t MAX_ELEMS = (int64_t)1 << 31;

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

bool sizes_ok(int64_t N, int64_t h, int64_t Vs) { return N >= 1 && h >= 1 && Vs >= 1; }

// Row lengths are limited to 2^20 elements: the GEMM epilogues address 256 rows of an output with 32-bit byte offsets.
constexpr int64_t MAX_ROW = (int64_t)1 << 20;

bool sizes_supported(int64_t N, int64_t h, int64_t Vs) {
    return N < MAX_ELEMS && h <= MAX_ROW && Vs <= MAX_ROW && N * Vs < MAX_ELEMS && N * h < MAX_ELEMS &&
           Vs * h < MAX_ELEMS;
}

bool dtype_ok(vp_dtype dt) { return dt == VP_F32 || dt == VP_BF16; }

int64_t fwd_tiles(int64_t Vs) { return ceil_div(Vs, GEMM_BN); }

// Row stride (elements) of the bf16 D matrix in the backward workspace: rows start on 128-byte
// boundaries, so the 128-byte row pieces the dH product fetches never straddle two cache lines
// (worth 9 % on that product when Vs * 2 is not a multiple of 128).
int64_t d_row_stride(int64_t Vs) { return (Vs + 63) / 64 * 64; }

size_t max3(size_t a, size_t b, size_t c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }

// fp32 path: bytes of K-slice scratch behind the [N, Vs] matrix at the start of the workspace
size_t f32_fwd_scratch(int64_t N, int64_t h, int64_t Vs) { return gemm_f32_scratch_floats(N, Vs, h) * sizeof(float); }
size_t f32_bwd_scratch(int64_t N, int64_t h, int64_t Vs) {
    return max3(gemm_f32_scratch_floats(N, Vs, h), gemm_f32_scratch_floats(N, h, Vs), gemm_f32_scratch_floats(Vs, h, N)) *
           sizeof(float);
}
size_t f32_matrix_bytes(int64_t N, int64_t Vs) { return align_up((size_t)N * Vs * sizeof(float), 256); }

vp_status dev(hipError_t e) { return e == hipSuccess ? VP_OK : VP_ERR_DEVICE; }

// Scratch of vp_output_fwd_noalloc: device memory that belongs to the library's code object, so the
// entry point has nothing to allocate.  Every GPU the library runs on holds its own copy until the
// process ends.  In host code the array's name is only a handle: its device address is looked up
// once per device (with that device current) and that address is what the kernels are given.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)4 << 20;
constexpr int NOALLOC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
std::mutex g_scratch_mu;
void* g_scratch_ptr[NOALLOC_MAX_DEVICES] = {nullptr};

// Device address of `scratch` on the current device, nullptr if the runtime refuses.
void* scratch_of_current_device() {
    int d = -1;
    if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= NOALLOC_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[d]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[d] = ptr;
    }
    return g_scratch_ptr[d];
}

}  // namespace

extern "C" {

int vp_version(void) { return 100; }

const char* vp_status_string(vp_status s) {
    switch (s) {
        case VP_OK: return "VP_OK";
        case VP_ERR_INVALID_ARG: return "VP_ERR_INVALID_ARG";
        case VP_ERR_UNSUPPORTED: return "VP_ERR_UNSUPPORTED";
        case VP_ERR_WORKSPACE: return "VP_ERR_WORKSPACE";
        case VP_ERR_DEVICE: return "VP_ERR_DEVICE";
    }
    return "VP_ERR_UNKNOWN";
}

size_t vp_workspace_bytes(vp_call which, int64_t N, int64_t h, int64_t Vs, vp_dtype dt, uint32_t flags) {
    const uint32_t allowed =
        which == VP_CALL_OUTPUT_BWD ? (uint32_t)(VP_SAVE_LOGITS | VP_SKIP_DH | VP_DH_OVERWRITE) : (uint32_t)VP_SAVE_LOGITS;
    if (!dtype_ok(dt) || (flags & ~allowed)) return (size_t)-1;
    switch (which) {
        case VP_CALL_OUTPUT_FWD_ALG2:
            // the statistics partials of the forward pass, then the softmax' operand of A = softmax' W
            if (!sizes_ok(N, h, Vs) || !sizes_supported(N, h, Vs)) return (size_t)-1;
            if (dt == VP_BF16) {
                if (N * d_row_stride(Vs) >= MAX_ELEMS) return (size_t)-1;
                return align_up((size_t)(2 * fwd_tiles(Vs) + 1) * N * sizeof(float), 256) +
                       align_up((size_t)N * d_row_stride(Vs) * 2, 256);
            }
            return f32_matrix_bytes(N, Vs) + align_up(f32_bwd_scratch(N, h, Vs), 256);
        case VP_CALL_OUTPUT_DX_ALG2:
            return 0;
        case VP_CALL_OUTPUT_FWD:
            if (!sizes_ok(N, h, Vs) || !sizes_supported(N, h, Vs)) return (size_t)-1;
            if (dt == VP_BF16) return align_up((size_t)(2 * fwd_tiles(Vs) + 1) * N * sizeof(float), 256);
            // fp32: the logits live in the workspace unless the caller keeps them; then K-slice scratch
            return ((flags & VP_SAVE_LOGITS) ? 0 : f32_matrix_bytes(N, Vs)) + align_up(f32_fwd_scratch(N, h, Vs), 256);
        case VP_CALL_OUTPUT_BWD:
            if (!sizes_ok(N, h, Vs) || !sizes_supported(N, h, Vs)) return (size_t)-1;
            if (dt == VP_BF16) {
                if (N * d_row_stride(Vs) >= MAX_ELEMS) return (size_t)-1;
                return align_up((size_t)N * d_row_stride(Vs) * 2, 256);
            }
            return f32_matrix_bytes(N, Vs) + align_up(f32_bwd_scratch(N, h, Vs), 256);
        case VP_CALL_EMBED_BWD:
            if (N < 1 || N > ((int64_t)1 << 24)) return (size_t)-1;
            return align_up(embed_bwd_workspace(N), 256);
        case VP_CALL_COMBINE_STATS:
        case VP_CALL_EMBED_FWD:
            return 0;
    }
    return (size_t)-1;
}

vp_status vp_output_fwd(const void* H, const void* W_shard, const int64_t* labels, int64_t N, int64_t h, int64_t Vs,
                        int64_t shard_offset, vp_dtype dt, uint32_t flags, float* local_max, float* local_sumexp,
                        float* local_target, void* logits_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!H || !W_shard || !labels || !local_max || !local_sumexp || !local_target) return VP_ERR_INVALID_ARG;
    if (!sizes_ok(N, h, Vs) || !dtype_ok(dt) || shard_offset < 0) return VP_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)VP_SAVE_LOGITS) return VP_ERR_INVALID_ARG;
    if (((flags & VP_SAVE_LOGITS) != 0) != (logits_out != nullptr)) return VP_ERR_INVALID_ARG;
    if (!aligned16(H) || !aligned16(W_shard) || !aligned16(logits_out) || !aligned16(workspace))
        return VP_ERR_INVALID_ARG;
    if (!sizes_supported(N, h, Vs)) return VP_ERR_UNSUPPORTED;
    const size_t need = vp_workspace_bytes(VP_CALL_OUTPUT_FWD, N, h, Vs, dt, flags);
    if (need > 0 && (!workspace || workspace_bytes < need)) return VP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;

    if (dt == VP_BF16) {
        const int64_t tiles = fwd_tiles(Vs);
        float* pm = (float*)workspace;
        float* ps = pm + tiles * N;
        float* pt = ps + tiles * N;
        GemmBf16Params g{};
        g.A = (const u16*)H; g.B = (const u16*)W_shard;
        g.M = (int)N; g.N = (int)Vs; g.K = (int)h;
        g.lda = (int)h; g.ldb = (int)h;
        g.a_kcontig = 1; g.b_kcontig = 1;
        g.vec_ok = (h % 8 == 0) ? 1 : 0;
        g.epi = Epi::FwdStats;
        g.Y = (u16*)logits_out; g.ldy = (int)Vs;
        g.labels = labels; g.shard_offset = shard_offset;
        g.part_max = pm; g.part_sum = ps; g.part_tgt = pt;
        hipError_t e = launch_gemm_bf16(g, st);
        if (e != hipSuccess) return VP_ERR_DEVICE;
        return dev(launch_fold_partials(pm, ps, pt, (int)tiles, (int)N, labels, shard_offset, (int)Vs, local_max,
                                        local_sumexp, local_target, st));
    }
    float* Y = logits_out ? (float*)logits_out : (float*)workspace;
    float* scratch = f32_fwd_scratch(N, h, Vs) ? (float*)((char*)workspace + (logits_out ? 0 : f32_matrix_bytes(N, Vs)))
                                               : nullptr;
    hipError_t e = launch_gemm_f32((const float*)H, h, 1, (const float*)W_shard, h, 1, Y, Vs, (int)N, (int)Vs, (int)h,
                                   false, scratch, st);
    if (e != hipSuccess) return VP_ERR_DEVICE;
    return dev(launch_row_stats_f32(Y, Vs, labels, shard_offset, (int)N, (int)Vs, local_max, local_sumexp,
                                    local_target, st));
}

size_t vp_output_fwd_noalloc_max_scratch(void) { return NOALLOC_SCRATCH_BYTES; }

vp_status vp_output_fwd_noalloc(const void* H, const void* W_shard, const int64_t* labels, int64_t N, int64_t h,
                                int64_t Vs, int64_t shard_offset, vp_dtype dt, uint32_t flags, float* local_max,
                                float* local_sumexp, float* local_target, void* logits_out, void* stream) {
    // sizes first: a request whose scratch does not fit the static array is refused before anything else
    if (!sizes_ok(N, h, Vs) || !dtype_ok(dt)) return VP_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)VP_SAVE_LOGITS) return VP_ERR_INVALID_ARG;
    if (!sizes_supported(N, h, Vs)) return VP_ERR_UNSUPPORTED;
    const size_t need = vp_workspace_bytes(VP_CALL_OUTPUT_FWD, N, h, Vs, dt, flags);
    if (need == (size_t)-1 || need > NOALLOC_SCRATCH_BYTES) return VP_ERR_UNSUPPORTED;
    void* ws = scratch_of_current_device();
    if (!ws) return VP_ERR_DEVICE;
    // nothing in the scratch has to start at zero: every partial the fold reads is written by this call's
    // GEMM first (the target partial only for rows whose label the shard owns, and only those are read)
    return vp_output_fwd(H, W_shard, labels, N, h, Vs, shard_offset, dt, flags, local_max, local_sumexp, local_target,
                         logits_out, ws, NOALLOC_SCRATCH_BYTES, stream);
}

vp_status vp_combine_stats(const float* local_max, const float* local_sumexp, const float* local_target, int32_t p,
                           int64_t N, float* global_max, float* global_sumexp, float* loss_per_row, float* loss_mean,
                           void* stream) {
    if (!local_max || !local_sumexp || !local_target || !global_max || !global_sumexp || !loss_mean)
        return VP_ERR_INVALID_ARG;
    if (p < 1 || N < 1) return VP_ERR_INVALID_ARG;
    if (N >= MAX_ELEMS || (int64_t)p * N >= MAX_ELEMS) return VP_ERR_UNSUPPORTED;
    return dev(launch_combine(local_max, local_sumexp, local_target, p, (int)N, global_max, global_sumexp,
                              loss_per_row, loss_mean, (hipStream_t)stream));
}

int64_t vp_dlogits_row_stride(int64_t Vs, vp_dtype dt) {
    if (Vs < 1 || !dtype_ok(dt)) return -1;
    return dt == VP_BF16 ? d_row_stride(Vs) : Vs;
}

vp_status vp_output_bwd(const void* H, const void* W_shard, const int64_t* labels, int64_t N, int64_t h, int64_t Vs,
                        int64_t shard_offset, vp_dtype dt, uint32_t flags, const float* global_max,
                        const float* global_sumexp, const void* logits_saved, float grad_scale, float* dH_accum,
                        float* dW_shard, void* workspace, size_t workspace_bytes, void* stream) {
    if (!H || !W_shard || !labels || !global_max || !global_sumexp || !dW_shard) return VP_ERR_INVALID_ARG;
    if (!dH_accum && !(flags & VP_SKIP_DH)) return VP_ERR_INVALID_ARG;
    if (!sizes_ok(N, h, Vs) || !dtype_ok(dt) || shard_offset < 0) return VP_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)(VP_SAVE_LOGITS | VP_SKIP_DH | VP_DH_OVERWRITE)) return VP_ERR_INVALID_ARG;
    if ((flags & VP_SKIP_DH) && (flags & VP_DH_OVERWRITE)) return VP_ERR_INVALID_ARG;
    if (((flags & VP_SAVE_LOGITS) != 0) != (logits_saved != nullptr)) return VP_ERR_INVALID_ARG;
    if (!aligned16(H) || !aligned16(W_shard) || !aligned16(logits_saved) || !aligned16(workspace) ||
        !aligned16(dH_accum) || !aligned16(dW_shard))
        return VP_ERR_INVALID_ARG;
    const bool skip_dh = (flags & VP_SKIP_DH) != 0;
    const bool dh_overwrite = (flags & VP_DH_OVERWRITE) != 0;
    if (!sizes_supported(N, h, Vs)) return VP_ERR_UNSUPPORTED;
    const size_t need = vp_workspace_bytes(VP_CALL_OUTPUT_BWD, N, h, Vs, dt, flags);
    if (need == (size_t)-1) return VP_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < need) return VP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;

    if (dt == VP_BF16) {
        u16* D = (u16*)workspace;
        const int64_t ldd = d_row_stride(Vs);
        const int vec_ok = (h % 8 == 0) ? 1 : 0;
        if (logits_saved) {
            e = launch_dlogits(logits_saved, Vs, D, ldd, 1, labels, shard_offset, global_max, global_sumexp, grad_scale,
                               (int)N, (int)Vs, st);
        } else {
            GemmBf16Params g{};
            g.A = (const u16*)H; g.B = (const u16*)W_shard;
            g.M = (int)N; g.N = (int)Vs; g.K = (int)h;
            g.lda = (int)h; g.ldb = (int)h;
            g.a_kcontig = 1; g.b_kcontig = 1;
            g.vec_ok = (h % 8 == 0) ? 1 : 0;
            g.epi = Epi::DLogits;
            g.Y = D; g.ldy = (int)ldd;
            g.labels = labels; g.shard_offset = shard_offset;
            g.gmax = global_max; g.gsum = global_sumexp; g.scale = grad_scale;
            e = launch_gemm_bf16(g, st);
            if (e == hipSuccess) e = launch_zero_pad_columns(D, (int)N, (int)Vs, ldd, st);
        }
        if (e != hipSuccess) return VP_ERR_DEVICE;
        if (!skip_dh) {   // dH += D W_shard : M = N tokens, N = h, K = Vs; W_shard is stored [K][N]
            GemmBf16Params g{};
            g.A = D; g.B = (const u16*)W_shard;
            g.M = (int)N; g.N = (int)h; g.K = (int)Vs;
            g.lda = (int)ldd; g.ldb = (int)h;
            g.a_kcontig = 1; g.b_kcontig = 0;
            g.vec_ok = vec_ok;
            g.epi = dh_overwrite ? Epi::StoreF32 : Epi::AccumF32;
            g.kernel_id = K_GEMM_DH;
            g.C = dH_accum; g.ldc = (int)h;
            e = launch_gemm_bf16(g, st);
            if (e != hipSuccess) return VP_ERR_DEVICE;
        }
        {   // dW = D^T H : M = Vs, N = h, K = N tokens; D is stored [K][M], H is stored [K][N]
            GemmBf16Params g{};
            g.A = D; g.B = (const u16*)H;
            g.M = (int)Vs; g.N = (int)h; g.K = (int)N;
            g.lda = (int)ldd; g.ldb = (int)h;
            g.a_kcontig = 0; g.b_kcontig = 0;
            g.vec_ok = vec_ok;
            g.epi = Epi::StoreF32;
            g.C = dW_shard; g.ldc = (int)h;
            e = launch_gemm_bf16(g, st);
        }
        return dev(e);
    }

    // fp32: every step in fp32
    float* D = (float*)workspace;
    float* scratch = f32_bwd_scratch(N, h, Vs) ? (float*)((char*)workspace + f32_matrix_bytes(N, Vs)) : nullptr;
    const float* Y = (const float*)logits_saved;
    if (!Y) {
        e = launch_gemm_f32((const float*)H, h, 1, (const float*)W_shard, h, 1, D, Vs, (int)N, (int)Vs, (int)h, false,
                            scratch, st);
        if (e != hipSuccess) return VP_ERR_DEVICE;
        Y = D;   // D is formed in place
    }
    e = launch_dlogits(Y, Vs, D, Vs, 0, labels, shard_offset, global_max, global_sumexp, grad_scale, (int)N, (int)Vs, st);
    if (e != hipSuccess) return VP_ERR_DEVICE;
    if (!skip_dh) {
        e = launch_gemm_f32(D, Vs, 1, (const float*)W_shard, 1, h, dH_accum, h, (int)N, (int)h, (int)Vs, !dh_overwrite,
                            scratch, st);
        if (e != hipSuccess) return VP_ERR_DEVICE;
    }
    e = launch_gemm_f32(D, 1, Vs, (const float*)H, 1, h, dW_shard, h, (int)Vs, (int)h, (int)N, false, scratch, st);
    return dev(e);
}

vp_status vp_output_fwd_alg2(const void* H, const void* W_shard, const int64_t* labels, int64_t N, int64_t h,
                             int64_t Vs, int64_t shard_offset, vp_dtype dt, uint32_t flags, float* local_max,
                             float* local_sumexp, float* local_target, void* logits_out, float* A_out, void* B_out,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!H || !W_shard || !labels || !local_max || !local_sumexp || !local_target || !A_out || !B_out)
        return VP_ERR_INVALID_ARG;
    if (!sizes_ok(N, h, Vs) || !dtype_ok(dt) || shard_offset < 0) return VP_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)VP_SAVE_LOGITS) return VP_ERR_INVALID_ARG;
    if (((flags & VP_SAVE_LOGITS) != 0) != (logits_out != nullptr)) return VP_ERR_INVALID_ARG;
    if (!aligned16(H) || !aligned16(W_shard) || !aligned16(logits_out) || !aligned16(workspace) ||
        !aligned16(A_out) || !aligned16(B_out))
        return VP_ERR_INVALID_ARG;
    if (!sizes_supported(N, h, Vs)) return VP_ERR_UNSUPPORTED;
    const size_t need = vp_workspace_bytes(VP_CALL_OUTPUT_FWD_ALG2, N, h, Vs, dt, flags);
    if (need == (size_t)-1) return VP_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < need) return VP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;

    if (dt == VP_BF16) {
        const int64_t tiles = fwd_tiles(Vs);
        const int64_t ldd = d_row_stride(Vs);
        float* pm = (float*)workspace;
        float* ps = pm + tiles * N;
        float* pt = ps + tiles * N;
        u16* P = (u16*)((char*)workspace + align_up((size_t)(2 * tiles + 1) * N * sizeof(float), 256));
        // the logits go to the caller's buffer when it keeps them, else into the softmax' buffer (in place)
        u16* Y = logits_out ? (u16*)logits_out : P;
        const int64_t ldy = logits_out ? Vs : ldd;
        GemmBf16Params g{};
        g.A = (const u16*)H; g.B = (const u16*)W_shard;
        g.M = (int)N; g.N = (int)Vs; g.K = (int)h;
        g.lda = (int)h; g.ldb = (int)h;
        g.a_kcontig = 1; g.b_kcontig = 1;
        g.vec_ok = (h % 8 == 0) ? 1 : 0;
        g.epi = Epi::FwdStats;
        g.Y = Y; g.ldy = (int)ldy;
        g.labels = labels; g.shard_offset = shard_offset;
        g.part_max = pm; g.part_sum = ps; g.part_tgt = pt;
        if ((e = launch_gemm_bf16(g, st)) != hipSuccess) return VP_ERR_DEVICE;
        if ((e = launch_fold_partials(pm, ps, pt, (int)tiles, (int)N, labels, shard_offset, (int)Vs, local_max,
                                      local_sumexp, local_target, st)) != hipSuccess)
            return VP_ERR_DEVICE;
        // softmax' with the shard's own statistics (no one-hot term, scale 1), rows padded and zero-filled
        if ((e = launch_dlogits(Y, ldy, P, ldd, 1, nullptr, shard_offset, local_max, local_sumexp, 1.0f, (int)N,
                                (int)Vs, st)) != hipSuccess)
            return VP_ERR_DEVICE;
        GemmBf16Params a{};   // A = softmax' W_shard : M = N tokens, N = h, K = Vs; W_shard is stored [K][N]
        a.A = P; a.B = (const u16*)W_shard;
        a.M = (int)N; a.N = (int)h; a.K = (int)Vs;
        a.lda = (int)ldd; a.ldb = (int)h;
        a.a_kcontig = 1; a.b_kcontig = 0;
        a.vec_ok = (h % 8 == 0) ? 1 : 0;
        a.epi = Epi::StoreF32;
        a.C = A_out; a.ldc = (int)h;
        a.kernel_id = K_GEMM_A_ALG2;
        if ((e = launch_gemm_bf16(a, st)) != hipSuccess) return VP_ERR_DEVICE;
        return dev(launch_embed_fwd(W_shard, labels, (int)N, (int)h, (int)Vs, shard_offset, 2, B_out, st));
    }

    // fp32: logits in the caller's buffer or the workspace, softmax' in the workspace (in place when they coincide)
    float* P = (float*)workspace;
    float* Y = logits_out ? (float*)logits_out : P;
    float* scratch = f32_bwd_scratch(N, h, Vs) ? (float*)((char*)workspace + f32_matrix_bytes(N, Vs)) : nullptr;
    if ((e = launch_gemm_f32((const float*)H, h, 1, (const float*)W_shard, h, 1, Y, Vs, (int)N, (int)Vs, (int)h, false,
                             scratch, st)) != hipSuccess)
        return VP_ERR_DEVICE;
    if ((e = launch_row_stats_f32(Y, Vs, labels, shard_offset, (int)N, (int)Vs, local_max, local_sumexp, local_target,
                                  st)) != hipSuccess)
        return VP_ERR_DEVICE;
    if ((e = launch_dlogits(Y, Vs, P, Vs, 0, nullptr, shard_offset, local_max, local_sumexp, 1.0f, (int)N, (int)Vs,
                            st)) != hipSuccess)
        return VP_ERR_DEVICE;
    if ((e = launch_gemm_f32(P, Vs, 1, (const float*)W_shard, 1, h, A_out, h, (int)N, (int)h, (int)Vs, false, scratch,
                             st)) !=
        hipSuccess)
        return VP_ERR_DEVICE;
    return dev(launch_embed_fwd(W_shard, labels, (int)N, (int)h, (int)Vs, shard_offset, 4, B_out, st));
}

vp_status vp_output_dx_alg2(const float* A, const void* B, const float* local_max, const float* local_sumexp,
                            const float* global_max, const float* global_sumexp, int64_t N, int64_t h, vp_dtype dt,
                            uint32_t flags, float grad_scale, float* dH_accum, void* stream) {
    if (!A || !B || !local_max || !local_sumexp || !global_max || !global_sumexp || !dH_accum)
        return VP_ERR_INVALID_ARG;
    if (N < 1 || h < 1 || !dtype_ok(dt) || (flags & ~(uint32_t)VP_DH_OVERWRITE)) return VP_ERR_INVALID_ARG;
    if (!aligned16(A) || !aligned16(B) || !aligned16(dH_accum)) return VP_ERR_INVALID_ARG;
    if (N >= MAX_ELEMS || h >= MAX_ELEMS || N * h >= MAX_ELEMS) return VP_ERR_UNSUPPORTED;
    return dev(launch_dx_alg2(A, B, dt == VP_BF16 ? 1 : 0, local_max, local_sumexp, global_max, global_sumexp, (int)N,
                              (int)h, grad_scale, (flags & VP_DH_OVERWRITE) != 0, dH_accum, (hipStream_t)stream));
}

vp_status vp_embed_fwd(const void* table_shard, const int64_t* ids, int64_t N, int64_t h, int64_t Vs,
                       int64_t shard_offset, vp_dtype dt, void* out, void* stream) {
    if (!table_shard || !ids || !out) return VP_ERR_INVALID_ARG;
    if (!sizes_ok(N, h, Vs) || !dtype_ok(dt) || shard_offset < 0) return VP_ERR_INVALID_ARG;
    if (!aligned16(table_shard) || !aligned16(out)) return VP_ERR_INVALID_ARG;
    if (!sizes_supported(N, h, Vs)) return VP_ERR_UNSUPPORTED;
    return dev(launch_embed_fwd(table_shard, ids, (int)N, (int)h, (int)Vs, shard_offset, dt == VP_BF16 ? 2 : 4, out,
                                (hipStream_t)stream));
}

vp_status vp_embed_bwd(const void* grad_out, const int64_t* ids, int64_t N, int64_t h, int64_t Vs,
                       int64_t shard_offset, vp_dtype dt, float* dtable_shard, void* workspace, size_t workspace_bytes,
                       void* stream) {
    if (!grad_out || !ids || !dtable_shard) return VP_ERR_INVALID_ARG;
    if (!sizes_ok(N, h, Vs) || !dtype_ok(dt) || shard_offset < 0) return VP_ERR_INVALID_ARG;
    if (!aligned16(grad_out) || !aligned16(dtable_shard) || !aligned16(workspace)) return VP_ERR_INVALID_ARG;
    if (!sizes_supported(N, h, Vs) || N > ((int64_t)1 << 24)) return VP_ERR_UNSUPPORTED;
    const size_t need = vp_workspace_bytes(VP_CALL_EMBED_BWD, N, h, Vs, dt, 0);
    if (!workspace || workspace_bytes < need) return VP_ERR_WORKSPACE;
    return dev(launch_embed_bwd(grad_out, ids, (int)N, (int)h, (int)Vs, shard_offset, dt == VP_BF16 ? 1 : 0,
                                dtable_shard, workspace, (hipStream_t)stream));
}

}  // extern "C"
