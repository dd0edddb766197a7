/*
 * vp.h - C ABI of libvp: one device's shard of the vocabulary layers of Vocabulary
 * Parallelism (arXiv 2411.05288) on AMD MI355X (gfx950).
 *
 * Notation (paper, section 4): N = b*s token rows, h hidden size, V vocabulary size,
 * p shards, Vs rows of the vocabulary owned by this shard, shard_offset the global id of
 * the shard's first row.  X (here H) is [N, h]; the shard of the embedding weights W is
 * [Vs, h]; Y = X W^T are the logits; m_i and sum_i the row maximum and the row sum of
 * exponentials; g_i the label of token i.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, dense row-major,
 *     16-byte aligned.  The library allocates nothing, frees nothing and keeps no state
 *     between calls; scratch memory is the caller's `workspace`, at least
 *     vp_workspace_bytes(...) bytes, 256-byte aligned, contents undefined on entry/exit.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return; there is no host synchronisation inside.
 *   - Arguments are validated on the host before anything is launched.  An invalid
 *     argument returns an error code and launches nothing.  Nothing is thrown or aborted
 *     across this boundary.
 *   - `dt` is the storage type of H, W, the embedding table, the stored logits and the
 *     incoming embedding gradient.  Statistics, the loss and all gradients leaving the
 *     library are fp32.  With VP_BF16 the products are bf16 x bf16 MFMA with fp32
 *     accumulation; with VP_F32 everything is computed in fp32.
 *   - Labels / token ids are global vocabulary ids (int64).  An id outside the shard's
 *     range [shard_offset, shard_offset + Vs) - including ids outside [0, V) - is treated
 *     as "not owned": target logit 0, all-zero one-hot row, zero output row, no scatter.
 *   - Sizes: 1 <= N, h, Vs; h, Vs <= 2^20; and N*Vs, N*h, Vs*h < 2^31 elements each.
 */
#ifndef VP_H_
#define VP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VP_OK = 0,
    VP_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bad enum, misaligned pointer */
    VP_ERR_UNSUPPORTED = 2, /* valid request outside the implemented size limits */
    VP_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than vp_workspace_bytes() */
    VP_ERR_DEVICE = 4       /* the HIP runtime reported an error at launch */
} vp_status;

typedef enum { VP_F32 = 0, VP_BF16 = 1 } vp_dtype;

typedef enum {
    VP_CALL_OUTPUT_FWD = 0,
    VP_CALL_COMBINE_STATS = 1,
    VP_CALL_OUTPUT_BWD = 2,
    VP_CALL_EMBED_FWD = 3,
    VP_CALL_EMBED_BWD = 4,
    VP_CALL_OUTPUT_FWD_ALG2 = 5,
    VP_CALL_OUTPUT_DX_ALG2 = 6
} vp_call;

/* flags */
enum {
    VP_SAVE_LOGITS = 1u, /* fwd: store the logits; bwd: the stored logits are supplied */
    VP_SKIP_DH = 2u,     /* vp_output_bwd only: pass T of Algorithm 2, dW_shard alone (dH_accum may be NULL) */
    VP_DH_OVERWRITE = 4u /* vp_output_bwd, vp_output_dx_alg2: dH_accum = (this shard's term) instead of +=: the first
                            term of the reduce C2, which saves zero-filling dH_accum and reading the zeros back */
};

/* Library version (major*10000 + minor*100 + patch). Host-only, no device work. */
int vp_version(void);

/* Static, human-readable name of a status code. */
const char* vp_status_string(vp_status s);

/*
 * Bytes of scratch the given call needs for these sizes (0 if none).  Host-only.
 * Returns (size_t)-1 for invalid arguments.
 */
size_t vp_workspace_bytes(vp_call which, int64_t N, int64_t h, int64_t Vs, vp_dtype dt, uint32_t flags);

/*
 * Pass S of Algorithm 1 (section 4.3) for one shard: Y = H W_shard^T over the shard's Vs
 * vocabulary rows, fused with the shard-local softmax statistics, so the logits are never
 * re-read:
 *     local_max[i]    = m'_i   = max_k Y_ik
 *     local_sumexp[i] = sum'_i = sum_k exp(Y_ik - m'_i)
 *     local_target[i] = Y[i, labels[i] - shard_offset] if the shard owns labels[i], else 0
 * The paper's softmax' matrix is not materialised.  If logits_out != NULL (flag
 * VP_SAVE_LOGITS must then be set) Y is also stored there as [N, Vs] in type `dt`.
 *   H [N,h], W_shard [Vs,h] : in, type dt.     labels [N] : in, int64.
 *   local_* [N] : out, fp32.                   logits_out : out or NULL.
 */
vp_status vp_output_fwd(const void* H, const void* W_shard, const int64_t* labels,
                        int64_t N, int64_t h, int64_t Vs, int64_t shard_offset,
                        vp_dtype dt, uint32_t flags,
                        float* local_max, float* local_sumexp, float* local_target,
                        void* logits_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * vp_output_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops that evaluate a loss, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as vp_output_fwd, except that the scratch (the per-column-tile partial
 * statistics; with VP_F32 the logits when they are not kept, and K-slice partials) lives in a static device
 * array inside the library, vp_output_fwd_noalloc_max_scratch() bytes (4 MiB) on every GPU the library
 * runs on, held until the process ends.  The call allocates and frees nothing.
 *   - A request whose vp_workspace_bytes(VP_CALL_OUTPUT_FWD, ...) exceeds that size returns
 *     VP_ERR_UNSUPPORTED and launches nothing (bf16: (2 ceil(Vs/256) + 1) * N * 4 bytes, so all five
 *     benchmark configurations fit).
 *   - All calls on one GPU share the one array: calls that overlap on a GPU (two streams, two threads)
 *     race on it.  Calls on one stream are ordered and safe.  The array keeps the last call's contents;
 *     nothing in it needs to start at zero.
 *   - The array's device address is looked up on the first call on each device (with that device current).
 */
vp_status vp_output_fwd_noalloc(const void* H, const void* W_shard, const int64_t* labels,
                                int64_t N, int64_t h, int64_t Vs, int64_t shard_offset,
                                vp_dtype dt, uint32_t flags,
                                float* local_max, float* local_sumexp, float* local_target,
                                void* logits_out, void* stream);
size_t vp_output_fwd_noalloc_max_scratch(void);

/*
 * Barrier C1 of Algorithm 1 (section 4.3) as an on-device fold over the p shards' rows
 * (it stands in for the two all-reduces):
 *     m_i   = max_r m'_{r,i}
 *     sum_i = sum_r sum'_{r,i} * exp(m'_{r,i} - m_i)      (ascending r)
 *     loss_i = m_i + ln(sum_i) - sum_r t'_{r,i};   loss_mean = (1/N) sum_i loss_i
 * The mean is taken with one fixed reduction tree, so results repeat bit for bit.
 *   local_* [p,N] : in, fp32 (row r = shard r's vp_output_fwd outputs).
 *   global_max, global_sumexp [N] : out.  loss_per_row [N] : out or NULL.  loss_mean [1] : out.
 */
vp_status vp_combine_stats(const float* local_max, const float* local_sumexp, const float* local_target,
                           int32_t p, int64_t N,
                           float* global_max, float* global_sumexp,
                           float* loss_per_row, float* loss_mean, void* stream);

/*
 * Pass T of Algorithm 1 plus this shard's term of the reduce C2 (section 4.3; gradients
 * of section 4.2):
 *     D_ij      = ( exp(Y_ij - m_i) / sum_i  -  [labels[i] == shard_offset + j] ) * grad_scale
 *                 (equal to softmax' * sum' e^{m'-m} / sum - G, the rescale identity)
 *     dH_accum += D W_shard          (fp32, accumulate: the caller zeroes it once per
 *                                     microbatch; calling the p shards in ascending order
 *                                     is the deterministic reduce)
 *     dW_shard  = D^T H              (fp32, overwritten)
 * grad_scale = 1/N gives the gradients of the mean loss, 1 the paper's unscaled form.
 * logits_saved != NULL (with VP_SAVE_LOGITS): Y is read from there ([N,Vs], type dt);
 * NULL: Y is recomputed from H and W_shard.
 * With VP_SKIP_DH only dW_shard is formed (pass T of Algorithm 2, section 4.4, where the input
 * gradient has already left through vp_output_dx_alg2); dH_accum is then ignored and may be NULL.
 */
/*
 * Row stride (elements) of the D matrix that vp_output_bwd leaves at the start of its workspace:
 * on return (once the stream has run the call) the workspace begins with D as [N, stride] in type
 * dt, columns Vs .. stride-1 zero.  With VP_BF16 rows are padded to 128 bytes, with VP_F32 the
 * matrix is dense.  This is how tests compare D itself with the definition; the rest of the
 * workspace stays undefined.  Host-only; returns -1 for invalid arguments.
 */
int64_t vp_dlogits_row_stride(int64_t Vs, vp_dtype dt);

vp_status vp_output_bwd(const void* H, const void* W_shard, const int64_t* labels,
                        int64_t N, int64_t h, int64_t Vs, int64_t shard_offset,
                        vp_dtype dt, uint32_t flags,
                        const float* global_max, const float* global_sumexp,
                        const void* logits_saved, float grad_scale,
                        float* dH_accum, float* dW_shard,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Pass S of Algorithm 2 (section 4.4, one barrier instead of two) for one shard: everything
 * vp_output_fwd produces, plus the two [N,h] matrices from which the input gradient is formed
 * inside the barrier, before the global statistics are known:
 *     A = softmax'(Y) W_shard,   softmax'_ij = exp(Y_ij - m'_i) / sum'_i      (fp32)
 *     B = G W_shard              (row i = W_shard[labels[i] - shard_offset] when the shard owns
 *                                 labels[i], else zero; type dt, an exact copy of rows of W)
 *   A_out [N,h] : out, fp32.   B_out [N,h] : out, type dt.   Everything else as vp_output_fwd.
 */
vp_status vp_output_fwd_alg2(const void* H, const void* W_shard, const int64_t* labels,
                             int64_t N, int64_t h, int64_t Vs, int64_t shard_offset,
                             vp_dtype dt, uint32_t flags,
                             float* local_max, float* local_sumexp, float* local_target,
                             void* logits_out, float* A_out, void* B_out,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * This shard's term of the input gradient of Algorithm 2 (section 4.4, the identity
 * dX = sum_r ( A_r * sum'_r e^{m'_r - m} / sum  -  B_r )), evaluated once the barrier has
 * produced the global statistics:
 *     dH_accum[i,:] += ( A[i,:] * c_i - B[i,:] ) * grad_scale,
 *     c_i = local_sumexp[i] * exp(local_max[i] - global_max[i]) / global_sumexp[i]
 * (c_i = 0 for a shard whose local_max is -inf).  Calling the p shards in ascending order is
 * the deterministic reduce.  Pass T of Algorithm 2 is vp_output_bwd with VP_SKIP_DH.
 * flags: 0, or VP_DH_OVERWRITE for the first term of the reduce (dH_accum = ... instead of +=, so the
 * caller need not zero-fill it).
 *   A [N,h] : in, fp32.  B [N,h] : in, type dt.  local_* / global_* [N] : in, fp32.
 *   dH_accum [N,h] : in/out (out only with VP_DH_OVERWRITE), fp32.
 */
vp_status vp_output_dx_alg2(const float* A, const void* B,
                            const float* local_max, const float* local_sumexp,
                            const float* global_max, const float* global_sumexp,
                            int64_t N, int64_t h, vp_dtype dt, uint32_t flags, float grad_scale,
                            float* dH_accum, void* stream);

/*
 * Input layer forward on one shard (appendix C): the full-size [N,h] output, row i being
 * table_shard[ids[i] - shard_offset] when the shard owns ids[i] and all +0 otherwise, so
 * that the sum over shards is the embedding lookup.  Pure data movement, bit exact.
 *   table_shard [Vs,h] : in, type dt.  ids [N] : in.  out [N,h] : out, type dt.
 */
vp_status vp_embed_fwd(const void* table_shard, const int64_t* ids,
                       int64_t N, int64_t h, int64_t Vs, int64_t shard_offset, vp_dtype dt,
                       void* out, void* stream);

/*
 * Input layer backward on one shard (appendix C): scatter-add of the output gradient,
 *     dtable_shard[ids[i] - shard_offset, :] += (float) grad_out[i, :]   for owned ids,
 * with repeated ids accumulated in increasing token position i.  No atomics: tokens are
 * grouped by row with a sort and every row is summed, per slab of columns, by one workgroup, so the result is
 * bit-identical from run to run.
 *   grad_out [N,h] : in, type dt.  dtable_shard [Vs,h] : in/out, fp32, accumulate.
 * Limit: N <= 2^24.
 */
vp_status vp_embed_bwd(const void* grad_out, const int64_t* ids,
                       int64_t N, int64_t h, int64_t Vs, int64_t shard_offset, vp_dtype dt,
                       float* dtable_shard, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aid, not part of the method.  While enabled, every kernel launch made by the
 * entry points above is bracketed by two HIP events on the launch stream (events are created
 * on demand and pooled; this is the only state the library ever holds, and none exists while
 * timing is off, the default).  vp_profile_read waits for the recorded events, writes the
 * summed elapsed milliseconds and the launch count per kernel id into the two host arrays
 * (length n >= vp_profile_kernel_count()), and clears the records.
 */
int vp_profile_kernel_count(void);
const char* vp_profile_kernel_name(int id);
vp_status vp_profile_enable(int on);
vp_status vp_profile_read(double* ms_total, int64_t* launches, int n);

/*
 * Test switch, not part of the method: while on, every bf16 product goes through the generic GEMM
 * kernel (element-wise predicated loads) instead of the fast one, so that tests can compare the two on
 * shapes the fast kernel would normally take.  Process-wide; off by default.
 */
vp_status vp_profile_force_generic_gemm(int on);

/*
 * Measurement aid, not part of the method: a timeline of the fast bf16 GEMM kernel.  While `buffer`
 * (device memory, 8-byte aligned, owned by the caller) is set, every launch of that kernel whose records
 * fit writes, per workgroup and output tile, four phase stamps - tile start, operands of the first k
 * tile landed, main loop done, epilogue done (stores issued) - each as {100 MHz counter, shader clock}:
 *     word 0: workgroups; word 1: output tiles; word 2: tiles per workgroup T;
 *     words 8 + ((w * T + t) * 8) .. +7 : stamps of tile t of workgroup w.
 * A launch overwrites the previous one's records.  kernel_id >= 0 (an index of vp_profile_kernel_name)
 * restricts the trace to the launches timed under that name, < 0 takes every fast GEMM launch.
 * buffer = NULL switches it off (the default).  Process-wide; launches that race with a change of the
 * buffer see either setting.
 */
vp_status vp_profile_gemm_trace(void* buffer, size_t bytes, int kernel_id);

/*
 * Measurement aid, not part of the method: `blocks` workgroups of 4 wavefronts each run `iters` x 16
 * back-to-back v_mfma_f32_32x32x16_bf16 on register operands, with no memory traffic inside the loop
 * (blocks * 4 * iters * 16 * 32768 flops in total).  The matrix cores are power limited and the rate they
 * sustain depends on the operand VALUES; this gives the ceiling for a given value distribution.
 *   operands : in, device, 8 * 256 * 16 bytes of bf16 (the 8 operand fragments of every lane).
 *   out      : out, device, blocks * 256 floats (keeps the work observable; contents are meaningless).
 */
vp_status vp_profile_mfma_loop(const void* operands, float* out, int32_t iters, int32_t blocks, void* stream);

/*
 * The same measurement for other instruction shapes and issue orders, so that the ceiling is an
 * envelope and not one point.  Every wavefront owns a 128 x 128 block of accumulators:
 *   variant 0  v_mfma_f32_32x32x16_bf16, 4 x 4 tiles column by column (= vp_profile_mfma_loop)
 *           1  the same in a snake (one operand changes between consecutive instructions)
 *           2  two k sub-steps chained back to back on each accumulator
 *           3  four k sub-steps chained back to back on each accumulator
 *           4  v_mfma_f32_16x16x32_bf16, 8 x 8 tiles column by column
 *           5  the same in a snake
 * vp_profile_mfma_variant_flops(variant) is the flop count of one wavefront in one iteration
 * (total = blocks * 4 * iters * that); vp_profile_mfma_variant_count() the number of variants.
 *   operands : in, device, 32 * 256 * 16 bytes of bf16.   out : out, device, blocks * 256 floats.
 */
vp_status vp_profile_mfma_variant(const void* operands, float* out, int32_t iters, int32_t blocks, int32_t variant,
                                  void* stream);
int vp_profile_mfma_variant_count(void);
double vp_profile_mfma_variant_flops(int32_t variant);

#ifdef __cplusplus
}
#endif
#endif /* VP_H_ */
