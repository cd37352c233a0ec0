/*
 * moe_hip.h - C ABI of the MI355X (gfx950) MoE expert-layer library.
 *
 * The calls follow the paper's statement of the layer: Route -> Dispatch
 * (permute) -> Expert computation (Grouped GEMM) -> Combine (Sec. 2.1.1), with
 * the backward MLP split into a data-gradient and a weight-gradient call
 * (Sec. 4.2.3, "W/D split") and every dynamic shape left on the device
 * (Sec. 4.3.7, "device-initiated kernels").
 *
 * Conventions that hold for every call unless the call says otherwise
 *   - Pointers are DEVICE pointers owned by the caller, except the ones marked
 *     "host".  The library allocates nothing in these calls; its only memory is
 *     the context workspace (moe_ctx_create).
 *   - Tensors are row-major with the innermost dimension contiguous and the
 *     base address 16-byte aligned.  bf16 = 16-bit brain float, fp8 = OCP E4M3
 *     (bias 7, no infinities, max 448) stored one code per byte.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work: no host synchronisation, no device-to-host copy
 *     of the per-expert counts (Sec. 4.3.7, challenge 1).  Launch sizes come from
 *     the static arguments (T, k, E, Rcap ...); the kernels read the actual
 *     extents from `offsets` on the device and skip what lies beyond them.
 *   - Return value: MOE_OK or a negative moe_status.  Argument errors are found
 *     on the host before anything is launched; nothing is written then.
 *     moe_last_error gives a host string describing the last failure on a context.
 *   - Calls on one context from several host threads at once are not supported, and all calls on one
 *     context must be stream-ordered with respect to each other (use one context per stream): several calls
 *     keep device-side state in the context workspace (the row-ID map's histograms, the auxiliary loss's
 *     partial sums, the gate GEMM's offsets, the weight gradient's tile counter and partial tiles), and two such
 *     calls running at the same time on different streams would race silently.
 *   - Same inputs give bit-identical outputs from run to run (no floating-point
 *     atomics anywhere; integer atomics only where the result is order-free).
 */
#ifndef MOE_HIP_H
#define MOE_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx; /* opaque: device id, workspace, last error */

typedef enum {
    MOE_OK = 0,
    MOE_ERR_ARG = -1,         /* NULL pointer, size out of range, misaligned size */
    MOE_ERR_UNSUPPORTED = -2, /* valid request the library has no kernel for */
    MOE_ERR_WORKSPACE = -3,   /* context workspace too small for this call */
    MOE_ERR_HIP = -4          /* a HIP runtime call or kernel launch failed */
} moe_status;

typedef enum { MOE_BF16 = 0, MOE_FP8_E4M3 = 1, MOE_F32 = 2, MOE_MXFP8_E4M3 = 3 } moe_dtype;
typedef enum { MOE_SCORE_SOFTMAX = 0, MOE_SCORE_SIGMOID = 1 } moe_score;
typedef enum { MOE_EPI_NONE = 0, MOE_EPI_SWIGLU = 1 } moe_epilogue;

/* ------------------------------------------------------------------------- */
/* Context                                                                   */
/* ------------------------------------------------------------------------- */

/* Bytes of workspace the calls below need for problems up to the given sizes
 * (host, pure function).  T tokens, k slots per token, E experts, h hidden,
 * f_max the largest expert width used with this context.  The largest part is
 * the room for the weight gradient's split contraction (see
 * moe_grouped_gemm_wgrad): 8 fp32 copies of one expert's largest weight gradient,
 * 8 * 2 f_max * h * 4 bytes rounded up to whole 256 x 256 tiles. */
size_t moe_workspace_bytes(int T, int k, int E, int h, int f_max);

/* Create a context on `device` and allocate `workspace_bytes` of device memory
 * for it (hipMalloc; the only allocation the library ever makes).  *out is
 * written only on success.  Host call; synchronises the device. */
moe_status moe_ctx_create(moe_ctx** out, int device, size_t workspace_bytes);

/* Free the workspace and the context.  Pending work that uses the context
 * must have finished.  NULL is accepted. */
moe_status moe_ctx_destroy(moe_ctx* ctx);

/* Host string for the last error recorded on ctx ("" if none); owned by ctx.  ctx = NULL: the message of the
 * calling host thread's last failed call that takes no context (moe_permute_static). */
const char* moe_last_error(const moe_ctx* ctx);

/* Kernels that find a device-side inconsistency (offsets[E] > Rcap) skip the
 * work and set a device error word instead of writing out of bounds.  This
 * call waits for `stream`, copies the word to *device_error (host; 0 = none)
 * and clears it.  It is the only call that synchronises. */
moe_status moe_ctx_poll_error(moe_ctx* ctx, void* stream, int* device_error);

/* ------------------------------------------------------------------------- */
/* Stage 1: Route (Sec. 2.1.1 stage 1; Sec. 2.1.2 item 2; fused as in Sec. 4.3.4)*/
/* ------------------------------------------------------------------------- */
/*
 * Per token: score function over the E logits, the k highest experts, their
 * combine weights, and the per-expert histogram, in one fused kernel.  The gate
 * projection x*W_r is not part of this call (Sec. 4.3.4 leaves the GEMM outside
 * the fused router): `logits` [T,E] fp32 is the input.
 *
 *   fn = SOFTMAX : p_i = exp(l_i) / sum over all E;   fn = SIGMOID : p_i = 1/(1+exp(-l_i)).
 *   Selection: the k largest logits (both score functions are strictly
 *   increasing, so this is the set with the k highest scores); equal logits go
 *   to the lower expert index; slot 0 holds the largest.
 *   Weights: w = p_i, divided by the sum of the k selected p when norm_topk != 0,
 *   then multiplied by `scale`.
 * Outputs: topk_idx [T,k] int32, topk_prob [T,k] fp32, counts [E] int32
 * (counts may be NULL).  Limits: 1 <= k <= 32, k <= E <= 1024.  NaN logits are
 * not supported (selection is then unspecified, nothing faults).
 */
moe_status moe_route_topk(moe_ctx* ctx, void* stream, const float* logits, int T, int E, int k,
                          moe_score fn, int norm_topk, float scale,
                          int32_t* topk_idx, float* topk_prob, int32_t* counts);

/*
 * Gate GEMM in front of the router (Sec. 2.1.2 item 1): logits[t,e] = sum_i X[t,i] * Wr[e,i].
 * X [T,h] and Wr [E,h] bf16 (Wr is W_r of the paper stored expert-major, like an expert's Linear
 * weight), fp32 accumulation, logits [T,E] fp32 (Sec. 5.1 keeps the router in FP32).  E must be a
 * multiple of 8, h of 64.  Stream-ordered, no allocation or copy; uses 8 bytes of the context's
 * reserved workspace (calls on one context must not overlap).
 */
moe_status moe_gate_gemm(moe_ctx* ctx, void* stream, const void* X, const void* Wr, int T, int E, int h,
                         float* logits);

/*
 * Router with the branches Sec. 4.3.4 item 1 lists for the fused score kernel: group-limited
 * top-k, the load-balancing expert bias of the auxiliary-loss-free strategy (Sec. 7) and score
 * scaling.  The paper names them and cites their source; the published DeepSeek-V3 router is taken
 * as their definition:
 *   s = score function of the logits over all E experts; c = s + expert_bias (expert_bias [E] fp32
 *   or NULL) decides the routing, the weights use s; the experts form n_group contiguous groups of
 *   E / n_group; a group scores the sum of its k / topk_group largest c; only experts of the
 *   topk_group best groups can be selected; the k largest c among them are selected, slots in
 *   selection order; topk_prob = s of the selected (/ their sum when norm_topk) * scale.
 *   Ties go to the lower index (experts and groups).  n_group = topk_group = 1 with no bias selects
 *   what moe_route_topk selects.
 * The decisions are taken on fp32 values: s is evaluated in double and rounded to fp32 once, the
 * bias add and the group sums (largest first) are fp32 additions.
 * Limits: as moe_route_topk, and n_group <= 64, E % n_group == 0, topk_group <= n_group,
 * k % topk_group == 0, k / topk_group <= E / n_group.  moe_route_topk_bwd is its backward too (the
 * bias does not enter the weights).
 */
moe_status moe_route_topk_grouped(moe_ctx* ctx, void* stream, const float* logits, const float* expert_bias,
                                  int T, int E, int k, int n_group, int topk_group,
                                  moe_score fn, int norm_topk, float scale,
                                  int32_t* topk_idx, float* topk_prob, int32_t* counts);

/*
 * Load-balancing auxiliary loss and its gradient (Sec. 4.3.4 items 2 and 3: the score computation for the
 * loss and the loss itself, here one pass over the logits).  The paper cites the loss without restating it;
 * the Switch-Transformer form is taken:
 *   p[t,:] = softmax(logits[t,:]), or sigmoid(logits[t,:]) divided by its sum over the E experts
 *            (the probabilities of Sec. 2.1.2 item 2);
 *   loss   = coeff * E * sum_e f_e * P_e,  f_e = counts[e] / (T k),  P_e = (1/T) sum_t p[t,e];
 *   dlogits[t,:] = dloss * d loss / d logits[t,:] with the counts held constant (written, or added to
 *            what dlogits holds when accumulate != 0, e.g. the result of moe_route_topk_bwd);
 *            dlogits may be NULL to get the loss only.
 * counts [E] int32 is the routing histogram the loss balances (the router's counts output), loss one
 * fp32 on the device.  fp32 arithmetic per token, per-token terms summed in double in a fixed order
 * (run-to-run identical).  Uses the context's workspace (8 bytes per 32 tokens); calls on one context
 * must not overlap with each other or with moe_permute.  Limits: T >= 1, E <= 1024.
 */
moe_status moe_aux_loss(moe_ctx* ctx, void* stream, const float* logits, const int32_t* counts,
                        int T, int E, int k, moe_score fn, float coeff, float dloss, int accumulate,
                        float* loss, float* dlogits);

/*
 * Backward of the routing weights (Sec. 2.1.2 item 2) with the selection frozen:
 * dlogits[t,:] = sum_s dprob[t,s] * d topk_prob[t,s] / d logits[t,:], for the same score function,
 * normalisation and scale as the forward call.  logits [T,E] fp32, topk_idx [T,k] as returned by
 * moe_route_topk, dprob [T,k] fp32, dlogits [T,E] fp32 (every element is written; experts that
 * were not selected get a non-zero gradient only through the softmax denominator).
 */
moe_status moe_route_topk_bwd(moe_ctx* ctx, void* stream, const float* logits, const int32_t* topk_idx,
                              const float* dprob, int T, int E, int k, moe_score fn, int norm_topk,
                              float scale, float* dlogits);

/* ------------------------------------------------------------------------- */
/* Stage 2: Dispatch = permute (Sec. 4.3.3 "Preprocessing" + "Permute")      */
/* ------------------------------------------------------------------------- */
/*
 * Builds the row-ID map once (a stable counting sort of the T*k (token, slot)
 * pairs by expert) and moves the token rows into expert-contiguous order, each
 * token copied once per slot.  Per-expert zero padding to a multiple of `align`
 * rows is fused into the move (Sec. 5.4.1).
 *
 *   idx [T,k] int32: expert of each slot; values < 0 or >= E mean "not on this
 *       GPU" and produce no row.
 *   X [T,h] of dtype dt (MOE_BF16 or MOE_F32), or NULL to build the maps only.
 *   Xp [Rcap,h]: rows [offsets[e], offsets[e]+counts[e]) hold expert e's tokens in
 *       increasing flattened index t*k+s; rows up to offsets[e+1] are zero;
 *       rows >= offsets[E] are left untouched.
 *   row_of [T,k]: row of each slot, -1 if skipped.  src_of [Rcap]: t*k+s of each
 *       row, -1 for padding and for rows >= offsets[E].
 *   offsets [E+1]: padded group starts (offsets[0] = 0).  counts [E]: unpadded.
 *   Rcap must be >= T*k + E*(align-1) (checked on the host, so the device can
 *   never overflow it); align >= 1; h*sizeof(dt) must be a multiple of 16.
 * Uses the context workspace (moe_workspace_bytes).
 */
moe_status moe_permute(moe_ctx* ctx, void* stream, const void* X, moe_dtype dt,
                       const int32_t* idx, int T, int k, int h, int E, int align,
                       void* Xp, int64_t Rcap,
                       int32_t* row_of, int32_t* src_of, int32_t* offsets, int32_t* counts);

/*
 * moe_permute for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It takes no context (moe_ctx_create allocates) and calls no
 * hipMalloc / hipFree or allocating library routine: the per-chunk histograms that moe_permute keeps in the
 * context workspace live in a file-scope device array of 1 MiB inside the library (each GPU the library runs on
 * holds it until the process ends; its address is looked up once per device, on the first call made with that
 * device current).  Arguments, results and limits are those of moe_permute, bit for bit, and in addition
 *   ceil(T*k / 1024) * E * 4 bytes <= 1 MiB   (e.g. T*k <= 262144 pairs at E = 1024, 8.4 M pairs at E = 32);
 * larger problems return MOE_ERR_WORKSPACE and launch nothing.  The device current on the calling thread must be
 * the one that owns the buffers and `stream`.  The array needs no clearing between calls (every entry is written
 * before it is read), but every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU
 * (two streams, two host threads) race.  Failures: status as above, message through moe_last_error(NULL).
 */
moe_status moe_permute_static(void* stream, const void* X, moe_dtype dt,
                              const int32_t* idx, int T, int k, int h, int E, int align,
                              void* Xp, int64_t Rcap,
                              int32_t* row_of, int32_t* src_of, int32_t* offsets, int32_t* counts);

/* ------------------------------------------------------------------------- */
/* Stage 3: Expert computation = Grouped GEMM (Sec. 2.1.4, 4.3.2, 4.3.7)      */
/* ------------------------------------------------------------------------- */
/*
 * All three calls run every expert's GEMM in one persistent launch.  Rows
 * [offsets[e], offsets[e+1]) of the row-indexed operands belong to expert e;
 * `offsets` [E+1] int32 stays on the device.  Rows >= offsets[E] are neither
 * read nor written.  Weights are B [E,N,K] ("out, in" per expert: the layout of
 * an expert's Linear weight), no bias (Sec. 4.1.2 needs bias-free experts).
 * dt is the operand type: MOE_BF16 (fp32 accumulation, bf16 result) or
 * MOE_FP8_E4M3 (blockwise recipe of Sec. 5.3.2: operands are E4M3 codes with
 * fp32 scales, fp32 accumulation, bf16 result; the accumulators are carried in units of
 * the current 128-wide block's scales, so every scale must be a normal number and the product
 * of the two operands' scales may change from one block of a contraction to the next by a
 * factor of at most 2^100 either way; amax / 448 of bf16 data meets that unless blocks with
 * amax below 2^-60 alternate with blocks near the top of the bf16 range).  N and K must be multiples of
 * 128 (fp8) / 16 (bf16); in bf16 the contraction dimension of fwd (K) and of
 * dgrad (N) must also be a multiple of 64 (one 128-byte operand row per stage);
 * wgrad contracts over the expert's rows, any count.  N, K <= 2^24 and N*K <= 2^31 elements per
 * expert (32-bit offsets inside one expert's weights).  Sizes outside these limits
 * return MOE_ERR_UNSUPPORTED and touch nothing.  dt = MOE_F32: every operand and result is fp32
 * (fp32 accumulation in increasing contraction index; wgrad needs out_dt = MOE_F32; any N, K >= 1);
 * a plain one-thread-per-output path for parity runs at the 1e-5 level on small layers, not tuned.
 * dt = MOE_MXFP8_E4M3 (Sec. 5.3.3) is described with moe_mx_quantize below; all three calls take
 * both one-byte types.
 *
 * fwd:   C[r,n] = sum_k A[r,k] * B[e(r),n,k]                    A [Rcap,K], C [Rcap,N]
 *        epi = MOE_EPI_SWIGLU (N = 2f): C holds the pre-activation Z = [gate | up]
 *        (kept for backward) and C_act [Rcap,f] = silu(gate) * up, computed from
 *        the fp32 accumulators.  C may be NULL with SWIGLU to skip storing Z.
 *        fp8: a_scale [Rcap,K/128] (1x128 tiles along K), b_scale [E,N/128,K/128].
 */
moe_status moe_grouped_gemm_fwd(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                moe_dtype dt, moe_epilogue epi,
                                const float* a_scale, const float* b_scale,
                                void* C, void* C_act);

/*
 * dgrad: dA[r,k] = sum_n dC[r,n] * B[e(r),n,k]                  dC [Rcap,N], dA [Rcap,K]
 *        Z_saved != NULL (the fc2 data gradient, K = f): Z_saved [Rcap,2K] is the
 *        pre-activation fc1 stored; the SwiGLU backward is fused into the epilogue
 *        and the output is dZ [Rcap,2K] = [dA*up*silu'(gate) | dA*silu(gate)].
 *        fp8: dc_scale [Rcap,N/128] (1x128 tiles along N), b_scale as in fwd.
 */
moe_status moe_grouped_gemm_dgrad(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                  const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                  moe_dtype dt, const void* Z_saved,
                                  const float* dc_scale, const float* b_scale, void* dA);

/*
 * wgrad: dB[e,n,k] = sum over rows r of expert e of dC[r,n] * A[r,k]
 *        The contraction length is the expert's (padded) row count, read from
 *        `offsets`; an expert with no rows gets dB_e = 0 (accumulate = 0) or is
 *        left as it is (accumulate != 0: dB += ...).  out_dt: MOE_BF16 or MOE_F32.
 *        Under a skewed load (largest expert above twice the mean; decided on the device from
 *        `offsets`) the tiles are handed out through a counter in the context's reserved workspace
 *        and, for bf16 operands, the contraction of every expert above twice the mean is split into
 *        up to 8 pieces whose fp32 partial tiles go to the workspace and are added in piece order by
 *        a second kernel of the same call.  Which workgroup computes what varies from run to run,
 *        what is added to what, and in which order, does not: results are bit-identical run to
 *        run.  wgrad calls on one context must not overlap in time.
 *        One-byte operands are quantised down the token dimension, the contraction of this call
 *        (Sec. 5.4.1): blockwise fp8 in 128x1 tiles (moe_fp8_quantize, MOE_Q_128x1),
 *        a_scale [Rcap/128, K], dc_scale [Rcap/128, N] fp32; MXFP8 in 32x1 blocks (see
 *        moe_mx_quantize).  A scale block must not straddle two experts: every offsets[e] must be a
 *        multiple of 128 (moe_permute with align = 128), otherwise the error word is raised and dB is
 *        left untouched.  Blockwise: the product of a row's and a column's block scales may change from
 *        one 128-row block to the next by a factor of at most 2^100 either way (the accumulators are
 *        carried in units of the current block's scales).
 */
moe_status moe_grouped_gemm_wgrad(moe_ctx* ctx, void* stream, const void* A, const void* dC,
                                  const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                  moe_dtype dt, const float* a_scale, const float* dc_scale,
                                  int accumulate, moe_dtype out_dt, void* dB);

/*
 * Memory-efficient permutation (Sec. 4.1.2, eq. (2)): the routing weight multiplies the
 * activation before fc2, the combine is then a plain sum (moe_unpermute_combine with
 * prob = NULL), and dL/dp needs only the saved pre-activations, not the expert outputs.
 *
 * fwd_weighted:   as moe_grouped_gemm_fwd; with epi = MOE_EPI_SWIGLU and row_prob != NULL
 *                 (fp32 [Rcap], one weight per permuted row, see moe_gather_row_prob)
 *                 C_act[r,:] = row_prob[r] * silu(gate) * up.  C (the pre-activation) is
 *                 not weighted.  row_prob = NULL is exactly moe_grouped_gemm_fwd.
 * dgrad_weighted: as moe_grouped_gemm_dgrad with Z_saved; the output is
 *                 dZ[r,:] = row_prob[r] * SwiGLU-backward(dA[r,:], Z_saved[r,:]) and, if
 *                 dprob_part != NULL (fp32 [Rcap, 2 * ceil(K/256)]), dprob_part[r, 2j] +
 *                 dprob_part[r, 2j + 1] = sum over the 256 columns c of column tile j of
 *                 dA[r,c] * silu(gate)*up (each entry covers 128 of the tile's columns; which
 *                 ones is the kernel's business): the partial sums of dL/d row_prob[r], in
 *                 fp32, written once each (no atomics; moe_scatter_row_dprob adds them in a
 *                 fixed order).  Rows of padding get partials of 0; rows >= offsets[E] are
 *                 not written.
 */
moe_status moe_grouped_gemm_fwd_weighted(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                         const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                         moe_dtype dt, moe_epilogue epi,
                                         const float* a_scale, const float* b_scale,
                                         const float* row_prob, void* C, void* C_act);
moe_status moe_grouped_gemm_dgrad_weighted(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                           const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                           moe_dtype dt, const void* Z_saved,
                                           const float* dc_scale, const float* b_scale,
                                           const float* row_prob, void* dA, float* dprob_part);

/*
 * The permute's row move fused into the GEMMs that read the permuted tensor (Permutation Fusion, Sec. 4.3.3,
 * taken one step further: the move disappears).  bf16 only.  An operand indexed by permuted rows is never
 * stored: its row r is row src_of[r] / k of an unpermuted tensor of T rows, and all zeros where src_of[r] < 0
 * (padding rows, rows >= offsets[E]); src_of is moe_permute's map, which can be had without the move
 * (moe_permute with X = NULL).  Results are bit for bit those of the plain calls on the permuted copy.
 *
 * fwd_gather:   moe_grouped_gemm_fwd_weighted(dt = MOE_BF16) with A[r,:] = X[src_of[r]/k,:], X [T,K].
 * dgrad_gather: moe_grouped_gemm_dgrad_weighted(dt = MOE_BF16) with dC[r,:] = G[src_of[r]/k,:], G [T,N]
 *               (under eq. (2) the combine's backward is a plain copy of dY rows, so G = dY).
 * wgrad_gather: moe_grouped_gemm_wgrad(dt = MOE_BF16) with one operand gathered: which = MOE_GATHER_A:
 *               `A` points to X [T,K] and A[r,:] = X[src_of[r]/k,:]; which = MOE_GATHER_DC: `dC` points to
 *               G [T,N] and dC[r,:] = G[src_of[r]/k,:].  The other operand is read as it lies, [Rcap, .].
 * Limits (MOE_ERR_UNSUPPORTED otherwise): T * row bytes <= 0xE0000000, Rcap < 2^29, T*k*k < 2^30 (32-bit
 * offsets inside the gathered tensor; the division by k is a multiplication).  Every src_of[r] >= 0 must be
 * below T*k, as moe_permute's are (the fetch is bounds-checked against the T rows, so a larger entry cannot
 * fault, but what it reads is unspecified).
 */
typedef enum { MOE_GATHER_A = 0, MOE_GATHER_DC = 1 } moe_gather;
moe_status moe_grouped_gemm_fwd_gather(moe_ctx* ctx, void* stream, const void* X, int T, const int32_t* src_of,
                                       int k, const void* B, const int32_t* offsets, int E, int N, int K,
                                       int64_t Rcap, moe_epilogue epi, const float* row_prob, void* C,
                                       void* C_act);
moe_status moe_grouped_gemm_dgrad_gather(moe_ctx* ctx, void* stream, const void* G, int T, const int32_t* src_of,
                                         int k, const void* B, const int32_t* offsets, int E, int N, int K,
                                         int64_t Rcap, const void* Z_saved, const float* row_prob, void* dA,
                                         float* dprob_part);
moe_status moe_grouped_gemm_wgrad_gather(moe_ctx* ctx, void* stream, const void* A, const void* dC,
                                         moe_gather which, int T, const int32_t* src_of, int k,
                                         const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                         int accumulate, moe_dtype out_dt, void* dB);

/*
 * Quantisation of a GEMM's output fused into its epilogue (Sec. 5.4.2; the activation + quantisation
 * epilogue of Sec. 4.3.2), blockwise recipe (dt = MOE_FP8_E4M3) only.  The calls are the _weighted ones
 * with two more outputs, which receive the 1x128 codes and scales of the bf16 tensor the epilogue
 * stores, bit for bit what moe_fp8_quantize(MOE_Q_1x128) would make of it:
 *   fwd  (epi = MOE_EPI_SWIGLU): act_q [Rcap, N/2] codes, act_q_scale [Rcap, N/256] of C_act;
 *   dgrad (Z_saved != NULL)    : dz_q  [Rcap, 2K] codes,  dz_q_scale [Rcap, 2K/128] of dZ.
 * Both NULL = the _weighted call.  Rows >= offsets[E] are not written.
 */
moe_status moe_grouped_gemm_fwd_quant(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                      const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                      moe_dtype dt, moe_epilogue epi,
                                      const float* a_scale, const float* b_scale,
                                      const float* row_prob, void* C, void* C_act,
                                      void* act_q, float* act_q_scale);
moe_status moe_grouped_gemm_dgrad_quant(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                        const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                        moe_dtype dt, const void* Z_saved,
                                        const float* dc_scale, const float* b_scale,
                                        const float* row_prob, void* dA, float* dprob_part,
                                        void* dz_q, float* dz_q_scale);

/*
 * The same fusion for the MXFP8 recipe (Sec. 5.3.3, 5.4.2; dt = MOE_MXFP8_E4M3 implied, operands and scales as
 * for the plain MXFP8 calls): the SwiGLU epilogue of fc1 / the SwiGLU-backward epilogue of the fc2 data gradient
 * also emit the quantised copies of the bf16 tensor they store (C_act [Rcap, N/2] / dZ [Rcap, 2K]; "cols" below is
 * that tensor's width), bit for bit what moe_mx_quantize_rowcol would make of it:
 *   q_row [Rcap, cols] codes, e8_row [Rcap, cols/32] E8M0 bytes: the 1x32 copy (operand of the next forward /
 *         data-gradient GEMM); required.
 *   q_col [Rcap, cols] codes, e8_col [Rcap/128, cols, 4] E8M0 bytes: the 32x1 copy (operand of the weight
 *         gradients); both NULL = not made.  Needs Rcap % 128 == 0 and every expert's range to start and end on a
 *         multiple of 128 rows (moe_permute with align = 128); otherwise the device error word is raised
 *         (moe_ctx_poll_error) and the outputs are undefined.
 * Rows >= offsets[E] are not written.  All device pointers; nothing is allocated.
 */
moe_status moe_grouped_gemm_fwd_quant_mx(moe_ctx* ctx, void* stream, const void* A, const void* B,
                                         const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                         const void* a_scale, const void* b_scale, const float* row_prob,
                                         void* C, void* C_act, void* act_q_row, uint8_t* act_e8_row,
                                         void* act_q_col, uint8_t* act_e8_col);
moe_status moe_grouped_gemm_dgrad_quant_mx(moe_ctx* ctx, void* stream, const void* dC, const void* B,
                                           const int32_t* offsets, int E, int N, int K, int64_t Rcap,
                                           const void* Z_saved, const void* dc_scale, const void* b_scale,
                                           const float* row_prob, void* dZ, float* dprob_part,
                                           void* dz_q_row, uint8_t* dz_e8_row, void* dz_q_col, uint8_t* dz_e8_col);

/*
 * Row-indexed view of the routing weights for eq. (2) and its inverse:
 *   gather:  row_prob[r] = prob[src_of[r]] for r < Rcap, 0 where src_of[r] < 0 (padding).
 *   scatter: dprob[t,s] = sum_j dprob_part[row_of[t,s], j], j = 0..parts-1 in increasing
 *            order; 0 for skipped slots (row_of < 0).
 */
moe_status moe_gather_row_prob(moe_ctx* ctx, void* stream, const float* prob, const int32_t* src_of,
                               int64_t Rcap, float* row_prob);
moe_status moe_scatter_row_dprob(moe_ctx* ctx, void* stream, const float* dprob_part, int parts,
                                 const int32_t* row_of, int T, int k, float* dprob);

/* ------------------------------------------------------------------------- */
/* Stage 4: Combine = unpermute + weighted sum (Sec. 4.3.3 "Unpermute"; eq. (1))*/
/* ------------------------------------------------------------------------- */
/*
 * Y[t,:] = sum_s prob[t,s] * O[row_of[t,s],:]  (+ residual[t,:]),  accumulated in
 * fp32 and rounded once to dt.  prob == NULL means weight 1 (the plain sum used
 * for the backward of permute and for eq. (2)); residual [T,h] is the shared
 * expert's output, added here (Sec. 2.1.1 stage 4), or NULL.  Slots with
 * row_of < 0 contribute nothing.  dt: MOE_BF16 or MOE_F32 (O, residual and Y).
 */
moe_status moe_unpermute_combine(moe_ctx* ctx, void* stream, const void* O, moe_dtype dt,
                                 const int32_t* row_of, const float* prob, const void* residual,
                                 int T, int k, int h, void* Y);

/*
 * Backward of the combine for L = <dY, Y>:
 *   dO[r,:] = prob[t,s] * dY[t,:] for the slot (t,s) = src_of[r], zero for padding
 *   rows (src_of[r] < 0);  dprob[t,s] = <dY[t,:], O[row_of[t,s],:]> in fp32 (0 for
 *   skipped slots).  O may be NULL together with dprob to skip the dot products.
 *   dO is written for all Rcap rows; dO may be NULL to get dprob only (when the rows of dO are
 *   produced elsewhere, e.g. quantised straight from dY by moe_mx_quantize_rowcol_gather).
 */
moe_status moe_unpermute_combine_bwd(moe_ctx* ctx, void* stream, const void* dY, const void* O,
                                     moe_dtype dt, const int32_t* row_of, const int32_t* src_of,
                                     const float* prob, int T, int k, int h, int64_t Rcap,
                                     void* dO, float* dprob);

/* ------------------------------------------------------------------------- */
/* Blockwise FP8 quantisation (Sec. 5.3.2; grouped, shapes on device: Sec. 5.4.2)*/
/* ------------------------------------------------------------------------- */
/*
 * X bf16 -> E4M3 codes q (same shape, one byte each) + fp32 scales.
 *   scale = amax(block) / 448 (1 if the block is all zero), code = nearest E4M3
 *   to clamp(x / scale, +-448), division and rounding in fp32, ties to even.
 *   block = MOE_Q_1x128  : 128 consecutive elements of a row;   scale [rows, cols/128]
 *           MOE_Q_128x1  : 128 consecutive rows of a column;    scale [rows/128, cols]
 *           MOE_Q_128x128: square blocks of each [rows,cols] matrix of a stack of
 *                          `groups` matrices;                   scale [groups, rows/128, cols/128]
 *   rows_dev: optional device int32 holding the number of rows actually in use
 *   (e.g. &offsets[E]); rows beyond it are skipped.  NULL = all `rows`.
 */
typedef enum { MOE_Q_1x128 = 0, MOE_Q_128x1 = 1, MOE_Q_128x128 = 2 } moe_qblock;
moe_status moe_fp8_quantize(moe_ctx* ctx, void* stream, const void* X, moe_qblock block,
                            int groups, int64_t rows, int cols, const int32_t* rows_dev,
                            void* q, float* scale);

/*
 * Both copies of a row-indexed tensor in one pass over it (Sec. 5.3.3: a tensor that two GEMMs read with
 * different contraction dimensions is quantised once per direction; Sec. 5.4.2: one grouped launch for all
 * experts): (q_row, scale_row) as MOE_Q_1x128, (q_col, scale_col) as MOE_Q_128x1, bit for bit.  Either pair may
 * be NULL to make only the other copy.  rows and cols must be multiples of 128; rows_dev as above (whole tiles
 * of 128 rows that start below *rows_dev are quantised).
 * _gather: the same for a tensor that is never stored in bf16 (quantisation fused into the permute, padding
 * included, and into the backward of the combine: Sec. 5.4.1, 5.4.2):
 *   V[r,:] = X[s / k, :] with s = src_of[r]                         (pair_scale == NULL: the permuted tokens)
 *   V[r,:] = bf16(pair_scale[s] * X[s / k, :]), product in fp32     (pair_scale [T*k]: dO = p * dY)
 *   V[r,:] = 0 where src_of[r] < 0 (padding rows)
 * X [T,cols] bf16, src_of [rows] as moe_permute returns it (call it with X = Xp = NULL for the maps alone),
 * rows = Rcap, k <= 32; `groups` (>= 1, normally E) only steers the order in which the row tiles are visited.
 */
moe_status moe_fp8_quantize_rowcol(moe_ctx* ctx, void* stream, const void* X, int64_t rows, int cols,
                                   const int32_t* rows_dev, void* q_row, float* scale_row,
                                   void* q_col, float* scale_col);
moe_status moe_fp8_quantize_rowcol_gather(moe_ctx* ctx, void* stream, const void* X, const int32_t* src_of, int k,
                                          const float* pair_scale, int groups, int64_t rows, int cols,
                                          const int32_t* rows_dev, void* q_row, float* scale_row,
                                          void* q_col, float* scale_col);

/* ------------------------------------------------------------------------- */
/* MXFP8 quantisation (Sec. 5.3.3): E4M3 elements, 1x32 blocks, E8M0 scales    */
/* ------------------------------------------------------------------------- */
/*
 * X bf16 -> E4M3 codes q (same shape, one byte each) + one E8M0 byte per block of 32
 * elements along the contraction dimension of the GEMM that will read the tensor.
 *   scale = 2^e, e = ceil(log2(amax(block) / 448)) clamped to +-127 (no element
 *   saturates), e8m0 byte = e + 127, an all-zero block gets 127;
 *   code = nearest E4M3 to x / 2^e, ties to even.
 *   block = MOE_MX_1x32: 32 consecutive elements of a row; X [rows,cols], groups = 1
 *                        (a weight stack [E,N,K] is passed as rows = E*N); e8m0 [rows, cols/32].
 *           MOE_MX_32x1: 32 consecutive rows of a column, for a tensor that a GEMM reads with its
 *                        row index as the contraction: the copy of a weight stack [groups, rows = N,
 *                        cols = K] for the data gradient, and both operands of the weight gradient
 *                        (groups = 1, rows = Rcap).  q keeps the layout of X; the scales are stored in
 *                        units of 128 rows, the step in which the GEMMs walk such a contraction:
 *                        e8m0 [groups*rows/128, cols, 4], byte j of entry (R, c) = block of rows
 *                        128 R + 32 j .. + 31 of column c.  rows and cols must be multiples of 128.
 *   rows_dev: as in moe_fp8_quantize (groups = 1 only).  With 32x1 blocks, whole tiles of 128 rows
 *   that start below *rows_dev are quantised.
 * moe_mx_quantize_rowcol makes both copies of X [rows,cols] in one pass over it (Sec. 5.3.3: a
 * tensor used in two GEMMs with different contraction dimensions needs both; Sec. 5.4.2: one grouped
 * launch for all experts): (q_row, e8m0_row) as MOE_MX_1x32, (q_col, e8m0_col) as MOE_MX_32x1, bit
 * for bit.  rows and cols must be multiples of 128.
 * The grouped GEMMs take these with dt = MOE_MXFP8_E4M3: the scale arguments then point to
 * the E8M0 bytes and the scaling is done by the matrix instruction itself:
 *   fwd  : A 1x32 codes, a_scale [Rcap, K/32];  B 1x32 codes of [E*N, K], b_scale [E*N, K/32]
 *   dgrad: dC 1x32 codes, dc_scale [Rcap, N/32]; B 32x1 codes, b_scale [E*N/128, K, 4]
 *   wgrad: A and dC 32x1 codes, a_scale [Rcap/128, K, 4], dc_scale [Rcap/128, N, 4]; every expert's
 *          row range must start and end on a multiple of 128 (moe_permute with align = 128),
 *          otherwise the error word is raised and dB is left untouched.
 * N and K must be multiples of 128.
 */
typedef enum { MOE_MX_1x32 = 0, MOE_MX_32x1 = 1 } moe_mxblock;
moe_status moe_mx_quantize(moe_ctx* ctx, void* stream, const void* X, moe_mxblock block,
                           int groups, int64_t rows, int cols, const int32_t* rows_dev,
                           void* q, uint8_t* e8m0);
moe_status moe_mx_quantize_rowcol(moe_ctx* ctx, void* stream, const void* X, int64_t rows, int cols,
                                  const int32_t* rows_dev, void* q_row, uint8_t* e8m0_row,
                                  void* q_col, uint8_t* e8m0_col);
/*
 * The same two copies of a tensor that is never stored in bf16 (quantisation fused into the permute,
 * padding included: Sec. 5.4.1, 5.4.2, and into the backward of the combine):
 *   V[r,:] = X[s / k, :] with s = src_of[r]                         (pair_scale == NULL: the permuted tokens)
 *   V[r,:] = bf16(pair_scale[s] * X[s / k, :]), product in fp32     (pair_scale [T*k]: dO = p * dY)
 *   V[r,:] = 0 where src_of[r] < 0 (padding rows)
 * X [T,cols] bf16, src_of [rows] as moe_permute returns it (call it with X = Xp = NULL for the maps
 * alone), rows = Rcap, k <= 32.  `groups` (>= 1, normally E) only steers the order in which the row
 * tiles are visited (expert-interleaved, so that the k copies of a token are read close together in
 * time); any value gives the same result.  Outputs and limits as moe_mx_quantize_rowcol, bit for bit
 * what it gives on V.
 */
moe_status moe_mx_quantize_rowcol_gather(moe_ctx* ctx, void* stream, const void* X, const int32_t* src_of, int k,
                                         const float* pair_scale, int groups, int64_t rows, int cols,
                                         const int32_t* rows_dev, void* q_row, uint8_t* e8m0_row,
                                         void* q_col, uint8_t* e8m0_col);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HIP_H */
