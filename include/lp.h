/*
 * lp.h -- C ABI of the MI355X (gfx950) hot path of Latent Parallelism (LP).
 *
 * LP serves a video diffusion model on K devices by splitting, at every
 * denoising step, the latent tensor itself: the step's partition dimension
 * rotates over temporal / height / width (Sec. 3.2, Eq. 3), the latent is cut
 * into K patch-aligned overlapping sub-latents along it (Sec. 3.3, Eq. 7-10),
 * each sub-latent is denoised independently (its DiT blocks run global
 * self-attention over that sub-latent's patch tokens only; supplement, proof
 * of Theorem 1, step 3), and the K predictions are stitched back with
 * position-aware weights (Sec. 3.4, Eq. 11-17).
 *
 * This library is that per-device work for one GPU: the integer plan (host),
 * lp_partition, lp_attention and lp_reconstruct (device).  The K sub-latents
 * that LP places on K devices are processed in turn on the one device.
 * With classifier-free guidance every sub-latent is denoised twice per step
 * (Eq. 4); lp_attention_batch serves the pair in one launch and
 * lp_reconstruct_guided_step folds guidance, reconstruction and the sampler's
 * update (Eq. 4-6) into one pass.
 *
 * Conventions
 *  - Every call returns an int status: LP_OK (0) or a negative LP_ERR_* code;
 *    lp_strerror() names it.  Nothing throws across this boundary.
 *  - "device pointer" = memory the current HIP device can access (hipMalloc);
 *    "host pointer" = ordinary process memory.  Device pointers are borrowed
 *    until the work enqueued by the call has finished; the caller owns them.
 *  - Where a call says that buffers must not alias or overlap, passing the very same address
 *    for both is refused with LP_ERR_INVALID_ARG; partial overlaps are not detected.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Device work is enqueued on it and the call returns without waiting.  No
 *    call here synchronises, allocates or frees device memory.
 *  - Dimensions: 0 = temporal (T), 1 = height (H), 2 = width (W).
 *    Partition index k is 0-based here (the paper counts from 1).
 *  - Latent layout: binary32 [C, T, H, W], contiguous, W fastest.  Sub-latent k
 *    is [C, T_k, H_k, W_k] contiguous (only the partition dimension differs
 *    from the latent's); the K sub-latents are packed back to back in k order,
 *    sub-latent k starting at element lp_part_info.elem_offset.
 */
#ifndef LP_H
#define LP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LP_OK 0
#define LP_ERR_INVALID_ARG (-1) /* null pointer, bad index, bad stride, aliased buffers       */
#define LP_ERR_SHAPE (-2)       /* a problem statement the method does not define: extent < 1, */
                                /* patch < 1 or not dividing its extent, K < 1, K above        */
                                /* LP_MAX_PARTS, r outside [0, K-1] (Sec. 3.3)                 */
#define LP_ERR_UNSUPPORTED (-3) /* head_dim not in {64, 128}, sizes past 32-bit addressing    */
#define LP_ERR_HIP (-4)         /* a HIP call failed; see lp_last_hip_error()                 */
#define LP_ERR_NOMEM (-5)       /* host allocation failed                                     */
#define LP_ERR_LIMIT (-6)       /* beyond the fixed scratch of a non-allocating entry point   */

#define LP_MAX_PARTS 64

/* Problem statement of one LP step (Sec. 3.3: latent size, patch sizes, K, r). */
typedef struct lp_config {
    int32_t C, T, H, W;       /* latent extents; C is never partitioned                     */
    int32_t pT, pH, pW;       /* patch sizes (p_T, p_H, p_W); each must divide its extent   */
    int32_t K;                /* number of partitions, 1 .. LP_MAX_PARTS                    */
    int32_t overlap_patches;  /* O >= 0 given directly, or -1: O = floor(L * overlap_ratio) */
    double overlap_ratio;     /* r in [0, K-1] (Sec. 3.3); read only if overlap_patches < 0 */
} lp_config;

/* Everything Eq. 7-9 and 11 give for one partition, plus its place in the packed buffer. */
typedef struct lp_part_info {
    int32_t alpha, beta;         /* core [alpha, beta) in patches, Eq. 7 (beta may exceed N)  */
    int32_t alpha_ext, beta_ext; /* extended [alpha', beta') in patches, Eq. 8               */
    int32_t s, e;                /* latent range [s, e) along the partition dim, Eq. 9       */
    int32_t len;                 /* l_k = e - s; 0 for an empty partition                    */
    int32_t delta_start;         /* Eq. 11 front ramp length (latent units)                  */
    int32_t delta_end;           /* Eq. 11 rear ramp length; <= 0 when the core passes N     */
    int32_t shape[4];            /* C, T_k, H_k, W_k                                          */
    int64_t elem_offset;         /* first element of sub-latent k in the packed buffer       */
    int64_t n_elems;             /* C * T_k * H_k * W_k                                       */
    int64_t n_tokens;            /* patches in the sub-latent = attention sequence length    */
} lp_part_info;

typedef struct lp_plan lp_plan; /* opaque; host memory owned by the library */

/*
 * Eq. 3: partition dimension of the step_1based-th forward pass (1, 2, 3 ->
 * T, H, W, repeating).  Returns 0, 1 or 2; LP_ERR_INVALID_ARG if step < 1.
 */
int lp_rotation_dim(int64_t step_1based);

/*
 * Eq. 7-9, 11: build the plan of K partitions of cfg's latent along `dim`.
 * Host only; no GPU work.  On success *out holds a plan the caller releases
 * with lp_plan_destroy.  With N = D/p patches along dim: L = ceil(N/K),
 * core_k = [k L, k L + L), O = overlap_patches or floor(L r),
 * extended = [max(0, alpha - O), min(N, beta + O)), latent range = extended * p.
 * Errors: LP_ERR_INVALID_ARG (null, dim not 0..2), LP_ERR_SHAPE (extent or patch
 * < 1, patch not dividing its extent, K < 1, K > LP_MAX_PARTS, r outside
 * [0, K-1] or O > L (K-1)), LP_ERR_UNSUPPORTED (latent of 2^40 elements or
 * more), LP_ERR_NOMEM.
 */
int lp_plan_create(const lp_config *cfg, int32_t dim, lp_plan **out);
void lp_plan_destroy(lp_plan *plan); /* NULL is allowed */

int32_t lp_plan_num_parts(const lp_plan *plan);   /* K, or LP_ERR_INVALID_ARG            */
int32_t lp_plan_dim(const lp_plan *plan);         /* 0..2, or LP_ERR_INVALID_ARG         */
int64_t lp_plan_total_elems(const lp_plan *plan); /* floats in the packed buffer (S_ext) */
int64_t lp_plan_latent_elems(const lp_plan *plan);/* C*T*H*W (S_z)                       */
/* Fill *out (host pointer) for partition k in [0, K). */
int lp_plan_query(const lp_plan *plan, int32_t k, lp_part_info *out);

/*
 * Eq. 10: subs_packed[elem_offset_k + (c, t, h, w)] = z[c, t + s_k [dim=T],
 * h + s_k [dim=H], w + s_k [dim=W]] for all K partitions, one launch.
 * z: device, lp_plan_latent_elems floats, read only.  subs_packed: device,
 * lp_plan_total_elems floats, fully overwritten; must not alias z.
 * A pure copy: results are bit-identical to the input elements.
 */
int lp_partition(const lp_plan *plan, const float *z, float *subs_packed, void *stream);

/*
 * Eq. 12-17: out[x] = A(x) / Z(x) with A = sum_k I_k(x) W^(k)_j pred_k[j],
 * Z = sum_k I_k(x) W^(k)_j, j = x - s_k, weights by Eq. 12 (front ramp
 * j/Delta_start, 1 on the core, rear ramp (l_k - j)/Delta_end).
 * preds_packed: device, same packing as lp_partition's output, read only.
 * out: device, lp_plan_latent_elems floats, fully overwritten; must not alias preds_packed.
 * Arithmetic is binary32 in a fixed order -- k ascending from A = Z = 0,
 * w by one IEEE division, A += (w * pred) as a rounded product then a rounded
 * sum, out = A / Z by IEEE division -- so results are reproducible bit for bit.
 */
int lp_reconstruct(const lp_plan *plan, const float *preds_packed, float *out, void *stream);

/*
 * Eq. 4-6 as one pass: the denoising step on the reconstructed guided prediction,
 *   g_k = u_k + guidance * (c_k - u_k)          per element of every sub-latent (Eq. 4)
 *   pred = A / Z of the g_k                      as lp_reconstruct (Eq. 5, 12-17)
 *   out = coef_z * z + coef_pred * pred          the sampler's update (Eq. 6)
 * The paper leaves the sampler S open; this is the affine form z' = a z + b pred with
 * per-step scalars (an Euler step of a flow-matching sampler: a = 1, b = sigma' - sigma).
 * cond_packed, uncond_packed: device, conditional and unconditional predictions, both packed
 * like lp_partition's output, read only.  z: device, lp_plan_latent_elems floats.  out: device,
 * lp_plan_latent_elems floats, fully overwritten; out may be z itself (update in place) but must
 * not overlap cond_packed or uncond_packed.
 * Arithmetic is binary32, every operation rounded on its own, in this order: d = c - u,
 * m = guidance * d, g = u + m; lp_reconstruct's order on g; p = coef_z * z, q = coef_pred * pred,
 * out = p + q.  Results are reproducible bit for bit.
 * Reads (2 gamma + 1) S_z bytes and writes S_z, against (4 gamma + 4) S_z for guidance,
 * reconstruction and update as three passes.
 */
int lp_reconstruct_guided_step(const lp_plan *plan, const float *cond_packed, const float *uncond_packed,
                               float guidance, const float *z, float coef_z, float coef_pred, float *out,
                               void *stream);

/*
 * lp_reconstruct_guided_step followed by lp_partition of its result for the NEXT step (Eq. 4-6,
 * then Eq. 10 along the next rotating dimension), in one pass: every element of the updated
 * latent is written to `out` and to each sub-latent of next_plan that contains it, which saves
 * the next step's partition launch and its read of the latent.  next_plan: a plan over the same
 * latent extents (else LP_ERR_INVALID_ARG), normally along lp_rotation_dim(i + 1).
 * next_subs_packed: device, lp_plan_total_elems(next_plan) floats, fully overwritten, must not
 * overlap any other buffer.  Everything else, and every value written, as the two calls it replaces.
 */
int lp_reconstruct_guided_step_partition(const lp_plan *plan, const float *cond_packed, const float *uncond_packed,
                                         float guidance, const float *z, float coef_z, float coef_pred, float *out,
                                         const lp_plan *next_plan, float *next_subs_packed, void *stream);

/*
 * Self-attention inside one sub-latent: for every head h and token i,
 *   o[i,h,:] = sum_j softmax_j(scale * <q[i,h,:], k[j,h,:]>) v[j,h,:]
 * over all n_tokens tokens j of the sub-latent (no mask, not causal): inside a
 * sub-latent the DiT blocks attend globally over all of its positions
 * (supplement, proof of Theorem 1, step 3).
 * q, k, v, o: device, bfloat16; element (token, head, d) lives at
 * token * stride_tok + head * stride_head + d (strides in elements, the same
 * for all four tensors; d contiguous).  Required: head_dim in {64, 128}; both
 * strides multiples of 8 and all four base pointers 16-byte aligned; rows must
 * not overlap, i.e. either stride_tok >= heads * stride_head >= heads * head_dim
 * (token-major) or stride_head >= n_tokens * stride_tok, stride_tok >= head_dim
 * (head-major); (n_tokens * stride_tok + head_dim) * 2 < 2^31 (else
 * LP_ERR_UNSUPPORTED).  o must not alias q, k or v.
 * scale <= 0 selects 1/sqrt(head_dim).  n_tokens = 0 is a successful no-op.
 * workspace: optional device scratch of at least
 * lp_attention_workspace_size(head_dim) bytes, 16-byte aligned, contents
 * irrelevant on entry and undefined on return.  With it the work is dealt evenly
 * over the compute units whatever n_tokens and heads are (partial results of a
 * query tile that two workgroups share pass through the workspace and a second
 * small kernel merges them); with NULL (or too small a workspace) one workgroup
 * is launched per 256-row query tile and head, which leaves compute units idle
 * when their number does not divide the tile count.  Two calls that overlap in
 * time must not share a workspace.
 * Products run on bf16 MFMA with binary32 accumulation; q is multiplied by
 * scale*log2(e) and re-rounded to bf16 once; the softmax is binary32;
 * probabilities are rounded to bf16 before the second product and the result is
 * rounded to bf16 on store.
 * Scores of any finite size are handled.  A workgroup first takes its stretch of
 * keys relative to the largest score among its first 32; if some later score
 * lies so far above that one (about 2^7 in log2 units) that a probability, a row
 * sum or an output accumulator overflows binary32, it takes the stretch again
 * with a running maximum.  Such inputs cost up to twice the time, not accuracy.
 * Inputs must be finite.  With an infinity or a NaN in q, k or v the affected
 * output rows are unspecified (typically NaN, also where the definition would
 * give an infinity: rows of v beyond a probability of exactly 0 are still
 * multiplied); no memory outside o is written and the call still succeeds.
 * The workspace parameters are this library's own addition to the operation:
 * the method defines only q, k, v -> o.  NULL keeps the call allocation- and
 * scratch-free at the cost of idle compute units (see above).
 */
int lp_attention(const void *q, const void *k, const void *v, void *o, int64_t n_tokens,
                 int32_t heads, int32_t head_dim, int64_t stride_tok, int64_t stride_head,
                 float scale, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * lp_attention over `batch` independent items in one launch -- the conditional and the
 * unconditional pass of a guided step (Eq. 4) are batch = 2.  Item b, token i, head h, element d
 * lives at b * stride_batch + i * stride_tok + h * stride_head + d; items never attend to each
 * other.  Everything else as lp_attention (batch = 1 is lp_attention).  Allowed layouts for
 * batch > 1: the items one after the other (stride_batch at least the extent of one item), or,
 * token-major, the items of a token side by side (stride_tok >= batch * stride_batch,
 * stride_batch >= heads * stride_head); stride_batch a multiple of 8.  One launch deals all
 * batch * heads * ceil(n_tokens / 256) query tiles over the compute units together, which for
 * sequences of a few thousand tokens is measurably faster than one call per item.
 */
int lp_attention_batch(const void *q, const void *k, const void *v, void *o, int32_t batch, int64_t n_tokens,
                       int32_t heads, int32_t head_dim, int64_t stride_batch, int64_t stride_tok,
                       int64_t stride_head, float scale, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Bytes of workspace lp_attention can use on the current device for this
 * head_dim (2 partial-result slots per compute unit; about 35 MB for head_dim
 * 128 on 256 compute units).  Negative LP_ERR_* on failure.
 */
int64_t lp_attention_workspace_size(int32_t head_dim);

/*
 * ---- The DiT-block operations on either side of the attention core -------------------------
 * The paper says only that the denoiser is a stack of DiT blocks (Sec. 5.1) whose atomic units
 * are the patches (Sec. 3.1); it fixes none of the block's internals.  The form taken here is
 * the common one and is this library's stated reading, not the paper's:
 *   y = x W^T + b,  cut into q | k | v sections of d_model = heads * head_dim features each;
 *   q, k <- x / sqrt(mean_d x^2 + eps) * gain[head, d]   per (token, head), over head_dim;
 *   q, k <- rotated pairwise: elements (2 j, 2 j + 1) of a part of size p of head_dim turn by
 *           pos * base^(-2 j / p), the three parts split[0..2] (even, adding up to head_dim)
 *           taking pos = the token's t, h, w patch coordinate in turn;
 *   out = o W_o^T + b_o after attention.
 * Tokens are the patches of the sub-latent in row-major (t, h, w) order (grid[0..2], whose
 * product is n_tokens); offset[0..2] is added to the coordinates (0 = coordinates local to
 * the sub-latent; alpha'_k along the partition dimension places it in the global grid).
 */
typedef struct lp_rope {
    int32_t grid[3];   /* patches of the sub-latent along T, H, W                      */
    int32_t offset[3]; /* added to the patch coordinates                               */
    int32_t split[3];  /* head_dim features rotated by t, h, w: even, sum = head_dim   */
    float base;        /* > 0, e.g. 10000                                              */
} lp_rope;

/*
 * q | k | v = x w_qkv^T + bias with the normalisation and rotation of q and k done in the
 * product's epilogue (one launch; q, k, v are written once, in the layout lp_attention reads).
 * x: device, bf16 [n_tokens, d_model].  w_qkv: device, bf16 [3 d_model, d_model], row o holding
 * the weights of output feature o; rows [0, d_model) produce q, [d_model, 2 d_model) k, the rest v.
 * bias: device, binary32 [3 d_model], or NULL.  gain_q, gain_k: device, binary32 [heads, head_dim].
 * q, k, v: device, bf16 [n_tokens, heads, head_dim] contiguous, fully overwritten; they must not
 * alias each other or x.  All pointers 16-byte aligned.  rope: host pointer.
 * head_dim in {64, 128}, d_model a multiple of 128 (else LP_ERR_UNSUPPORTED); n_tokens = 0 is a
 * successful no-op.  The product runs on bf16 MFMA with binary32 accumulation; bias, normalisation
 * and rotation are binary32 (angles via the hardware sine / cosine of the fractional turn count);
 * the result is rounded to bf16 once, on store.
 */
int lp_qkv_projection(const void *x, const void *w_qkv, const float *bias, const float *gain_q, const float *gain_k,
                      float eps, const lp_rope *rope, void *q, void *k, void *v, int64_t n_tokens, int32_t heads,
                      int32_t head_dim, void *stream);

/*
 * y = x w^T + bias: the block's output projection (or any linear layer of these shapes).
 * x: device, bf16 [n, d_in]; w: device, bf16 [d_out, d_in]; bias: device, binary32 [d_out] or NULL;
 * y: device, bf16 [n, d_out], fully overwritten, must not alias x or w.  d_in a multiple of 64,
 * d_out a multiple of 128 (else LP_ERR_UNSUPPORTED).  bf16 MFMA, binary32 accumulation, one
 * rounding to bf16 on store.
 */
int lp_linear(const void *x, const void *w, const float *bias, void *y, int64_t n, int32_t d_in, int32_t d_out,
              void *stream);

/*
 * The normalisation + rotation of lp_qkv_projection alone, in place, for q or k projected
 * elsewhere.  x: device, bf16, element (token, head, d) at token * stride_tok + head * stride_head
 * + d (strides as in lp_attention).  gain: device, binary32 [heads, head_dim].
 */
int lp_qk_norm_rope(void *x, const float *gain, float eps, const lp_rope *rope, int64_t n_tokens, int32_t heads,
                    int32_t head_dim, int64_t stride_tok, int64_t stride_head, void *stream);

/*
 * lp_attention for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same kernels, with the scratch for shared query tiles taken from a fixed array that
 * lives in the library's device image (lp_attention_static_scratch_bytes() bytes, about
 * 35 MB, held by every device the library runs on until the process ends).  Arguments,
 * results and errors as lp_attention without its workspace pair.  The call allocates and
 * frees nothing; its first call on a device looks the array's address up once.
 * LP_ERR_LIMIT if the device has more compute units than the array has slots for
 * (2 per compute unit, 256 compute units at head_dim 128).
 * All calls on one device share the one array: calls that overlap in time on the same
 * device (two streams, two threads) race on it and must be serialised by the caller.
 */
int lp_attention_static(const void *q, const void *k, const void *v, void *o, int64_t n_tokens,
                        int32_t heads, int32_t head_dim, int64_t stride_tok, int64_t stride_head,
                        float scale, void *stream);
int64_t lp_attention_static_scratch_bytes(void); /* size of that array, bytes */

const char *lp_strerror(int status); /* static string, never NULL              */
int lp_last_hip_error(void);         /* hipError_t of the last LP_ERR_HIP (thread local) */
const char *lp_version(void);        /* "lp-mi355x x.y (gfx950)"               */

#ifdef __cplusplus
}
#endif
#endif /* LP_H */
