/*
 * lp_oracle.c -- CPU oracle for the single-GPU hot path of Latent Parallelism (LP).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * path computes.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may build, load or call it.  It shares no code, header or table with the
 * HIP library and the HIP library never calls it.
 *
 * What is here, each written straight from the paper's definitions:
 *   lpo_rotation_dim   rotating partition dimension            (Sec. 3.2, Eq. 3)
 *   lpo_plan           patch-aligned overlapping partition     (Sec. 3.3, Eq. 7-9)
 *                      and ramp lengths                         (Sec. 3.4, Eq. 11)
 *   lpo_weight         position-aware weight mask              (Sec. 3.4, Eq. 12)
 *   lpo_partition      sub-latent extraction                   (Sec. 3.3, Eq. 10)
 *   lpo_reconstruct    weighted averaging A/Z                  (Sec. 3.4, Eq. 13-17)
 *   lpo_guided_step    per-partition classifier-free guidance, reconstruction and
 *                      the sampler's update as one denoising step  (Sec. 3.2, Eq. 4-6)
 *   lpo_attention      global softmax self-attention inside one sub-latent
 *                      (supplement, proof of Theorem 1, step 3: attention acts
 *                      over all positions of the sub-latent) -- the textbook
 *                      definition softmax(scale * Q K^T) V, three passes per row.
 *
 * Equation numbers count the paper's displayed equations of the main body in
 * order of appearance (the source leaves them unnumbered):
 *   1 sampler step, 2 CFG, 3 rotation, 4 per-partition CFG, 5 reconstruction F,
 *   6 sampler on the reconstructed prediction, 7 core bounds, 8 extended bounds,
 *   9 latent bounds, 10 partition map, 11 ramp lengths, 12 weights,
 *   13 pi_k, 14 indicator, 15 A, 16 Z, 17 A/Z.
 *
 * Precision.  Partition is a copy.  Weights and reconstruction are evaluated in
 * IEEE binary32 with a fixed operation order (see lpo_reconstruct) so that an
 * independent implementation following the same order agrees bit for bit; this
 * file must be compiled with -ffp-contract=off and without -ffast-math.
 * Attention takes binary32 inputs (bf16 values widened), does every product,
 * sum and exponential in binary64 and returns binary32.
 *
 * Pins (tests/test_oracle_*.py): the paper's Table 1 LP rows for the integer
 * plan; closed forms and hand-derived weight tables; round-trip and
 * slice-consistency identities for reconstruction; a separate pure-Python
 * brute force and analytic special cases for attention.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct lpo_part {
    int32_t alpha, beta;         /* core region in patch space, Eq. 7 (beta may exceed N) */
    int32_t alpha_ext, beta_ext; /* extended region in patch space, Eq. 8                 */
    int32_t s, e;                /* latent range along the partition dim, Eq. 9           */
    int32_t len;                 /* l_k = e - s                                           */
    int32_t delta_start;         /* Eq. 11, front ramp length in latent units             */
    int32_t delta_end;           /* Eq. 11, rear ramp length; <= 0 when beta > N          */
    int32_t shape[4];            /* C, T_k, H_k, W_k of the packed sub-latent             */
    int64_t elem_offset;         /* start of sub-latent k in the packed buffer (floats)   */
    int64_t n_elems;             /* C*T_k*H_k*W_k                                         */
    int64_t n_tokens;            /* patches in the sub-latent                             */
} lpo_part;

/* Eq. 3: step i (1-based) -> 0 = temporal, 1 = height, 2 = width. */
int lpo_rotation_dim(int64_t step_1based)
{
    if (step_1based < 1) return -1;
    return (int)((step_1based - 1) % 3);
}

/*
 * Eq. 7-9 and 11 along dimension `dim` (0=T,1=H,2=W) of a latent [C,T,H,W].
 * overlap_patches >= 0 gives O directly; otherwise O = floor(L * r).
 * Returns 0, or -1 on arguments the method does not define (K < 1, a patch
 * size that does not divide its extent, r outside [0, K-1]).
 *
 * When K*L > N the last cores run past N.  Eq. 8 clamps only the extended
 * bounds, so Eq. 11 evaluated as written gives delta_end <= 0 there (and a
 * delta_start that may exceed len when alpha_k > N).  Both are kept as the
 * equations give them: Eq. 12's cases, tested in the order written, stay well
 * defined (a non-positive delta_end makes the third range empty and lets the
 * second run to l_k).  If alpha - O >= N the partition is empty (len 0).
 */
int lpo_plan(const int32_t latent[4], const int32_t patch[3], int32_t K,
             int32_t overlap_patches, double r, int32_t dim, lpo_part *parts)
{
    if (K < 1 || dim < 0 || dim > 2) return -1;
    for (int d = 0; d < 4; ++d) if (latent[d] < 1) return -1;
    for (int d = 0; d < 3; ++d) {
        if (patch[d] < 1) return -1;
        if (latent[1 + d] % patch[d] != 0) return -1;
    }
    const int32_t D = latent[1 + dim];
    const int32_t p = patch[dim];
    const int32_t N = D / p;                 /* number of patches along dim      */
    const int32_t L = (N + K - 1) / K;       /* ceil(N / K), core patches        */
    int32_t O;
    if (overlap_patches >= 0) {
        O = overlap_patches;
    } else {
        if (!(r >= 0.0) || r > (double)(K - 1)) return -1;
        O = (int32_t)floor((double)L * r);
    }
    if ((int64_t)O > (int64_t)L * (K - 1)) return -1;

    int64_t offset = 0;
    for (int32_t k1 = 1; k1 <= K; ++k1) {    /* the paper's 1-based k            */
        lpo_part *q = &parts[k1 - 1];
        const int64_t alpha = (int64_t)(k1 - 1) * L;             /* Eq. 7 */
        const int64_t beta = alpha + L;
        int64_t alpha_ext = alpha - O; if (alpha_ext < 0) alpha_ext = 0;   /* Eq. 8 */
        int64_t beta_ext = beta + O;   if (beta_ext > N) beta_ext = N;
        if (alpha_ext > beta_ext) alpha_ext = beta_ext;          /* empty partition */
        q->alpha = (int32_t)alpha; q->beta = (int32_t)beta;
        q->alpha_ext = (int32_t)alpha_ext; q->beta_ext = (int32_t)beta_ext;
        q->s = (int32_t)(alpha_ext * p);                         /* Eq. 9 */
        q->e = (int32_t)(beta_ext * p);
        q->len = q->e - q->s;
        q->delta_start = (int32_t)((alpha - alpha_ext) * p);     /* Eq. 11 */
        q->delta_end = (int32_t)((beta_ext - beta) * p);
        q->shape[0] = latent[0];
        for (int d = 0; d < 3; ++d) q->shape[1 + d] = (d == dim) ? q->len : latent[1 + d];
        q->n_elems = (int64_t)q->shape[0] * q->shape[1] * q->shape[2] * q->shape[3];
        q->n_tokens = 1;
        for (int d = 0; d < 3; ++d) q->n_tokens *= q->shape[1 + d] / patch[d];
        q->elem_offset = offset;
        offset += q->n_elems;
    }
    return 0;
}

/*
 * Eq. 12: weight of local position j in [0, len).  The three cases are tested
 * in the order the paper writes them, so a zero-length ramp never divides.
 */
float lpo_weight(int32_t j, int32_t len, int32_t delta_start, int32_t delta_end)
{
    if (j < delta_start) return (float)j / (float)delta_start;
    if (j < len - delta_end) return 1.0f;
    return (float)(len - j) / (float)delta_end;
}

static int64_t lat_index(const int32_t latent[4], int64_t c, int64_t t, int64_t h, int64_t w)
{
    return ((c * latent[1] + t) * latent[2] + h) * latent[3] + w;
}

/* Eq. 10: z^(k) = z[..., s_k:e_k, ...] along dim, packed [C,T_k,H_k,W_k] back to back. */
void lpo_partition(const int32_t latent[4], int32_t dim, int32_t K, const lpo_part *parts,
                   const float *z, float *subs)
{
    for (int32_t k = 0; k < K; ++k) {
        const lpo_part *q = &parts[k];
        float *dst = subs + q->elem_offset;
        const int64_t st = (dim == 0) ? q->s : 0;
        const int64_t sh = (dim == 1) ? q->s : 0;
        const int64_t sw = (dim == 2) ? q->s : 0;
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t c = 0; c < q->shape[0]; ++c)
            for (int64_t t = 0; t < q->shape[1]; ++t)
                for (int64_t h = 0; h < q->shape[2]; ++h)
                    for (int64_t w = 0; w < q->shape[3]; ++w) {
                        const int64_t li = ((c * q->shape[1] + t) * q->shape[2] + h) * q->shape[3] + w;
                        dst[li] = z[lat_index(latent, c, t + st, h + sh, w + sw)];
                    }
    }
}

/*
 * Eq. 13-17.  For every latent position, k ascending from A = 0, Z = 0:
 *   if s_k <= x < e_k (Eq. 14):  j = x - s_k (Eq. 13);  w = W^(k)_j (Eq. 12);
 *       A = A + (w * pred_k[j])   -- product rounded, then sum rounded (Eq. 15)
 *       Z = Z + w                                                   (Eq. 16)
 *   out = A / Z                                                     (Eq. 17)
 * all in binary32.
 */
void lpo_reconstruct(const int32_t latent[4], int32_t dim, int32_t K, const lpo_part *parts,
                     const float *preds, float *out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t c = 0; c < latent[0]; ++c)
        for (int64_t t = 0; t < latent[1]; ++t)
            for (int64_t h = 0; h < latent[2]; ++h)
                for (int64_t w = 0; w < latent[3]; ++w) {
                    const int64_t x = (dim == 0) ? t : (dim == 1) ? h : w;
                    float A = 0.0f, Z = 0.0f;
                    for (int32_t k = 0; k < K; ++k) {
                        const lpo_part *q = &parts[k];
                        if (x < q->s || x >= q->e) continue;
                        const int32_t j = (int32_t)(x - q->s);
                        const float wt = lpo_weight(j, q->len, q->delta_start, q->delta_end);
                        const int64_t lt = (dim == 0) ? j : t;
                        const int64_t lh = (dim == 1) ? j : h;
                        const int64_t lw = (dim == 2) ? j : w;
                        const int64_t li = ((c * q->shape[1] + lt) * q->shape[2] + lh) * q->shape[3] + lw;
                        const float prod = wt * preds[q->elem_offset + li];
                        A = A + prod;
                        Z = Z + wt;
                    }
                    out[lat_index(latent, c, t, h, w)] = A / Z;
                }
}

/*
 * One denoising step on the reconstructed prediction, in the paper's order:
 *   Eq. 4  g_k = u_k + w (c_k - u_k)       on every element of every sub-latent prediction
 *                                          (c = conditional, u = unconditional, w = guidance scale)
 *   Eq. 5  pred = F({g_k}, d)              lpo_reconstruct
 *   Eq. 6  z' = S(z, pred, t)              the sampler.  The paper leaves S open; taken here as
 *                                          the affine update z' = a z + b pred with per-step
 *                                          scalars a, b (an Euler step of a flow-matching
 *                                          sampler is a = 1, b = sigma' - sigma).
 * binary32 throughout, every operation rounded on its own: d = c - u, m = w d, g = u + m;
 * then lpo_reconstruct's order; then p = a z, q = b pred, z' = p + q.
 * `guided` is caller-provided scratch of the packed size.
 */
void lpo_guided_step(const int32_t latent[4], int32_t dim, int32_t K, const lpo_part *parts, int64_t total_elems,
                     const float *cond, const float *uncond, float w, const float *z, float a, float b,
                     float *guided, float *out)
{
    for (int64_t i = 0; i < total_elems; ++i) {
        const float d = cond[i] - uncond[i];
        const float m = w * d;
        guided[i] = uncond[i] + m;
    }
    lpo_reconstruct(latent, dim, K, parts, guided, out);
    const int64_t n = (int64_t)latent[0] * latent[1] * latent[2] * latent[3];
    for (int64_t i = 0; i < n; ++i) {
        const float p = a * z[i];
        const float q = b * out[i];
        out[i] = p + q;
    }
}

static float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/*
 * Softmax attention over the n tokens of one sub-latent, per head:
 *   s_j = scale * sum_d q[i,d] k[j,d];  p_j = exp(s_j - max_j s_j) / sum_j exp(.)
 *   o[i,:] = sum_j p_j v[j,:]
 * q, k, v: bf16 bit patterns, element (token, head, d) at token*stride_tok +
 * head*stride_head + d (strides in elements).  Only the query rows listed in
 * `rows` (n_rows of them; NULL = all n rows in order) are evaluated, each over
 * all n keys.  out is [n_rows, heads, head_dim] binary32, dense.
 * The K and V rows of the current head are widened to binary64 once up front
 * (a change of storage, not of arithmetic).  Returns 0, or -1 if memory for
 * that copy or for the per-thread score rows cannot be had (all of it is
 * requested before the first parallel loop).
 */
int lpo_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v, float *out,
                  int64_t n, int32_t heads, int32_t head_dim,
                  int64_t stride_tok, int64_t stride_head, double scale,
                  const int64_t *rows, int64_t n_rows)
{
    if (rows == NULL) n_rows = n;
    if (n <= 0 || n_rows <= 0) return 0;
    const int64_t D = head_dim;
    /* work buffers, one set per thread, all allocated before any parallel region */
#ifdef _OPENMP
    const int64_t nt = omp_get_max_threads();
#else
    const int64_t nt = 1;
#endif
    double *kd = (double *)malloc((size_t)(n * D) * sizeof(double));
    double *vd = (double *)malloc((size_t)(n * D) * sizeof(double));
    double *score_all = (double *)malloc((size_t)(nt * n) * sizeof(double));
    double *acc_all = (double *)malloc((size_t)(nt * D) * sizeof(double));
    double *qrow_all = (double *)malloc((size_t)(nt * D) * sizeof(double));
    if (!kd || !vd || !score_all || !acc_all || !qrow_all) {
        free(kd); free(vd); free(score_all); free(acc_all); free(qrow_all);
        return -1;
    }
    for (int32_t h = 0; h < heads; ++h) {
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < n; ++j) {
            const uint16_t *kj = k + j * stride_tok + (int64_t)h * stride_head;
            const uint16_t *vj = v + j * stride_tok + (int64_t)h * stride_head;
            for (int64_t d = 0; d < D; ++d) {
                kd[j * D + d] = (double)bf16_to_f32(kj[d]);
                vd[j * D + d] = (double)bf16_to_f32(vj[d]);
            }
        }
#pragma omp parallel for schedule(dynamic, 4)
        for (int64_t ri = 0; ri < n_rows; ++ri) {
#ifdef _OPENMP
            const int64_t me = omp_get_thread_num();
#else
            const int64_t me = 0;
#endif
            double *score = score_all + me * n, *acc = acc_all + me * D, *qrow = qrow_all + me * D;
            const int64_t i = rows ? rows[ri] : ri;
            const uint16_t *qi = q + i * stride_tok + (int64_t)h * stride_head;
            for (int64_t d = 0; d < D; ++d) qrow[d] = (double)bf16_to_f32(qi[d]);
            /* pass 1: scores and their maximum */
            double mx = -INFINITY;
            for (int64_t j = 0; j < n; ++j) {
                const double *kj = kd + j * D;
                double dot = 0.0;
#pragma omp simd reduction(+ : dot)
                for (int64_t d = 0; d < D; ++d) dot += qrow[d] * kj[d];
                const double sj = scale * dot;
                score[j] = sj;
                if (sj > mx) mx = sj;
            }
            /* pass 2: exponentials and their sum */
            double denom = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                score[j] = exp(score[j] - mx);
                denom += score[j];
            }
            /* pass 3: weighted sum of value rows */
            for (int64_t d = 0; d < D; ++d) acc[d] = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                const double *vj = vd + j * D;
                const double pj = score[j] / denom;
                for (int64_t d = 0; d < D; ++d) acc[d] += pj * vj[d];
            }
            float *o = out + (ri * heads + h) * D;
            for (int64_t d = 0; d < D; ++d) o[d] = (float)acc[d];
        }
    }
    free(kd); free(vd); free(score_all); free(acc_all); free(qrow_all);
    return 0;
}

/* Threads the parallel loops above run on (1 when built without OpenMP). */
int lpo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
