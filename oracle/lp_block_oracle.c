/*
 * lp_block_oracle.c -- CPU oracle for the DiT-block operations next to the attention core:
 * the QKV projection, the per-head RMS normalisation of queries and keys, the 3-D rotary
 * position encoding over the (t, h, w) patch grid of a sub-latent, and the output projection.
 *
 * TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's CPU-baseline leg
 * may build, load or call it; it shares no code, header or table with the HIP library.
 *
 * The paper says only that the denoiser is a stack of DiT blocks (Sec. 5.1: 30 of them) whose
 * atomic units are the spatio-temporal patches (Sec. 3.1) and that attention acts over all
 * positions of a sub-latent (supplement, proof of Theorem 1, step 3).  It fixes none of the
 * block's internals, so what is below is a stated reading, the common form of such a block:
 *
 *   y      = x W^T + b                      x: [n, d_model], W: [3 d_model, d_model]
 *   q|k|v  = the three d_model-wide sections of y, each seen as [n, heads, head_dim]
 *   q, k   <- RMS-normalised per (token, head) over head_dim, times a learned gain
 *   q, k   <- rotated pairwise by angles that depend on the token's patch coordinates
 *   o      = attention(q, k, v)             (lp_oracle.c)
 *   out    = o W_o^T + b_o
 *
 * Every function evaluates its definition in binary64 with plain loops; inputs are bf16
 * (bit patterns) or binary32, outputs binary32 (so a chain of them rounds to binary32 between
 * its links, far below the bf16 resolution the HIP path is compared at).  The chain itself --
 * projection, split into q | k | v, normalisation and rotation of q and k -- is put together
 * by the Python front end from these functions.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * Linear layer: y[i, o] = sum_c x[i, c] * w[o, c] + bias[o]  (bias may be NULL).
 * x: bf16 [n, d_in] row-major, w: bf16 [d_out, d_in] row-major (one row per output feature).
 */
void lpo_linear(const uint16_t *x, const uint16_t *w, const float *bias, int64_t n, int64_t d_in, int64_t d_out,
                float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t o = 0; o < d_out; ++o) {
            double acc = 0.0;
            for (int64_t c = 0; c < d_in; ++c) acc += bf16_to_f64(x[i * d_in + c]) * bf16_to_f64(w[o * d_in + c]);
            if (bias) acc += (double)bias[o];
            y[i * d_out + o] = (float)acc;
        }
}

/*
 * Per-head RMS normalisation, in place: for every (token, head)
 *   x[d] <- x[d] / sqrt(mean_d x[d]^2 + eps) * gain[head, d].
 * x: binary32 [n, heads, head_dim]; gain: binary32 [heads, head_dim].
 */
void lpo_rms_norm_heads(float *x, const float *gain, int64_t n, int32_t heads, int32_t head_dim, double eps)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int32_t h = 0; h < heads; ++h) {
            float *row = x + (i * heads + h) * head_dim;
            double ss = 0.0;
            for (int32_t d = 0; d < head_dim; ++d) ss += (double)row[d] * (double)row[d];
            const double r = sqrt(ss / (double)head_dim + eps);
            for (int32_t d = 0; d < head_dim; ++d) row[d] = (float)((double)row[d] / r * (double)gain[h * head_dim + d]);
        }
}

/*
 * 3-D rotary position encoding, in place.  Token i of the sub-latent sits at patch coordinates
 *   (t, h, w) = (i / (grid_h grid_w), (i / grid_w) % grid_h, i % grid_w) + (off_t, off_h, off_w)
 * (tokens are the patches in row-major (t, h, w) order; the offsets place the sub-latent in the
 * global grid, 0 for coordinates local to the sub-latent).  head_dim is cut into three parts of
 * even sizes split[0] + split[1] + split[2] = head_dim, rotated by the t, h and w coordinate in
 * turn.  Inside a part of size p, elements (2 j, 2 j + 1) form pair j, turned by the angle
 *   pos * base^(-2 j / p):    (a, b) <- (a cos - b sin, a sin + b cos).
 * x: binary32 [n, heads, head_dim].  Returns -1 if the split is not even / does not add up.
 */
int lpo_rope3d(float *x, int64_t n, int32_t heads, int32_t head_dim, const int32_t grid[3], const int32_t offset[3],
               const int32_t split[3], double base)
{
    if (split[0] + split[1] + split[2] != head_dim) return -1;
    for (int a = 0; a < 3; ++a) if (split[a] < 0 || split[a] % 2 != 0) return -1;
    if ((int64_t)grid[0] * grid[1] * grid[2] != n) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const int64_t pos[3] = {i / ((int64_t)grid[1] * grid[2]) + offset[0], (i / grid[2]) % grid[1] + offset[1],
                                i % grid[2] + offset[2]};
        for (int32_t h = 0; h < heads; ++h) {
            float *row = x + (i * heads + h) * head_dim;
            int32_t d0 = 0;
            for (int a = 0; a < 3; ++a) {
                const int32_t p = split[a];
                for (int32_t j = 0; j < p / 2; ++j) {
                    const double angle = (double)pos[a] * pow(base, -2.0 * (double)j / (double)p);
                    const double c = cos(angle), s = sin(angle);
                    const double u = (double)row[d0 + 2 * j], v = (double)row[d0 + 2 * j + 1];
                    row[d0 + 2 * j] = (float)(u * c - v * s);
                    row[d0 + 2 * j + 1] = (float)(u * s + v * c);
                }
                d0 += p;
            }
        }
    }
    return 0;
}
