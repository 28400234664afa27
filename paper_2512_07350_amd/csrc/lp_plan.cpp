// Host part of the library: rotation schedule, partition plan, status strings.
#include <cmath>
#include <cstdlib>
#include <new>

#include "lp_internal.h"

namespace {
thread_local int g_last_hip_error = 0;
}

namespace lp {
void set_last_hip_error(int err) { g_last_hip_error = err; }
}  // namespace lp

extern "C" {

// Sec. 3.2, Eq. 3.
int lp_rotation_dim(int64_t step_1based) {
    if (step_1based < 1) return LP_ERR_INVALID_ARG;
    return static_cast<int>((step_1based - 1) % 3);
}

// Sec. 3.3, Eq. 7-9; Sec. 3.4, Eq. 11.
int lp_plan_create(const lp_config *cfg, int32_t dim, lp_plan **out) {
    if (out == nullptr) return LP_ERR_INVALID_ARG;
    *out = nullptr;
    if (cfg == nullptr || dim < 0 || dim > 2) return LP_ERR_INVALID_ARG;
    if (cfg->K < 1 || cfg->K > LP_MAX_PARTS) return LP_ERR_SHAPE;
    const int32_t ext[3] = {cfg->T, cfg->H, cfg->W};
    const int32_t pat[3] = {cfg->pT, cfg->pH, cfg->pW};
    if (cfg->C < 1) return LP_ERR_SHAPE;
    for (int d = 0; d < 3; ++d) {
        if (ext[d] < 1 || pat[d] < 1) return LP_ERR_SHAPE;
        if (ext[d] % pat[d] != 0) return LP_ERR_SHAPE;
    }
    const int64_t latent_elems = int64_t(cfg->C) * cfg->T * cfg->H * cfg->W;
    if (latent_elems >= (int64_t(1) << 40)) return LP_ERR_UNSUPPORTED;

    const int32_t K = cfg->K;
    const int32_t p = pat[dim];
    const int32_t N = ext[dim] / p;
    const int32_t L = (N + K - 1) / K;
    int64_t O;
    if (cfg->overlap_patches >= 0) {
        O = cfg->overlap_patches;
    } else {
        const double r = cfg->overlap_ratio;
        if (!(r >= 0.0) || r > double(K - 1)) return LP_ERR_SHAPE;   // Sec. 3.3: r in [0, K-1]
        O = static_cast<int64_t>(std::floor(double(L) * r));
    }
    if (O > int64_t(L) * (K - 1)) return LP_ERR_SHAPE;                // the same bound, for O given directly

    lp_plan *pl = new (std::nothrow) lp_plan();
    if (pl == nullptr) return LP_ERR_NOMEM;
    pl->cfg = *cfg;
    pl->dim = dim;
    pl->K = K;
    pl->N = N;
    pl->L = L;
    pl->O = static_cast<int32_t>(O);
    pl->extent = ext[dim];
    pl->inner = 1;
    for (int d = dim + 1; d < 3; ++d) pl->inner *= ext[d];
    pl->outer = cfg->C;
    for (int d = 0; d < dim; ++d) pl->outer *= ext[d];
    pl->latent_elems = latent_elems;

    int64_t offset = 0;
    for (int32_t k = 0; k < K; ++k) {
        lp_part_info &q = pl->part[k];
        const int64_t core_begin = int64_t(k) * L;              // alpha_k with k counted from 0
        const int64_t core_end = core_begin + L;
        int64_t lo = core_begin - O;
        int64_t hi = core_end + O;
        if (lo < 0) lo = 0;
        if (hi > N) hi = N;
        if (lo > hi) lo = hi;                                    // nothing left of [0, N): empty
        q.alpha = int32_t(core_begin);
        q.beta = int32_t(core_end);
        q.alpha_ext = int32_t(lo);
        q.beta_ext = int32_t(hi);
        q.s = int32_t(lo * p);
        q.e = int32_t(hi * p);
        q.len = q.e - q.s;
        q.delta_start = int32_t((core_begin - lo) * p);
        q.delta_end = int32_t((hi - core_end) * p);
        q.shape[0] = cfg->C;
        q.n_tokens = 1;
        for (int d = 0; d < 3; ++d) {
            q.shape[1 + d] = (d == dim) ? q.len : ext[d];
            q.n_tokens *= q.shape[1 + d] / pat[d];
        }
        q.n_elems = pl->outer * q.len * pl->inner;
        q.elem_offset = offset;
        offset += q.n_elems;
    }
    pl->total_elems = offset;
    *out = pl;
    return LP_OK;
}

void lp_plan_destroy(lp_plan *plan) { delete plan; }

int32_t lp_plan_num_parts(const lp_plan *plan) { return plan ? plan->K : LP_ERR_INVALID_ARG; }
int32_t lp_plan_dim(const lp_plan *plan) { return plan ? plan->dim : LP_ERR_INVALID_ARG; }
int64_t lp_plan_total_elems(const lp_plan *plan) { return plan ? plan->total_elems : LP_ERR_INVALID_ARG; }
int64_t lp_plan_latent_elems(const lp_plan *plan) { return plan ? plan->latent_elems : LP_ERR_INVALID_ARG; }

int lp_plan_query(const lp_plan *plan, int32_t k, lp_part_info *out) {
    if (plan == nullptr || out == nullptr || k < 0 || k >= plan->K) return LP_ERR_INVALID_ARG;
    *out = plan->part[k];
    return LP_OK;
}

const char *lp_strerror(int status) {
    switch (status) {
        case LP_OK: return "ok";
        case LP_ERR_INVALID_ARG: return "invalid argument";
        case LP_ERR_SHAPE: return "problem statement outside what the method defines (patch must divide extent, 1 <= K <= 64, r in [0, K-1])";
        case LP_ERR_UNSUPPORTED: return "unsupported size or head_dim";
        case LP_ERR_HIP: return "HIP call failed (see lp_last_hip_error)";
        case LP_ERR_NOMEM: return "host allocation failed";
        case LP_ERR_LIMIT: return "request exceeds the fixed scratch of the non-allocating entry point";
        default: return "unknown status";
    }
}

int lp_last_hip_error(void) { return g_last_hip_error; }

const char *lp_version(void) { return "lp-mi355x 0.2 (gfx950)"; }

}  // extern "C"
