// lp_partition / lp_reconstruct: the latent-space halves of an LP step as
// HBM-bound gather and blend kernels for gfx950.
//
//   lp_partition    Sec. 3.3, Eq. 10   sub-latent k = z[..., s_k:e_k, ...]
//   lp_reconstruct  Sec. 3.4, Eq. 12-17   out = A / Z, weights by Eq. 12
//   lp_reconstruct_guided_step  Sec. 3.2, Eq. 4-6 around it: guidance before, sampler update after
//
// Both kernels see the latent as [outer, extent, inner] (outer = channels and
// the dims before the partition dim, inner = the dims after it) and move
// VEC-float vectors; VEC is the widest of {4, 2, 1} that every run length,
// every slice start and both base pointers are aligned to.  One thread owns
// UNROLL vectors; there is no cross-thread communication and every output
// element has exactly one writer.
#include <hip/hip_runtime.h>

#include "lp_internal.h"

namespace {

constexpr int kThreads = 256;

// floor(n / d) for 0 <= n < 2^31 as (n * magic) >> shift with a 64-bit product.
// With l = ceil(log2 d), magic = floor(2^(31+l) / d) + 1 < 2^32 and shift = 31 + l,
// magic*d = 2^shift + e with 0 < e <= 2^l, so the error term n*e/(d*2^shift) < 1/d.
struct FastDiv {
    uint32_t magic;
    uint32_t shift;
    uint32_t d;
};

FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;
    f.shift = 31 + l;
    f.magic = uint32_t(((unsigned __int128)1 << f.shift) / d + 1);
    return f;
}

__device__ __forceinline__ uint32_t fastdiv(uint32_t n, const FastDiv &f) {
    return uint32_t((uint64_t(n) * f.magic) >> f.shift);
}

template <int VEC>
struct VecT;
template <>
struct VecT<4> { using type = float4; };
template <>
struct VecT<2> { using type = float2; };
template <>
struct VecT<1> { using type = float; };

struct PartitionArgs {
    uint32_t n_vec[LP_MAX_PARTS];     // vectors in sub-latent k
    uint32_t dst_off[LP_MAX_PARTS];   // first vector of sub-latent k in the packed buffer
    uint32_t src_off[LP_MAX_PARTS];   // s_k * inner, in vectors
    FastDiv run[LP_MAX_PARTS];        // len_k * inner, in vectors (contiguous run per outer index)
    uint32_t src_stride;              // extent * inner, in vectors
};

// Eq. 10.  grid = (blocks over the largest sub-latent, K).
template <int VEC, int UNROLL>
__global__ __launch_bounds__(kThreads) void partition_kernel(const float *__restrict__ z,
                                                             float *__restrict__ subs,
                                                             const PartitionArgs a) {
    using V = typename VecT<VEC>::type;
    const int k = blockIdx.y;
    const uint32_t n_vec = a.n_vec[k];
    const uint32_t base = blockIdx.x * (kThreads * UNROLL) + threadIdx.x;
    if (blockIdx.x * (kThreads * UNROLL) >= n_vec) return;
    const FastDiv run = a.run[k];
    const V *src = reinterpret_cast<const V *>(z) + a.src_off[k];
    V *dst = reinterpret_cast<V *>(subs) + a.dst_off[k];
    if (blockIdx.x * (kThreads * UNROLL) + kThreads * UNROLL <= n_vec) {
        // whole block in range: all loads in flight before the first store
        V val[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t i = base + u * kThreads;
            const uint32_t o = fastdiv(i, run);
            const uint32_t r = i - o * run.d;
            val[u] = src[uint64_t(o) * a.src_stride + r];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) dst[base + u * kThreads] = val[u];
    } else {
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t i = base + u * kThreads;
            if (i < n_vec) {
                const uint32_t o = fastdiv(i, run);
                const uint32_t r = i - o * run.d;
                dst[i] = src[uint64_t(o) * a.src_stride + r];
            }
        }
    }
}

struct ReconstructArgs {
    int32_t s[LP_MAX_PARTS];            // Eq. 9
    int32_t e[LP_MAX_PARTS];
    int32_t len[LP_MAX_PARTS];          // l_k
    int32_t delta_start[LP_MAX_PARTS];  // Eq. 11
    int32_t delta_end[LP_MAX_PARTS];
    uint32_t off[LP_MAX_PARTS];         // first vector of prediction k
    int32_t K;
    uint32_t n_vec;                     // vectors in the latent
    uint32_t inner_vec;                 // inner / VEC (X_PER_ELEM = false), else unused
    FastDiv lat_run;                    // extent * inner, in vectors
    FastDiv inner_div;                  // inner, in vectors (X_PER_ELEM = false)
    FastDiv core_div;                   // L * p: core length in latent units (LANE_K)
    int32_t ovl;                        // O * p: overlap in latent units (LANE_K)
};

// What the guided step adds to the reconstruction (Eq. 4 before it, Eq. 6 after it).
struct GuidedArgs {
    const float *uncond;   // unconditional predictions, packed like the conditional ones
    const float *z;        // current latent
    float w;               // guidance scale
    float a, b;            // z' = a z + b pred
};

// Where the updated latent goes besides `out`: the sub-latents of the NEXT step's partition
// (Eq. 10 along the next rotating dimension), written in the same pass.
struct ScatterArgs {
    float *subs;                        // packed sub-latents of the next step; nullptr = none
    int32_t s[LP_MAX_PARTS];            // Eq. 9 of the next step's plan
    int32_t e[LP_MAX_PARTS];
    int32_t len[LP_MAX_PARTS];
    uint32_t off[LP_MAX_PARTS];         // first vector of sub-latent k
    int32_t K;
    uint32_t inner_vec;                 // inner / VEC, or 1 when the next partition dim is the vectorised one
    int32_t x_per_elem;                 // the next partition dim is the vectorised one
    FastDiv lat_run;                    // extent * inner of the next dim, in vectors
    FastDiv inner_div;                  // inner of the next dim, in vectors
};

// Eq. 12 at local position j; the cases in the order the paper gives them.
__device__ __forceinline__ float ramp_weight(int32_t j, int32_t len, int32_t ds, int32_t de) {
    if (j < ds) return __fdiv_rn(float(j), float(ds));
    if (j < len - de) return 1.0f;
    return __fdiv_rn(float(len - j), float(de));
}

// Eq. 4 on one vector: u + w (c - u), difference, product and sum each rounded.
template <int VEC>
__device__ __forceinline__ typename VecT<VEC>::type guide(const typename VecT<VEC>::type c,
                                                          const typename VecT<VEC>::type u, float w) {
    typename VecT<VEC>::type r;
    const float *cf = reinterpret_cast<const float *>(&c), *uf = reinterpret_cast<const float *>(&u);
    float *rf = reinterpret_cast<float *>(&r);
#pragma unroll
    for (int e = 0; e < VEC; ++e) rf[e] = __fadd_rn(uf[e], __fmul_rn(w, __fsub_rn(cf[e], uf[e])));
    return r;
}

// One partition's term of Eq. 15-16 for the vector at x0 (local position j0 in partition k).
template <int VEC, bool X_PER_ELEM>
__device__ __forceinline__ void blend_term(const typename VecT<VEC>::type p, int32_t j0, int32_t len, int32_t ds,
                                           int32_t de, float (&A)[VEC], float (&Z)[VEC]) {
    const float *pf = reinterpret_cast<const float *>(&p);
    if (X_PER_ELEM) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const float w = ramp_weight(j0 + c, len, ds, de);
            A[c] = __fadd_rn(A[c], __fmul_rn(w, pf[c]));   // Eq. 15: rounded product, rounded sum
            Z[c] = __fadd_rn(Z[c], w);                      // Eq. 16
        }
    } else {
        const float w = ramp_weight(j0, len, ds, de);
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            A[c] = __fadd_rn(A[c], __fmul_rn(w, pf[c]));
            Z[c] = __fadd_rn(Z[c], w);
        }
    }
}

// Eq. 13-17.  X_PER_ELEM: the partition dim is the vectorised (fastest) one, so
// each element of a vector has its own coordinate x and its own weight.
// LANE_K: the lanes of a wave sit at many different x (short inner runs), so a
// wave as a whole touches every partition.  Each lane then walks only the k
// range that can cover its x -- from s_k >= k L p - O p and e_k <= (k+1) L p + O p,
// floor((x - O p) / (L p)) <= k <= floor((x + O p) / (L p)) -- with the plan
// held in LDS; the test against s_k and e_k still decides.  Otherwise a wave
// shares one or two x and the loop over all k with scalar loads is cheaper.
// Both visit the covering partitions in ascending k, so the sums are identical.
// GUIDED: the prediction of partition k is formed on the fly as u + w (c - u) from the
// conditional (`preds`) and unconditional sets (Eq. 4), and the result is the sampler's
// update a z + b pred (Eq. 6); every operation is rounded on its own, in that order.
// `out` may be the same buffer as g.z (each element is read and then written by one thread).
// SCATTER: the updated latent is also written into every sub-latent of the next step's
// partition that contains it (Eq. 10 along the next dimension), which saves that step's
// lp_partition launch and its read of the latent.
template <int VEC, bool X_PER_ELEM, bool LANE_K, bool GUIDED, bool SCATTER>
__global__ __launch_bounds__(kThreads) void reconstruct_kernel(const float *__restrict__ preds, float *out,
                                                               const ReconstructArgs a, const GuidedArgs g,
                                                               const ScatterArgs sc) {
    using V = typename VecT<VEC>::type;
    __shared__ int32_t plan_s[LANE_K ? LP_MAX_PARTS : 1], plan_e[LANE_K ? LP_MAX_PARTS : 1],
        plan_len[LANE_K ? LP_MAX_PARTS : 1], plan_ds[LANE_K ? LP_MAX_PARTS : 1], plan_de[LANE_K ? LP_MAX_PARTS : 1];
    __shared__ uint32_t plan_off[LANE_K ? LP_MAX_PARTS : 1];
    if (LANE_K) {
        const int t = threadIdx.x;
        if (t < a.K) {
            plan_s[t] = a.s[t];
            plan_e[t] = a.e[t];
            plan_len[t] = a.len[t];
            plan_ds[t] = a.delta_start[t];
            plan_de[t] = a.delta_end[t];
            plan_off[t] = a.off[t];
        }
        __syncthreads();
    }
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= a.n_vec) return;
    const uint32_t o = fastdiv(i, a.lat_run);
    const uint32_t rem = i - o * a.lat_run.d;
    int32_t x0;       // coordinate along the partition dim of element 0 of this vector
    uint32_t r_in;    // vector offset inside one x-slab
    if (X_PER_ELEM) {
        x0 = int32_t(rem) * VEC;
        r_in = 0;
    } else {
        const uint32_t xq = fastdiv(rem, a.inner_div);
        x0 = int32_t(xq);
        r_in = rem - xq * a.inner_div.d;
    }
    float A[VEC], Z[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) { A[c] = 0.0f; Z[c] = 0.0f; }
    const V *pv = reinterpret_cast<const V *>(preds);
    const V *uv = reinterpret_cast<const V *>(g.uncond);
    if (LANE_K) {
        const int k_lo = x0 >= a.ovl ? int(fastdiv(uint32_t(x0 - a.ovl), a.core_div)) : 0;
        const int k_hi = min(a.K - 1, int(fastdiv(uint32_t(x0 + a.ovl), a.core_div)));
        for (int k = k_lo; k <= k_hi; ++k) {
            const int32_t s = plan_s[k];
            if (x0 < s || x0 >= plan_e[k]) continue;   // Eq. 14 (a vector never straddles s_k or e_k)
            const int32_t j0 = x0 - s;                  // Eq. 13
            const int32_t len = plan_len[k];
            uint64_t idx;
            if (X_PER_ELEM)
                idx = uint64_t(plan_off[k]) + (uint64_t(o) * uint32_t(len) + uint32_t(j0)) / VEC;
            else
                idx = uint64_t(plan_off[k]) + (uint64_t(o) * uint32_t(len) + uint32_t(j0)) * a.inner_vec + r_in;
            blend_term<VEC, X_PER_ELEM>(GUIDED ? guide<VEC>(pv[idx], uv[idx], g.w) : pv[idx], j0, len, plan_ds[k],
                                        plan_de[k], A, Z);
        }
    } else {
        for (int k = 0; k < a.K; ++k) {
            const int32_t s = a.s[k];
            if (x0 < s || x0 >= a.e[k]) continue;
            const int32_t j0 = x0 - s;
            const int32_t len = a.len[k];
            const uint64_t idx = uint64_t(a.off[k]) + (uint64_t(o) * uint32_t(len) + uint32_t(j0)) * a.inner_vec + r_in;
            blend_term<VEC, false>(GUIDED ? guide<VEC>(pv[idx], uv[idx], g.w) : pv[idx], j0, len, a.delta_start[k],
                                   a.delta_end[k], A, Z);
        }
    }
    V res;
    float *rf = reinterpret_cast<float *>(&res);
#pragma unroll
    for (int c = 0; c < VEC; ++c) rf[c] = (Z[c] == 1.0f) ? A[c] : __fdiv_rn(A[c], Z[c]);   // Eq. 17 (A/1 = A)
    if (GUIDED) {
        const V zv = reinterpret_cast<const V *>(g.z)[i];
        const float *zf = reinterpret_cast<const float *>(&zv);
#pragma unroll
        for (int c = 0; c < VEC; ++c) rf[c] = __fadd_rn(__fmul_rn(g.a, zf[c]), __fmul_rn(g.b, rf[c]));   // Eq. 6
    }
    reinterpret_cast<V *>(out)[i] = res;
    if (SCATTER) {
        // this vector in the [outer, extent, inner] view around the next step's partition dim
        const uint32_t o2 = fastdiv(i, sc.lat_run);
        const uint32_t rem2 = i - o2 * sc.lat_run.d;
        int32_t x2;
        uint32_t r2;
        if (sc.x_per_elem) {
            x2 = int32_t(rem2) * VEC;
            r2 = 0;
        } else {
            const uint32_t xq = fastdiv(rem2, sc.inner_div);
            x2 = int32_t(xq);
            r2 = rem2 - xq * sc.inner_div.d;
        }
        V *dst = reinterpret_cast<V *>(sc.subs);
        for (int k = 0; k < sc.K; ++k) {
            const int32_t s = sc.s[k];
            if (x2 < s || x2 >= sc.e[k]) continue;      // (a vector never straddles s_k or e_k)
            const uint64_t row = uint64_t(o2) * uint32_t(sc.len[k]) + uint32_t(x2 - s);
            dst[sc.x_per_elem ? uint64_t(sc.off[k]) + row / VEC : uint64_t(sc.off[k]) + row * sc.inner_vec + r2] = res;
        }
    }
}

// ---- Partition along the fastest dimension (inner == 1), four floats per vector.
// A sub-latent's row is then a run of only len_k floats (96-112 bytes on the 720p latent): lanes
// that write one side contiguously touch two or three partial 128-byte lines per run on the other
// side, and partition_kernel spends its time in the address path, not on bandwidth.  The kernel
// below takes R consecutive rows per workgroup and passes them through LDS: the R rows of the
// latent are one contiguous block, and so are the R rows of every sub-latent (rows are packed back
// to back), so every global access is a contiguous stream of whole lines, and the short runs are
// taken apart in LDS.  (The same staging for lp_reconstruct was built and measured slower than
// reconstruct_kernel, 21-26 us against 14.6 us on the 19.4 MB latent, and is not kept.)
constexpr uint32_t kRowsLdsBytes = 32768;   // LDS per workgroup for the rows held by the kernel below

struct RowsArgs {
    int32_t s[LP_MAX_PARTS];            // Eq. 9
    int32_t len[LP_MAX_PARTS];          // l_k
    uint32_t off[LP_MAX_PARTS];         // first float4 of sub-latent k in the packed buffer
    FastDiv len4[LP_MAX_PARTS];         // len_k / 4
    int32_t K;
    uint32_t rows;                      // outer
    uint32_t R;                         // rows per workgroup
    uint32_t w4;                        // extent / 4
};

// Eq. 10: LDS holds the R latent rows; sub-latent k's R rows leave as one contiguous block.
__global__ __launch_bounds__(kThreads) void partition_rows_kernel(const float4 *__restrict__ z, float4 *__restrict__ subs,
                                                                  const RowsArgs a) {
    extern __shared__ float4 rows_lds[];
    const uint32_t o0 = blockIdx.x * a.R;
    const uint32_t rows = min(a.R, a.rows - o0);
    const float4 *src = z + uint64_t(o0) * a.w4;
    for (uint32_t i = threadIdx.x; i < rows * a.w4; i += kThreads) rows_lds[i] = src[i];
    __syncthreads();
    for (int k = 0; k < a.K; ++k) {
        const uint32_t l4 = a.len4[k].d;
        if (a.len[k] == 0) continue;
        float4 *dst = subs + a.off[k] + uint64_t(o0) * l4;
        const uint32_t s4 = uint32_t(a.s[k]) / 4;
        for (uint32_t i = threadIdx.x; i < rows * l4; i += kThreads) {
            const uint32_t r = fastdiv(i, a.len4[k]);
            dst[i] = rows_lds[r * a.w4 + s4 + (i - r * l4)];
        }
    }
}

// Fills the arguments of partition_rows_kernel; false if this plan is not for it (the partition
// dimension is not the fastest one, vectors of four do not fit, or a latent row exceeds the LDS share).
bool make_rows_args(const lp_plan *pl, RowsArgs *a) {
    if (pl->inner != 1 || pl->extent % 4 != 0) return false;
    a->K = pl->K;
    for (int k = 0; k < pl->K; ++k) {
        const lp_part_info &q = pl->part[k];
        if (q.len % 4 != 0 || q.s % 4 != 0 || q.elem_offset % 4 != 0) return false;
        a->s[k] = q.s;
        a->len[k] = q.len;
        a->off[k] = uint32_t(q.elem_offset / 4);
        a->len4[k] = make_fastdiv(q.len ? uint32_t(q.len / 4) : 1);
    }
    const uint32_t w4 = uint32_t(pl->extent / 4);
    if (w4 * 16 > kRowsLdsBytes) return false;
    const uint32_t R = kRowsLdsBytes / (w4 * 16);
    a->rows = uint32_t(pl->latent_elems / pl->extent);
    a->R = R > 32 ? 32 : R;
    a->w4 = w4;
    return true;
}

bool aligned_to(const void *p, int bytes) { return (reinterpret_cast<uintptr_t>(p) % bytes) == 0; }

// Widest vector usable for this plan and these pointers.  Either the vector lies
// inside one coordinate of the partition dim (inner is a multiple of it), or the
// partition dim is the fastest one (inner == 1) and every slice start, slice
// length and the extent are multiples of it, so no vector straddles a boundary.
int pick_vec(const lp_plan *pl, const void *a, const void *b) {
    for (int vec = 4; vec > 1; vec /= 2) {
        if (!aligned_to(a, 4 * vec) || !aligned_to(b, 4 * vec)) continue;
        if (pl->inner % vec == 0) return vec;
        if (pl->inner != 1 || pl->extent % vec != 0) continue;
        bool ok = true;
        for (int k = 0; ok && k < pl->K; ++k) ok = pl->part[k].len % vec == 0 && pl->part[k].s % vec == 0;
        if (ok) return vec;
    }
    return 1;
}

template <int VEC>
int launch_partition(const lp_plan *pl, const float *z, float *subs, hipStream_t stream) {
    constexpr int UNROLL = 4;
    PartitionArgs a;
    uint32_t max_vec = 0;
    for (int k = 0; k < pl->K; ++k) {
        const lp_part_info &q = pl->part[k];
        a.n_vec[k] = uint32_t(q.n_elems / VEC);
        a.dst_off[k] = uint32_t(q.elem_offset / VEC);
        a.src_off[k] = uint32_t(int64_t(q.s) * pl->inner / VEC);
        const uint32_t run = uint32_t(int64_t(q.len) * pl->inner / VEC);
        a.run[k] = make_fastdiv(run ? run : 1);
        if (a.n_vec[k] > max_vec) max_vec = a.n_vec[k];
    }
    a.src_stride = uint32_t(int64_t(pl->extent) * pl->inner / VEC);
    if (max_vec == 0) return LP_OK;
    const uint32_t per_block = kThreads * UNROLL;
    dim3 grid((max_vec + per_block - 1) / per_block, pl->K);
    return lp::launch_kernel(reinterpret_cast<const void *>(&partition_kernel<VEC, UNROLL>), grid, dim3(kThreads), 0,
                             stream, z, subs, a);
}

template <int VEC, bool GUIDED, bool SCATTER>
int launch_reconstruct(const lp_plan *pl, const float *preds, float *out, const GuidedArgs g, const lp_plan *next,
                       float *next_subs, hipStream_t stream) {
    ReconstructArgs a;
    a.K = pl->K;
    for (int k = 0; k < pl->K; ++k) {
        const lp_part_info &q = pl->part[k];
        a.s[k] = q.s;
        a.e[k] = q.e;
        a.len[k] = q.len;
        a.delta_start[k] = q.delta_start;
        a.delta_end[k] = q.delta_end;
        a.off[k] = uint32_t(q.elem_offset / VEC);
    }
    a.n_vec = uint32_t(pl->latent_elems / VEC);
    a.lat_run = make_fastdiv(uint32_t(int64_t(pl->extent) * pl->inner / VEC));
    const bool x_per_elem = (pl->inner % VEC) != 0;   // pick_vec allows this only for inner == 1
    a.inner_vec = x_per_elem ? 1 : uint32_t(pl->inner / VEC);
    a.inner_div = make_fastdiv(a.inner_vec);
    const int32_t p = pl->dim == 0 ? pl->cfg.pT : pl->dim == 1 ? pl->cfg.pH : pl->cfg.pW;
    a.core_div = make_fastdiv(uint32_t(pl->L) * uint32_t(p));
    a.ovl = pl->O * p;
    // a wave of 64 vectors sits on at least 64 / inner_vec different x
    const bool lane_k = x_per_elem || a.inner_vec < 16;
    dim3 grid((a.n_vec + kThreads - 1) / kThreads);
    ScatterArgs sc{};
    if (SCATTER) {
        sc.subs = next_subs;
        sc.K = next->K;
        for (int k = 0; k < next->K; ++k) {
            const lp_part_info &q = next->part[k];
            sc.s[k] = q.s;
            sc.e[k] = q.e;
            sc.len[k] = q.len;
            sc.off[k] = uint32_t(q.elem_offset / VEC);
        }
        sc.x_per_elem = (next->inner % VEC) != 0;
        sc.inner_vec = sc.x_per_elem ? 1 : uint32_t(next->inner / VEC);
        sc.lat_run = make_fastdiv(uint32_t(int64_t(next->extent) * next->inner / VEC));
        sc.inner_div = make_fastdiv(sc.inner_vec);
    }
    const void *fn = x_per_elem ? reinterpret_cast<const void *>(&reconstruct_kernel<VEC, true, true, GUIDED, SCATTER>)
                     : lane_k   ? reinterpret_cast<const void *>(&reconstruct_kernel<VEC, false, true, GUIDED, SCATTER>)
                                : reinterpret_cast<const void *>(&reconstruct_kernel<VEC, false, false, GUIDED, SCATTER>);
    return lp::launch_kernel(fn, grid, dim3(kThreads), 0, stream, preds, out, a, g, sc);
}

// The kernels index with 32-bit vector counts; 2^31 vectors is far beyond any latent.
bool fits_32bit(const lp_plan *pl) {
    return pl->total_elems < (int64_t(1) << 31) && pl->latent_elems < (int64_t(1) << 31);
}

}  // namespace

extern "C" {

int lp_partition(const lp_plan *plan, const float *z, float *subs_packed, void *stream) {
    if (plan == nullptr || z == nullptr || subs_packed == nullptr) return LP_ERR_INVALID_ARG;
    if (!aligned_to(z, 4) || !aligned_to(subs_packed, 4) || z == subs_packed) return LP_ERR_INVALID_ARG;
    if (!fits_32bit(plan)) return LP_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int vec = pick_vec(plan, z, subs_packed);
    RowsArgs rows;
    if (vec == 4 && make_rows_args(plan, &rows))
        return lp::launch_kernel(reinterpret_cast<const void *>(&partition_rows_kernel), dim3((rows.rows + rows.R - 1) / rows.R),
                                 dim3(kThreads), rows.R * rows.w4 * 16, st, reinterpret_cast<const float4 *>(z),
                                 reinterpret_cast<float4 *>(subs_packed), rows);
    switch (vec) {
        case 4: return launch_partition<4>(plan, z, subs_packed, st);
        case 2: return launch_partition<2>(plan, z, subs_packed, st);
        default: return launch_partition<1>(plan, z, subs_packed, st);
    }
}

int lp_reconstruct(const lp_plan *plan, const float *preds_packed, float *out, void *stream) {
    if (plan == nullptr || preds_packed == nullptr || out == nullptr) return LP_ERR_INVALID_ARG;
    if (!aligned_to(preds_packed, 4) || !aligned_to(out, 4) || out == preds_packed) return LP_ERR_INVALID_ARG;
    if (!fits_32bit(plan)) return LP_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const GuidedArgs none{};
    switch (pick_vec(plan, preds_packed, out)) {
        case 4: return launch_reconstruct<4, false, false>(plan, preds_packed, out, none, nullptr, nullptr, st);
        case 2: return launch_reconstruct<2, false, false>(plan, preds_packed, out, none, nullptr, nullptr, st);
        default: return launch_reconstruct<1, false, false>(plan, preds_packed, out, none, nullptr, nullptr, st);
    }
}

int lp_reconstruct_guided_step(const lp_plan *plan, const float *cond_packed, const float *uncond_packed, float guidance,
                               const float *z, float coef_z, float coef_pred, float *out, void *stream) {
    if (plan == nullptr || cond_packed == nullptr || uncond_packed == nullptr || z == nullptr || out == nullptr)
        return LP_ERR_INVALID_ARG;
    if (!aligned_to(cond_packed, 4) || !aligned_to(uncond_packed, 4) || !aligned_to(z, 4) || !aligned_to(out, 4))
        return LP_ERR_INVALID_ARG;
    if (out == cond_packed || out == uncond_packed) return LP_ERR_INVALID_ARG;   // only z may be updated in place
    if (!fits_32bit(plan)) return LP_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    GuidedArgs g;
    g.uncond = uncond_packed;
    g.z = z;
    g.w = guidance;
    g.a = coef_z;
    g.b = coef_pred;
    const int v1 = pick_vec(plan, cond_packed, out), v2 = pick_vec(plan, uncond_packed, z);
    switch (v1 < v2 ? v1 : v2) {
        case 4: return launch_reconstruct<4, true, false>(plan, cond_packed, out, g, nullptr, nullptr, st);
        case 2: return launch_reconstruct<2, true, false>(plan, cond_packed, out, g, nullptr, nullptr, st);
        default: return launch_reconstruct<1, true, false>(plan, cond_packed, out, g, nullptr, nullptr, st);
    }
}

int lp_reconstruct_guided_step_partition(const lp_plan *plan, const float *cond_packed, const float *uncond_packed,
                                         float guidance, const float *z, float coef_z, float coef_pred, float *out,
                                         const lp_plan *next_plan, float *next_subs_packed, void *stream) {
    if (plan == nullptr || cond_packed == nullptr || uncond_packed == nullptr || z == nullptr || out == nullptr ||
        next_plan == nullptr || next_subs_packed == nullptr)
        return LP_ERR_INVALID_ARG;
    if (!aligned_to(cond_packed, 4) || !aligned_to(uncond_packed, 4) || !aligned_to(z, 4) || !aligned_to(out, 4) ||
        !aligned_to(next_subs_packed, 4))
        return LP_ERR_INVALID_ARG;
    if (out == cond_packed || out == uncond_packed || next_subs_packed == cond_packed ||
        next_subs_packed == uncond_packed || next_subs_packed == z || next_subs_packed == out)
        return LP_ERR_INVALID_ARG;
    const lp_config &c0 = plan->cfg, &c1 = next_plan->cfg;
    if (c0.C != c1.C || c0.T != c1.T || c0.H != c1.H || c0.W != c1.W) return LP_ERR_INVALID_ARG;   // one latent
    if (!fits_32bit(plan) || !fits_32bit(next_plan)) return LP_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    GuidedArgs g;
    g.uncond = uncond_packed;
    g.z = z;
    g.w = guidance;
    g.a = coef_z;
    g.b = coef_pred;
    int vec = pick_vec(plan, cond_packed, out);
    const int v2 = pick_vec(plan, uncond_packed, z), v3 = pick_vec(next_plan, next_subs_packed, out);
    vec = v2 < vec ? v2 : vec;
    vec = v3 < vec ? v3 : vec;
    switch (vec) {
        case 4: return launch_reconstruct<4, true, true>(plan, cond_packed, out, g, next_plan, next_subs_packed, st);
        case 2: return launch_reconstruct<2, true, true>(plan, cond_packed, out, g, next_plan, next_subs_packed, st);
        default: return launch_reconstruct<1, true, true>(plan, cond_packed, out, g, next_plan, next_subs_packed, st);
    }
}

}  // extern "C"
