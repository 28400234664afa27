// lp_attention: non-causal multi-head self-attention over the patch tokens of one
// sub-latent (supplement, proof of Theorem 1, step 3: inside a sub-latent the DiT
// blocks attend globally over all of its positions), as a flash-style kernel for
// gfx950: bf16 MFMA 32x32x16 for both products, binary32 online softmax, K and
// V^T tiles staged through LDS.
//
// Work decomposition.  One workgroup = 4 wavefronts = 256 query rows of one
// head; each wavefront owns 64 query rows (two 32-column MFMA blocks) and walks
// all keys in tiles of 64.  Per tile it forms the TRANSPOSED scores
//     S^T[key, query] = K_tile . Q^T        (A = K rows from LDS, B = Q in registers)
// so that in the MFMA accumulator layout a lane holds 16 scores of ONE query:
// row maxima and row sums are in-lane reductions plus one exchange between the
// two half-waves, the rescale factor of the running output is a per-lane scalar,
// and the bf16 probabilities are already laid out as the B operand of
//     O^T[d, query] += V^T_tile . P^T       (A = V^T rows from LDS).
// The key order inside a 32-key block is permuted (bits 2 and 3 of the MFMA row
// index swapped when K rows are read) so that the 8 probabilities a lane feeds
// to one MFMA belong to 8 consecutive keys, which makes the V^T operand a single
// 16-byte LDS read.  V is transposed on its way from global memory into LDS.
#include <hip/hip_runtime.h>

#include "lp_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kQPerWave = 64;                 // two MFMA column blocks of 32 queries
constexpr int kBM = kWaves * kQPerWave;       // query rows per workgroup
constexpr int kBN = 64;                       // keys per tile
constexpr int kPad = 8;                       // bf16 elements of row padding in LDS (16 bytes)
constexpr float kRescaleThreshold = 8.0f;     // log2 units the running max may lag behind

template <int D>
struct Smem {
    static constexpr int kRowK = D + kPad;            // K tile row (one key), in bf16
    static constexpr int kRowV = kBN + kPad;          // V^T tile row (one d), in bf16
    static constexpr int kTileK = kBN * kRowK;
    static constexpr int kTileV = D * kRowV;
    static constexpr int kBytes = 2 * (kTileK + kTileV) * 2;   // double buffered
};

union Pack16 {
    uint4 u;
    bf16x8 v;
};

__device__ __forceinline__ float half_swap(float x) {
    // value held by the lane 32 away (the other half-wave)
    return __shfl_xor(x, 32, 64);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

template <int D>
__global__ __launch_bounds__(kThreads, 1) void attention_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
    __bf16 *__restrict__ o, int n, int heads, int64_t stride_tok, int64_t stride_head,
    float scale_log2e, int n_qtiles) {
    using S = Smem<D>;
    constexpr int KS = D / 16;        // MFMA steps along d for S^T
    constexpr int MB = D / 32;        // 32-row blocks of O^T
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __bf16 *smem = reinterpret_cast<__bf16 *>(smem_raw);
    // layout: K tile 0, K tile 1, V^T tile 0, V^T tile 1

    // Workgroup -> (head, query tile).  Consecutive workgroup ids are dealt round
    // robin to the 8 XCDs; remap so each XCD works on a contiguous range of
    // (head, tile) pairs and the K/V of a head stay in one XCD's L2.
    const uint32_t n_wg = gridDim.x;
    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b % 8, slot = b / 8;
    const uint32_t base = n_wg / 8, rem = n_wg % 8;
    const uint32_t logical = xcd * base + (xcd < rem ? xcd : rem) + slot;
    const int head = logical / n_qtiles;
    const int qtile = logical % n_qtiles;

    const int tid = threadIdx.x;
    const int wave = tid / 64;
    const int lane = tid % 64;
    const int col = lane % 32;        // MFMA column (query) / A-operand row
    const int half = lane / 32;

    const int64_t head_off = int64_t(head) * stride_head;
    const __bf16 *qh = q + head_off;
    const __bf16 *kh = k + head_off;
    const __bf16 *vh = v + head_off;
    __bf16 *oh = o + head_off;

    // ---- Q^T operands: lane holds, for query `col` of block nb, d = 16*kk + 8*half .. +7
    const int q0 = qtile * kBM + wave * kQPerWave;
    bf16x8 qreg[2][KS];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int qi = q0 + nb * 32 + col;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            Pack16 t;
            t.u = make_uint4(0, 0, 0, 0);
            if (qi < n) t.u = *reinterpret_cast<const uint4 *>(qh + int64_t(qi) * stride_tok + kk * 16 + half * 8);
            qreg[nb][kk] = t.v;
        }
    }

    f32x16 acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.0f;
    float m_run[2] = {-INFINITY, -INFINITY};   // running max, raw score units
    float l_run[2] = {0.0f, 0.0f};             // this lane's share of the running sum

    // ---- tile loader: global -> registers -> LDS
    constexpr int kKChunks = kBN * (D / 8) / kThreads;    // 16-byte chunks of K per thread
    constexpr int kVUnits = (kBN / 4) * (D / 8);          // (4 keys x 8 d) units of V per tile
    uint4 kst[kKChunks];
    uint4 vst[4];
    const int v_kg = tid % 16;        // key group (4 keys)
    const int v_dc = tid / 16;        // d chunk (8 d)

    auto load_tile = [&](int key0) {
#pragma unroll
        for (int c = 0; c < kKChunks; ++c) {
            const int id = tid + c * kThreads;
            const int row = id / (D / 8), cc = id % (D / 8);
            const int key = key0 + row;
            kst[c] = make_uint4(0, 0, 0, 0);
            if (key < n) kst[c] = *reinterpret_cast<const uint4 *>(kh + int64_t(key) * stride_tok + cc * 8);
        }
        if (tid < kVUnits) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int key = key0 + v_kg * 4 + j;
                vst[j] = make_uint4(0, 0, 0, 0);
                if (key < n) vst[j] = *reinterpret_cast<const uint4 *>(vh + int64_t(key) * stride_tok + v_dc * 8);
            }
        }
    };
    auto store_tile = [&](int buf) {
        __bf16 *ksb = smem + buf * S::kTileK;
#pragma unroll
        for (int c = 0; c < kKChunks; ++c) {
            const int id = tid + c * kThreads;
            const int row = id / (D / 8), cc = id % (D / 8);
            *reinterpret_cast<uint4 *>(ksb + row * S::kRowK + cc * 8) = kst[c];
        }
        if (tid < kVUnits) {
            __bf16 *vtb = smem + 2 * S::kTileK + buf * S::kTileV;
            const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&vst[0]);
            const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&vst[1]);
            const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&vst[2]);
            const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&vst[3]);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                // dword w of a row holds d = 2w (low half) and 2w+1 (high half)
                uint2 even, odd;
                even.x = (w0[w] & 0xffffu) | (w1[w] << 16);
                even.y = (w2[w] & 0xffffu) | (w3[w] << 16);
                odd.x = (w0[w] >> 16) | (w1[w] & 0xffff0000u);
                odd.y = (w2[w] >> 16) | (w3[w] & 0xffff0000u);
                const int drow = v_dc * 8 + 2 * w;
                *reinterpret_cast<uint2 *>(vtb + drow * S::kRowV + v_kg * 4) = even;
                *reinterpret_cast<uint2 *>(vtb + (drow + 1) * S::kRowV + v_kg * 4) = odd;
            }
        }
    };

    const int n_tiles = (n + kBN - 1) / kBN;
    load_tile(0);
    store_tile(0);
    __syncthreads();

    // A-operand row of K this lane reads: bits 2 and 3 of `col` swapped
    const int krow = (col & 0x13) | ((col & 4) << 1) | ((col & 8) >> 1);

    for (int jt = 0; jt < n_tiles; ++jt) {
        const int buf = jt & 1;
        const int key0 = jt * kBN;
        const bool has_next = jt + 1 < n_tiles;
        if (has_next) load_tile(key0 + kBN);
        const __bf16 *ksb = smem + buf * S::kTileK;
        const __bf16 *vtb = smem + 2 * S::kTileK + buf * S::kTileV;
        const bool ragged = key0 + kBN > n;

#pragma unroll
        for (int sub = 0; sub < kBN / 32; ++sub) {
            // ---- S^T = K . Q^T for 32 keys x 64 queries
            f32x16 s[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[nb][r] = 0.0f;
            const __bf16 *krow_ptr = ksb + (sub * 32 + krow) * S::kRowK + half * 8;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(krow_ptr + kk * 16);
                s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[0][kk], s[0], 0, 0, 0);
                s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[1][kk], s[1], 0, 0, 0);
            }
            // accumulator register r of this lane is key  key0 + 32*sub + 16*(r/8) + 8*half + r%8
            if (ragged) {
                const int kbase = key0 + sub * 32 + half * 8;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kbase + 16 * (r / 8) + (r % 8);
                    if (key >= n) {
                        s[0][r] = -INFINITY;
                        s[1][r] = -INFINITY;
                    }
                }
            }
            // ---- online softmax (base 2), lazily rescaled
            bf16x8 p[2][2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                float tmax = s[nb][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, s[nb][r]);
                tmax = fmaxf(tmax, half_swap(tmax));
                const bool need = (tmax - m_run[nb]) * scale_log2e > kRescaleThreshold;
                if (__any(need)) {
                    const float m_new = fmaxf(m_run[nb], tmax);
                    const float alpha = __builtin_amdgcn_exp2f((m_run[nb] - m_new) * scale_log2e);
                    m_run[nb] = m_new;
                    l_run[nb] *= alpha;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[mb][nb][r] *= alpha;
                }
                const float mc = m_run[nb] * scale_log2e;
                float e[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(fmaf(s[nb][r], scale_log2e, -mc));
                Pack16 lo, hi;
                lo.u = make_uint4(pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3]), pack_bf16(e[4], e[5]), pack_bf16(e[6], e[7]));
                hi.u = make_uint4(pack_bf16(e[8], e[9]), pack_bf16(e[10], e[11]), pack_bf16(e[12], e[13]), pack_bf16(e[14], e[15]));
                p[nb][0] = lo.v;
                p[nb][1] = hi.v;
                float psum = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) psum += e[r];
                l_run[nb] += psum;
            }
            // ---- O^T += V^T . P^T
            const __bf16 *vrow_ptr = vtb + col * S::kRowV + sub * 32 + half * 8;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(vrow_ptr + mb * 32 * S::kRowV + ks * 16);
                    acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[0][ks], acc[mb][0], 0, 0, 0);
                    acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[1][ks], acc[mb][1], 0, 0, 0);
                }
            }
        }

        if (has_next) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- normalise and store: lane holds, for query `col` of block nb, rows
    // d = 32*mb + 8*(r/4) + 4*half + r%4 of O^T
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float l_tot = l_run[nb] + half_swap(l_run[nb]);
        const float inv = 1.0f / l_tot;
        const int qi = q0 + nb * 32 + col;
        if (qi < n) {
            __bf16 *orow = oh + int64_t(qi) * stride_tok;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint2 w;
                    w.x = pack_bf16(acc[mb][nb][4 * g + 0] * inv, acc[mb][nb][4 * g + 1] * inv);
                    w.y = pack_bf16(acc[mb][nb][4 * g + 2] * inv, acc[mb][nb][4 * g + 3] * inv);
                    *reinterpret_cast<uint2 *>(orow + mb * 32 + g * 8 + half * 4) = w;
                }
        }
    }
}

template <int D>
int launch(const void *q, const void *k, const void *v, void *o, int n, int heads, int64_t stride_tok,
           int64_t stride_head, float scale, hipStream_t stream) {
    static bool attr_set = false;   // per process; the attribute is per function
    auto kern = attention_kernel<D>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Smem<D>::kBytes);
        if (e != hipSuccess) {
            lp::set_last_hip_error(int(e));
            return LP_ERR_HIP;
        }
        attr_set = true;
    }
    const int n_qtiles = (n + kBM - 1) / kBM;
    const dim3 grid(uint32_t(n_qtiles) * uint32_t(heads));
    const float scale_log2e = scale * 1.4426950408889634f;
    return lp::launch_kernel(reinterpret_cast<const void *>(kern), grid, dim3(kThreads), Smem<D>::kBytes, stream,
                             static_cast<const __bf16 *>(q), static_cast<const __bf16 *>(k),
                             static_cast<const __bf16 *>(v), static_cast<__bf16 *>(o), n, heads, stride_tok,
                             stride_head, scale_log2e, n_qtiles);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

extern "C" int lp_attention(const void *q, const void *k, const void *v, void *o, int64_t n_tokens,
                            int32_t heads, int32_t head_dim, int64_t stride_tok, int64_t stride_head,
                            float scale, void *stream) {
    if (n_tokens < 0 || heads < 1) return LP_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return LP_ERR_UNSUPPORTED;
    if (n_tokens == 0) return LP_OK;
    if (q == nullptr || k == nullptr || v == nullptr || o == nullptr) return LP_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return LP_ERR_INVALID_ARG;
    if (stride_head < head_dim || stride_head % 8 != 0 || stride_tok % 8 != 0) return LP_ERR_INVALID_ARG;
    // rows of different (token, head) pairs must not overlap: either token-major or head-major
    const bool token_major = stride_tok >= int64_t(heads) * stride_head;
    const bool head_major = stride_head >= n_tokens * stride_tok && stride_tok >= head_dim;
    if (!token_major && !head_major) return LP_ERR_INVALID_ARG;
    if (n_tokens > (int64_t(1) << 24) || int64_t(heads) * ((n_tokens + kBM - 1) / kBM) > (int64_t(1) << 30))
        return LP_ERR_UNSUPPORTED;
    if (!(scale > 0.0f)) scale = 1.0f / sqrtf(float(head_dim));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (head_dim == 128)
        return launch<128>(q, k, v, o, int(n_tokens), heads, stride_tok, stride_head, scale, st);
    return launch<64>(q, k, v, o, int(n_tokens), heads, stride_tok, stride_head, scale, st);
}
