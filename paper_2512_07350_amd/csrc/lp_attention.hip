// lp_attention: non-causal multi-head self-attention over the patch tokens of one
// sub-latent (supplement, proof of Theorem 1, step 3: inside a sub-latent the DiT
// blocks attend globally over all of its positions), as a flash-style kernel for
// gfx950: bf16 MFMA 32x32x16 for both products, binary32 online softmax, K and V
// tiles streamed global -> LDS without passing through registers.
//
// Work decomposition.  One workgroup = 4 wavefronts = 256 query rows of one head;
// each wavefront owns 64 query rows (two 32-column MFMA blocks) and walks all keys
// in rounds of 32.  Per round it forms the TRANSPOSED scores
//     S^T[key, query] = K . Q^T            (A = K rows from LDS, B = Q in registers)
// so that in the MFMA accumulator layout a lane holds 16 scores of ONE query: the
// row maximum and row sum are in-lane reductions, the rescale factor of the running
// output is a per-lane scalar, and the bf16 probabilities are already laid out as
// the B operand of
//     O^T[d, query] += V^T . P^T           (A = V^T, read transposed from LDS).
//
// Details that matter for speed:
//  * Q is multiplied by scale*log2(e) once and re-rounded to bf16, and the score
//    accumulators start at -m (m = running maximum, log2 units), so a probability
//    is a bare exp2 of the accumulator.
//  * The running maximum is only raised when some score exceeds it by more than
//    kRescaleThreshold; probabilities then stay below 2^kRescaleThreshold and the
//    output accumulators are rescaled in a rarely taken, wave-uniform branch.
//  * The score product of round r+1 is issued before the softmax of round r, so
//    MFMA and VALU work of one wavefront overlap.
//  * The key order inside a 32-key round is permuted (bits 2 and 3 of the MFMA row
//    index swapped when K rows are read) so that the 8 probabilities a lane feeds
//    to one MFMA belong to 8 consecutive keys; V^T operands then come from two
//    ds_read_b64_tr_b16 (transposing LDS reads) of the row-major V tile.
//  * K/V tiles go global -> LDS with global_load_lds_dwordx4 (kStages tiles
//    resident), with XOR swizzles of the 16-byte granules chosen so that the K
//    reads (ds_read_b128) and the V reads are free of bank conflicts.
#include <hip/hip_runtime.h>

#include "lp_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

#define LP_LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int kBM = 256;                      // query rows per workgroup
// A wavefront owns NB blocks of 32 query rows; the workgroup has kBM / (32 NB) wavefronts.
constexpr int waves_of(int nb) { return kBM / (32 * nb); }
constexpr int kBlocksPerWave = 1;             // NB used by lp_attention
constexpr int kBN = 64;                       // keys per LDS tile (two rounds of 32)
constexpr int kStages = 3;                    // LDS tiles resident (>= 3)
constexpr float kRescaleThreshold = 8.0f;     // log2 units the running max may lag behind

template <int D, int NB>
struct Tile {
    static constexpr int kWaves = waves_of(NB);
    static constexpr int kRowBytes = D * 2;
    static constexpr int kGran = kRowBytes / 16;            // 16-byte granules per row
    static constexpr int kTileBytes = kBN * kRowBytes;      // one K or one V tile
    static constexpr int kStageBytes = 2 * kTileBytes;      // K tile then V tile
    static constexpr int kBytes = kStages * kStageBytes;
    static constexpr int kRowsPerInstr = 1024 / kRowBytes;  // rows one wave-wide 16-byte load covers
    static constexpr int kInstrPerTile = kBN / kRowsPerInstr;
    static constexpr int kLoadsPerWave = 2 * kInstrPerTile / kWaves;   // K and V, per tile
    // granule XOR masks; reader and writer use the same functions
    __device__ static int swz_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
    __device__ static int swz_v(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row & 3) >> 1); }
};

union Pack16 {
    uint4 u;
    bf16x8 v;
    bf16x4 h[2];
    bf16x2 p[4];
};

__device__ __forceinline__ float other_half(float x) {
    return __shfl_xor(x, 32, 64);   // value held by the lane 32 away
}

__device__ __forceinline__ bf16x2 to_bf16x2(float lo, float hi) {
    f32x2 f = {lo, hi};
    return __builtin_convertvector(f, bf16x2);
}

// Wait until at most `pending` of this wave's global->LDS loads are still in flight.
template <int PENDING>
__device__ __forceinline__ void wait_tile_loads() {
    static_assert(PENDING >= 0 && PENDING < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
}

// Per-lane constants of the tile traffic.
struct LaneCtx {
    const __bf16 *kh, *vh;   // K and V of this head
    int64_t stride_tok;
    int n, n_tiles, n_rounds;
    int wave;                // wave index inside the workgroup (wave-uniform)
    int half;                // lane / 32
    int krow;                // K row this lane feeds to the MFMA: lane%32 with bits 2 and 3 swapped
    int vj, vg;              // lane%16 and (lane/16)%2 for the transposing V reads
    int ld_row, ld_gran;     // row and physical granule this lane fills in a 1024-byte load block
};

// global -> LDS loads of one K/V tile.  One wave-wide instruction moves 1024 bytes
// (lane L fills bytes 16L..16L+15 of the block); waves take blocks round robin.
template <int D, int NB>
__device__ __forceinline__ void issue_tile(unsigned char *smem, const LaneCtx &c, int tile) {
    using T = Tile<D, NB>;
    unsigned char *stage = smem + (tile % kStages) * T::kStageBytes;
    const int key0 = tile * kBN;
#pragma unroll
    for (int i = 0; i < T::kInstrPerTile / T::kWaves; ++i) {
        const int instr = c.wave + i * T::kWaves;
        const int row = instr * T::kRowsPerInstr + c.ld_row;       // row inside the tile
        int key = key0 + row;
        key = key < c.n ? key : c.n - 1;                            // rows past the end repeat the last key
        const int64_t goff = int64_t(key) * c.stride_tok;
        // (operands go through plainly typed locals: the builtin is checked where it is written)
        const int gk = c.ld_gran ^ T::swz_k(row), gv = c.ld_gran ^ T::swz_v(row);
        const __bf16 *src_k = c.kh + goff + 8 * gk;
        const __bf16 *src_v = c.vh + goff + 8 * gv;
        unsigned char *dst_k = stage + instr * 1024;
        unsigned char *dst_v = dst_k + T::kTileBytes;
        __builtin_amdgcn_global_load_lds(src_k, LP_LDS_PTR(void, dst_k), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(src_v, LP_LDS_PTR(void, dst_v), 16, 0, 0);
    }
}

// S^T of round r (32 keys) for both query blocks.
template <int D, int NB>
__device__ __forceinline__ void score_round(const unsigned char *smem, const LaneCtx &c, int r,
                                            const bf16x8 (&qreg)[NB][D / 16], f32x16 (&s)[NB]) {
    using T = Tile<D, NB>;
    const int tile = r / 2, sub = r % 2;
    const unsigned char *kt = smem + (tile % kStages) * T::kStageBytes;
    const int row = sub * 32 + c.krow;
    const unsigned char *rp = kt + row * T::kRowBytes;
    const int sw = T::swz_k(row);
    f32x16 zero16;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero16[i] = 0.0f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
        const bf16x8 a = *LP_LDS_PTR(const bf16x8, rp + 16 * ((2 * kk + c.half) ^ sw));
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[nb][kk], kk == 0 ? zero16 : s[nb], 0, 0, 0);
    }
}

// Keys past the end get score -inf.  Accumulator register i of a lane is key
// 32*r + 16*(i/8) + 8*half + i%8.
template <int NB>
__device__ __forceinline__ void mask_round(const LaneCtx &c, int r, f32x16 (&s)[NB]) {
    const int kbase = r * 32 + c.half * 8;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (kbase + 16 * (i / 8) + (i % 8) >= c.n) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) s[nb][i] = -INFINITY;
        }
    }
}

// O^T += V^T . P^T for round r.  Inside a group of 16 lanes, lane j supplies the 8-byte
// chunk (row j/4, columns 4*(j%4)..+3) to the transposing read and receives column j of
// that 4x16 block, i.e. 4 consecutive keys of one d.
template <int D, int NB>
__device__ __forceinline__ void pv_round(const unsigned char *smem, const LaneCtx &c, int r,
                                         const bf16x8 (&p)[NB][2], f32x16 (&acc)[D / 32][NB]) {
    using T = Tile<D, NB>;
    const int tile = r / 2, sub = r % 2;
    const unsigned char *vt = smem + (tile % kStages) * T::kStageBytes + T::kTileBytes;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int row0 = sub * 32 + ks * 16 + c.half * 8 + c.vj / 4;      // + 4 for the second read
        const unsigned char *r0 = vt + row0 * T::kRowBytes + 8 * ((c.vj % 4) % 2);
        const unsigned char *r1 = r0 + 4 * T::kRowBytes;
        const int sw0 = T::swz_v(row0), sw1 = T::swz_v(row0 + 4);
#pragma unroll
        for (int mb = 0; mb < D / 32; ++mb) {
            const int gran = 4 * mb + 2 * c.vg + (c.vj % 4) / 2;
            Pack16 a;
            a.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LP_LDS_PTR(bf16x4, r0 + 16 * (gran ^ sw0)));
            a.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LP_LDS_PTR(bf16x4, r1 + 16 * (gran ^ sw1)));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, p[nb][ks], acc[mb][nb], 0, 0, 0);
        }
    }
}

__device__ __forceinline__ float max16(const f32x16 &s) {
    float t = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) t = fmaxf(t, s[i]);
    return t;
}

// One round: issue S^T of round r+1 (MFMA), then softmax of round r (VALU), then PV of
// round r (MFMA).  s_cur / s_nxt swap roles from round to round.
template <int D, int NB>
__device__ __forceinline__ void round_body(unsigned char *smem, const LaneCtx &c, int r,
                                           const bf16x8 (&qreg)[NB][D / 16], f32x16 (&s_cur)[NB],
                                           f32x16 (&s_nxt)[NB], f32x16 (&acc)[D / 32][NB],
                                           float (&m_run)[NB], float (&l_run)[NB]) {
    using T = Tile<D, NB>;
    if (r + 1 < c.n_rounds) {
        if ((r & 1) == 1) {
            // The next round opens tile t.  Tiles t .. t+kStages-3 are in flight; t must
            // have landed.  After the barrier every wave has left tile t-2, whose stage
            // then takes tile t+kStages-2.  (Tile t-1 still feeds this round's V reads.)
            const int t = (r + 1) / 2;
            if (t + kStages - 3 < c.n_tiles)
                wait_tile_loads<(kStages - 3) * T::kLoadsPerWave>();
            else
                wait_tile_loads<0>();          // near the end fewer tiles are in flight
            __syncthreads();
            if (t + kStages - 2 < c.n_tiles) issue_tile<D, NB>(smem, c, t + kStages - 2);
        }
        score_round<D, NB>(smem, c, r + 1, qreg, s_nxt);
    }
    if ((r + 1) * 32 > c.n) mask_round<NB>(c, r, s_cur);

    // ---- lazy running maximum: only act when some score is far above it
    bool raise = false;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) raise = raise || (max16(s_cur[nb]) - m_run[nb] > kRescaleThreshold);
    if (__any(raise)) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float tmax = max16(s_cur[nb]);
            tmax = fmaxf(tmax, other_half(tmax));
            const float m_new = fmaxf(m_run[nb], tmax);      // the maximum never goes down
            const float alpha = __builtin_amdgcn_exp2f(m_run[nb] - m_new);
            m_run[nb] = m_new;
            l_run[nb] *= alpha;
#pragma unroll
            for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mb][nb][i] *= alpha;
        }
    }

    // ---- probabilities, rounded to bf16; the row sum adds the rounded values
    bf16x8 p[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        Pack16 lo, hi;
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        const float m = m_run[nb];
        float l = l_run[nb];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lo.p[e] = to_bf16x2(__builtin_amdgcn_exp2f(s_cur[nb][2 * e] - m), __builtin_amdgcn_exp2f(s_cur[nb][2 * e + 1] - m));
            hi.p[e] = to_bf16x2(__builtin_amdgcn_exp2f(s_cur[nb][8 + 2 * e] - m), __builtin_amdgcn_exp2f(s_cur[nb][8 + 2 * e + 1] - m));
            l = __builtin_amdgcn_fdot2_f32_bf16(lo.p[e], ones, l, false);
            l = __builtin_amdgcn_fdot2_f32_bf16(hi.p[e], ones, l, false);
        }
        l_run[nb] = l;
        p[nb][0] = lo.v;
        p[nb][1] = hi.v;
    }
    pv_round<D, NB>(smem, c, r, p, acc);
}

template <int D, int NB>
__global__ __launch_bounds__(waves_of(NB) * 64) void attention_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
    __bf16 *__restrict__ o, int n, int heads, int64_t stride_tok, int64_t stride_head,
    float scale_log2e, int n_qtiles) {
    using T = Tile<D, NB>;
    constexpr int KS = D / 16;        // MFMA steps along d for S^T
    constexpr int MB = D / 32;        // 32-row blocks of O^T
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

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
    const int lane = tid % 64;
    const int col = lane % 32;        // MFMA column (query) / A-operand row
    const int64_t head_off = int64_t(head) * stride_head;
    const __bf16 *qh = q + head_off;
    __bf16 *oh = o + head_off;

    LaneCtx c;
    c.kh = k + head_off;
    c.vh = v + head_off;
    c.stride_tok = stride_tok;
    c.n = n;
    c.n_tiles = (n + kBN - 1) / kBN;
    c.n_rounds = (n + 31) / 32;
    c.wave = __builtin_amdgcn_readfirstlane(tid / 64);
    c.half = lane / 32;
    c.krow = (col & 0x13) | ((col & 4) << 1) | ((col & 8) >> 1);
    c.vj = lane % 16;
    c.vg = (lane / 16) % 2;
    c.ld_row = lane / T::kGran;
    c.ld_gran = lane % T::kGran;

#pragma unroll
    for (int t = 0; t < kStages - 1; ++t)
        if (t < c.n_tiles) issue_tile<D, NB>(smem, c, t);

    // ---- Q^T operands, pre-multiplied by scale*log2(e): lane holds, for query `col`
    // of block nb, d = 16*kk + 8*half .. +7
    const int q0 = qtile * kBM + c.wave * (32 * NB);
    bf16x8 qreg[NB][KS];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int qi = q0 + nb * 32 + col;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            Pack16 t;
            t.u = make_uint4(0, 0, 0, 0);
            if (qi < n) t.u = *reinterpret_cast<const uint4 *>(qh + int64_t(qi) * stride_tok + kk * 16 + c.half * 8);
            const uint32_t w[4] = {t.u.x, t.u.y, t.u.z, t.u.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)   // a bf16 is the upper half of the binary32 with the same value
                t.p[e] = to_bf16x2(__uint_as_float(w[e] << 16) * scale_log2e, __uint_as_float(w[e] & 0xffff0000u) * scale_log2e);
            qreg[nb][kk] = t.v;
        }
    }

    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.0f;
    float m_run[NB];                  // running maximum (log2 units), common to both half-waves
    float l_run[NB];                  // this lane's share of the running sum
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) l_run[nb] = 0.0f;

    // ---- round 0 fixes the initial maximum
    wait_tile_loads<0>();
    __syncthreads();
    f32x16 s_a[NB], s_b[NB];
    score_round<D, NB>(smem, c, 0, qreg, s_a);
    if (n < 32) mask_round<NB>(c, 0, s_a);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float tmax = max16(s_a[nb]);
        m_run[nb] = fmaxf(tmax, other_half(tmax));
        s_b[nb] = s_a[nb];
    }

    for (int r = 0; r < c.n_rounds; r += 2) {
        round_body<D, NB>(smem, c, r, qreg, s_a, s_b, acc, m_run, l_run);
        if (r + 1 < c.n_rounds) round_body<D, NB>(smem, c, r + 1, qreg, s_b, s_a, acc, m_run, l_run);
    }

    // ---- normalise and store: lane holds, for query `col` of block nb, rows
    // d = 32*mb + 8*(i/4) + 4*half + i%4 of O^T
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float l_tot = l_run[nb] + other_half(l_run[nb]);
        const float inv = 1.0f / l_tot;
        const int qi = q0 + nb * 32 + col;
        if (qi < n) {
            __bf16 *orow = oh + int64_t(qi) * stride_tok;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    union { uint2 u; bf16x2 p[2]; } w;
                    w.p[0] = to_bf16x2(acc[mb][nb][4 * g + 0] * inv, acc[mb][nb][4 * g + 1] * inv);
                    w.p[1] = to_bf16x2(acc[mb][nb][4 * g + 2] * inv, acc[mb][nb][4 * g + 3] * inv);
                    *reinterpret_cast<uint2 *>(orow + mb * 32 + g * 8 + c.half * 4) = w.u;
                }
        }
    }
}

template <int D, int NB>
int launch(const void *q, const void *k, const void *v, void *o, int n, int heads, int64_t stride_tok,
           int64_t stride_head, float scale, hipStream_t stream) {
    static bool attr_set = false;   // per process; the attribute is per function
    auto kern = attention_kernel<D, NB>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Tile<D, NB>::kBytes);
        if (e != hipSuccess) {
            lp::set_last_hip_error(int(e));
            return LP_ERR_HIP;
        }
        attr_set = true;
    }
    const int n_qtiles = (n + kBM - 1) / kBM;
    const dim3 grid(uint32_t(n_qtiles) * uint32_t(heads));
    const float scale_log2e = scale * 1.4426950408889634f;
    return lp::launch_kernel(reinterpret_cast<const void *>(kern), grid, dim3(waves_of(NB) * 64), Tile<D, NB>::kBytes, stream,
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
        return launch<128, kBlocksPerWave>(q, k, v, o, int(n_tokens), heads, stride_tok, stride_head, scale, st);
    return launch<64, kBlocksPerWave>(q, k, v, o, int(n_tokens), heads, stride_tok, stride_head, scale, st);
}
