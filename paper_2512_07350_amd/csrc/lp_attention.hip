// lp_attention: non-causal multi-head self-attention over the patch tokens of one
// sub-latent (supplement, proof of Theorem 1, step 3: inside a sub-latent the DiT
// blocks attend globally over all of its positions), as a flash-style kernel for
// gfx950: bf16 MFMA 32x32x16 for both products, binary32 online softmax, K and V
// tiles streamed global -> LDS without passing through registers.
//
// Work decomposition.  One workgroup = 4 wavefronts = 256 query rows of one head, one
// wavefront per SIMD; each wavefront owns 64 query rows (two 32-column MFMA blocks) and
// walks all keys in rounds of 32.  Per round it forms the TRANSPOSED scores
//     S^T[key, query] = K . Q^T            (A = K rows from LDS, B = Q in registers)
// so that in the MFMA accumulator layout a lane holds 16 scores of ONE query: the
// row maximum and row sum are in-lane reductions, the rescale factor of the running
// output is a per-lane scalar, and the bf16 probabilities are already laid out as
// the B operand of
//     O^T[d, query] += V^T . P^T           (A = V^T, read transposed from LDS).
// Every operand fetched from LDS feeds two products (one per 32-query block): 0.75 LDS
// reads per matrix instruction.  The 64 rows need more than 256 registers per lane: the
// O^T accumulators and the Q^T operands are kept in the accumulation registers (AGPRs) by
// writing the matrix instructions as assembly statements with the register file of every
// operand spelled out (see mfma_score / mfma_pv).
//
// Details that matter for speed:
//  * Q is multiplied by scale*log2(e) once and re-rounded to bf16, and the score
//    accumulators start at -m (m = running maximum, log2 units), so a probability
//    is a bare exp2 of the accumulator.
//  * A segment's rounds run first with the maximum fixed at what the segment's first round made
//    it and no look at the scores at all: exp2 of a score 100 log2 units above that maximum is
//    still an ordinary binary32 / bf16 number, and numerator and denominator of the final
//    division carry the same power of two.  Only if a row sum or an accumulator comes out
//    non-finite (a score about 2^7 log2 units above the first round's) does the workgroup run
//    the segment again, this time raising the maximum lazily: when some score exceeds it by
//    more than kRescaleThreshold, in a rarely taken, wave-uniform branch that rescales the
//    output accumulators.
//  * The score product of round r+1, the softmax of round r and the PV product of round
//    r-1 share one step, and the step's vector and LDS work is cut into one small window
//    per matrix instruction (pipeline_step), so that the one wavefront of a SIMD has its
//    next product ready when the matrix pipeline takes it.
//  * The key order inside a 32-key round is permuted (bits 2 and 3 of the MFMA row
//    index swapped when K rows are read) so that the 8 probabilities a lane feeds
//    to one MFMA belong to 8 consecutive keys; V^T operands then come from two
//    ds_read_b64_tr_b16 (transposing LDS reads) of the row-major V tile.
//  * K/V tiles go global -> LDS with buffer_load_dwordx4 ... lds (kStages tiles
//    resident), with XOR swizzles of the 16-byte granules chosen so that the K
//    reads (ds_read_b128) and the V reads are free of bank conflicts.
//  * One persistent workgroup per compute unit; the (query tile, key tile) space is
//    dealt so that every workgroup gets the same cost, and a query tile shared by
//    several workgroups is merged by combine_kernel (see AttnParams).
//  * A segment's results leave as whole 128-byte lines through per-wave LDS
//    staging, after the next segment's first tiles and Q rows have been sent for.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "lp_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define LP_LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

// f(integral_constant<int, I>) for I = FROM .. TO-1: a loop whose index is a constant
// expression inside the body.
template <int FROM, int TO, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (FROM < TO) {
        f(std::integral_constant<int, FROM>{});
        static_for<FROM + 1, TO>(f);
    }
}

constexpr int kBM = 256;                      // query rows per workgroup
// A wavefront owns NB blocks of 32 query rows; the workgroup has kBM / (32 NB) wavefronts.
constexpr int waves_of(int nb) { return kBM / (32 * nb); }
// NB used by lp_attention: 64 query rows per wavefront (one wavefront per SIMD, four per workgroup)
constexpr int blocks_per_wave(int /* head_dim */) { return 2; }
constexpr int kBN = 64;                       // keys per LDS tile (two rounds of 32)
constexpr int kStages = 4;                    // LDS stages: three tiles in use plus one arriving
constexpr float kRescaleThreshold = 8.0f;     // log2 units the running max may lag behind
constexpr uint32_t kBoundaryTiles = 4;        // what changing units costs a workgroup, in tile times

template <int D, int NB>
struct Tile {
    static constexpr int kWaves = waves_of(NB);
    static constexpr int kRowBytes = D * 2;
    static constexpr int kGran = kRowBytes / 16;            // 16-byte granules per row
    static constexpr int kTileBytes = kBN * kRowBytes;      // one K or one V tile
    static constexpr int kStageBytes = 2 * kTileBytes;      // K tile then V tile
    static constexpr int kRingBytes = kStages * kStageBytes;
    static constexpr int kOutBytes = 4096;                  // per wave: 32 result rows of 64 d in bf16
    static constexpr int kBytes = kRingBytes + kWaves * kOutBytes;
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

// At most N LDS operations of this wavefront still outstanding (the compiler sees this wait
// and leaves out its own for everything older).
template <int N>
__device__ __forceinline__ void lds_wait() {
    static_assert(N >= 0 && N < 16, "lgkmcnt range");
    __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));
}

// LDS accesses below use 32-bit LDS byte addresses held in registers.
// The same value, but not a loop invariant as far as the compiler can tell.
__device__ __forceinline__ int opaque(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

template <typename V>
__device__ __forceinline__ V lds_load(uint32_t addr) {
    return *LP_LDS_PTR(const V, uintptr_t(addr));
}

__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ float max16(const f32x16 &s) {
    float t = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) t = fmaxf(t, s[i]);
    return t;
}

// What a lane needs to know to move tiles from global memory into LDS.
template <int D, int NB>
struct Lane {
    using T = Tile<D, NB>;
    static constexpr int kLd = T::kInstrPerTile / T::kWaves;   // K (and V) load instructions per wave per tile
    __amdgpu_buffer_rsrc_t k_rsrc, v_rsrc;   // K and V of this head as raw buffers ending with token n-1
    uint32_t k_voff[kLd], v_voff[kLd];       // byte offset of this lane's 16 bytes in tile 0
    uint32_t ld_dst[kLd];                    // LDS offset of the 1024-byte block inside a K tile (wave-uniform)
    uint32_t tile_bytes;                     // global byte distance between consecutive tiles
    uint32_t valid_bytes;                    // size of the K (and V) buffer of the current head: a load at or past it reads zeros and fetches nothing
    int half;                                // lane / 32
    int key_end;                             // keys at and past this index do not exist for the current segment
    int t_end;                               // one past the segment's last tile
};

// One wave-wide global -> LDS load: lane L fetches the 16 bytes at byte offset voff + soff of
// the buffer and they land at LDS address lds_addr + 16 L (lds_addr is wave-uniform and goes
// through M0; bytes outside the buffer arrive as zeros).  Written as an assembly statement so
// that the compiler keeps no record of it: told about such a load, it waits for ALL of them
// (vmcnt(0)) before the next LDS read of any address, which would put the whole memory latency
// of the tile just sent for in front of the operand reads of the tiles in use.  The waits that
// order these loads against the reads of their own stage are wait_tile_loads + barrier.
// Nothing else in this file uses M0.
template <int V_LDS_OFFSET>
__device__ __forceinline__ void load_kv_to_lds_16(__amdgpu_buffer_rsrc_t k_rsrc, __amdgpu_buffer_rsrc_t v_rsrc, uint32_t k_lds,
                                                  uint32_t k_voff, uint32_t v_voff, uint32_t soff) {
    // K block, then the V block V_LDS_OFFSET bytes further on.  M0 must be written one
    // instruction before the load that uses it: the address of the V block is formed between
    // the first write and its use, an s_nop stands between the second write and its use.
    uint32_t v_lds;
    asm volatile("s_mov_b32 m0, %1\n\ts_add_u32 %0, %1, %2\n\tbuffer_load_dwordx4 %3, %5, %7 offen lds\n\t"
                 "s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %4, %6, %7 offen lds"
                 : "=&s"(v_lds)
                 : "s"(k_lds), "n"(V_LDS_OFFSET), "v"(k_voff), "v"(v_voff), "s"(k_rsrc), "s"(v_rsrc), "s"(soff)
                 : "memory", "m0", "scc");
}

// global -> LDS loads of one K/V tile into the stage at byte offset stage_off.  One
// wave-wide instruction moves 1024 bytes.  Rows past token n-1 lie outside the buffers
// and arrive as zeros.
template <int D, int NB>
__device__ __forceinline__ void issue_tile(uint32_t lds0, const Lane<D, NB> &c, int tile, uint32_t stage_off) {
    using T = Tile<D, NB>;
    const uint32_t soff = uint32_t(tile) * c.tile_bytes;
#pragma unroll
    for (int i = 0; i < Lane<D, NB>::kLd; ++i) {
        const uint32_t dst_k = __builtin_amdgcn_readfirstlane(lds0 + stage_off + c.ld_dst[i]);
        load_kv_to_lds_16<T::kTileBytes>(c.k_rsrc, c.v_rsrc, dst_k, c.k_voff[i], c.v_voff[i], soff);
    }
}

// The I-th of a wave's kLd load statements of a tile (K block and V block), at scalar byte offset
// soff (which takes part in the buffer's range check, like the lane's own offset).
template <int D, int NB, int I>
__device__ __forceinline__ void issue_tile_part(uint32_t lds0, const Lane<D, NB> &c, uint32_t soff, uint32_t stage_off) {
    using T = Tile<D, NB>;
    const uint32_t dst_k = __builtin_amdgcn_readfirstlane(lds0 + stage_off + c.ld_dst[I]);
    load_kv_to_lds_16<T::kTileBytes>(c.k_rsrc, c.v_rsrc, dst_k, c.k_voff[I], c.v_voff[I], soff);
}

// Keys past the end get score -inf.  Accumulator register i of a lane is key
// 32*r + 16*(i/8) + 8*half + i%8.
template <int NB>
__device__ __forceinline__ void mask_scores(int r, int half, int n, f32x16 (&s)[NB]) {
    const int kbase = r * 32 + half * 8;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (kbase + 16 * (i / 8) + (i % 8) >= n) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) s[nb][i] = -INFINITY;
        }
    }
}

// ---- the matrix instructions, with the register file of every operand chosen here.
// A wavefront that owns 64 query rows needs more than 256 registers: the O^T accumulators
// (D/32 * NB * 16) and the Q^T operands (NB * D/16 * 4) live in the accumulation registers
// (AGPRs) and are touched by matrix instructions only; scores, probabilities and the LDS
// operands live in the ordinary ones, where the vector ALU works on them.  The compiler is
// not told what these statements are, so it neither moves operands between the two files
// nor inserts the wait states that separate a matrix instruction's result from a vector
// instruction reading it; settle_scores / settle_acc below do that where such a read follows.
__device__ __forceinline__ void mfma_score_init(f32x16 &d, const bf16x8 &k, const bf16x8 &q, const f32x16 &c) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(k), "a"(q), "v"(c));
}
__device__ __forceinline__ void mfma_score(f32x16 &d, const bf16x8 &k, const bf16x8 &q) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_pv(f32x16 &acc, const bf16x8 &vt, const bf16x8 &p) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(vt), "v"(p));
}

// Ordering points for the vector work between matrix instructions.  Statements of this kind
// keep their program order among themselves, so whatever produces x comes before this point
// and whatever uses x afterwards comes after it; no instruction is emitted.
__device__ __forceinline__ void pin(float &x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(uint32_t &x) { asm volatile("" : "+v"(x)); }

// Scores written by matrix instructions become readable by vector instructions: 16 wait
// states cover the 8 passes of the last product plus its write-back.
template <int NB>
__device__ __forceinline__ void settle_scores(f32x16 (&s)[NB], bool wait) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        if (wait) asm volatile("s_nop 15" : "+v"(s[nb]));
        else asm volatile("" : "+v"(s[nb]));
    }
}

// The same for the accumulators in the AGPRs (before they are rescaled or stored), and, with
// after = true, between vector writes to them and the next matrix instruction.
template <int D, int NB>
__device__ __forceinline__ void settle_acc(f32x16 (&acc)[D / 32][NB], bool after) {
    if (after) asm volatile("s_nop 3");
    else asm volatile("s_nop 15\n\ts_nop 7");
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+a"(acc[mb][nb]));
}

// The row sum adds the rounded probabilities.
__device__ __forceinline__ void add_to_row_sum(uint32_t pair, float &l) {
    union { bf16x2 p; uint32_t u; } w;
    w.u = pair;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    l = __builtin_amdgcn_fdot2_f32_bf16(w.p, ones, l, false);
}

// Lazy running maximum.  Score accumulators start at neg_m = -m (m = running maximum, log2
// units), so s holds scores relative to m that will be exponentiated NEXT.  If any of them
// exceeds kRescaleThreshold, raise the maximum by delta and rescale what was accumulated
// under the old one: these scores, the output accumulators, the row sums, and the
// probabilities p_pending that have been computed but not yet multiplied into acc.
template <int D, int NB>
__device__ __forceinline__ void raise_maximum(const float (&lane_max)[NB], f32x16 (&s)[NB], f32x16 (&neg_m)[NB],
                                              bf16x8 (&p_pending)[NB][2], f32x16 (&acc)[D / 32][NB], float (&l_run)[NB]) {
    bool raise = false;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) raise = raise || (lane_max[nb] > kRescaleThreshold);
    if (__builtin_expect(__any(raise) != 0, 0)) {     // the branch body is laid out away from the loop
        settle_acc<D, NB>(acc, false);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float tmax = lane_max[nb];
            tmax = fmaxf(tmax, other_half(tmax));
            const float delta = fmaxf(tmax, 0.0f);           // the maximum never goes down
            const float alpha = __builtin_amdgcn_exp2f(-delta);
            l_run[nb] *= alpha;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s[nb][i] -= delta;
                neg_m[nb][i] -= delta;
            }
#pragma unroll
            for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mb][nb][i] *= alpha;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                Pack16 t;
                t.v = p_pending[nb][ks];
                const uint32_t w[4] = {t.u.x, t.u.y, t.u.z, t.u.w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    t.p[e] = to_bf16x2(__uint_as_float(w[e] << 16) * alpha, __uint_as_float(w[e] & 0xffff0000u) * alpha);
                p_pending[nb][ks] = t.v;
            }
        }
        settle_acc<D, NB>(acc, true);
    }
}

// One K operand (16 bytes of a K row) from LDS: SUB selects the first or second round of
// the tile whose operand addresses are k_addr.
template <int D, int NB, int SUB>
__device__ __forceinline__ bf16x8 load_k_operand(const uint32_t (&k_addr)[D / 16], int kk) {
    return lds_load<bf16x8>(k_addr[kk] + SUB * 32 * Tile<D, NB>::kRowBytes);
}

// One V^T operand via two transposing reads.  Inside a group of 16 lanes, lane j supplies
// the 8-byte chunk (row j/4, columns 4*(j%4)..+3) and receives column j of that 4x16 block,
// i.e. 4 consecutive keys of one d.  Operand j covers keys 16*(j / MB).. of the round and
// rows 32*(j % MB).. of O^T; HALF selects its first or second four keys.
template <int D, int NB, int SUB, int HALF>
__device__ __forceinline__ bf16x4 load_v_half(const uint32_t (&v_addr)[D / 32], int j) {
    using T = Tile<D, NB>;
    constexpr int MB = D / 32;
    const uint32_t a0 = v_addr[j % MB] + (SUB * 32 + (j / MB) * 16 + HALF * 4) * T::kRowBytes;
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LP_LDS_PTR(bf16x4, uintptr_t(a0)));
}

// Everything one wavefront carries from step to step.
template <int D, int NB>
struct Pipe {
    bf16x8 qreg[NB][D / 16];       // Q^T operands (pre-scaled)
    bf16x8 opreg[D / 16];          // LDS operands: K rows before a score product, V^T blocks before a PV product
    f32x16 acc[D / 32][NB];        // O^T accumulators
    f32x16 neg_m[NB];              // -m in every element (m = running maximum, log2 units, common to
                                   // both half-waves): the initial value of every score accumulator
    float l_run[NB];               // this lane's share of the running sum
    uint32_t k_addr[D / 16];       // LDS addresses of the K operands in the stage at k_off
    uint32_t v_addr[D / 32];       // LDS addresses of the V operands in the stage at v_off
    uint32_t k_off, v_off;         // stage offsets k_addr / v_addr currently point into
    uint32_t tile_off;             // stage offset of tile i/2
    uint32_t issue_off;            // stage offset the next issued tile goes to
    int issue_t;                   // index of the next tile to issue
};

// Writes this wave's 32 result rows (acc scaled by `inv`, rounded to bf16) to rows
// dst + r * row_stride, r < rows_valid.  A lane holds, for query `col`, rows
// d = 32*mb + 8*(i/4) + 4*half + i%4 of O^T, i.e. 8-byte pieces of many rows; the pieces
// pass through the wave's own 4 KB of LDS (64 d at a time, 16-byte granules XORed with
// the row so that both directions are conflict free) and leave as whole 128-byte lines.
template <int D, int NB>
__device__ __forceinline__ void store_rows(uint32_t out_lds, const f32x16 (&acc)[D / 32][NB], int nb, float inv, __bf16 *dst,
                                           int64_t row_stride, int rows_valid, int lane) {
    const int col = lane % 32, half = lane / 32;
#pragma unroll
    for (int pass = 0; pass < D / 64; ++pass) {
#pragma unroll
        for (int mbl = 0; mbl < 2; ++mbl)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x16 &x = acc[2 * pass + mbl][nb];
                union { u32x2 u; bf16x2 p[2]; } ow;
                ow.p[0] = to_bf16x2(x[4 * g + 0] * inv, x[4 * g + 1] * inv);
                ow.p[1] = to_bf16x2(x[4 * g + 2] * inv, x[4 * g + 3] * inv);
                *LP_LDS_PTR(u32x2, uintptr_t(out_lds + col * 128 + 16 * ((4 * mbl + g) ^ (col & 7)) + 8 * half)) = ow.u;
            }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = lane / 8 + 8 * j, gran = lane % 8;
            const u32x4 u = lds_load<u32x4>(out_lds + r * 128 + 16 * (gran ^ (r & 7)));
            if (r < rows_valid) *reinterpret_cast<u32x4 *>(dst + r * row_stride + 64 * pass + 8 * gran) = u;
        }
    }
}

// The part of the softmax that trails the exponentials: converts the pairs [CVT_FROM, CVT_TO)
// to packed bf16 words (and completes an operand with its fourth word), then adds the words
// [SUM_FROM, CVT_FROM) to the row sums.  Pair k holds scores 2 k, 2 k + 1 counted across both
// blocks: word k % 4 of operand (k % 8) / 4 of block k / 8.
template <int NB, int CVT_TO, int CVT_FROM, int SUM_FROM>
__device__ __forceinline__ void vector_tail(const float (&ex)[NB * 16], uint32_t (&pw)[NB][2][4], bf16x8 (&p_cur)[NB][2],
                                            float (&l_run)[NB]) {
    static_for<CVT_FROM, CVT_TO>([&](auto kc) {
        constexpr int k = decltype(kc)::value, nb = k / 8, part = (k % 8) / 4, e = k % 4;
        union { bf16x2 p; uint32_t u; } cv;
        cv.p = to_bf16x2(ex[2 * k], ex[2 * k + 1]);
        pw[nb][part][e] = cv.u;
        pin(pw[nb][part][e]);
        if constexpr (e == 3) {
            Pack16 t;
            t.u = make_uint4(pw[nb][part][0], pw[nb][part][1], pw[nb][part][2], pw[nb][part][3]);
            p_cur[nb][part] = t.v;
        }
    });
    static_for<SUM_FROM, CVT_FROM>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        add_to_row_sum(pw[k / 8][(k % 8) / 4][k % 4], l_run[k / 8]);
        pin(l_run[k / 8]);
    });
}

template <int BYTES>
__device__ __forceinline__ uint32_t next_stage(uint32_t off) {
    off += BYTES;
    return off == kStages * BYTES ? 0u : off;
}

// Step i of the software pipeline (SUB = i % 2).  For ONE wavefront a step issues
//   MFMA:  S^T of round i+1, then O^T += V^T P^T of round i-1
//   VALU:  probabilities of round i (spread over the whole step), then the maximum check
//          for round i+1
//   LDS :  each score group is followed by the fetch of a V operand of round i-1 into the
//          registers it has just read, each PV group by the fetch of a K operand of round i+2
// so that an LDS operand is fetched half a step before its products, and K and V operands
// share one set of registers.
// Even steps open tile t+1 (t = i/2): at the end of their score phase they wait for its loads
// and pass the barrier (after which every wave has fetched its last operand from tile t-2), and
// over their PV phase they refill that stage with tile t+kStages-2.
// The same code runs at the ends of a segment: with MASK, keys past the segment's end get
// scores -inf (probabilities 0), and the round before the first has probabilities 0, so
// the products issued for rounds that do not exist add nothing; their operands are read
// from valid, if stale, LDS addresses.  MASK = false is for steps whose rounds i+1 lie
// wholly inside the segment and keeps the step free of conditionals.
template <int D, int NB, int SUB, bool MASK, bool CHECK>
__device__ __forceinline__ void pipeline_step(uint32_t lds0, const Lane<D, NB> &c, int i, bool first,
                                              Pipe<D, NB> &w, f32x16 (&s_cur)[NB], f32x16 (&s_nxt)[NB],
                                              bf16x8 (&p_prev)[NB][2], bf16x8 (&p_cur)[NB][2]) {
    using T = Tile<D, NB>;
    constexpr int KS = D / 16, MB = D / 32;
    // Per-tile bookkeeping is scalar and happens here; what it decides is carried out inside the
    // windows below, so that no stretch of the step is without a product to issue:
    //  * SUB == 0 opens tile t+1 (t = i/2).  Its K operands are first fetched in the PV phase, so
    //    the wait for its loads and the barrier (after which every wave has fetched its last
    //    operand from tile t-2) stand at the end of the score phase; each K operand address moves
    //    to the new stage right before its first fetch there; and the kLd load statements that
    //    refill tile t-2's stage with tile t+kStages-2 are spread over the PV phase.  Past the
    //    segment's end the loads are given an offset outside the buffer: they fetch nothing.
    //  * SUB == 1: round i-1 is the first of tile i/2, the V fetches move on to that tile --
    //    unless it lies past the segment and was never loaded (its probabilities are 0, and 0
    //    times whatever an unwritten stage holds need not be 0); each V operand address moves
    //    right before its first fetch of the step.
    uint32_t k_delta = 0, v_delta = 0, issue_soff = 0, issue_stage = 0;
    if (SUB == 0) {
        if (!first) w.tile_off = next_stage<T::kStageBytes>(w.tile_off);
        const uint32_t nxt_off = next_stage<T::kStageBytes>(w.tile_off);
        k_delta = nxt_off - w.k_off;       // wraps; the sums do not
        w.k_off = nxt_off;
        issue_soff = w.issue_t < c.t_end ? uint32_t(w.issue_t) * c.tile_bytes : c.valid_bytes;
        issue_stage = w.issue_off;
        ++w.issue_t;
        w.issue_off = next_stage<T::kStageBytes>(w.issue_off);
    } else {
        if (i / 2 < c.t_end) {
            v_delta = w.tile_off - w.v_off;
            w.v_off = w.tile_off;
        }
    }

    // The step's 2 KS NB products, in KS score groups and then KS PV groups (a group is the
    // NB products that share one LDS operand).  The wavefront is alone on its SIMD, so the
    // matrix pipeline is busy only if the next product is issued within the 8 passes of the
    // one before: the vector and LDS work of the step is therefore cut into one window per
    // product -- the exponentials of round i (8 / KS per window), a conversion and a row-sum
    // update for every second of them, the refill of the operand registers the group has just
    // read (half a V^T operand or one K operand per window), in even steps a quarter of the next
    // tile's loads in every second PV group, and, from four windows after the last score product
    // to the end of the step, the per-lane maximum of round i+1's scores.
    static_assert(NB == 2, "the windows below are laid out for two 32-row blocks per wavefront");
    constexpr int M = 2 * KS * NB;              // products per step
    constexpr int X = (NB * 16) / M;            // exponentials per window
    // the maximum of round i+1's scores: from four windows after its last product (whose result
    // has then left the pipeline) to the end of the step, both blocks in turn
    constexpr int kMaxFrom = KS * NB + 4, kMaxWin = (M - kMaxFrom) / NB;   // windows per block
    uint32_t pw[NB][2][4];
    float ex[NB * 16];
    float lane_max[NB];
    Pack16 vop;
    static_for<0, M>([&](auto mc) {
        constexpr int m = decltype(mc)::value, g = m / NB, nb = m % NB;
        // Operand arrivals are checked for half a phase at a time.  In issue order the LDS queue
        // holds, at the start of the score phase, the KS K fetches of the previous PV phase: all
        // but the newest KS/2 cover groups 0 .. KS/2-1; by group KS/2 the newest are KS/2 groups
        // of V fetches (2 each), so lgkmcnt(KS) covers the rest.  The PV phase mirrors this with
        // 2 KS V fetches followed by one K fetch per group.
        if constexpr (nb == 0 && g == 0) lds_wait<KS / 2>();
        if constexpr (nb == 0 && g == KS / 2) lds_wait<KS>();
        if constexpr (nb == 0 && g == KS) lds_wait<KS>();
        if constexpr (nb == 0 && g == KS + KS / 2) lds_wait<KS / 2>();
        if constexpr (g < KS) {
            if constexpr (g == 0) mfma_score_init(s_nxt[nb], w.opreg[g], w.qreg[nb][g], w.neg_m[nb]);
            else mfma_score(s_nxt[nb], w.opreg[g], w.qreg[nb][g]);
            if constexpr (SUB == 1 && nb == 0 && g < MB) w.v_addr[g] += v_delta;
            if constexpr (nb == 0) vop.h[0] = load_v_half<D, NB, 1 - SUB, 0>(w.v_addr, g);
            else {
                vop.h[1] = load_v_half<D, NB, 1 - SUB, 1>(w.v_addr, g);
                w.opreg[g] = vop.v;
            }
        } else {
            constexpr int j = g - KS;
            mfma_pv(w.acc[j % MB][nb], w.opreg[j], p_prev[nb][j / MB]);
            if constexpr (nb == NB - 1) {
                if constexpr (SUB == 0) w.k_addr[j] += k_delta;
                w.opreg[j] = load_k_operand<D, NB, SUB>(w.k_addr, j);
            } else if constexpr (SUB == 0 && nb == 0) {
                // the tile's load statements, evenly over the PV groups
                constexpr int kLd = Lane<D, NB>::kLd, every = KS / kLd;
                if constexpr (j % every == 0) issue_tile_part<D, NB, j / every>(lds0, c, issue_soff, issue_stage);
            }
        }
        if constexpr (SUB == 0 && m == KS * NB - 1) {
            wait_tile_loads<0>();              // tile t+1, issued one tile ago
            __syncthreads();
        }
        // exponentials x = m X .. of the round's NB * 16 scores.  A pair is converted in the
        // window after its second exponential (a conversion must not directly follow the
        // exponential it reads) and joins the row sum one window later.
        static_for<m * X, (m + 1) * X>([&](auto xc) {
            constexpr int x = decltype(xc)::value;
            float sc = s_cur[x / 16][x % 16];
            pin(sc);
            ex[x] = __builtin_amdgcn_exp2f(sc);
        });
        vector_tail<NB, m * X / 2, (m > 0 ? (m - 1) * X / 2 : 0), (m > 1 ? (m - 2) * X / 2 : 0)>(ex, pw, p_cur, w.l_run);
        static_for<m * X, (m + 1) * X>([&](auto xc) { pin(ex[decltype(xc)::value]); });
        if constexpr (m == kMaxFrom - 1) {
            settle_scores<NB>(s_nxt, false);
            if (MASK) mask_scores<NB>(i + 1, c.half, c.key_end, s_nxt);
        }
        if constexpr (CHECK && m >= kMaxFrom) {
            constexpr int wdx = m - kMaxFrom, nbm = wdx % NB, first = (16 * (wdx / NB)) / kMaxWin;
            // three-operand maxima, written out so that no operand is first passed through a
            // quieting v_max (the scores come from assembly statements, so the compiler cannot
            // tell that they are ordinary numbers)
            float mx = first == 0 ? s_nxt[nbm][0] : lane_max[nbm];
            constexpr int lo = first == 0 ? 1 : first, hi = (16 * (wdx / NB + 1)) / kMaxWin;
            static_for<0, (hi - lo) / 2>([&](auto rc) {
                constexpr int r = lo + 2 * decltype(rc)::value;
                mx = max3(mx, s_nxt[nbm][r], s_nxt[nbm][r + 1]);
            });
            if constexpr ((hi - lo) % 2 == 1) mx = max3(mx, s_nxt[nbm][hi - 1], s_nxt[nbm][hi - 1]);
            lane_max[nbm] = mx;
            pin(lane_max[nbm]);
        }
    });
    // what the last two windows left to convert and to add
    vector_tail<NB, NB * 8, (M - 1) * X / 2, (M - 2) * X / 2>(ex, pw, p_cur, w.l_run);
    vector_tail<NB, NB * 8, NB * 8, (M - 1) * X / 2>(ex, pw, p_cur, w.l_run);
    if constexpr (CHECK) raise_maximum<D, NB>(lane_max, s_nxt, w.neg_m, p_cur, w.acc, w.l_run);
}

// Launch parameters.  A unit is one 256-row query tile of one head; every unit walks
// tiles_per_unit tiles of 64 keys.  With P workgroups, the units are served in two parts:
//  * the first shared_units units form a (unit, key tile) iteration space that is cut into
//    shared_wgs <= P contiguous ranges (never empty), so a workgroup may start and end in
//    the middle of a unit; such partial results go to `ws` and are merged by combine_kernel.
//    The cut is even in COST, not in tiles: every unit is preceded by kBoundaryTiles
//    imaginary tiles that stand for what a workgroup pays to change units (drain and
//    refill of the pipeline, stores, a new Q), the space of shared_units * unit_cost
//    real and imaginary tiles is cut into equal ranges, and a range's imaginary tiles are
//    dropped.  A workgroup that changes units thus gets fewer tiles than one that does not.
//  * the remaining whole_rounds * P units are taken whole, unit shared_units + r*P + p by
//    workgroup p in round r: the workgroups of an XCD then walk the keys of one head in
//    step and share its K/V stream through the L2.
// One workgroup per unit (nothing shared) is shared_units = 0, whole_rounds = 1.
struct AttnParams {
    const __bf16 *q, *k, *v;
    __bf16 *o;
    float *ws;                 // slots for partial results: 2 per workgroup
    int64_t stride_tok, stride_head, stride_batch;
    int heads;                 // heads per batch item; a unit's head index counts batch * heads + head
    float scale_log2e;
    int n, n_qtiles, tiles_per_unit;
    int shared_units, whole_rounds;
    uint32_t shared_work;      // shared_units * unit_cost
    uint32_t unit_cost;        // tiles_per_unit + kBoundaryTiles
    uint32_t shared_wgs;       // workgroups 0 .. shared_wgs-1 (logical order) take part in the shared space
};

// A slot holds, for the 256 query rows of a unit: m[256] and l[256] in binary32, then the
// unnormalised O rows [256][D] rounded to bf16 (the merged row is rounded to bf16 on store
// anyway; halving the rows halves the traffic of the merge).
template <int D>
constexpr int slot_floats() { return kBM * (D / 2 + 2); }

// Element offset of the first token of head index bh = batch_item * heads + head.
__device__ __forceinline__ int64_t head_offset(const AttnParams &a, int bh) {
    const int b = bh / a.heads;
    return int64_t(b) * a.stride_batch + int64_t(bh - b * a.heads) * a.stride_head;
}

// First iteration of (logical) workgroup p when W iterations are dealt to P workgroups.
__device__ __forceinline__ uint32_t range_start(uint32_t p, uint32_t W, uint32_t P) {
    return uint32_t(uint64_t(p) * W / P);
}

// Position x in the space with imaginary tiles -> index of the first real tile at or after it.
__device__ __forceinline__ uint32_t real_tile(uint32_t x, uint32_t unit_cost, uint32_t tpu) {
    const uint32_t unit = x / unit_cost, r = x - unit * unit_cost, imaginary = unit_cost - tpu;
    return unit * tpu + (r > imaginary ? r - imaginary : 0u);
}

// Workgroup ids are dealt round robin to the 8 XCDs; remap so that each XCD owns a
// contiguous stretch of the iteration space and the K/V of a head stay in one XCD's L2.
__device__ __forceinline__ uint32_t logical_workgroup(uint32_t b, uint32_t n_wg) {
    const uint32_t xcd = b % 8, slot = b / 8;
    const uint32_t base = n_wg / 8, rem = n_wg % 8;
    return xcd * base + (xcd < rem ? xcd : rem) + slot;
}

// A segment: the tiles [t_begin, t_stop) of one unit.
struct Segment {
    uint32_t unit;
    int t_begin, t_stop;
    bool valid;
};

// Where a workgroup stands in its work: its range of the shared space first, then whole units.
struct Walk {
    uint32_t it, it_end;
    int whole_round;
};

__device__ __forceinline__ Segment next_segment(Walk &k, const AttnParams &a, uint32_t tpu, uint32_t lp, uint32_t n_wg) {
    Segment s;
    s.valid = true;
    if (k.it < k.it_end) {
        s.unit = k.it / tpu;
        s.t_begin = int(k.it - s.unit * tpu);
        s.t_stop = int(min(tpu, uint32_t(s.t_begin) + (k.it_end - k.it)));
        k.it += uint32_t(s.t_stop - s.t_begin);
    } else if (k.whole_round < a.whole_rounds) {
        s.unit = uint32_t(a.shared_units) + uint32_t(k.whole_round) * n_wg + lp;
        s.t_begin = 0;
        s.t_stop = int(tpu);
        ++k.whole_round;
    } else {
        s.unit = 0;
        s.t_begin = s.t_stop = 0;
        s.valid = false;
    }
    return s;
}

// Points the tile traffic at a segment and sends for its first kStages-2 tiles (the
// segment's tiles use the LDS stages in turn, from stage 0).  The caller has made sure
// that no wave still reads the stages.
template <int D, int NB>
__device__ __forceinline__ void start_tiles(uint32_t lds0, const AttnParams &a, const Segment &seg,
                                            Lane<D, NB> &c, Pipe<D, NB> &w, int n, int64_t stride_tok) {
    using T = Tile<D, NB>;
    const int64_t head_off = head_offset(a, int(seg.unit) / a.n_qtiles);
    c.key_end = min(n, seg.t_stop * kBN);
    c.t_end = seg.t_stop;
    {
        // raw buffers over this head's K and V, ending with the last element of token n-1
        // (flags: 32-bit data format, as every untyped buffer on this architecture)
        const int valid_bytes = int((int64_t(n - 1) * stride_tok + D) * 2);
        c.valid_bytes = uint32_t(valid_bytes);
        const __bf16 *kh = a.k + head_off, *vh = a.v + head_off;
        c.k_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16 *>(kh), 0, valid_bytes, 0x00020000);
        c.v_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16 *>(vh), 0, valid_bytes, 0x00020000);
    }
    w.issue_off = 0;
    w.issue_t = seg.t_begin;
#pragma unroll
    for (int t = 0; t < kStages - 2; ++t) {
        if (w.issue_t < c.t_end) issue_tile<D, NB>(lds0, c, w.issue_t, w.issue_off);
        w.issue_off += T::kStageBytes;
        ++w.issue_t;
    }
}

// Loads a segment's raw Q rows: a lane holds, for query `col`, d = 16*kk + 8*half .. +7.
template <int D, int NB>
__device__ __forceinline__ void load_q(const AttnParams &a, const Segment &seg, Pipe<D, NB> &w, int n,
                                       int64_t stride_tok, int wave, int col, int half) {
    const int head = int(seg.unit) / a.n_qtiles;
    const int qtile = int(seg.unit) % a.n_qtiles;
    const __bf16 *qh = a.q + head_offset(a, head);
    const int q0 = qtile * kBM + wave * (32 * NB);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int qi = q0 + nb * 32 + col;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
            Pack16 t;
            t.u = make_uint4(0, 0, 0, 0);
            if (qi < n) t.u = *reinterpret_cast<const uint4 *>(qh + int64_t(qi) * stride_tok + kk * 16 + half * 8);
            w.qreg[nb][kk] = t.v;
        }
    }
}

template <int D, int NB>
__global__ __launch_bounds__(waves_of(NB) * 64) void attention_kernel(const AttnParams a) {
    using T = Tile<D, NB>;
    using L = Lane<D, NB>;
    constexpr int KS = D / 16;        // MFMA steps along d for S^T
    constexpr int MB = D / 32;        // 32-row blocks of O^T
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const uint32_t lds0 = uint32_t(uintptr_t(LP_LDS_PTR(unsigned char, smem)));

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int lane_id = tid % 64;
    const int lane = lane_id;
    const int col = lane % 32;        // MFMA column (query) / A-operand row
    const int half = lane / 32;
    const int n = a.n;
    const int64_t stride_tok = a.stride_tok;
    const int n_rounds = (n + 31) / 32;

    // ---- lane constants of the tile traffic
    L c;
    c.half = half;
    c.tile_bytes = uint32_t(kBN * stride_tok * 2);
#pragma unroll
    for (int i = 0; i < L::kLd; ++i) {
        const int instr = wave + i * T::kWaves;
        const int row = instr * T::kRowsPerInstr + lane / T::kGran;
        const int gran = lane % T::kGran;          // physical granule this lane fills
        c.ld_dst[i] = instr * 1024;
        c.k_voff[i] = uint32_t(row * stride_tok * 2) + 16 * (gran ^ T::swz_k(row));
        c.v_voff[i] = uint32_t(row * stride_tok * 2) + 16 * (gran ^ T::swz_v(row));
    }

    // ---- this workgroup's range of the shared (unit, tile) space, then its whole units
    const uint32_t lp = logical_workgroup(blockIdx.x, gridDim.x);
    const bool sharing = lp < a.shared_wgs;
    const uint32_t tpu = uint32_t(a.tiles_per_unit);
    Walk walk;
    walk.it = sharing ? real_tile(range_start(lp, a.shared_work, a.shared_wgs), a.unit_cost, tpu) : 0u;
    walk.it_end = sharing ? real_tile(range_start(lp + 1, a.shared_work, a.shared_wgs), a.unit_cost, tpu) : 0u;
    walk.whole_round = 0;
    const uint32_t out_lds = lds0 + T::kRingBytes + wave * T::kOutBytes;
    bool first_segment = true;

    Segment seg = next_segment(walk, a, tpu, lp, gridDim.x);
    if (!seg.valid) return;
    Pipe<D, NB> w;
    start_tiles<D, NB>(lds0, a, seg, c, w, n, stride_tok);
    load_q<D, NB>(a, seg, w, n, stride_tok, wave, col, half);

    while (true) {
        const int qtile = int(seg.unit) % a.n_qtiles;
        const int64_t head_off = head_offset(a, int(seg.unit) / a.n_qtiles);
        const int t_begin = seg.t_begin, t_stop = seg.t_stop;
        const int i_begin = 2 * t_begin;                 // rounds [i_begin, i_end) of 32 keys
        const int i_end = min(2 * t_stop, n_rounds);

        // ---- Q^T operands arrive raw; multiply by scale*log2(e) and round to bf16 again
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                Pack16 t;
                t.v = w.qreg[nb][kk];
                const uint32_t u[4] = {t.u.x, t.u.y, t.u.z, t.u.w};
#pragma unroll
                for (int e = 0; e < 4; ++e)   // a bf16 is the upper half of the binary32 with the same value
                    t.p[e] = to_bf16x2(__uint_as_float(u[e] << 16) * a.scale_log2e,
                                       __uint_as_float(u[e] & 0xffff0000u) * a.scale_log2e);
                w.qreg[nb][kk] = t.v;
            }
        // the Q^T operands now live in AGPRs for the whole segment (left to itself the register
        // allocator may keep them elsewhere and copy each into one shared AGPR quad right before
        // its product, overwriting the quad the product issued just before is still reading)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) asm volatile("" : "+a"(w.qreg[nb][kk]));

        // ---- the segment's rounds.  Run first without the running-maximum check (CHECK = false):
        // the maximum stays what the first round made it, a probability is exp2 of whatever the
        // score is above that, and as long as nothing overflows binary32 / bf16 (2^127) the result
        // is the same sum of the same terms, only scaled by another power of two on both sides of
        // the final division.  If a row sum or an accumulator does come out non-finite -- some
        // score exceeded the first round's maximum by about 2^7 in log2 units -- the workgroup
        // runs the segment again with the check (CHECK = true), which raises the maximum as it goes.
        auto run_segment = [&](auto checked_c) {
        constexpr bool CHECK = decltype(checked_c)::value;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) w.acc[mb][nb][r] = 0.0f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) w.l_run[nb] = 0.0f;
        settle_acc<D, NB>(w.acc, true);

        // ---- LDS operand addresses in stage 0 (recomputed from an opaque copy of the lane
        // index: kept as loop invariants they would be held in registers through the pipeline)
        w.tile_off = 0;
        w.k_off = 0;
        w.v_off = 0;
        {
            const int lane = opaque(lane_id), col = lane % 32, half = lane / 32;
            // K operand: row = col with bits 2 and 3 swapped, so that accumulator register i
            // of a lane is key 16*(i/8) + 8*half + i%8 of the round
            const int krow = (col & 0x13) | ((col & 4) << 1) | ((col & 8) >> 1);
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                w.k_addr[kk] = lds0 + krow * T::kRowBytes + 16 * ((2 * kk + half) ^ T::swz_k(krow));
            const int vj = lane % 16, vg = (lane / 16) % 2;
            const int vrow = half * 8 + vj / 4;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                w.v_addr[mb] = lds0 + T::kTileBytes + vrow * T::kRowBytes + 8 * ((vj % 4) % 2) +
                               16 * ((4 * mb + 2 * vg + (vj % 4) / 2) ^ T::swz_v(vrow));
        }

        // ---- the segment's first round fixes the initial maximum
        wait_tile_loads<0>();
        __syncthreads();
        f32x16 s_a[NB], s_b[NB];
        bf16x8 p_a[NB][2], p_b[NB][2];
        {
            f32x16 zero16;
#pragma unroll
            for (int r = 0; r < 16; ++r) zero16[r] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) w.opreg[kk] = load_k_operand<D, NB, 0>(w.k_addr, kk);
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    if (kk == 0) mfma_score_init(s_a[nb], w.opreg[kk], w.qreg[nb][kk], zero16);
                    else mfma_score(s_a[nb], w.opreg[kk], w.qreg[nb][kk]);
                }
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) w.opreg[kk] = load_k_operand<D, NB, 1>(w.k_addr, kk);
            settle_scores<NB>(s_a, true);
        }
        if ((i_begin + 1) * 32 > c.key_end) mask_scores<NB>(i_begin, half, c.key_end, s_a);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float tmax = max16(s_a[nb]);
            tmax = fmaxf(tmax, other_half(tmax));
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                w.neg_m[nb][r] = -tmax;
                s_a[nb][r] -= tmax;
            }
            s_b[nb] = s_a[nb];
            Pack16 z;
            z.u = make_uint4(0, 0, 0, 0);
            p_b[nb][0] = z.v;               // probabilities of the round before the first: none
            p_b[nb][1] = z.v;
        }

        // ---- the pipeline, two steps at a time; step i_end only flushes the PV product of
        // the last round (and a step past it, if the count is odd, adds nothing)
        int i = i_begin;
        for (; (i + 3) * 32 <= c.key_end; i += 2) {      // rounds i+1 and i+2 are whole
            pipeline_step<D, NB, 0, false, CHECK>(lds0, c, i, i == i_begin, w, s_a, s_b, p_b, p_a);
            pipeline_step<D, NB, 1, false, CHECK>(lds0, c, i + 1, false, w, s_b, s_a, p_a, p_b);
        }
        for (; i <= i_end; i += 2) {
            pipeline_step<D, NB, 0, true, CHECK>(lds0, c, i, i == i_begin, w, s_a, s_b, p_b, p_a);
            pipeline_step<D, NB, 1, true, CHECK>(lds0, c, i + 1, false, w, s_b, s_a, p_a, p_b);
        }
        };   // run_segment

        run_segment(std::false_type{});
        {
            // anything in this lane's row sums or accumulators that is not finite, or within 2^7 of
            // not being so (partial rows are stored as bf16)?  y - y is 0 for every finite y
            settle_acc<D, NB>(w.acc, false);
            float probe = 0.0f;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const float yl = w.l_run[nb] * 128.0f;
                probe += yl - yl;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float y = w.acc[mb][nb][r] * 128.0f;
                        probe += y - y;
                    }
            }
            // the barrier also makes sure that every wave has left the segment's tiles
            if (__syncthreads_or(!(probe == 0.0f))) {
                start_tiles<D, NB>(lds0, a, seg, c, w, n, stride_tok);
                run_segment(std::true_type{});
            }
        }

        // ---- the next segment's first tiles set out before this segment's results are
        // stored, so that their latency hides behind the stores
        const Segment nxt = next_segment(walk, a, tpu, lp, gridDim.x);
        if (nxt.valid) {
            __syncthreads();        // every wave has left this segment's tiles before their stages are refilled
            start_tiles<D, NB>(lds0, a, nxt, c, w, n, stride_tok);
            load_q<D, NB>(a, nxt, w, n, stride_tok, wave, opaque(lane_id) % 32, opaque(lane_id) / 32);
        }

        // ---- results of this segment: final rows, or (a unit shared with other workgroups)
        // running maximum, row sum and unnormalised rows into this workgroup's slot
        settle_acc<D, NB>(w.acc, false);
        const int lane = opaque(lane_id), col = lane % 32, half = lane / 32;
        const bool whole = (t_begin == 0) && (uint32_t(t_stop) == tpu);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const float l_tot = w.l_run[nb] + other_half(w.l_run[nb]);
            const int row0 = wave * (32 * NB) + nb * 32;
            if (whole) {
                const int q0 = qtile * kBM + row0;
                store_rows<D, NB>(out_lds, w.acc, nb, 1.0f / l_tot, a.o + head_off + int64_t(q0) * stride_tok, stride_tok, n - q0, lane);
            } else {
                float *slot = a.ws + (size_t(2) * lp + (first_segment ? 0 : 1)) * slot_floats<D>();
                if (half == 0) {
                    slot[row0 + col] = -w.neg_m[nb][0];
                    slot[kBM + row0 + col] = l_tot;
                }
                store_rows<D, NB>(out_lds, w.acc, nb, 1.0f, reinterpret_cast<__bf16 *>(slot + 2 * kBM) + row0 * D, D, 32, lane);
            }
        }
        first_segment = false;
        if (!nxt.valid) break;
        seg = nxt;
    }
}

// Merges the partial results of every unit that more than one workgroup worked on:
//   m = max_s m_s,  l = sum_s l_s 2^(m_s - m),  O = sum_s O_s 2^(m_s - m) / l.
// grid = (units, kBM / 32): a workgroup takes 32 query rows of one unit, a thread one row
// and 16 consecutive d.
template <int D>
__global__ __launch_bounds__(32 * (D / 16)) void combine_kernel(const AttnParams a, uint32_t n_wg) {
    constexpr int kChunks = D / 16;
    const uint32_t unit = blockIdx.x;
    const uint32_t W = a.shared_work, tpu = uint32_t(a.tiles_per_unit);
    // the unit's real tiles sit at [x_lo, x_hi) of the shared space, after its imaginary ones
    const uint32_t x_hi = (unit + 1) * a.unit_cost, x_lo = x_hi - tpu;
    // workgroup holding position x: the largest p with range_start(p) <= x
    const uint32_t pf = uint32_t((uint64_t(x_lo + 1) * n_wg - 1) / W);
    const uint32_t pl = uint32_t((uint64_t(x_hi) * n_wg - 1) / W);
    if (pf == pl) return;                                      // computed whole by one workgroup
    const int head = int(unit) / a.n_qtiles, qtile = int(unit) % a.n_qtiles;
    const int row = int(blockIdx.y) * 32 + int(threadIdx.x) / kChunks, ch = int(threadIdx.x) % kChunks;
    const int qi = qtile * kBM + row;
    if (qi >= a.n) return;
    // a workgroup's first segment lies in slot 0, a later (its last) one in slot 1
    const bool pf_starts_here = range_start(pf, W, n_wg) >= unit * a.unit_cost;
    const float *slot0 = a.ws + (size_t(2) * pf + (pf_starts_here ? 0 : 1)) * slot_floats<D>();
    const size_t slot_step = size_t(2) * slot_floats<D>();    // every later workgroup starts inside the unit: slot 0
    const float *first_later = a.ws + size_t(2) * (pf + 1) * slot_floats<D>();
    float m = slot0[row];
    for (uint32_t p = pf + 1; p <= pl; ++p) m = fmaxf(m, first_later[(p - pf - 1) * slot_step + row]);
    float l = 0.0f, acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
    for (uint32_t p = pf; p <= pl; ++p) {
        const float *slot = p == pf ? slot0 : first_later + (p - pf - 1) * slot_step;
        const float f = __builtin_amdgcn_exp2f(slot[row] - m);
        l += slot[kBM + row] * f;
        const uint4 *src = reinterpret_cast<const uint4 *>(reinterpret_cast<const __bf16 *>(slot + 2 * kBM) + row * D + ch * 16);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const uint4 x = src[e];
            const uint32_t wds[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {     // a bf16 is the upper half of the binary32 of the same value
                acc[8 * e + 2 * j + 0] += __uint_as_float(wds[j] << 16) * f;
                acc[8 * e + 2 * j + 1] += __uint_as_float(wds[j] & 0xffff0000u) * f;
            }
        }
    }
    const float inv = 1.0f / l;
    union { uint4 u[2]; bf16x2 p[8]; } ow;
#pragma unroll
    for (int e = 0; e < 8; ++e) ow.p[e] = to_bf16x2(acc[2 * e] * inv, acc[2 * e + 1] * inv);
    uint4 *dst = reinterpret_cast<uint4 *>(a.o + head_offset(a, head) + int64_t(qi) * a.stride_tok + ch * 16);
    dst[0] = ow.u[0];
    dst[1] = ow.u[1];
}

// Compute units of the current device (each host thread remembers the last device it asked about).
int device_compute_units(int *device = nullptr) {
    static thread_local int cached_dev = -1, cached_cus = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (dev != cached_dev) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached_cus = cus;
        cached_dev = dev;
    }
    if (device != nullptr) *device = dev;
    return cached_cus;
}

template <int D>
int64_t workspace_bytes_for(int cus) { return int64_t(2) * cus * slot_floats<D>() * int64_t(sizeof(float)); }

template <int D, int NB>
int launch(AttnParams a, int heads, void *workspace, int64_t workspace_bytes, hipStream_t stream) {
    // The dynamic-LDS limit is an attribute of the function on a device: set once per device
    // (a repeated set by a racing host thread is harmless).
    static std::atomic<uint64_t> attr_set{0};
    const void *kern = reinterpret_cast<const void *>(&attention_kernel<D, NB>);
    int dev = 0;
    const int cus = device_compute_units(&dev);
    const uint64_t dev_bit = dev < 64 ? (uint64_t(1) << dev) : 0;
    if ((attr_set.load(std::memory_order_relaxed) & dev_bit) == 0) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, Tile<D, NB>::kBytes);
        if (e != hipSuccess) {
            lp::set_last_hip_error(int(e));
            return LP_ERR_HIP;
        }
        attr_set.fetch_or(dev_bit, std::memory_order_relaxed);
    }
    a.n_qtiles = (a.n + kBM - 1) / kBM;
    a.tiles_per_unit = (a.n + kBN - 1) / kBN;
    const uint32_t units = uint32_t(a.n_qtiles) * uint32_t(heads), tpu = uint32_t(a.tiles_per_unit);
    // default: one workgroup per unit, nothing shared
    uint32_t n_wg = units;
    a.ws = nullptr;
    a.shared_units = 0;
    a.whole_rounds = 1;
    a.shared_work = 0;
    a.unit_cost = tpu;
    a.shared_wgs = 0;
    if (workspace != nullptr && cus > 0 && workspace_bytes >= workspace_bytes_for<D>(cus)) {
        // Candidate: one workgroup per compute unit takes floor(units / #CU) rounds of whole
        // units, and the units left over are shared evenly by as many workgroups as get at least
        // kMinTiles tiles each.  Costs in units of one tile's time: a workgroup that starts or
        // ends inside a unit pays a second prologue and a partial store, and the merge kernel
        // follows.
        constexpr uint32_t kMinTiles = 8, kSplitCost = 6, kMergeCost = 3;
        static_assert(kBoundaryTiles < kMinTiles, "a range of kMinTiles positions must hold a real tile");
        const uint32_t p = units < uint32_t(cus) ? units : uint32_t(cus);     // workgroups
        const uint32_t rounds = units >= uint32_t(cus) ? units / p : 0;       // whole-unit rounds
        const uint32_t shared = units - rounds * p;
        if (shared > 0) {
            uint32_t sharers = shared * tpu / kMinTiles;                      // never more than tiles
            if (sharers > uint32_t(cus)) sharers = uint32_t(cus);
            if (sharers > shared || rounds > 0) {                             // else sharing adds no parallelism
                if (sharers < 1) sharers = 1;
                const uint32_t wgs = rounds > 0 ? p : sharers;
                const uint32_t t_plain = ((units + cus - 1) / cus) * tpu;
                const uint32_t t_split = rounds * tpu + (shared * tpu + sharers - 1) / sharers + kSplitCost + kMergeCost;
                if (t_split < t_plain) {
                    n_wg = wgs;
                    a.ws = static_cast<float *>(workspace);
                    a.shared_units = int(shared);
                    a.whole_rounds = int(rounds);
                    a.unit_cost = tpu + kBoundaryTiles;
                    a.shared_work = shared * a.unit_cost;
                    a.shared_wgs = sharers;
                }
            }
        }
    }
    int rc = lp::launch_kernel(kern, dim3(n_wg), dim3(waves_of(NB) * 64), Tile<D, NB>::kBytes, stream, a);
    if (rc != LP_OK || a.ws == nullptr) return rc;
    return lp::launch_kernel(reinterpret_cast<const void *>(&combine_kernel<D>), dim3(uint32_t(a.shared_units), kBM / 32),
                             dim3(32 * (D / 16)), 0, stream, a, a.shared_wgs);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

extern "C" int64_t lp_attention_workspace_size(int32_t head_dim) {
    if (head_dim != 64 && head_dim != 128) return LP_ERR_UNSUPPORTED;
    const int cus = device_compute_units();
    if (cus <= 0) return LP_ERR_HIP;
    return head_dim == 128 ? workspace_bytes_for<128>(cus) : workspace_bytes_for<64>(cus);
}

namespace {

// Argument checks shared by the entry points; no HIP call.  LP_OK: launch; kNothingToDo: succeed
// without a launch; negative: the error to return.
constexpr int kNothingToDo = 1;

int attention_check(const void *q, const void *k, const void *v, void *o, int32_t batch, int64_t n_tokens, int32_t heads,
                    int32_t head_dim, int64_t stride_batch, int64_t stride_tok, int64_t stride_head,
                    void *workspace, int64_t workspace_bytes) {
    if (n_tokens < 0 || heads < 1 || batch < 1) return LP_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return LP_ERR_UNSUPPORTED;
    if (n_tokens == 0) return kNothingToDo;
    if (q == nullptr || k == nullptr || v == nullptr || o == nullptr) return LP_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return LP_ERR_INVALID_ARG;
    if (o == q || o == k || o == v) return LP_ERR_INVALID_ARG;   // the output is written while inputs are still read
    if (workspace != nullptr && (!aligned16(workspace) || workspace_bytes < 0)) return LP_ERR_INVALID_ARG;
    if (stride_head < head_dim || stride_head % 8 != 0 || stride_tok % 8 != 0) return LP_ERR_INVALID_ARG;
    // rows of different (token, head) pairs must not overlap: either token-major or head-major
    const bool token_major = stride_tok >= int64_t(heads) * stride_head;
    const bool head_major = stride_head >= n_tokens * stride_tok && stride_tok >= head_dim;
    if (!token_major && !head_major) return LP_ERR_INVALID_ARG;
    if (batch > 1) {
        // items one after the other, or (token-major) the items of a token side by side
        if (stride_batch < 0 || stride_batch % 8 != 0) return LP_ERR_INVALID_ARG;
        const int64_t item = token_major ? n_tokens * stride_tok : int64_t(heads) * stride_head;
        const bool outer = stride_batch >= item;
        const bool inner = stride_tok >= int64_t(batch) * stride_batch && stride_batch >= int64_t(heads) * stride_head;
        if (!outer && !inner) return LP_ERR_INVALID_ARG;
    }
    // 32-bit addressing inside one head: byte offsets below 2^31, work items below 2^31
    if (n_tokens > (int64_t(1) << 24) || (n_tokens * stride_tok + head_dim) * 2 >= (int64_t(1) << 31)) return LP_ERR_UNSUPPORTED;
    const int64_t all_heads = int64_t(batch) * heads;
    if (all_heads >= (int64_t(1) << 24)) return LP_ERR_UNSUPPORTED;
    const int64_t units = all_heads * ((n_tokens + kBM - 1) / kBM);
    if (units * ((n_tokens + kBN - 1) / kBN + kBoundaryTiles) >= (int64_t(1) << 31)) return LP_ERR_UNSUPPORTED;
    return LP_OK;
}

int attention_call(const void *q, const void *k, const void *v, void *o, int32_t batch, int64_t n_tokens, int32_t heads,
                   int32_t head_dim, int64_t stride_batch, int64_t stride_tok, int64_t stride_head, float scale,
                   void *workspace, int64_t workspace_bytes, void *stream) {
    const int chk = attention_check(q, k, v, o, batch, n_tokens, heads, head_dim, stride_batch, stride_tok, stride_head,
                                    workspace, workspace_bytes);
    if (chk != LP_OK) return chk == kNothingToDo ? LP_OK : chk;
    const int64_t all_heads = int64_t(batch) * heads;
    if (!(scale > 0.0f)) scale = 1.0f / sqrtf(float(head_dim));
    AttnParams a{};
    a.q = static_cast<const __bf16 *>(q);
    a.k = static_cast<const __bf16 *>(k);
    a.v = static_cast<const __bf16 *>(v);
    a.o = static_cast<__bf16 *>(o);
    a.stride_tok = stride_tok;
    a.stride_head = stride_head;
    a.stride_batch = batch > 1 ? stride_batch : 0;
    a.heads = heads;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.n = int(n_tokens);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (head_dim == 128) return launch<128, blocks_per_wave(128)>(a, int(all_heads), workspace, workspace_bytes, st);
    return launch<64, blocks_per_wave(64)>(a, int(all_heads), workspace, workspace_bytes, st);
}

}  // namespace

// ---- scratch for callers that cannot allocate (lp_attention_static)
// Sized for the partial-result slots of head_dim 128 on kStaticMaxCUs compute units (the
// largest case; head_dim 64 needs less).  Every device the library runs on holds its own copy
// of this array, at its own address, until the process ends.  In host code the array's name
// is only a handle for hipGetSymbolAddress: kernels are given the address that call returns.
constexpr int kStaticMaxCUs = 256;
constexpr size_t kStaticScratchFloats = size_t(2) * kStaticMaxCUs * slot_floats<128>();
static __device__ __align__(256) float scratch[kStaticScratchFloats];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<float *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device; looked up once per device, with that
// device current.  Returns nullptr (and records the HIP error) on failure.
float *static_scratch(int *status) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        lp::set_last_hip_error(int(e));
        *status = LP_ERR_HIP;
        return nullptr;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        *status = LP_ERR_LIMIT;
        return nullptr;
    }
    float *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void *sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess || sym == nullptr) {
            lp::set_last_hip_error(int(e));
            *status = LP_ERR_HIP;
            return nullptr;
        }
        p = static_cast<float *>(sym);
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // a racing thread stores the same address
    }
    *status = LP_OK;
    return p;
}

}  // namespace

extern "C" int64_t lp_attention_static_scratch_bytes(void) { return int64_t(kStaticScratchFloats * sizeof(float)); }

extern "C" int lp_attention_static(const void *q, const void *k, const void *v, void *o, int64_t n_tokens,
                                   int32_t heads, int32_t head_dim, int64_t stride_tok, int64_t stride_head,
                                   float scale, void *stream) {
    const int chk = attention_check(q, k, v, o, 1, n_tokens, heads, head_dim, 0, stride_tok, stride_head, nullptr, 0);
    if (chk != LP_OK) return chk == kNothingToDo ? LP_OK : chk;
    const int cus = device_compute_units();
    if (cus <= 0) return LP_ERR_HIP;
    // the slots of every compute unit must fit the fixed array
    const int64_t need = head_dim == 128 ? workspace_bytes_for<128>(cus) : workspace_bytes_for<64>(cus);
    if (need > int64_t(kStaticScratchFloats * sizeof(float))) return LP_ERR_LIMIT;
    int status = LP_OK;
    float *ws = static_scratch(&status);
    if (ws == nullptr) return status;
    return attention_call(q, k, v, o, 1, n_tokens, heads, head_dim, 0, stride_tok, stride_head, scale, ws, need, stream);
}

extern "C" int lp_attention(const void *q, const void *k, const void *v, void *o, int64_t n_tokens,
                            int32_t heads, int32_t head_dim, int64_t stride_tok, int64_t stride_head,
                            float scale, void *workspace, int64_t workspace_bytes, void *stream) {
    return attention_call(q, k, v, o, 1, n_tokens, heads, head_dim, 0, stride_tok, stride_head, scale, workspace,
                          workspace_bytes, stream);
}

extern "C" int lp_attention_batch(const void *q, const void *k, const void *v, void *o, int32_t batch, int64_t n_tokens,
                                  int32_t heads, int32_t head_dim, int64_t stride_batch, int64_t stride_tok,
                                  int64_t stride_head, float scale, void *workspace, int64_t workspace_bytes,
                                  void *stream) {
    return attention_call(q, k, v, o, batch, n_tokens, heads, head_dim, stride_batch, stride_tok, stride_head, scale,
                          workspace, workspace_bytes, stream);
}
