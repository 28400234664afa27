// The DiT-block operations on either side of the attention core, for gfx950:
//
//   lp_qkv_projection   y = x W^T + b cut into q | k | v, with the per-head RMS normalisation
//                       and the 3-D rotary encoding of q and k done in the product's epilogue
//   lp_linear           y = x W^T + b (the block's output projection)
//   lp_qk_norm_rope     the normalisation + rotation alone, in place, for q / k that were
//                       projected elsewhere
//
// The paper leaves the block's internals open (Sec. 5.1: 30 DiT blocks whose atomic units are
// the patches of Sec. 3.1); the form taken is stated in include/lp.h.
//
// The product is computed TRANSPOSED, C^T[feature, token] = W . X^T with bf16 MFMA 32x32x16
// (A = rows of W, B = rows of x, both k-contiguous, both streamed global -> LDS without
// passing through registers): in the accumulator layout a lane then holds 64 features of ONE
// token, so the sum of squares of a head is an in-lane sum plus one exchange with the other
// half-wave, and the two elements of a rotary pair sit in neighbouring registers.
//
// Work decomposition.  A workgroup (8 wavefronts, two per SIMD) owns 256 features x 256
// tokens; a wavefront 128 features (one head of 128, or two of 64) x 64 tokens: 4 x 2 MFMA
// blocks, 128 accumulator registers, 6 LDS operand reads per 8 products.  k advances in tiles
// of 64 through two LDS stages (W tile + x tile, 64 KB per stage).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>

#include "lp_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define LP_LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int kTF = 256;                 // features per workgroup
constexpr int kTT = 256;                 // tokens per workgroup
constexpr int kBK = 64;                  // k per LDS stage
constexpr int kRowBytes = kBK * 2;       // one tile row: 64 bf16
constexpr int kTileBytes = 256 * kRowBytes;      // W tile or x tile: 32 KB
constexpr int kStageBytes = 2 * kTileBytes;      // W tile then x tile
constexpr int kStagesG = 2;
constexpr int kLdsBytes = kStagesG * kStageBytes;
constexpr int kThreadsG = 512;
constexpr int kPanel = 4;                // token tiles per panel of the tile order
constexpr int kMaxPairs = 64;            // rotary pairs per head (head_dim <= 128)

// floor(n / d) for 0 <= n < 2^31 as (n * magic) >> shift (64-bit product); see make_fastdiv.
struct FastDiv {
    uint32_t magic, shift, d;
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

// What the normalisation + rotation needs besides the data.
struct RopeArgs {
    float turns[kMaxPairs][4];   // pair p: turns (angle / 2 pi) per unit of the t, h, w coordinate; [3] unused
    FastDiv hw, w;               // grid_h * grid_w and grid_w
    int32_t grid_h;
    int32_t off[3];
    float eps;
};

struct GemmArgs {
    const __bf16 *x, *w;
    const float *bias;           // [d_out] or nullptr
    __bf16 *out[3];              // plain: out[0] = y [n, d_out]; qkv: q, k, v [n, heads, head_dim]
    const float *gain[2];        // qkv: gain_q, gain_k [heads, head_dim]
    int32_t n, d_in, d_out;
    int32_t heads;               // qkv: heads; d_out = 3 * heads * head_dim
    int32_t n_ftiles, n_ttiles;
    RopeArgs rope;
};

__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

__device__ __forceinline__ bf16x2 to_bf16x2(float lo, float hi) {
    f32x2 f = {lo, hi};
    return __builtin_convertvector(f, bf16x2);
}

template <typename V>
__device__ __forceinline__ V lds_load(uint32_t addr) {
    return *LP_LDS_PTR(const V, uintptr_t(addr));
}

// granule XOR mask of a tile row (reader and writer use the same function): with 128-byte rows
// the 16-byte granule g of row r lives at position g ^ swz(r), which makes the ds_read_b128 of
// 32 rows x one granule free of bank conflicts
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// One wave-wide global -> LDS load of 1024 bytes (see lp_attention.hip for why this is an
// assembly statement): lane L's 16 bytes at byte offset voff + soff of the buffer land at
// lds_addr + 16 L; bytes outside the buffer arrive as zeros.
__device__ __forceinline__ void load_to_lds_16(__amdgpu_buffer_rsrc_t rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}

__device__ __forceinline__ void wait_all_tile_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Workgroup ids are dealt round robin to the 8 XCDs; remap so that each XCD owns a contiguous
// stretch of the tile order (see the panels in gemm_kernel) and what neighbouring tiles share
// stays in one XCD's L2.
__device__ __forceinline__ uint32_t logical_workgroup(uint32_t b, uint32_t n_wg) {
    const uint32_t xcd = b % 8, slot = b / 8;
    const uint32_t base = n_wg / 8, rem = n_wg % 8;
    return xcd * base + (xcd < rem ? xcd : rem) + slot;
}

// One matrix instruction, acc += a . b, as an assembly statement: such statements keep their
// program order, and the LDS reads written between them stay between them.  The compiler does
// not know what the statement is and adds no wait states after it: settle() stands between the
// last product and the first vector instruction that reads an accumulator.
__device__ __forceinline__ void mfma(f32x16 &acc, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void settle(f32x16 (&acc)[4][2]) {
    asm volatile("s_nop 15\n\ts_nop 7");
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) asm volatile("" : "+v"(acc[mb][nb]));
}

// Writes 32 result rows (tokens) of 128 features, rounded to bf16, to dst + r * row_stride
// (r < rows_valid).  A lane holds, for token `col`, features 32 mb + 8 (i / 4) + 4 half + i % 4;
// the 8-byte pieces pass through 4 KB of the wave's LDS (64 features at a time, granules XORed
// with the row) and leave as whole 128-byte lines.
__device__ __forceinline__ void store_rows(uint32_t out_lds, const float (&val)[4][16], __bf16 *dst, int64_t row_stride,
                                           int rows_valid, int lane) {
    const int col = lane % 32, half = lane / 32;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int mbl = 0; mbl < 2; ++mbl)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float (&x)[16] = val[2 * pass + mbl];
                union { u32x2 u; bf16x2 p[2]; } ow;
                ow.p[0] = to_bf16x2(x[4 * g + 0], x[4 * g + 1]);
                ow.p[1] = to_bf16x2(x[4 * g + 2], x[4 * g + 3]);
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

// Per-head RMS normalisation and rotary encoding of the 128 features x 32 tokens a wave holds
// in val (layout as store_rows).  HD = 128: the 128 features are one head; HD = 64: two heads
// (blocks 0-1 and 2-3).  gain points at the first of these features; tk is this lane's token.
// The rotary table sits in LDS at rope_lds: float4 per pair.
template <int HD>
__device__ __forceinline__ void norm_rope(float (&val)[4][16], const float *gain, const RopeArgs &r, uint32_t rope_lds,
                                          uint32_t tk, int half) {
    // coordinates of this lane's token
    const uint32_t t = fastdiv(tk, r.hw);
    const uint32_t rem = tk - t * r.hw.d;
    const uint32_t h = fastdiv(rem, r.w);
    const float pt = float(int32_t(t) + r.off[0]), ph = float(int32_t(h) + r.off[1]),
                pw = float(int32_t(rem - h * r.w.d) + r.off[2]);
    constexpr int kHeads = 128 / HD, kBlocks = HD / 32;
#pragma unroll
    for (int hh = 0; hh < kHeads; ++hh) {
        float ss = 0.0f;
#pragma unroll
        for (int b = 0; b < kBlocks; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) ss += val[hh * kBlocks + b][i] * val[hh * kBlocks + b][i];
        ss += other_half(ss);
        const float inv = 1.0f / sqrtf(ss * (1.0f / float(HD)) + r.eps);
#pragma unroll
        for (int b = 0; b < kBlocks; ++b) {
            const int mb = hh * kBlocks + b;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // features 32 mb + 8 g + 4 half + 0..3 of the wave's 128: two rotary pairs
                const int f_local = 32 * b + 8 * g + 4 * half;             // inside the head
                const float4 gn = *reinterpret_cast<const float4 *>(gain + hh * HD + f_local);
                const float gv[4] = {gn.x, gn.y, gn.z, gn.w};
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    const f32x4 tb = lds_load<f32x4>(rope_lds + 16 * (f_local / 2 + pr));
                    float turns = pt * tb.x + ph * tb.y + pw * tb.z;
                    turns = turns - floorf(turns);
                    const float c = __builtin_amdgcn_cosf(turns), s = __builtin_amdgcn_sinf(turns);
                    const float a = val[mb][4 * g + 2 * pr] * inv * gv[2 * pr];
                    const float bb = val[mb][4 * g + 2 * pr + 1] * inv * gv[2 * pr + 1];
                    val[mb][4 * g + 2 * pr] = a * c - bb * s;
                    val[mb][4 * g + 2 * pr + 1] = a * s + bb * c;
                }
            }
        }
    }
}

// QKV = true: the epilogue cuts the features into q | k | v sections of heads * HD, normalises
// and rotates q and k.  QKV = false: plain y = x W^T + b.
template <bool QKV, int HD>
__global__ __launch_bounds__(kThreadsG) void gemm_kernel(const GemmArgs a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const uint32_t lds0 = uint32_t(uintptr_t(LP_LDS_PTR(unsigned char, smem)));
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int lane = tid % 64, col = lane % 32, half = lane / 32;
    const int fw = wave / 4, tq = wave % 4;              // feature half, token quarter of the workgroup tile

    // Tiles are ordered in panels of kPanel token tiles, feature tile by feature tile inside a
    // panel: the 32 workgroups an XCD runs at a time then cover 8 feature tiles x 4 token tiles
    // and share their W and x rows through its L2 (12 operand tiles fetched for 32 products).
    const uint32_t lw = logical_workgroup(blockIdx.x, gridDim.x);
    const int panel_tiles = kPanel * a.n_ftiles;
    const int panel = int(lw) / panel_tiles, in_panel = int(lw) - panel * panel_tiles;
    const int panel_h = min(kPanel, a.n_ttiles - panel * kPanel);
    const int ftile = in_panel / panel_h, ttile = panel * kPanel + in_panel - ftile * panel_h;
    const int f0 = ftile * kTF, t0 = ttile * kTT;

    // raw buffers over the rows this tile can touch (rows past the end read as zeros)
    const int64_t w_rows = min(int64_t(kTF), int64_t(a.d_out) - f0), x_rows = min(int64_t(kTT), int64_t(a.n) - t0);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__bf16 *>(a.w + int64_t(f0) * a.d_in), 0, int(w_rows * a.d_in * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__bf16 *>(a.x + int64_t(t0) * a.d_in), 0, int(x_rows * a.d_in * 2), 0x00020000);

    // this lane's part of the tile traffic: 4 wave-wide loads per operand tile and stage
    uint32_t voff[4], ld_dst[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int instr = wave + 8 * i;                  // 32 instructions of 8 rows per operand tile
        const int row = instr * 8 + lane / 8, gran = lane % 8;
        ld_dst[i] = instr * 1024;
        voff[i] = uint32_t(row) * uint32_t(a.d_in * 2) + 16 * (gran ^ swz(row));
    }
    auto issue = [&](int kt, uint32_t stage_off) {
        const uint32_t soff = uint32_t(kt) * kRowBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + stage_off + ld_dst[i]);
            load_to_lds_16(w_rsrc, dst, voff[i], soff);
            load_to_lds_16(x_rsrc, dst + kTileBytes, voff[i], soff);
        }
    };

    // LDS operand addresses in stage 0: A = W rows (4 blocks of 32 features), B = x rows (2 blocks of 32 tokens)
    uint32_t a_addr[4], b_addr[2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
        const int row = fw * 128 + mb * 32 + col;
        a_addr[mb] = lds0 + row * kRowBytes + 16 * (half ^ swz(row));       // granule 2 s + half is (2 s) ^ ... below
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int row = tq * 64 + nb * 32 + col;
        b_addr[nb] = lds0 + kTileBytes + row * kRowBytes + 16 * (half ^ swz(row));
    }

    f32x16 acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.0f;

    const int n_kt = a.d_in / kBK;
    issue(0, 0);
    for (int kt = 0; kt < n_kt; ++kt) {
        const uint32_t stage = (kt & 1) * kStageBytes;
        wait_all_tile_loads();
        __syncthreads();          // stage kt has landed for everyone; everyone has left the other stage
        if (kt + 1 < n_kt) issue(kt + 1, kStageBytes - stage);
        // Operands of k-step s+1 are fetched from LDS while the products of step s run: two
        // register sets, one fetch after each of the first six products of a step.  The products
        // are assembly statements so that this order stands (left to the scheduler, an operand is
        // fetched right before its two products and the wave sits out the LDS latency every time);
        // LDS reads keep their place between such statements.
        // granule (2 s + half) ^ swz(row) = (half ^ swz(row)) ^ (2 s): a step flips bits 1-2 of the granule index
        bf16x8 aop[2][4], bop[2][2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) bop[0][nb] = lds_load<bf16x8>(b_addr[nb] + stage);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) aop[0][mb] = lds_load<bf16x8>(a_addr[mb] + stage);
#pragma unroll
        for (int s = 0; s < kBK / 16; ++s) {
            const int cur = s & 1, nxt = cur ^ 1;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int mb = i / 2, nb = i % 2;
                mfma(acc[mb][nb], aop[cur][mb], bop[cur][nb]);
                if (s + 1 < kBK / 16) {
                    if (i < 2) bop[nxt][i] = lds_load<bf16x8>((b_addr[i] + stage) ^ uint32_t(32 * (s + 1)));
                    else if (i < 6) aop[nxt][i - 2] = lds_load<bf16x8>((a_addr[i - 2] + stage) ^ uint32_t(32 * (s + 1)));
                }
            }
        }
    }
    settle(acc);

    // ---- epilogue; the tile ring is free once every wave has left it
    __syncthreads();
    const uint32_t out_lds = lds0 + wave * 4096;
    const uint32_t rope_lds = lds0 + 8 * 4096;
    if (QKV) {
        if (tid < kMaxPairs)
            *LP_LDS_PTR(f32x4, uintptr_t(rope_lds + 16 * tid)) =
                f32x4{a.rope.turns[tid][0], a.rope.turns[tid][1], a.rope.turns[tid][2], 0.0f};
        __syncthreads();
    }
    const int fbase = f0 + fw * 128;                     // first of this wave's 128 features
    if (fbase >= a.d_out) return;
    int section = 0, f_in_section = fbase;
    if (QKV) {
        const int dm = a.heads * HD;
        section = fbase / dm;
        f_in_section = fbase - section * dm;
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int tok_first = t0 + tq * 64 + nb * 32;    // first token of this 32-token block
        if (tok_first >= a.n) break;
        float val[4][16];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float bv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (a.bias != nullptr) {
                    const int f = fbase + 32 * mb + 8 * g + 4 * half;
                    if (f + 3 < a.d_out) {
                        const float4 b4 = *reinterpret_cast<const float4 *>(a.bias + f);
                        bv[0] = b4.x; bv[1] = b4.y; bv[2] = b4.z; bv[3] = b4.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) if (f + e < a.d_out) bv[e] = a.bias[f + e];
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) val[mb][4 * g + e] = acc[mb][nb][4 * g + e] + bv[e];
            }
        }
        __bf16 *dst;
        int64_t row_stride;
        if (QKV) {
            if (section < 2) norm_rope<HD>(val, a.gain[section] + f_in_section, a.rope, rope_lds, uint32_t(min(tok_first + col, a.n - 1)), half);
            row_stride = int64_t(a.heads) * HD;
            dst = a.out[section] + int64_t(tok_first) * row_stride + f_in_section;
        } else {
            row_stride = a.d_out;
            dst = a.out[0] + int64_t(tok_first) * row_stride + fbase;
        }
        store_rows(out_lds, val, dst, row_stride, a.n - tok_first, lane);
    }
}

// Normalisation + rotation alone, in place: one thread per 8 consecutive features of a
// (token, head) row, HD / 8 threads per row.
template <int HD>
__global__ __launch_bounds__(256) void norm_rope_kernel(__bf16 *x, const float *gain, int64_t n, int32_t heads,
                                                        int64_t stride_tok, int64_t stride_head, const RopeArgs r) {
    __shared__ float4 table[kMaxPairs];
    if (threadIdx.x < kMaxPairs)
        table[threadIdx.x] = make_float4(r.turns[threadIdx.x][0], r.turns[threadIdx.x][1], r.turns[threadIdx.x][2], 0.0f);
    __syncthreads();
    constexpr int kPer = HD / 8;                          // threads per row
    const int64_t row = (int64_t(blockIdx.x) * 256 + threadIdx.x) / kPer;
    const int part = threadIdx.x % kPer;
    const bool live = row < n * heads;
    const int64_t rc = live ? row : 0;
    const int64_t tk = rc / heads;
    const int head = int(rc - tk * heads);
    __bf16 *p = x + tk * stride_tok + int64_t(head) * stride_head + part * 8;
    union { uint4 u; bf16x2 p[4]; } in;
    in.u = *reinterpret_cast<const uint4 *>(p);
    float v[8];
    const uint32_t wds[4] = {in.u.x, in.u.y, in.u.z, in.u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {      // a bf16 is the upper half of the binary32 with the same value
        v[2 * e] = __uint_as_float(wds[e] << 16);
        v[2 * e + 1] = __uint_as_float(wds[e] & 0xffff0000u);
    }
    float ss = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
#pragma unroll
    for (int m = 1; m < kPer; m *= 2) ss += __shfl_xor(ss, m, 64);
    const float inv = 1.0f / sqrtf(ss * (1.0f / float(HD)) + r.eps);
    const uint32_t t = fastdiv(uint32_t(tk), r.hw);
    const uint32_t rem = uint32_t(tk) - t * r.hw.d;
    const uint32_t h = fastdiv(rem, r.w);
    const float pt = float(int32_t(t) + r.off[0]), ph = float(int32_t(h) + r.off[1]), pw = float(int32_t(rem - h * r.w.d) + r.off[2]);
    const float *gr = gain + head * HD + part * 8;
    const float4 g0 = *reinterpret_cast<const float4 *>(gr), g1 = *reinterpret_cast<const float4 *>(gr + 4);
    const float gv[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    union { uint4 u; bf16x2 p[4]; } out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float4 tb = table[part * 4 + e];
        float turns = pt * tb.x + ph * tb.y + pw * tb.z;
        turns = turns - floorf(turns);
        const float c = __builtin_amdgcn_cosf(turns), s = __builtin_amdgcn_sinf(turns);
        const float a = v[2 * e] * inv * gv[2 * e], b = v[2 * e + 1] * inv * gv[2 * e + 1];
        out.p[e] = to_bf16x2(a * c - b * s, a * s + b * c);
    }
    if (live) *reinterpret_cast<uint4 *>(p) = out.u;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Fills the device-side rotary description; LP_OK or the error.
int make_rope_args(const lp_rope *rope, int64_t n, int32_t head_dim, float eps, RopeArgs *out) {
    if (rope == nullptr) return LP_ERR_INVALID_ARG;
    int64_t cells = 1;
    int32_t sum = 0;
    for (int ax = 0; ax < 3; ++ax) {
        if (rope->grid[ax] < 1 || rope->split[ax] < 0 || rope->split[ax] % 2 != 0) return LP_ERR_INVALID_ARG;
        cells *= rope->grid[ax];
        sum += rope->split[ax];
    }
    if (cells != n || sum != head_dim || !(rope->base > 0.0f) || !(eps >= 0.0f)) return LP_ERR_INVALID_ARG;
    if (n >= (int64_t(1) << 31)) return LP_ERR_UNSUPPORTED;
    RopeArgs r{};
    int pair = 0;
    for (int ax = 0; ax < 3; ++ax) {
        const int p = rope->split[ax];
        for (int j = 0; j < p / 2; ++j, ++pair) {
            // angle per unit coordinate base^(-2 j / p), stored in turns
            const double freq = std::pow(double(rope->base), -2.0 * double(j) / double(p));
            r.turns[pair][ax] = float(freq / (2.0 * M_PI));
        }
    }
    r.hw = make_fastdiv(uint32_t(rope->grid[1]) * uint32_t(rope->grid[2]));
    r.w = make_fastdiv(uint32_t(rope->grid[2]));
    r.grid_h = rope->grid[1];
    for (int ax = 0; ax < 3; ++ax) r.off[ax] = rope->offset[ax];
    r.eps = eps;
    *out = r;
    return LP_OK;
}

template <bool QKV, int HD>
int launch_gemm(GemmArgs a, hipStream_t stream) {
    static std::atomic<uint64_t> attr_set{0};
    const void *kern = reinterpret_cast<const void *>(&gemm_kernel<QKV, HD>);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        lp::set_last_hip_error(int(e));
        return LP_ERR_HIP;
    }
    const uint64_t dev_bit = dev < 64 ? (uint64_t(1) << dev) : 0;
    if ((attr_set.load(std::memory_order_relaxed) & dev_bit) == 0) {
        e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) {
            lp::set_last_hip_error(int(e));
            return LP_ERR_HIP;
        }
        attr_set.fetch_or(dev_bit, std::memory_order_relaxed);
    }
    a.n_ftiles = (a.d_out + kTF - 1) / kTF;
    a.n_ttiles = int32_t((a.n + kTT - 1) / kTT);
    const int64_t tiles = int64_t(a.n_ftiles) * a.n_ttiles;
    if (tiles >= (int64_t(1) << 31)) return LP_ERR_UNSUPPORTED;
    return lp::launch_kernel(kern, dim3(uint32_t(tiles)), dim3(kThreadsG), kLdsBytes, stream, a);
}

// shape limits of the product: k in whole tiles, 32-bit byte offsets inside a tile's rows
int check_gemm_shape(int64_t n, int32_t d_in, int32_t d_out) {
    if (n < 0 || d_in < 1 || d_out < 1) return LP_ERR_INVALID_ARG;
    if (d_in % kBK != 0 || d_out % 128 != 0) return LP_ERR_UNSUPPORTED;   // whole k tiles; a wave stores 128 features per token
    if (int64_t(256) * d_in * 2 >= (int64_t(1) << 31) || n >= (int64_t(1) << 31)) return LP_ERR_UNSUPPORTED;
    return LP_OK;
}

}  // namespace

extern "C" int lp_linear(const void *x, const void *w, const float *bias, void *y, int64_t n, int32_t d_in, int32_t d_out,
                         void *stream) {
    const int chk = check_gemm_shape(n, d_in, d_out);
    if (chk != LP_OK) return chk;
    if (n == 0) return LP_OK;
    if (x == nullptr || w == nullptr || y == nullptr) return LP_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(bias) || y == x || y == w) return LP_ERR_INVALID_ARG;
    GemmArgs a{};
    a.x = static_cast<const __bf16 *>(x);
    a.w = static_cast<const __bf16 *>(w);
    a.bias = bias;
    a.out[0] = static_cast<__bf16 *>(y);
    a.n = int32_t(n);
    a.d_in = d_in;
    a.d_out = d_out;
    return launch_gemm<false, 128>(a, static_cast<hipStream_t>(stream));
}

extern "C" int lp_qkv_projection(const void *x, const void *w_qkv, const float *bias, const float *gain_q, const float *gain_k,
                                 float eps, const lp_rope *rope, void *q, void *k, void *v, int64_t n_tokens, int32_t heads,
                                 int32_t head_dim, void *stream) {
    if (heads < 1) return LP_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return LP_ERR_UNSUPPORTED;
    const int64_t dm64 = int64_t(heads) * head_dim;
    if (3 * dm64 >= (int64_t(1) << 31)) return LP_ERR_UNSUPPORTED;
    const int32_t dm = int32_t(dm64);
    if (dm % 128 != 0) return LP_ERR_UNSUPPORTED;          // a wave's 128 features must not straddle q | k | v
    const int chk = check_gemm_shape(n_tokens, dm, 3 * dm);
    if (chk != LP_OK) return chk;
    if (n_tokens == 0) return LP_OK;
    if (x == nullptr || w_qkv == nullptr || gain_q == nullptr || gain_k == nullptr || q == nullptr || k == nullptr || v == nullptr)
        return LP_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_qkv) || !aligned16(bias) || !aligned16(gain_q) || !aligned16(gain_k) || !aligned16(q) ||
        !aligned16(k) || !aligned16(v))
        return LP_ERR_INVALID_ARG;
    if (q == k || q == v || k == v || q == x || k == x || v == x) return LP_ERR_INVALID_ARG;
    GemmArgs a{};
    const int rc = make_rope_args(rope, n_tokens, head_dim, eps, &a.rope);
    if (rc != LP_OK) return rc;
    a.x = static_cast<const __bf16 *>(x);
    a.w = static_cast<const __bf16 *>(w_qkv);
    a.bias = bias;
    a.out[0] = static_cast<__bf16 *>(q);
    a.out[1] = static_cast<__bf16 *>(k);
    a.out[2] = static_cast<__bf16 *>(v);
    a.gain[0] = gain_q;
    a.gain[1] = gain_k;
    a.n = int32_t(n_tokens);
    a.d_in = dm;
    a.d_out = 3 * dm;
    a.heads = heads;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return head_dim == 128 ? launch_gemm<true, 128>(a, st) : launch_gemm<true, 64>(a, st);
}

extern "C" int lp_qk_norm_rope(void *x, const float *gain, float eps, const lp_rope *rope, int64_t n_tokens, int32_t heads,
                               int32_t head_dim, int64_t stride_tok, int64_t stride_head, void *stream) {
    if (heads < 1 || n_tokens < 0) return LP_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return LP_ERR_UNSUPPORTED;
    if (n_tokens == 0) return LP_OK;
    if (x == nullptr || gain == nullptr || !aligned16(x) || !aligned16(gain)) return LP_ERR_INVALID_ARG;
    if (stride_head < head_dim || stride_head % 8 != 0 || stride_tok % 8 != 0) return LP_ERR_INVALID_ARG;
    const bool token_major = stride_tok >= int64_t(heads) * stride_head;
    const bool head_major = stride_head >= n_tokens * stride_tok && stride_tok >= head_dim;
    if (!token_major && !head_major) return LP_ERR_INVALID_ARG;
    RopeArgs r;
    const int rc = make_rope_args(rope, n_tokens, head_dim, eps, &r);
    if (rc != LP_OK) return rc;
    const int64_t threads = n_tokens * heads * (head_dim / 8);
    const int64_t blocks = (threads + 255) / 256;
    if (blocks >= (int64_t(1) << 31)) return LP_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const void *fn = head_dim == 128 ? reinterpret_cast<const void *>(&norm_rope_kernel<128>)
                                     : reinterpret_cast<const void *>(&norm_rope_kernel<64>);
    return lp::launch_kernel(fn, dim3(uint32_t(blocks)), dim3(256), 0, st, static_cast<__bf16 *>(x), gain, n_tokens, heads,
                             stride_tok, stride_head, r);
}
