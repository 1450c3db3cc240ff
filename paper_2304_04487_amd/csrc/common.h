// Shared device helpers and the argument structs passed from the host orchestration to the
// kernel launchers.  gfx950 (CDNA4) only: 64-wide wavefronts, MFMA 16x16x32 bf16.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef uint16_t bf16_t;                       // raw bfloat16 bit pattern

#define LLMA_NEG_INF (-__builtin_huge_valf())

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round-to-nearest-even; inputs are finite in this library
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
// x ~= hi + lo with hi = bf16(x), lo = bf16(x - hi): 16 significand bits kept
__device__ __forceinline__ void split_bf16(float x, bf16_t &hi, bf16_t &lo) {
    hi = f32_to_bf16(x);
    lo = f32_to_bf16(x - bf16_to_f32(hi));
}
__device__ __forceinline__ void split4(const float v[4], u32x2 &hi, u32x2 &lo) {
    bf16_t h[4], l[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) split_bf16(v[r], h[r], l[r]);
    hi = (u32x2){(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
    lo = (u32x2){(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
}
// ---- the 8-bit lo plane of the K/V cache ----------------------------------------------------
// A cached value x is kept as hi = bf16(x) plus lo = x - hi.  |lo| <= ulp(hi) / 2 = 2^-9 |x| at most, and four
// significant bits of it are enough (rounding lo to four bits costs a quarter of the logit tolerance at 32
// layers, rounding it away eleven times the tolerance), so the lo plane holds one byte per element:
// OCP fp8 e4m3 of 256 lo (|256 lo| <= |x|: saturates only for |x| > 448; spacing 2^-9 below 2^-6, i.e. lo is
// kept to 2^-17 absolutely).  The attention kernels widen it to bf16 (exactly) in registers.
__device__ __forceinline__ uint32_t lo8x2(float l0, float l1, uint32_t old, bool upper) {
    const float a = fminf(fmaxf(l0 * 256.f, -448.f), 448.f), b = fminf(fmaxf(l1 * 256.f, -448.f), 448.f);
    return upper ? (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, true)
                 : (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, false);
}
__device__ __forceinline__ uint32_t lo8x4(const float l[4]) { return lo8x2(l[2], l[3], lo8x2(l[0], l[1], 0u, false), true); }
__device__ __forceinline__ uint8_t lo8x1(float l) { return (uint8_t)(lo8x2(l, 0.f, 0u, false) & 0xffu); }
// eight lo bytes (one lane's share of a block) -> the eight bf16 values the MFMA takes
__device__ __forceinline__ u32x4 lo8_operand(u32x2 p) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    u32x4 r;
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const f32x2_t a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(p[w], 0.00390625f, false);
        const f32x2_t b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(p[w], 0.00390625f, true);
        r[2 * w] = (__float_as_uint(a.x) >> 16) | (__float_as_uint(a.y) & 0xffff0000u);      // (at most four significant
        r[2 * w + 1] = (__float_as_uint(b.x) >> 16) | (__float_as_uint(b.y) & 0xffff0000u);  //  bits: exact in bf16)
    }
    return r;
}
__device__ __forceinline__ f32x4 mfma16x16x32(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ---- tiled weight layout (bf16) ------------------------------------------------------------
// A row-major matrix W[N][K] (N % 16 == 0, K % 32 == 0) is stored as N/16 x KSp blocks of
// 1 KiB (KSp >= K/32 k-steps; blocks past K/32 are zero padding).  Block (ft, ks) holds
// W[16 ft .. 16 ft+15][32 ks .. 32 ks+31]; inside it lane l of a wavefront owns 16 contiguous
// bytes: W[16 ft + l%16][32 ks + 8 (l/16) .. +7].  That is the A-operand register image of
// v_mfma_f32_16x16x32_bf16, so a wavefront fetches one block with a single fully coalesced
// 16-byte-per-lane load and feeds it to the MFMA unchanged.
//
// ---- tiled activation layout (bf16) ---------------------------------------------------------
// Activations X[rows][K] that feed a GEMM are stored as the matching B-operand images, one
// plane for the hi part and one for the lo part of each value: block (t, ks) of 1 KiB holds rows
// 16 t .. 16 t+15, columns 32 ks .. +31; lane l owns X[16 t + l%16][32 ks + 8 (l/16) .. +7] and
// finds it in the block's 16-byte piece xtile_piece(l) = 4 (l%16) + l/16: the pieces of a row are
// adjacent (64 bytes), so a step with r live rows in a tile touches only the first 64 r bytes of
// each block (lanes of rows past the end do not load at all).
__host__ __device__ __forceinline__ int xtile_piece(int lane) { return ((lane & 15) << 2) | (lane >> 4); }
__host__ __device__ __forceinline__ size_t xtile_off(int row, int col, int KSp) {
    return ((size_t)((row >> 4) * KSp + (col >> 5)) * 64 + (size_t)((row & 15) * 4 + ((col & 31) >> 3))) * 8 + (col & 7);
}

// ---- KV cache layout (bf16), per (slot, head): max_seq x head_dim elements per plane ---------
// K: groups of 16 positions; group g16 holds head_dim/32 blocks of 1 KiB, block s = the
//    A-operand image of K[16 g16 .. +15][32 s .. 32 s+31] (lane l: position l%16, dims 8(l/16)..).
// V: groups of 32 positions; group g32 holds head_dim/16 blocks of 1 KiB, block dt = the
//    A-operand image of V^T[16 dt .. +15][32 positions], where slot (kb, j) of the 32-wide
//    reduction axis is position  16 (j/4) + 4 kb + j%4  of the group: exactly the order in
//    which the score MFMAs leave probabilities in a lane's registers.
// With kv_split the cache has a second plane of the same shape holding the lo parts.
__host__ __device__ __forceinline__ size_t kcache_off(int pos, int c, int dh) {
    int g16 = pos >> 4, i = pos & 15, s = c >> 5, kb = (c & 31) >> 3, j = c & 7;
    return (size_t)g16 * (16 * dh) + (size_t)s * 512 + (size_t)(kb * 16 + i) * 8 + j;
}
__host__ __device__ __forceinline__ size_t vcache_off(int pos, int c, int dh) {
    int g32 = pos >> 5, q = pos & 31, th = q >> 4, i16 = q & 15, kb = i16 >> 2, r = i16 & 3;
    int dt = c >> 4, i = c & 15;
    return (size_t)g32 * (32 * dh) + (size_t)dt * 512 + (size_t)(kb * 16 + i) * 8 + (th * 4 + r);
}

// ---- launcher argument structs --------------------------------------------------------------
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3, EPI_QKV = 4 };

// how one weight matrix is cut into work: a function of its shape only (never of the row count)
struct GemmPlan {
    int N, K;        // logical shape (SWIGLU: N = d_ffn, the matrix has 2N rows)
    int KSp;         // k-steps (of 32) per feature tile
    int tasks;       // feature tiles (SWIGLU: gate/up tile pairs)
    int tiles_per_task;   // 2 for the fused gate/up matrix, else 1
    int tk_ft[3];    // tile-K kernel: feature tiles (SWIGLU: pairs) per workgroup for 1, 2, 3 row tiles.  Work division
                     //   only -- every tile's sum is the same whatever the value -- so it may be tuned per device
    int tk_waves;    //   and K slices (= waves, or half as many waves taking two slices each): fixes the order of the sums
    int n_split;     // panel kernel, batched steps: ranges the K axis is cut into (1 = no split)
};

struct GemmArgs {          // bf16 path (fields marked f32 are used by the fp32 kernels only)
    const void *W;         // tiled bf16 weights, or row-major fp32 weights
    const void *Xhi;       // bf16: tiled activations, hi plane; f32: row-major [rows][K]
    const void *Xlo;       // bf16: lo plane
    GemmPlan plan;
    int N, K;              // f32: logical output features, reduction length
    int rows;              // valid rows
    int epi;
    int split;             // use Xlo
    // inputs of the epilogues
    const float *ssq_in;   // [rows][ssq_tiles] sums of squares of the producer's residual rows
    int ssq_tiles;         //   rstd[row] = rsqrt(sum / (16 ssq_tiles) + eps)
    float eps;
    const float *rstd_in;  // panel GEMM only: [rows] precomputed rstd (instead of ssq_in)
    float *rstd_out;       // panel GEMM, split-K form: if set, one extra workgroup computes every row's rstd from ssq_in into it (for the finishing kernel)
    const int *rows_live;  // tile-K GEMM only, may be null: device int, rows 0 .. *rows_live carry tokens (the rest of `rows` is padding)
    int panel_rb;          // panel GEMM only: row blocks (set by the launcher)
    int ksplit;            // panel GEMM only: > 1 = the K axis is cut into this many ranges of k-chunks, partial sums via `part`
    float *part;           //   [ksplit][tiles][row tiles][64 lanes x 4] fp32 partial sums (register images)
    // EPI_STORE (f32) / EPI_RESID / EPI_LMHEAD
    float *out;            // STORE: [rows][N]; RESID: h[rows][N] += ; LMHEAD: optional logits dump (may be null)
    // EPI_RESID: prepares the next RMSNorm'd GEMM input
    const float *gain;     // [N] gains of the next norm
    void *nx_hi, *nx_lo;   // tiled planes over N columns with nx_KSp k-steps per row tile: (h * gain) hi / lo
    int nx_KSp;
    float *ssq_out;        // [rows][N/16]
    // EPI_SWIGLU
    void *act_hi, *act_lo; // tiled planes over d_ffn (KSp of the down projection) ; f32: row-major in act_hi
    int act_KSp;
    // EPI_LMHEAD
    float *pval; int *pidx; int n_part;
    // EPI_QKV: rotate, write q (tiled planes over d_model), append k, v to the cache
    const int *row_pos, *row_slot;
    const float *row_cs;   // [rows][dh/2][2]: (cos, sin) of every row's position
    void *q_hi, *q_lo;
    void *k_hi, *k_lo, *v_hi, *v_lo;   // this layer's cache planes (lo may be null)
    int H, dh, max_seq;
};

struct AttnArgs {
    const void *Qhi, *Qlo;  // bf16: tiled planes over d_model; f32: Qhi = [R][d_model]
    const void *Khi, *Klo, *Vhi, *Vlo;   // this layer's cache (lo null without kv_split); f32: Khi, Vhi
    const int *T;           // [max_batch] device lengths before the step
    const int *batch_slots; // [n_seqs]
    int slot_const;         // >= 0: the single sequence's slot (saves a dependent load); -1: read batch_slots
    int n_seqs, m;          // rows per sequence
    int H, dh, max_seq;
    int n_chunks;           // launched chunks (upper bound over the batch); the partials' count per (sequence, head)
    int part_span;          // key positions one partial covers (ATTN_CHUNK, or a whole number of chunks); set by the launcher
    const int *rows_live;   // may be null: device int, rows 0 .. *rows_live of the (single) sequence carry tokens
    const int *lo_from;     // may be null: [max_batch] device ints, positions below lo_from[slot] have all-zero lo planes (imported bf16 caches)
    int n_rblocks;          // row blocks per sequence (set by the launcher)
    float scale;
    float *po, *pm, *pl;    // partials
    void *out_hi, *out_lo;  // bf16: tiled planes over d_model (out_KSp k-steps per row tile); f32: out_hi = [R][d_model]
    int out_KSp;
};

#define ATTN_CHUNK 128      // key positions per workgroup (4 waves x 32)
