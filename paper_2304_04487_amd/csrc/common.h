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
__device__ __forceinline__ f32x4 mfma16x16x32(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ---- tiled weight layout (bf16) ------------------------------------------------------------
// A row-major matrix W[N][K] (N % 16 == 0, K % 32 == 0) is stored as N/16 x K/32 blocks of
// 1 KiB.  Block (ft, ks) holds W[16 ft .. 16 ft+15][32 ks .. 32 ks+31]; inside it lane l of a
// wavefront owns 16 contiguous bytes: W[16 ft + l%16][32 ks + 8 (l/16) .. +7].  That is the
// A-operand register image of v_mfma_f32_16x16x32_bf16, so a wavefront fetches one block
// with a single fully coalesced 16-byte-per-lane load and feeds it to the MFMA unchanged.

// ---- KV cache layout (bf16), per (slot, head): max_seq x head_dim elements -------------------
// K: groups of 16 positions; group g16 holds head_dim/32 blocks of 1 KiB, block s = the
//    A-operand image of K[16 g16 .. +15][32 s .. 32 s+31] (lane l: position l%16, dims 8(l/16)..).
// V: groups of 32 positions; group g32 holds head_dim/16 blocks of 1 KiB, block dt = the
//    A-operand image of V^T[16 dt .. +15][32 positions], where slot (kb, j) of the 32-wide
//    reduction axis is position  16 (j/4) + 4 kb + j%4  of the group: exactly the order in
//    which the score MFMAs leave probabilities in a lane's registers.
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
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };

struct GemmArgs {
    const void *W;          // tiled bf16 weights, or row-major fp32 weights
    const void *Xhi;        // activations [rows_pad][K]: bf16 hi part, or fp32
    const void *Xlo;        // bf16 lo part (bf16 path with split), else unused
    int N, K;               // logical output features (for SWIGLU: d_ffn), reduction length
    int rows;               // valid rows
    int epi;
    float *out;             // STORE: [rows][N] fp32; RESID: h[rows][N] += ; LMHEAD: optional logits dump (may be null)
    void *act_hi, *act_lo;  // SWIGLU: [rows_pad][N] bf16 hi/lo, or fp32 in act_hi
    float *pval; int *pidx; // LMHEAD: per-row partial arg max [rows][n_part]
    int n_part;
    int split;              // use Xlo
};

struct AttnArgs {
    const void *Q;          // [R][d_model] bf16 (rotated) or fp32
    const void *Kc, *Vc;    // this layer's cache base
    const int *T;           // [max_batch] device lengths before the step
    const int *batch_slots; // [n_seqs]
    int n_seqs, m;          // rows per sequence
    int H, dh, max_seq;
    int n_chunks;           // launched chunks (upper bound over the batch)
    float scale;
    float *po, *pm, *pl;    // partials
    void *out_hi, *out_lo;  // [R_pad][d_model] bf16 hi/lo or fp32
    int split;
};

#define ATTN_CHUNK 256      // key positions per workgroup (4 waves x 2 groups of 32)
