// bf16 kernels of the verification forward (paper: Eq. 3 -- one causal forward over the
// pending token plus k copied tokens): weight re-tiling, the skinny weight-streaming GEMM
// with its fused epilogues (RMSNorm scaling, RoPE + KV append, SwiGLU, residual + next-norm
// preparation, vocabulary arg-max partials), and causal attention of a few query rows over a
// long KV cache.
//
// Everything here is HBM-bound at the row counts of a decoding step (1 + k <= 33 rows): the
// kernels are organised around streaming each weight / KV byte exactly once with fully
// coalesced 16-byte-per-lane loads, and use the MFMA unit because it consumes those
// registers directly.  Activations enter the MFMAs as hi + lo bf16 pairs (the extra MFMAs are
// free while memory-bound), which keeps 16 significand bits of every activation.
// Reduction orders are fixed by the matrix shapes and by absolute key positions, never by the
// number of rows in the step, so row j of a k-row step is bit-identical to the same token
// processed in a one-row step.
#include <stdlib.h>

#include <atomic>
#include <type_traits>
#include <utility>

#include "common.h"
#include "kernels.h"

// Kernels that use more than 64 KB of dynamic LDS need the limit raised once per device.  `done`
// (one per kernel instantiation) holds a bit per device id; concurrent first calls may both set the
// attribute, which is harmless.
static void allow_full_lds(const void *kernel, std::atomic<uint64_t> &done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 0;
    const uint64_t bit = 1ull << dev;
    if (done.load(std::memory_order_acquire) & bit) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    done.fetch_or(bit, std::memory_order_release);
}

// =============================================================================================
// weight re-tiling: row-major [N][K] bf16 -> 1 KiB MFMA A-operand blocks (see common.h)
// =============================================================================================
// rope_dh > 0 (the fused q/k/v matrix, d = model width): the 16 rows of a q or k tile are the
// rotary pairs (i, i + rope_dh/2) for 8 consecutive i -- rows 0..7 hold i, rows 8..15 hold
// i + rope_dh/2 -- so that the GEMM epilogue finds both elements of a pair in one wavefront.
__device__ __forceinline__ size_t src_row_of(size_t ft, int i, int rope_dh, int d) {
    if (rope_dh == 0) return ft * 16 + i;
    const int tiles_per_sec = d / 16;
    const int sec = (int)(ft / tiles_per_sec);
    if (sec == 2) return ft * 16 + i;
    const int tin = (int)(ft % tiles_per_sec);
    const int tph = rope_dh / 16;
    const int head = tin / tph, j = tin % tph;
    const int c = (i < 8) ? (8 * j + i) : (rope_dh / 2 + 8 * j + (i - 8));
    return (size_t)sec * d + (size_t)head * rope_dh + c;
}

__global__ void pack_weight_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int N, int K, int KSp,
                                   int rope_dh, int d) {
    // one thread per 16-byte piece of the destination
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)(N / 16) * KSp * 64;
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    size_t blk = idx >> 6;
    int ks = (int)(blk % KSp);
    size_t ft = blk / KSp;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (ks < K / 32) {
        size_t row = src_row_of(ft, lane & 15, rope_dh, d);
        size_t col = (size_t)ks * 32 + (size_t)(lane >> 4) * 8;
        v = src[(row * K + col) / 8];
    }
    dst[idx] = v;
}

void launch_pack_weight(const void *src, void *dst, int N, int K, int KSp, int rope_dh, int d, hipStream_t st) {
    size_t total = (size_t)(N / 16) * KSp * 64;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(pack_weight_kernel, dim3(blocks), dim3(256), 0, st, (const u32x4 *)src, (u32x4 *)dst, N, K, KSp, rope_dh, d);
}

// plain [H][len][dh] bf16 -> tiled K / V cache of one (slot, layer); lo planes (if any) are zeroed
__global__ void kv_import_bf16_kernel(const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                      bf16_t *__restrict__ kh, uint8_t *__restrict__ kl,
                                      bf16_t *__restrict__ vh, uint8_t *__restrict__ vl,
                                      int H, int len, int dh, int max_seq) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)H * len * dh;
    if (idx >= total) return;
    int c = (int)(idx % dh);
    int pos = (int)((idx / dh) % len);
    int h = (int)(idx / ((size_t)dh * len));
    size_t base = (size_t)h * max_seq * dh;
    size_t ko = base + kcache_off(pos, c, dh), vo = base + vcache_off(pos, c, dh);
    kh[ko] = k[idx];
    vh[vo] = v[idx];
    if (kl) { kl[ko] = 0; vl[vo] = 0; }
}

void launch_kv_import_bf16(const void *k, const void *v, void *kh, void *kl, void *vh, void *vl, int H, int len, int dh,
                           int max_seq, hipStream_t st) {
    size_t total = (size_t)H * len * dh;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(kv_import_bf16_kernel, dim3(blocks), dim3(256), 0, st, (const bf16_t *)k, (const bf16_t *)v,
                       (bf16_t *)kh, (uint8_t *)kl, (bf16_t *)vh, (uint8_t *)vl, H, len, dh, max_seq);
}

// =============================================================================================
// embedding gather + preparation of the first RMSNorm'd GEMM input
// =============================================================================================
// h[r] = E[tok_r]; x = h * gain as hi/lo tiled planes; per (row, 16-feature tile) sum of squares.
// One thread per 16-feature tile.
__global__ __launch_bounds__(256) void embed_prep_bf16_kernel(const bf16_t *__restrict__ embed, const int *__restrict__ row_tok,
                                                              const float *__restrict__ gain, float *__restrict__ h,
                                                              bf16_t *__restrict__ nx_hi, bf16_t *__restrict__ nx_lo,
                                                              float *__restrict__ ssq_out, int d, int KSp) {
    const int r = blockIdx.x;
    const size_t base = (size_t)row_tok[r] * d;
    const int n_tiles = d / 16;
    for (int ft = threadIdx.x; ft < n_tiles; ft += 256) {
        const u32x4 *src = (const u32x4 *)(embed + base + ft * 16);
        u32x4 raw[2] = {src[0], src[1]};
        float ss = 0.f;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            float v[8], x[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[2 * j] = __uint_as_float(raw[half][j] << 16);
                v[2 * j + 1] = __uint_as_float(raw[half][j] & 0xFFFF0000u);
            }
            const int c0 = ft * 16 + half * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) { ss += v[j] * v[j]; x[j] = v[j] * gain[c0 + j]; }
            *(f32x4 *)(h + (size_t)r * d + c0) = (f32x4){v[0], v[1], v[2], v[3]};
            *(f32x4 *)(h + (size_t)r * d + c0 + 4) = (f32x4){v[4], v[5], v[6], v[7]};
            u32x2 h0, l0, h1, l1;
            split4(x, h0, l0);
            split4(x + 4, h1, l1);
            const size_t o = xtile_off(r, c0, KSp);
            *(u32x4 *)(nx_hi + o) = (u32x4){h0[0], h0[1], h1[0], h1[1]};
            *(u32x4 *)(nx_lo + o) = (u32x4){l0[0], l0[1], l1[0], l1[1]};
        }
        ssq_out[(size_t)r * n_tiles + ft] = ss;
    }
}
void launch_embed_prep_bf16(const void *embed, const int *row_tok, const float *gain, float *h, void *nx_hi, void *nx_lo,
                            float *ssq_out, int R, int d, int KSp, hipStream_t st) {
    hipLaunchKernelGGL(embed_prep_bf16_kernel, dim3(R), dim3(256), 0, st, (const bf16_t *)embed, row_tok, gain, h,
                       (bf16_t *)nx_hi, (bf16_t *)nx_lo, ssq_out, d, KSp);
}

// =============================================================================================
// skinny GEMM  Y[rows][N] = X[rows][K] . W[N][K]^T,  rows <= 16*NT
// =============================================================================================
// Two kernels share the fused epilogues below: the tile-K kernel for decoding steps (few rows,
// HBM-bound weight streaming) and the panel kernel for prompt processing (hundreds of rows,
// MFMA-bound).  D[i][n] = sum_k A[i][k] B[k][n] with i = feature, n = activation row, so a lane
// ends with features 4(l/16)..+3 of row l%16 of every row tile.
// ---- fused epilogues.  Lane l holds features 16 task + 4 (l/16) .. +3 of row 16 t + l%16.
// Everything an epilogue reads from memory is fetched by epi_prefetch() before the partial sums
// are reduced, so the kernel has one memory round trip on its critical path instead of three.
template <int NT>
struct EpiIn {
    f32x4 hv[NT], gv;          // RESID: residual values, next norm's gains
    int pos[NT], slot[NT];     // QKV: position and cache slot of the row
    f32x4 cs01[NT], cs23[NT];  // QKV: (cos, sin) of the lane's four rotary pairs
};

template <int NT, int EPI>
__device__ __forceinline__ void epi_prefetch(const GemmArgs &a, const GemmPlan &p, int task, int lane, EpiIn<NT> &in) {
    const int n = lane & 15, g4 = lane >> 4;
    const int f0 = task * 16 + g4 * 4;
    if (EPI == EPI_RESID) in.gv = *(const f32x4 *)(a.gain + f0);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int row = t * 16 + n;
        const bool live = row < a.rows;
        if (EPI == EPI_RESID) {
            in.hv[t] = live ? *(const f32x4 *)(a.out + (size_t)row * p.N + f0) : (f32x4){0.f, 0.f, 0.f, 0.f};
        } else if (EPI == EPI_QKV) {
            in.pos[t] = live ? a.row_pos[row] : 0;
            in.slot[t] = live ? a.row_slot[row] : 0;
            const int tps = a.H * a.dh / 16, tph = a.dh / 16, half = a.dh / 2;
            const int j = (task % tps) % tph;
            const int i0 = 8 * j + (g4 & 1) * 4;
            const f32x4 *cp = (const f32x4 *)(a.row_cs + ((size_t)(live ? row : 0) * half + i0) * 2);
            in.cs01[t] = cp[0];
            in.cs23[t] = cp[1];
        }
    }
}

template <int NT, int EPI, int TILES>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, const GemmPlan &p, int task, int lane,
                                              f32x4 (&acc)[TILES][NT], const float *rstd_s, const EpiIn<NT> &in) {
    const int n = lane & 15, g4 = lane >> 4;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int row = t * 16 + n;
        const bool live = row < a.rows;
        const int f0 = task * 16 + g4 * 4;
        if (EPI == EPI_RESID) {
            float x[4];
            float ss = 0.f;
            const f32x4 hv = in.hv[t] + acc[0][t];
#pragma unroll
            for (int r = 0; r < 4; ++r) { ss += hv[r] * hv[r]; x[r] = hv[r] * in.gv[r]; }
            if (live) {
                *(f32x4 *)(a.out + (size_t)row * p.N + f0) = hv;
                u32x2 hi, lo;
                split4(x, hi, lo);
                const size_t o = xtile_off(row, f0, a.nx_KSp);
                *(u32x2 *)((bf16_t *)a.nx_hi + o) = hi;
                *(u32x2 *)((bf16_t *)a.nx_lo + o) = lo;
            }
            ss += __shfl_xor(ss, 16);
            ss += __shfl_xor(ss, 32);
            if (live && g4 == 0) a.ssq_out[(size_t)row * (p.N / 16) + task] = ss;
        } else if (EPI == EPI_SWIGLU) {
            if (live) {
                const float rs = rstd_s[row];
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float gg = acc[0][t][r] * rs, uu = acc[1][t][r] * rs;
                    v[r] = gg / (1.0f + __expf(-gg)) * uu;
                }
                u32x2 hi, lo;
                split4(v, hi, lo);
                const size_t o = xtile_off(row, f0, a.act_KSp);
                *(u32x2 *)((bf16_t *)a.act_hi + o) = hi;
                *(u32x2 *)((bf16_t *)a.act_lo + o) = lo;
            }
        } else if (EPI == EPI_LMHEAD) {
            const float rs = live ? rstd_s[row] : 0.f;
            const f32x4 lg = acc[0][t] * rs;
            if (a.out != nullptr && live) *(f32x4 *)(a.out + (size_t)row * p.N + f0) = lg;
            float bv = lg[0];
            int bi = f0;
#pragma unroll
            for (int r = 1; r < 4; ++r)
                if (lg[r] > bv) { bv = lg[r]; bi = f0 + r; }
#pragma unroll
            for (int sh = 16; sh <= 32; sh <<= 1) {
                const float ov = __shfl_xor(bv, sh);
                const int oi = __shfl_xor(bi, sh);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (g4 == 0 && live) {
                a.pval[(size_t)row * a.n_part + task] = bv;
                a.pidx[(size_t)row * a.n_part + task] = bi;
            }
        } else if (EPI == EPI_QKV) {
            // tile rows 0..7 = rotary first halves i, rows 8..15 = their partners i + dh/2
            const int d = a.H * a.dh, tps = d / 16, tph = a.dh / 16;
            const int sec = task / tps, tin = task % tps;
            const int head = tin / tph, j = tin % tph;
            const float rs = live ? rstd_s[row] : 0.f;
            float v[4], o4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = acc[0][t][r] * rs;
            const int pos = in.pos[t];
            const size_t head_base = ((size_t)in.slot[t] * a.H + head) * (size_t)a.max_seq * a.dh;
            if (sec < 2) {
                const int half = a.dh / 2;
                const int i0 = 8 * j + (g4 & 1) * 4;
                const float cs[8] = {in.cs01[t][0], in.cs01[t][1], in.cs01[t][2], in.cs01[t][3],
                                     in.cs23[t][0], in.cs23[t][1], in.cs23[t][2], in.cs23[t][3]};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float pr = __shfl_xor(v[r], 32);
                    o4[r] = (g4 < 2) ? (v[r] * cs[2 * r] - pr * cs[2 * r + 1]) : (v[r] * cs[2 * r] + pr * cs[2 * r + 1]);
                }
                const int c0 = (g4 < 2) ? i0 : half + i0;
                if (live) {
                    u32x2 hi, lo;
                    split4(o4, hi, lo);
                    if (sec == 0) {
                        const size_t o = xtile_off(row, head * a.dh + c0, d / 32);
                        *(u32x2 *)((bf16_t *)a.q_hi + o) = hi;
                        *(u32x2 *)((bf16_t *)a.q_lo + o) = lo;
                    } else {
                        const size_t o = head_base + kcache_off(pos, c0, a.dh);
                        *(u32x2 *)((bf16_t *)a.k_hi + o) = hi;
                        if (a.k_lo) {                                   // one byte per element (see lo8x2)
                            const float res[4] = {o4[0] - bf16_to_f32((bf16_t)(hi[0] & 0xffffu)), o4[1] - bf16_to_f32((bf16_t)(hi[0] >> 16)),
                                                  o4[2] - bf16_to_f32((bf16_t)(hi[1] & 0xffffu)), o4[3] - bf16_to_f32((bf16_t)(hi[1] >> 16))};
                            *(uint32_t *)((uint8_t *)a.k_lo + o) = lo8x4(res);
                        }
                    }
                }
            } else if (live) {
                const int c0 = j * 16 + g4 * 4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    bf16_t hi, lo;
                    split_bf16(v[r], hi, lo);
                    const size_t o = head_base + vcache_off(pos, c0 + r, a.dh);
                    ((bf16_t *)a.v_hi)[o] = hi;
                    if (a.v_lo) ((uint8_t *)a.v_lo)[o] = lo8x1(v[r] - bf16_to_f32(hi));
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// tile-K kernel (decoding steps): one workgroup per FT consecutive feature tiles, its waves split
// the K axis; each wave streams its weight blocks from HBM with non-temporal 1 KiB loads, the
// next batch in flight while the current one feeds the MFMAs; B operands come straight from the
// tiled activation planes (1 KiB contiguous per k-step and plane, shared through L2 by all
// workgroups); the waves' partial sums meet in LDS and are added in wave order; the first FT
// waves run the fused epilogue.  FT and the number of K slices depend on the matrix shape only, so
// the order of every sum is the same for any number of rows; with several feature tiles AND several
// row tiles (more than four tile pairs in all) a wave takes two K slices one after the other (half the
// waves, twice the registers).
// ---------------------------------------------------------------------------------------------
#ifndef TK_TRACE
#define TK_TRACE(slot)      // (timeline probe of the one-off microbenchmarks; nothing in the library build)
#endif
template <int NT, int FT>
struct TileKShape {
    static constexpr int SL = (FT > 1 && NT > 1 && FT * NT > 4) ? 2 : 1;   // K slices per wave
    static constexpr int MAX_THREADS = (NT == 1) ? 1024 : 512;     // one row tile: up to 16 waves of <= 128 registers
};
template <int NT, int EPI, bool SPLIT, int FT>
__global__ __launch_bounds__((TileKShape<NT, FT>::MAX_THREADS)) void gemm_tilek_bf16(GemmArgs a) {
    constexpr int SL = TileKShape<NT, FT>::SL;
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    constexpr int AT = FT * TILES;                 // weight tiles per k-step
    // k-steps per load batch (two batches in flight): one weight tile and one row tile per wave (O, down at
    // up to 16 rows: 256 workgroups, one per compute unit) need four for enough bytes in flight
    constexpr int UB = (AT * NT >= 4) ? 1 : (AT * NT == 1 ? 4 : 2);
    constexpr int PL = SPLIT ? 2 : 1;
    extern __shared__ f32x4 red[];                 // [S][AT][NT][64], then rstd[16*NT] floats
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, S = (blockDim.x >> 6) * SL;
    TK_TRACE(0);
    // llma_generate launches k + 1 rows in every step; how many of them carry a token (1 + the
    // drafts the trigger found) is only known on the device.  The dead rows cost nothing here:
    // their lanes re-read the first row's operands and the epilogue skips them.
    auto clamp_rows = [&]() {
        if (a.rows_live != nullptr) {
            const int live = *a.rows_live + 1;
            a.rows = live < a.rows ? live : a.rows;
        }
    };
    if (NT > 1) clamp_rows();
    const GemmPlan &p = a.plan;
    const int KSp = p.KSp;
    const int task0 = blockIdx.x * FT;
    // slice boundaries floor(KSp * slice / S); S is 8 or 16 (a shift; a 64-bit division here costs
    // a few hundred instructions before the kernel's first load)
    const int s_sh = 31 - __builtin_clz(S);
    int ks0 = 0, ks1 = 0, turn = 0;                // the K slice being streamed, and where in it the walk starts
    // If every workgroup walked its slices from their first k-step, the whole chip would at any moment
    // read the blocks of the same few k-steps of every tile -- addresses a fixed stride apart, which
    // fall on few memory channels.  So the walk over a slice starts `turn` k-steps in and wraps around
    // (QKV 18.9 -> 18.4 us, down 18.9 -> 17.9 us per launch at the 7B shapes).  The start is a
    // function of the tile's group of 12 -- the same for 1, 2, 3 or 4 tiles per workgroup -- and of the
    // slice length, so a tile's sums are added in an order that no launch parameter changes.
    const int turn_grp = task0 / 12;
    auto k_turn = [&](int len) { return len > 1 ? (turn_grp * 5) % len : 0; };
    float *rstd_s = (float *)(red + (size_t)S * AT * NT * 64);

    const u32x4 *wp[AT];
#pragma unroll
    for (int f = 0; f < FT; ++f)
#pragma unroll
        for (int i = 0; i < TILES; ++i) {
            int task = task0 + f;
            task = task < p.tasks ? task : p.tasks - 1;          // ragged last workgroup: recompute the last tile
            wp[f * TILES + i] = (const u32x4 *)a.W + ((size_t)(task + i * p.tasks) * KSp) * 64 + lane;
        }
    // One row tile (the usual decoding step): the wave's first weight blocks are requested before
    // the live-row count is read, which is a round trip to memory of its own.
    u32x4 avA[AT][UB];
    if (NT == 1) {
        const int k_lo = (KSp * wave * SL) >> s_sh, k_hi = (KSp * (wave * SL + 1)) >> s_sh;
        if (k_lo < k_hi) {
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                int k = (k_lo + u < k_hi ? k_lo + u : k_hi - 1) + k_turn(k_hi - k_lo);
                k = k >= k_hi ? k - (k_hi - k_lo) : k;
#pragma unroll
                for (int i = 0; i < AT; ++i) avA[i][u] = __builtin_nontemporal_load(wp[i] + (size_t)k * 64);
            }
        }
        clamp_rows();
    }
    const u32x4 *xh = (const u32x4 *)a.Xhi, *xl = (const u32x4 *)a.Xlo;
    const int nt_live = (a.rows + 15) >> 4;        // row tiles with at least one live row (uniform)
    int xpc[NT];                                   // lanes of rows past the end re-read the tile's first row:
#pragma unroll                                     // no extra cache line, no divergence; their results are dropped
    for (int t = 0; t < NT; ++t) xpc[t] = (t * 16 + (lane & 15) < a.rows) ? xtile_piece(lane) : (lane >> 4);

    auto issue = [&](int ks, u32x4 (&av)[AT][UB], u32x4 (&bv)[PL][NT][UB], bool weights = true) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            int k = ks + u;
            k = (k < ks1 ? k : ks1 - 1) + turn;
            k = k >= ks1 ? k - (ks1 - ks0) : k;
            if (weights)
#pragma unroll
            for (int i = 0; i < AT; ++i) av[i][u] = __builtin_nontemporal_load(wp[i] + (size_t)k * 64);
#pragma unroll
            for (int t = 0; t < NT; ++t)
                if (t == 0 || t < nt_live) {           // a row tile without a live row is skipped altogether
                    bv[0][t][u] = xh[((size_t)t * KSp + k) * 64 + xpc[t]];
                    if (SPLIT) bv[PL - 1][t][u] = xl[((size_t)t * KSp + k) * 64 + xpc[t]];
                }
        }
    };
    f32x4 acc[AT][NT];
    auto compute = [&](int ks, u32x4 (&av)[AT][UB], u32x4 (&bv)[PL][NT][UB]) {
#pragma unroll
        for (int u = 0; u < UB; ++u)
            if (ks + u < ks1) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    if (t == 0 || t < nt_live)
#pragma unroll
                    for (int i = 0; i < AT; ++i) {
                        acc[i][t] = mfma16x16x32(av[i][u], bv[0][t][u], acc[i][t]);
                        if (SPLIT) acc[i][t] = mfma16x16x32(av[i][u], bv[PL - 1][t][u], acc[i][t]);
                    }
            }
    };

    u32x4 bvA[PL][NT][UB], avB[AT][UB], bvB[PL][NT][UB];
    int slice = wave * SL;
    int ks = (KSp * slice) >> s_sh;
    ks1 = (KSp * (slice + 1)) >> s_sh;
    ks0 = ks; turn = k_turn(ks1 - ks0);
    if (ks < ks1) issue(ks, avA, bvA, NT > 1);      // (one row tile: the weights are already on their way)
    // epilogue inputs and rstd while the first batch is in flight
    EpiIn<NT> in;
    const int my_task = task0 + wave;                           // waves 0..FT-1 finish one tile each
    const bool finisher = wave < FT && my_task < p.tasks;
    if (finisher) epi_prefetch<NT, EPI>(a, p, my_task, lane, in);
    if (EPI != EPI_RESID && threadIdx.x < 256) {
        const int row = threadIdx.x >> 4, i = threadIdx.x & 15;
        const int chunk = (a.ssq_tiles + 15) / 16;
        const int j0 = i * chunk, j1 = (j0 + chunk < a.ssq_tiles) ? j0 + chunk : a.ssq_tiles;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int r = t * 16 + row;
            float ss = 0.f;
            if (r < a.rows) {
                const float *sp = a.ssq_in + (size_t)r * a.ssq_tiles;
                for (int j = j0; j < j1; j += 16) {
                    float v[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u)
                        if (j + u < j1) v[u] = sp[j + u];
#pragma unroll
                    for (int u = 0; u < 16; ++u)
                        if (j + u < j1) ss += v[u];
                }
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) ss += __shfl_xor(ss, off);
            if (i == 0) rstd_s[r] = 1.0f / sqrtf(ss / (float)(a.ssq_tiles * 16) + a.eps);
        }
    }
#pragma unroll
    for (int sl = 0; sl < SL; ++sl) {
        if (sl > 0) {
            slice = wave * SL + sl;
            ks = (KSp * slice) >> s_sh;
            ks1 = (KSp * (slice + 1)) >> s_sh;
            ks0 = ks; turn = k_turn(ks1 - ks0);
            if (ks < ks1) issue(ks, avA, bvA);
        }
#pragma unroll
        for (int i = 0; i < AT; ++i)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[i][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        while (ks < ks1) {
            if (ks + UB < ks1) issue(ks + UB, avB, bvB);
            compute(ks, avA, bvA);
            TK_TRACE(1);
            ks += UB;
            if (ks >= ks1) break;
            if (ks + UB < ks1) issue(ks + UB, avA, bvA);
            compute(ks, avB, bvB);
            ks += UB;
        }
        // ---- the slices' partial sums meet in LDS and are added in slice order
#pragma unroll
        for (int i = 0; i < AT; ++i)
#pragma unroll
            for (int t = 0; t < NT; ++t) red[((slice * AT + i) * NT + t) * 64 + lane] = acc[i][t];
    }
    TK_TRACE(2);
    __syncthreads();
    if (!finisher) return;
    f32x4 sum[TILES][NT];
#pragma unroll
    for (int i = 0; i < TILES; ++i)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            f32x4 v = red[((0 * AT + wave * TILES + i) * NT + t) * 64 + lane];
            for (int w = 1; w < S; ++w) v += red[((w * AT + wave * TILES + i) * NT + t) * 64 + lane];
            sum[i][t] = v;
        }
    gemm_epilogue<NT, EPI, TILES>(a, p, my_task, lane, sum, rstd_s, in);
    TK_TRACE(3);
}

// Which (feature tiles per workgroup) values the tile-K kernel can run for a matrix at nt row tiles: the
// waves' partial sums (K slices x tiles x row tiles KiB) must fit LDS, every finishing wave needs a tile,
// and a single-tile workgroup with several row tiles runs one slice per wave (at most 8 waves).
bool tilek_ft_valid(const GemmPlan &p, int nt, int ft) {
    if (ft < 1 || ft > 4 || nt < 1 || nt > 3) return false;
    const int tiles = p.tiles_per_task * ft;
    const int sl = (ft > 1 && nt > 1 && ft * nt > 4) ? 2 : 1, waves = p.tk_waves / sl;     // (TileKShape::SL)
    if (waves < ft || waves * 64 > (nt == 1 ? 1024 : 512)) return false;
    if (p.tiles_per_task == 2 && ft > 2) return false;
    return (size_t)p.tk_waves * tiles * nt * 1024 + 256 <= 160 * 1024 - 1024;
}
int tilek_ft_default(const GemmPlan &p, int nt) {
    const int want = (p.tiles_per_task == 2) ? 1 : (p.tk_waves == 16 ? 3 : 1);
    for (int ft = want; ft <= 4; ++ft)
        if (tilek_ft_valid(p, nt, ft)) return ft;
    for (int ft = want - 1; ft >= 1; --ft)
        if (tilek_ft_valid(p, nt, ft)) return ft;
    return 1;
}

template <int NT, int EPI, int FT>
static void launch_tilek(const GemmArgs &a, hipStream_t st) {
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    const GemmPlan &p = a.plan;
    const int S = p.tk_waves;                                        // K slices
    const int W = S / TileKShape<NT, FT>::SL;
    const size_t lds = (size_t)S * FT * TILES * NT * 1024 + 256;
    dim3 grid((p.tasks + FT - 1) / FT), block(W * 64);
    if (a.split) {
        static std::atomic<uint64_t> done{0};
        allow_full_lds((const void *)gemm_tilek_bf16<NT, EPI, true, FT>, done);
        hipLaunchKernelGGL((gemm_tilek_bf16<NT, EPI, true, FT>), grid, block, lds, st, a);
    } else {
        static std::atomic<uint64_t> done{0};
        allow_full_lds((const void *)gemm_tilek_bf16<NT, EPI, false, FT>, done);
        hipLaunchKernelGGL((gemm_tilek_bf16<NT, EPI, false, FT>), grid, block, lds, st, a);
    }
}

template <int NT, int EPI>
static void launch_gemm_nt_epi(const GemmArgs &a, hipStream_t st) {
    switch (tilek_ft_valid(a.plan, NT, a.plan.tk_ft[NT - 1]) ? a.plan.tk_ft[NT - 1] : tilek_ft_default(a.plan, NT)) {
        case 1: launch_tilek<NT, EPI, 1>(a, st); break;
        case 2: launch_tilek<NT, EPI, 2>(a, st); break;
        case 3: launch_tilek<NT, EPI, 3>(a, st); break;
        default: launch_tilek<NT, EPI, 4>(a, st); break;
    }
}

template <int NT>
static void launch_gemm_nt(const GemmArgs &a, hipStream_t st) {
    switch (a.epi) {
        case EPI_RESID: launch_gemm_nt_epi<NT, EPI_RESID>(a, st); break;
        case EPI_SWIGLU: launch_gemm_nt_epi<NT, EPI_SWIGLU>(a, st); break;
        case EPI_QKV: launch_gemm_nt_epi<NT, EPI_QKV>(a, st); break;
        default: launch_gemm_nt_epi<NT, EPI_LMHEAD>(a, st); break;
    }
}

// ---------------------------------------------------------------------------------------------
// Panel GEMM for prompt processing (hundreds of rows): a workgroup computes a block of
// WV*FT feature tiles x RT row tiles over the whole K axis -- no K split, no partial sums.  The
// block's activation rows are staged through LDS in chunks of KC k-steps (double-buffered,
// 16-byte pieces gathered from the planes' row-major piece order into lane order) and shared by the
// waves; every wave streams the weight blocks of its own FT feature tiles (TILES each) from
// global memory / L2, where the workgroups of the other row blocks find them again.  MFMA-bound
// by design: FT*TILES*RT*2 MFMAs per k-step and wave against RT*2 LDS operand reads.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void offset_rows(GemmArgs &a, const GemmPlan &p, int r0) {
    const int t0 = r0 / 16;
    a.rows = a.rows - r0;
    if (a.out) a.out += (size_t)r0 * p.N;
    if (a.nx_hi) { a.nx_hi = (bf16_t *)a.nx_hi + (size_t)t0 * a.nx_KSp * 512; a.nx_lo = (bf16_t *)a.nx_lo + (size_t)t0 * a.nx_KSp * 512; }
    if (a.ssq_out) a.ssq_out += (size_t)r0 * (p.N / 16);
    if (a.act_hi) { a.act_hi = (bf16_t *)a.act_hi + (size_t)t0 * a.act_KSp * 512; a.act_lo = (bf16_t *)a.act_lo + (size_t)t0 * a.act_KSp * 512; }
    if (a.pval) { a.pval += (size_t)r0 * a.n_part; a.pidx += (size_t)r0 * a.n_part; }
    if (a.row_pos) { a.row_pos += r0; a.row_slot += r0; a.row_cs += (size_t)r0 * a.dh; }
    if (a.q_hi) { a.q_hi = (bf16_t *)a.q_hi + (size_t)t0 * (a.H * a.dh / 32) * 512; a.q_lo = (bf16_t *)a.q_lo + (size_t)t0 * (a.H * a.dh / 32) * 512; }
}

// rstd[row] = rsqrt(sum of the row's per-tile sums of squares / d + eps), same summation order as
// the decoding kernels' in-kernel version (16 threads per row, contiguous chunks, butterfly); r = the
// calling thread's row (whole waves call this: the butterfly runs over 16-lane groups)
__device__ __forceinline__ void rstd_of_row(const float *__restrict__ ssq, int ssq_tiles, float eps, float *__restrict__ rstd, int rows, int r, int i) {
    const int chunk = (ssq_tiles + 15) / 16;
    const int j0 = i * chunk, j1 = (j0 + chunk < ssq_tiles) ? j0 + chunk : ssq_tiles;
    float ss = 0.f;
    if (r < rows) {
        const float *sp = ssq + (size_t)r * ssq_tiles;
        for (int j = j0; j < j1; j += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (j + u < j1) v[u] = sp[j + u];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (j + u < j1) ss += v[u];
        }
    }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) ss += __shfl_xor(ss, off);
    if (i == 0 && r < rows) rstd[r] = 1.0f / sqrtf(ss / (float)(ssq_tiles * 16) + eps);
}

// calls f(integral_constant<int, 0>), f(..1), ... in order until one returns false
template <class F, int... I>
__device__ __forceinline__ void chunks_in_order(std::integer_sequence<int, I...>, F &&f) {
    bool go = true;
    ((go = go && f(std::integral_constant<int, I>{})), ...);
}

#define PANEL_KC 2          // k-steps per LDS chunk
#ifndef PN_TRACE
#define PN_TRACE(slot, chunk)   // (timeline probe of the one-off microbenchmarks; nothing in the library build)
#endif
#ifndef PANEL_WD
#define PANEL_WD 8          // k-steps of weights in registers (one in use, the others in flight)
#endif
// (four or more weight tiles per wave: accumulators for up to 9 row tiles each need the whole register
//  file of a SIMD lane, 512 registers, i.e. one wave per SIMD; otherwise two)
template <int RT, int EPI, int FT, int WV>
__global__ __launch_bounds__(WV * 64, (FT * (EPI == EPI_SWIGLU ? 2 : 1) >= 4 ? 1 : 2)) void gemm_panel_bf16(GemmArgs a0) {
    constexpr int NTHR = WV * 64;
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    constexpr int AT = FT * TILES;
    constexpr int KC = PANEL_KC;                   // k-steps per LDS chunk
    constexpr int CH = RT * KC * 64;               // 16-byte pieces per plane and chunk
    constexpr int PER = (2 * CH + NTHR - 1) / NTHR; // pieces per thread and chunk (both planes)
    extern __shared__ u32x4 xs[];                  // [2 buffers][2 planes][RT][KC][64], then rstd[16*RT]
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const GemmPlan &p = a0.plan;
    const int KSp = p.KSp;
    if (a0.rstd_out != nullptr && blockIdx.x == gridDim.x - 1) {
        // split-K form: one workgroup more than the tiles need turns the rows' sums of squares into
        // rstd for the finishing kernel, beside the others instead of in a launch of its own
        if (blockIdx.y == 0)
            for (int r = threadIdx.x >> 4; r < ((a0.rows + 15) & ~15); r += NTHR / 16)
                rstd_of_row(a0.ssq_in, a0.ssq_tiles, a0.eps, a0.rstd_out, a0.rows, r, threadIdx.x & 15);
        return;
    }
    // Workgroup order: the row blocks of one feature block get ids that differ by multiples of 8, i.e.
    // they are dispatched close together and onto the same XCD, so the feature block's weights are
    // fetched from HBM once and found in that XCD's L2 by the other row blocks.
    const int RB = a0.panel_rb;
    const int grp = blockIdx.x / (8 * RB), within = blockIdx.x % (8 * RB);
    const int fb = grp * 8 + (within & 7), rb = within >> 3;
    const int r0 = rb * (16 * RT);
    const int rt0 = r0 / 16;
    float *rstd_s = (float *)(xs + 2 * 2 * CH);
    GemmArgs a = a0;
    offset_rows(a, p, r0);
    const int task0 = (fb * WV + wave) * FT;        // may lie past the last tile (padding feature blocks): clamped loads, no epilogue

    const char *wb[AT];                            // first weight block of each tile (wave-uniform)
#pragma unroll
    for (int f = 0; f < FT; ++f)
#pragma unroll
        for (int i = 0; i < TILES; ++i) {
            int task = task0 + f;
            task = task < p.tasks ? task : p.tasks - 1;
            wb[f * TILES + i] = (const char *)a.W + ((size_t)(task + i * p.tasks) * KSp) * 1024;
        }
    const char *xh = (const char *)a.Xhi, *xl = (const char *)a.Xlo;
    const int n_rt_total = (a0.rows + 15) / 16;    // row tiles that exist in the planes

    // Operand fetches.  Every address below is a wave-uniform base (scalar registers, scalar
    // arithmetic) plus one per-lane byte offset that never changes (the lane's 16 bytes of a 1 KiB
    // block), so the chunk loop spends no vector instructions on addressing; every load is
    // unconditional (indices are clamped instead): a load under a branch makes the compiler's count
    // of loads in flight inexact, and it then waits for all of them.
    // Activation chunk kc -> registers: wave w fetches the 1 KiB blocks q = j WV + w of the chunk's
    // [2 planes][RT][KC] blocks; blocks of row tiles past the end read tile 0.
    const unsigned x_lane = (unsigned)xtile_piece(lane) * 16u;     // LDS holds the block in lane order
    const unsigned w_lane = (unsigned)lane * 16u;
    auto fetch_x = [&](int kc, u32x4 (&v)[PER]) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            int q = j * WV + wave;
            q = q < 2 * RT * KC ? q : 2 * RT * KC - 1;
            const int pl = q / (RT * KC), t = (q % (RT * KC)) / KC, kk = q % KC;
            int k = kc * KC + kk;
            k = k < KSp ? k : KSp - 1;
            const int tt = (rt0 + t < n_rt_total) ? rt0 + t : 0;
            const char *blk = (const char *)(pl ? xl : xh) + ((size_t)tt * KSp + k) * 1024;
            v[j] = *(const u32x4 *)(blk + x_lane);
        }
    };
    auto stash_x = [&](int buf, u32x4 (&v)[PER]) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int q = j * WV + wave;
            if (q < 2 * RT * KC) xs[(buf * 2 * RT * KC + q) * 64 + lane] = v[j];
        }
    };
    // weights of k-step k0, one 1 KiB block per tile; a k-step past the end of K (ragged last chunk)
    // gets zeros and adds nothing
    auto fetch_w = [&](int k0, u32x4 (&av)[AT]) {
        const int k = k0 < KSp ? k0 : KSp - 1;
        const unsigned keep = k0 < KSp ? 0xffffffffu : 0u;          // (a mask, not a select: the load stays unconditional)
#pragma unroll
        for (int i = 0; i < AT; ++i) av[i] = *(const u32x4 *)(wb[i] + (size_t)k * 1024 + w_lane) & keep;
    };

    f32x4 acc[AT][RT];
#pragma unroll
    for (int i = 0; i < AT; ++i)
#pragma unroll
        for (int t = 0; t < RT; ++t) acc[i][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // split-K form (batched decoding steps, too few rows to fill the chip otherwise): blockIdx.y picks
    // one of a0.ksplit contiguous ranges of k-chunks; the raw sums go to a0.part and a second kernel
    // adds the ranges in order and runs the epilogue
    const int n_split = a0.ksplit > 1 ? a0.ksplit : 1;
    const int NC_all = (KSp + KC - 1) / KC;
    const int kc_lo = (int)((long)NC_all * blockIdx.y / n_split), NC = (int)((long)NC_all * (blockIdx.y + 1) / n_split);
    // The weights come straight from HBM, whose latency under load (2 us and more) is several chunks
    // of MFMA work, so they are requested WD - 1 k-steps ahead into a ring of WD register sets; the loop
    // below is unrolled over one turn of the ring (WD / KC chunks), which gives every set and both
    // activation staging arrays one fixed role per call site (one body taking either role made the
    // compiler copy registers between the roles every chunk, behind a wait for all loads in flight).
    // A wave's loads complete in the order it issued them, so an activation block (an L2 hit) waits
    // behind every weight block requested before it: the activations are requested two chunks before
    // they are parked in LDS.
    constexpr int WD = PANEL_WD;
    static_assert(WD % (2 * KC) == 0, "one turn of the weight ring is a whole number of LDS buffer pairs");
    u32x4 xvA[PER], xvB[PER], wr[WD][AT];
    PN_TRACE(0, 63);
    fetch_x(kc_lo, xvA);
#pragma unroll
    for (int j = 0; j < WD - 1; ++j) fetch_w(kc_lo * KC + j, wr[j]);
    fetch_x(kc_lo + 1, xvB);
    if (EPI != EPI_RESID && n_split == 1)
        for (int r = threadIdx.x; r < 16 * RT; r += NTHR) rstd_s[r] = (r < a.rows) ? a.rstd_in[r0 + r] : 0.f;
    stash_x(0, xvA);
    __syncthreads();
    PN_TRACE(1, 63);
    // One chunk: request operands (the weights WD - 1 k-steps ahead, the activations of the chunk after
    // the next: they still have to pass through LDS), run this chunk's MFMAs out of LDS buffer c & 1
    // and the ring, park the next chunk's activations (requested a chunk ago) in the other LDS buffer,
    // which was last read before the previous barrier.  (Requests past the end of the range or of K
    // are clamped, unused.)
    auto chunk = [&](int kc0, auto slot) -> bool {
        constexpr int c = decltype(slot)::value;        // chunk within the turn of the ring
        constexpr int buf = c & 1;
        const int kc = kc0 + c;
        if (kc >= NC) return false;
        PN_TRACE(0, kc - kc_lo);
        u32x4 (&x_park)[PER] = buf ? xvA : xvB;
        u32x4 (&x_req)[PER] = buf ? xvB : xvA;          // held this chunk's activations, in LDS since the last barrier
        fetch_x(kc + 2, x_req);
#pragma unroll
        for (int u = 0; u < KC; ++u) {
            const int j = c * KC + u;                   // ring set of this k-step (a constant after unrolling)
            fetch_w(kc * KC + u + WD - 1, wr[(j + WD - 1) % WD]);   // into the set the previous k-step used
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                const u32x4 bh = xs[buf * 2 * CH + (t * KC + u) * 64 + lane];
                const u32x4 bl = xs[buf * 2 * CH + CH + (t * KC + u) * 64 + lane];
#pragma unroll
                for (int i = 0; i < AT; ++i) {
                    acc[i][t] = mfma16x16x32(wr[j][i], bh, acc[i][t]);
                    acc[i][t] = mfma16x16x32(wr[j][i], bl, acc[i][t]);
                }
            }
        }
        PN_TRACE(1, kc - kc_lo);
        stash_x(buf ^ 1, x_park);
        PN_TRACE(2, kc - kc_lo);
        __syncthreads();
        PN_TRACE(3, kc - kc_lo);
        return true;
    };
    for (int kc = kc_lo; kc < NC; kc += WD / KC)
        chunks_in_order(std::make_integer_sequence<int, WD / KC>{}, [&](auto slot) { return chunk(kc, slot); });

    if (n_split > 1) {
        // partial sums as register images: [range][tile (SwiGLU: gate tiles, then up tiles)][row tile][lane]
        f32x4 *part = (f32x4 *)a0.part;
#pragma unroll
        for (int f = 0; f < FT; ++f)
#pragma unroll
            for (int i = 0; i < TILES; ++i)
#pragma unroll
                for (int t = 0; t < RT; ++t)
                    if (task0 + f < p.tasks && rt0 + t < n_rt_total)
                        part[(((size_t)blockIdx.y * (p.tasks * TILES) + task0 + f + i * p.tasks) * n_rt_total + rt0 + t) * 64 + lane] = acc[f * TILES + i][t];
        PN_TRACE(2, 63);
        return;
    }
    // ---- epilogues, one feature tile (pair) at a time
#pragma unroll
    for (int f = 0; f < FT; ++f) {
        const int task = task0 + f;
        if (task < p.tasks) {
            EpiIn<RT> in;
            epi_prefetch<RT, EPI>(a, p, task, lane, in);
            f32x4 sum[TILES][RT];
#pragma unroll
            for (int i = 0; i < TILES; ++i)
#pragma unroll
                for (int t = 0; t < RT; ++t) sum[i][t] = acc[f * TILES + i][t];
            gemm_epilogue<RT, EPI, TILES>(a, p, task, lane, sum, rstd_s, in);
        }
    }
}

__global__ __launch_bounds__(256) void rstd_rows_kernel(const float *__restrict__ ssq, int ssq_tiles, float eps, float *__restrict__ rstd, int rows) {
    rstd_of_row(ssq, ssq_tiles, eps, rstd, rows, blockIdx.x * 16 + (threadIdx.x >> 4), threadIdx.x & 15);
}
void launch_rstd_rows(const float *ssq, int ssq_tiles, float eps, float *rstd, int rows, hipStream_t st) {
    hipLaunchKernelGGL(rstd_rows_kernel, dim3((rows + 15) / 16), dim3(256), 0, st, ssq, ssq_tiles, eps, rstd, rows);
}

// second half of the split-K form: one wave per (feature tile (pair), row tile) adds the ranges'
// partial sums in range order and runs the fused epilogue on the result
template <int EPI>
__global__ __launch_bounds__(256) void gemm_splitk_finish_bf16(GemmArgs a0) {
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    __shared__ float rstd_sh[4][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GemmPlan &p = a0.plan;
    const int n_rt = (a0.rows + 15) / 16;
    const int unit = blockIdx.x * 4 + wave;
    if (unit >= p.tasks * n_rt) return;                         // (no workgroup barrier below)
    const int task = unit / n_rt, t = unit % n_rt;
    GemmArgs a = a0;
    offset_rows(a, p, t * 16);
    EpiIn<1> in;
    epi_prefetch<1, EPI>(a, p, task, lane, in);
    if (EPI != EPI_RESID && lane < 16) rstd_sh[wave][lane] = (lane < a.rows) ? a0.rstd_in[t * 16 + lane] : 0.f;
    const f32x4 *part = (const f32x4 *)a0.part;
    f32x4 sum[TILES][1];
#pragma unroll
    for (int i = 0; i < TILES; ++i) {
        const size_t tile = (size_t)(task + i * p.tasks) * n_rt + t, stride = (size_t)p.tasks * TILES * n_rt;
        f32x4 v = part[tile * 64 + lane];
        for (int s = 1; s < a0.ksplit; ++s) v += part[(s * stride + tile) * 64 + lane];
        sum[i][0] = v;
    }
    gemm_epilogue<1, EPI, TILES>(a, p, task, lane, sum, rstd_sh[wave], in);
}
template <int EPI>
static void launch_splitk_finish(const GemmArgs &a, hipStream_t st) {
    const int units = a.plan.tasks * ((a.rows + 15) / 16);
    hipLaunchKernelGGL((gemm_splitk_finish_bf16<EPI>), dim3((units + 3) / 4), dim3(256), 0, st, a);
}

template <int RT, int EPI, int FT, int WV>
static void launch_panel_cfg(const GemmArgs &a, hipStream_t st) {
    const GemmPlan &p = a.plan;
    const size_t lds = (size_t)2 * 2 * RT * PANEL_KC * 1024 + 16 * RT * sizeof(float);
    const int FB = ((p.tasks + WV * FT - 1) / (WV * FT) + 7) / 8 * 8;    // feature blocks, padded to whole groups of 8
    GemmArgs a2 = a;
    a2.panel_rb = (a.rows + 16 * RT - 1) / (16 * RT);
    if (a.ksplit <= 1) a2.rstd_out = nullptr;
    dim3 grid(FB * a2.panel_rb + (a2.rstd_out ? 1 : 0), a.ksplit > 1 ? a.ksplit : 1), block(WV * 64);
    static std::atomic<uint64_t> done{0};
    allow_full_lds((const void *)gemm_panel_bf16<RT, EPI, FT, WV>, done);
    hipLaunchKernelGGL((gemm_panel_bf16<RT, EPI, FT, WV>), grid, block, lds, st, a2);
}

// prompt-processing GEMM over any number of rows (needs a.rstd_in for the norm-scaled epilogues).
// A workgroup owns WV = 8 waves x FT feature tiles (FT = 2; SwiGLU: one gate/up pair) and RT = 5..9 row
// tiles, one workgroup per compute unit (two workgroups of 4 waves, whose chunk barriers fall at
// different times, were 8 % slower on the 1535-row prompt pass once the weights were requested a ring
// ahead: 46.7 vs 43.0 ms).  A launch runs in rounds of that many workgroups; a round costs about RT + 3
// (the weight stream and chunk barriers of a workgroup do not shrink with its height), and the height
// with the least rounds x (RT + 3) wins: 1535 prompt rows: 6 for QKV, O and down, 9 for gate/up; 144
// rows of a batched step: 9 for QKV and gate/up (one row block, the weights pass once: 64 -> 51 us,
// 104 -> 82 us), 5 for O and down (two row blocks fill the 256 compute units, one would leave half of
// them idle: 28 vs 33 us, 47 vs 58 us).
template <int EPI, int FT, int WV>
static void launch_panel_wv(const GemmArgs &a, hipStream_t st) {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n_cu = prop.multiProcessorCount;
        if (n_cu <= 0) n_cu = 256;
    }
    const int slots = n_cu * (8 / WV);                   // workgroups resident at once
    const int fb = ((a.plan.tasks + WV * FT - 1) / (WV * FT) + 7) / 8 * 8;
    const int row_tiles = (a.rows + 15) / 16;
    const int ns = a.ksplit > 1 ? a.ksplit : 1;
    auto cost = [&](int rt) { return (long)((fb * ((row_tiles + rt - 1) / rt) * ns + slots - 1) / slots) * (rt + 3); };
    constexpr int RT_MAX = (WV == 8) ? 9 : 8;            // (9 row tiles of accumulators need the 8-wave form's register budget)
    int best = 5;
    for (int rt = 6; rt <= RT_MAX; ++rt)
        if (cost(rt) <= cost(best)) best = rt;            // (ties: fewer, taller row blocks stream the weights less often)
    switch (best) {
        case 5: launch_panel_cfg<5, EPI, FT, WV>(a, st); break;
        case 6: launch_panel_cfg<6, EPI, FT, WV>(a, st); break;
        case 7: launch_panel_cfg<7, EPI, FT, WV>(a, st); break;
        case 8: launch_panel_cfg<8, EPI, FT, WV>(a, st); break;
        default:
            if constexpr (WV == 8) launch_panel_cfg<9, EPI, FT, WV>(a, st);
            else launch_panel_cfg<8, EPI, FT, WV>(a, st);
            break;
    }
    if (a.ksplit > 1) launch_splitk_finish<EPI>(a, st);
}
template <int EPI, int FT>
static void launch_panel_epi(const GemmArgs &a, hipStream_t st) {
    launch_panel_wv<EPI, FT, 8>(a, st);
}
void launch_gemm_panel_bf16(const GemmArgs &a, hipStream_t st) {
    switch (a.epi) {
        case EPI_RESID: launch_panel_epi<EPI_RESID, 2>(a, st); break;
        case EPI_SWIGLU: launch_panel_epi<EPI_SWIGLU, 1>(a, st); break;
        case EPI_QKV: launch_panel_epi<EPI_QKV, 2>(a, st); break;
        default: launch_panel_epi<EPI_LMHEAD, 2>(a, st); break;
    }
}

// decoding-step GEMM: one launch for up to 48 rows (three row tiles).  More rows are refused (false,
// nothing launched): every workgroup re-reads all rows' operands, so larger steps belong to the panel
// kernel, and processing them here in blocks would stream the weights once per block.
bool launch_gemm_bf16(const GemmArgs &a, hipStream_t st) {
    if (a.rows < 1 || a.rows > 48) return false;
    if (a.rows <= 16) launch_gemm_nt<1>(a, st);
    else if (a.rows <= 32) launch_gemm_nt<2>(a, st);
    else launch_gemm_nt<3>(a, st);
    return true;
}

// how a [N][K] weight matrix is cut into work for the tile-K kernel: three feature tiles per
// workgroup and 16 K slices for matrices of 640+ tiles (QKV, LM head), else one tile (pair) and 8
// slices -- the combinations measured fastest on the 7B and 13B shapes
GemmPlan make_gemm_plan(int N, int K, int tiles_per_task) {
    GemmPlan p;
    p.N = N; p.K = K;
    p.KSp = K / 32;
    p.tasks = N / 16;
    // K slices: 16 for matrices of 640+ tiles (QKV, LM head), else 8; feature tiles per workgroup: three
    // resp. one by default (the values measured fastest on the 7B shapes), re-tuned per context by timing
    // (llma_create), which cannot change any result
    p.tiles_per_task = tiles_per_task;
    p.tk_waves = (tiles_per_task != 2 && p.tasks >= 640) ? 16 : 8;
    for (int nt = 1; nt <= 3; ++nt) p.tk_ft[nt - 1] = tilek_ft_default(p, nt);
    // split-K form of the panel kernel: enough ranges that feature blocks x ranges is about 200
    // workgroups per row block (2..8, a function of the matrix only, so a row's sums do not depend on
    // how many rows share the step)
    const int fb = (p.tasks + (tiles_per_task == 2 ? 8 : 16) - 1) / (tiles_per_task == 2 ? 8 : 16);
    int ns = (192 + fb / 2) / fb;
    ns = ns < 2 ? 2 : (ns > 8 ? 8 : ns);
    const int chunks = (p.KSp + PANEL_KC - 1) / PANEL_KC;
    p.n_split = ns < chunks ? ns : (chunks > 0 ? chunks : 1);
    return p;
}

// Keeps the loads written above this point above it: the compiler may not sink a load into the
// branch that uses its value past something that could write memory.  No value is consumed here,
// so nothing waits.  Used where many loads must be in flight before a dependent value (the
// sequence length) arrives.
__device__ __forceinline__ void loads_stay_above() { asm volatile("" ::: "memory"); }

// =============================================================================================
// causal attention of m <= 16*NTQ query rows of one sequence over its KV cache
// =============================================================================================
// grid = (chunks of ATTN_CHUNK key positions, heads, sequences); 4 waves per workgroup, wave w
// owns the 32 positions [32 w, 32 w + 32) of the chunk and issues all of their K and V loads
// (whole 1 KiB blocks) before any arithmetic.  S^T = K_tile . Q^T (MFMA, keys on the A side;
// with hi/lo planes S = Khi.qhi + Khi.qlo + Klo.qhi), scale, causal mask by absolute position,
// softmax statistics per query row, O^T = V^T . P^T (again hi/lo).  The four waves' (max, sum, O)
// are merged in wave order, and the chunk's partial is written for the combine kernel.  Which
// keys a row sees, and in which order they are reduced, is a function of absolute positions only.
// COMPACT (three row tiles, at most ATTN_COMPACT_ROWS rows: the 33 rows per sequence of k = 32): the
// merge buffer holds only that many rows, every row tile is published as soon as it is done (one
// tile of accumulators in registers at a time) and the registers are capped, so that two workgroups
// fit a compute unit like they do with one or two row tiles.
#define ATTN_COMPACT_ROWS 36
template <int DH, int NTQ, bool KVS, bool LIVE, bool COMPACT = false>
__device__ __forceinline__ void attn_chunk_body(const AttnArgs &a, float (&sm)[4][NTQ * 16], float (&sl)[4][NTQ * 16],
                                                float (&so)[4][COMPACT ? ATTN_COMPACT_ROWS : NTQ * 16][DH + 4]) {
    constexpr int KSTEPS = DH / 32;   // MFMA k-steps of a q.k dot product
    constexpr int DT = DH / 16;       // 16-feature tiles of the head dimension
    constexpr int RQ = NTQ * 16;
    constexpr int OQ = COMPACT ? 1 : NTQ;                      // row tiles of accumulators held at once

    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z / a.n_rblocks, rb = blockIdx.z % a.n_rblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int slot = a.slot_const >= 0 ? a.slot_const : a.batch_slots[b];
    const int m = a.m;
    const int j0 = rb * RQ;                             // first row of this row block
    const int chunk0 = c * ATTN_CHUNK;
    const int d_model = a.H * DH;
    const int key0 = chunk0 + wave * 32;
    const size_t head_base = ((size_t)slot * a.H + h) * (size_t)a.max_seq * DH;
    // The sequence length and the live-row count are requested first and used last: both requests
    // are in flight together with the K/V blocks instead of one after the other behind them.
    const int T = a.T[slot];
    const int live_rows = LIVE ? *a.rows_live + 1 : m;
    loads_stay_above();
    // K and V blocks of the wave's 32 positions: issued before the sequence length is known (any
    // position below max_seq lies inside the cache allocation; unused blocks are simply dropped)
    u32x4 ka[2][KSTEPS], va[DT];
    u32x2 kb[2][KSTEPS], vb[DT];                     // lo planes: one byte per element
    {
        const bf16_t *kh = (const bf16_t *)a.Khi + head_base; const uint8_t *kl = (const uint8_t *)a.Klo + head_base;
        const bf16_t *vh = (const bf16_t *)a.Vhi + head_base; const uint8_t *vl = (const uint8_t *)a.Vlo + head_base;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const size_t off = (size_t)(key0 / 16 + t) * (16 * DH) + s * 512 + lane * 8;
                ka[t][s] = *(const u32x4 *)(kh + off);
                if (KVS) kb[t][s] = *(const u32x2 *)(kl + off);
            }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const size_t off = (size_t)(key0 / 32) * (32 * DH) + dt * 512 + lane * 8;
            va[dt] = (*(const u32x4 *)(vh + off));
            if (KVS) vb[dt] = *(const u32x2 *)(vl + off);
        }
    }
    // a single row tile's query operands do not depend on the sequence length either
    u32x4 qh0[KSTEPS], ql0[KSTEPS];
    if (NTQ == 1) {
        const int j = j0 + n;
        const int r = b * m + (j < m ? j : 0);
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const size_t off = xtile_off(r, h * DH + s * 32 + g * 8, d_model / 32);
            qh0[s] = (*(const u32x4 *)((const bf16_t *)a.Qhi + off));
            ql0[s] = (*(const u32x4 *)((const bf16_t *)a.Qlo + off));
        }
    }
    if (NTQ == 1) loads_stay_above();                   // (with more row tiles the registers are needed elsewhere)
    // generation steps: rows past the trigger's draft count are padding (see the GEMM); they are
    // masked like rows past m and a row tile made of them only is skipped
    const int m_live = live_rows < m ? live_rows : m;     // LIVE: rows_live is set
    if (j0 >= m_live) return;
    const int m_blk = (m_live - j0 < RQ) ? m_live - j0 : RQ;   // live rows of this block
    const int kv_len = T + j0 + m_blk;                  // positions the block's last row can see
    if (chunk0 >= kv_len) return;                       // uniform for the workgroup
    const bool active = key0 < kv_len;                  // uniform for the wave

    float mrow[NTQ], lrow[NTQ];
    f32x4 o[OQ][DT];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        mrow[q] = LLMA_NEG_INF;
        lrow[q] = 0.f;
    }
#pragma unroll
    for (int q = 0; q < OQ; ++q)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[q][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // every wave publishes (max, sum, O) of a row tile for the merge below
    auto publish = [&](int q, const f32x4 (&oq)[DT]) {
        float l = lrow[q];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (g == 0) { sm[wave][q * 16 + n] = mrow[q]; sl[wave][q * 16 + n] = l; }
        if (!COMPACT || q * 16 + n < ATTN_COMPACT_ROWS)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *(f32x4 *)&so[wave][q * 16 + n][dt * 16 + 4 * g] = oq[dt];
    };
    if (COMPACT && !active) {
#pragma unroll
        for (int q = 0; q < NTQ; ++q) publish(q, o[0]);         // (zeros)
    }

    if (active) {
#pragma unroll
        for (int q = 0; q < NTQ; ++q) {
            const int oi = COMPACT ? 0 : q;
            if (LIVE && q > 0 && j0 + q * 16 >= m_live) {           // uniform: no live row in this tile
                if (COMPACT) publish(q, o[0]);                      // (zeros: o[0] is cleared after every tile)
                continue;
            }
            const int j = j0 + q * 16 + n;
            const bool valid = j < m_live;
            const int rpos = valid ? T + j : -1;
            const int r = b * m + (valid ? j : 0);
            u32x4 qh[KSTEPS], ql[KSTEPS];
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                if (NTQ == 1) { qh[s] = qh0[s]; ql[s] = ql0[s]; continue; }
                const size_t off = xtile_off(r, h * DH + s * 32 + g * 8, d_model / 32);
                qh[s] = *(const u32x4 *)((const bf16_t *)a.Qhi + off);
                ql[s] = *(const u32x4 *)((const bf16_t *)a.Qlo + off);
            }
            float sv[8];
            float mx = LLMA_NEG_INF;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    acc = mfma16x16x32(ka[t][s], qh[s], acc);
                    acc = mfma16x16x32(ka[t][s], ql[s], acc);
                    if (KVS) acc = mfma16x16x32(lo8_operand(kb[t][s]), qh[s], acc);
                }
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int key = key0 + t * 16 + 4 * g + r4;
                    float v = acc[r4] * a.scale;
                    v = (key > rpos) ? LLMA_NEG_INF : v;
                    sv[t * 4 + r4] = v;
                    mx = fmaxf(mx, v);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            float psum = 0.f;
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = (mx == LLMA_NEG_INF) ? 0.f : __expf(sv[i] - mx);
                psum += p[i];
            }
            lrow[q] = psum;
            mrow[q] = mx;
            u32x2 h0, l0, h1, l1;
            split4(p, h0, l0);
            split4(p + 4, h1, l1);
            const u32x4 ph = (u32x4){h0[0], h0[1], h1[0], h1[1]};
            const u32x4 pl = (u32x4){l0[0], l0[1], l1[0], l1[1]};
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[oi][dt] = mfma16x16x32(va[dt], ph, o[oi][dt]);
                o[oi][dt] = mfma16x16x32(va[dt], pl, o[oi][dt]);
                if (KVS) o[oi][dt] = mfma16x16x32(lo8_operand(vb[dt]), ph, o[oi][dt]);
            }
            if (COMPACT) {
                publish(q, o[0]);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) o[0][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
            }
        }
    }

    // ---- merge the four waves in wave order: every wave publishes (max, sum, O), then all
    //      threads add the four contributions e^{m_w - M} O_w of an output element in wave order
    if (!COMPACT) {
#pragma unroll
        for (int q = 0; q < NTQ; ++q) publish(q, o[COMPACT ? 0 : q]);
    }
    __syncthreads();
    const size_t pbase = (((size_t)b * a.H + h) * a.n_chunks + c) * ((size_t)a.n_rblocks * RQ) + j0;
    for (int idx = threadIdx.x; idx < m_blk * (DH / 4); idx += 256) {
        const int j = idx / (DH / 4), d4 = idx % (DH / 4);
        float M = LLMA_NEG_INF;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sm[w][j]);
        f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = sm[w][j];
            const float sc = (mw == LLMA_NEG_INF) ? 0.f : __expf(mw - M);
            acc += *(const f32x4 *)&so[w][j][d4 * 4] * sc;
        }
        *(f32x4 *)(a.po + (pbase + j) * DH + d4 * 4) = acc;
    }
    if (threadIdx.x < m_blk) {
        int j = threadIdx.x;
        float M = LLMA_NEG_INF;
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sm[w][j]);
        float L = 0.f;
        for (int w = 0; w < 4; ++w) {
            float mw = sm[w][j];
            L += (mw == LLMA_NEG_INF) ? 0.f : sl[w][j] * __expf(mw - M);
        }
        a.pm[pbase + j] = M;
        a.pl[pbase + j] = L;
    }
}

// LOSKIP (batched steps on caches with hi + lo planes): positions below lo_from[slot] were imported
// as bf16 values -- their lo planes hold zeros -- so a chunk that lies entirely below it runs the
// single-plane form of the body: half the K/V bytes, the same sums (the skipped terms are zeros).
template <int DH, int NTQ, bool KVS, bool LIVE, bool LOSKIP = false, bool COMPACT = false>
__global__ __launch_bounds__(256, (COMPACT ? 2 : 1)) void attn_bf16_kernel(AttnArgs a) {
    constexpr int RQ = NTQ * 16;
    __shared__ float sm[4][RQ], sl[4][RQ];
    __shared__ float so[4][COMPACT ? ATTN_COMPACT_ROWS : RQ][DH + 4];
    if (KVS && LOSKIP) {
        const int slot = a.slot_const >= 0 ? a.slot_const : a.batch_slots[blockIdx.z / a.n_rblocks];
        if ((int)(blockIdx.x + 1) * ATTN_CHUNK <= a.lo_from[slot]) {     // uniform for the workgroup
            attn_chunk_body<DH, NTQ, false, LIVE, COMPACT>(a, sm, sl, so);
            return;
        }
    }
    attn_chunk_body<DH, NTQ, KVS, LIVE, COMPACT>(a, sm, sl, so);
}

// ---------------------------------------------------------------------------------------------
// Wide batched steps (several sequences, more than 48 rows in all; their GEMMs already add in an
// order of their own): a workgroup walks ATTN_WALK_CHUNKS consecutive chunks of one (sequence, head)
// instead of one.  Every chunk is computed like above -- four waves x 32 positions, all K/V blocks of
// the chunk requested at once, (max, sum, O) per wave merged through LDS in wave order -- and the merged
// chunk is folded into a running (max, sum, O) held in registers, in chunk order; one partial per
// walk goes to the combine kernel.  Four times fewer workgroups, partials and combine work than one
// chunk per workgroup (16 sequences x 4096 positions: 16384 -> 4096 workgroups per layer).  Chunks
// that lie entirely below lo_from[slot] (imported bf16 caches: all-zero lo planes) skip the lo planes.
// ---------------------------------------------------------------------------------------------
#define ATTN_WALK_CHUNKS 4
template <int DH, int NTQ, bool KVS>
__global__ __launch_bounds__(256, 2) void attn_walk_bf16_kernel(AttnArgs a) {
    constexpr int KSTEPS = DH / 32, DT = DH / 16;
    constexpr int RQ = NTQ * 16;
    constexpr int RS = (NTQ == 3) ? ATTN_COMPACT_ROWS : RQ;          // rows the merge buffer holds (a step has at most 33 per sequence)
    constexpr int OWN = (RS * (DH / 4) + 255) / 256;                  // merged output elements (float4) per thread
    __shared__ float sm[4][RQ], sl[4][RQ];
    __shared__ float so[4][RS][DH + 4];
    const int h = blockIdx.y, b = blockIdx.z / a.n_rblocks, rb = blockIdx.z % a.n_rblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int slot = a.batch_slots[b];
    const int T = a.T[slot];
    const int lo_from = (KVS && a.lo_from != nullptr) ? a.lo_from[slot] : 0;
    const int m = a.m, j0 = rb * RQ;
    if (j0 >= m) return;
    const int m_blk = (m - j0 < RQ) ? m - j0 : RQ;
    const int kv_len = T + j0 + m_blk;                               // positions the block's last row can see
    const int c0 = blockIdx.x * ATTN_WALK_CHUNKS;
    if (c0 * ATTN_CHUNK >= kv_len) return;                           // uniform for the workgroup
    const int c_need = (kv_len + ATTN_CHUNK - 1) / ATTN_CHUNK;
    const int c1 = c0 + ATTN_WALK_CHUNKS < c_need ? c0 + ATTN_WALK_CHUNKS : c_need;
    // chunks below c_lo lie entirely inside an imported bf16 cache: single plane
    int c_lo = KVS ? lo_from / ATTN_CHUNK : c1;
    c_lo = c_lo < c0 ? c0 : (c_lo > c1 ? c1 : c_lo);
    const int d_model = a.H * DH;
    const size_t head_base = ((size_t)slot * a.H + h) * (size_t)a.max_seq * DH;
    const bf16_t *kh = (const bf16_t *)a.Khi + head_base; const uint8_t *kl = (const uint8_t *)a.Klo + head_base;
    const bf16_t *vh = (const bf16_t *)a.Vhi + head_base; const uint8_t *vl = (const uint8_t *)a.Vlo + head_base;

    f32x4 acc_run[OWN];
    float M_run[OWN];
#pragma unroll
    for (int i = 0; i < OWN; ++i) { acc_run[i] = (f32x4){0.f, 0.f, 0.f, 0.f}; M_run[i] = LLMA_NEG_INF; }
    float M_row = LLMA_NEG_INF, L_row = 0.f;                         // thread j < m_blk: row j's running max / sum
    for (int c = c0; c < c1; ++c) {
        const int key0 = c * ATTN_CHUNK + wave * 32;
        const bool active = key0 < kv_len;                           // uniform for the wave
        const bool use_lo = KVS && c >= c_lo;                        // uniform for the workgroup
        u32x4 ka[2][KSTEPS], va[DT];
        u32x2 kb[2][KSTEPS], vb[DT];                     // lo planes: one byte per element
        if (active) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    const size_t off = (size_t)(key0 / 16 + t) * (16 * DH) + s * 512 + lane * 8;
                    ka[t][s] = *(const u32x4 *)(kh + off);
                    if (KVS && use_lo) kb[t][s] = *(const u32x2 *)(kl + off);
                }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const size_t off = (size_t)(key0 / 32) * (32 * DH) + dt * 512 + lane * 8;
                va[dt] = *(const u32x4 *)(vh + off);
                if (KVS && use_lo) vb[dt] = *(const u32x2 *)(vl + off);
            }
        }
#pragma unroll
        for (int q = 0; q < NTQ; ++q) {
            const int j = j0 + q * 16 + n;
            const bool valid = j < m;
            float mrow = LLMA_NEG_INF, lsum = 0.f;
            f32x4 o[DT];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (active && j0 + q * 16 < m) {                         // (a row tile past the block's rows: nothing to do, uniform)
                const int rpos = valid ? T + j : -1;
                const int r = b * m + (valid ? j : j0);
                u32x4 qh[KSTEPS], ql[KSTEPS];
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    const size_t off = xtile_off(r, h * DH + s * 32 + g * 8, d_model / 32);
                    qh[s] = *(const u32x4 *)((const bf16_t *)a.Qhi + off);
                    ql[s] = *(const u32x4 *)((const bf16_t *)a.Qlo + off);
                }
                float sv[8];
                float mx = LLMA_NEG_INF;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < KSTEPS; ++s) {
                        acc = mfma16x16x32(ka[t][s], qh[s], acc);
                        acc = mfma16x16x32(ka[t][s], ql[s], acc);
                        if (KVS && use_lo) acc = mfma16x16x32(lo8_operand(kb[t][s]), qh[s], acc);
                    }
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int key = key0 + t * 16 + 4 * g + r4;
                        float v = acc[r4] * a.scale;
                        v = (key > rpos) ? LLMA_NEG_INF : v;
                        sv[t * 4 + r4] = v;
                        mx = fmaxf(mx, v);
                    }
                }
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                float p[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    p[i] = (mx == LLMA_NEG_INF) ? 0.f : __expf(sv[i] - mx);
                    lsum += p[i];
                }
                mrow = mx;
                u32x2 h0, l0, h1, l1;
                split4(p, h0, l0);
                split4(p + 4, h1, l1);
                const u32x4 ph = (u32x4){h0[0], h0[1], h1[0], h1[1]};
                const u32x4 pl = (u32x4){l0[0], l0[1], l1[0], l1[1]};
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    o[dt] = mfma16x16x32(va[dt], ph, o[dt]);
                    o[dt] = mfma16x16x32(va[dt], pl, o[dt]);
                    if (KVS && use_lo) o[dt] = mfma16x16x32(lo8_operand(vb[dt]), ph, o[dt]);
                }
            }
            // publish this wave's (max, sum, O) of the row tile
            lsum += __shfl_xor(lsum, 16);
            lsum += __shfl_xor(lsum, 32);
            if (g == 0) { sm[wave][q * 16 + n] = mrow; sl[wave][q * 16 + n] = lsum; }
            if (q * 16 + n < RS)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) *(f32x4 *)&so[wave][q * 16 + n][dt * 16 + 4 * g] = o[dt];
        }
        __syncthreads();
        // merge the four waves in wave order, then fold the chunk into the running state (chunk order)
#pragma unroll
        for (int i = 0; i < OWN; ++i) {
            const int idx = threadIdx.x + 256 * i;
            if (idx < m_blk * (DH / 4)) {
                const int j = idx / (DH / 4), d4 = idx % (DH / 4);
                float Mc = LLMA_NEG_INF;
#pragma unroll
                for (int w = 0; w < 4; ++w) Mc = fmaxf(Mc, sm[w][j]);
                if (Mc != LLMA_NEG_INF) {
                    f32x4 accc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const float mw = sm[w][j];
                        const float sc = (mw == LLMA_NEG_INF) ? 0.f : __expf(mw - Mc);
                        accc += *(const f32x4 *)&so[w][j][d4 * 4] * sc;
                    }
                    const float Mn = fmaxf(M_run[i], Mc);
                    const float s_run = (M_run[i] == LLMA_NEG_INF) ? 0.f : __expf(M_run[i] - Mn);
                    acc_run[i] = acc_run[i] * s_run + accc * __expf(Mc - Mn);
                    M_run[i] = Mn;
                }
            }
        }
        if (threadIdx.x < m_blk) {
            const int j = threadIdx.x;
            float Mc = LLMA_NEG_INF;
            for (int w = 0; w < 4; ++w) Mc = fmaxf(Mc, sm[w][j]);
            if (Mc != LLMA_NEG_INF) {
                float Lc = 0.f;
                for (int w = 0; w < 4; ++w) {
                    const float mw = sm[w][j];
                    Lc += (mw == LLMA_NEG_INF) ? 0.f : sl[w][j] * __expf(mw - Mc);
                }
                const float Mn = fmaxf(M_row, Mc);
                const float s_run = (M_row == LLMA_NEG_INF) ? 0.f : __expf(M_row - Mn);
                L_row = L_row * s_run + Lc * __expf(Mc - Mn);
                M_row = Mn;
            }
        }
        __syncthreads();                                             // the merge buffers are written again by the next chunk
    }
    const size_t pbase = (((size_t)b * a.H + h) * a.n_chunks + blockIdx.x) * ((size_t)a.n_rblocks * RQ) + j0;
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
        const int idx = threadIdx.x + 256 * i;
        if (idx < m_blk * (DH / 4)) {
            const int j = idx / (DH / 4), d4 = idx % (DH / 4);
            *(f32x4 *)(a.po + (pbase + j) * DH + d4 * 4) = acc_run[i];
        }
    }
    if (threadIdx.x < m_blk) {
        a.pm[pbase + threadIdx.x] = M_row;
        a.pl[pbase + threadIdx.x] = L_row;
    }
}

// The same walk for one or two row tiles with the running state per WAVE: a wave folds its 32 positions
// of every chunk into its own (max, sum, O) in registers -- no LDS and no barrier inside the walk, so
// the eight waves of a compute unit drift apart and one wave's arithmetic hides the other's loads --
// and the four waves are merged once, in wave order, at the end of the walk.  A row's result is
// again a function of absolute positions only (wave w: positions 32 w .. 32 w + 31 of each chunk of
// the walk in chunk order; then the waves in order; then the walks in order in the combine kernel).
template <int DH, int NTQ, bool KVS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_walk_wave_bf16_kernel(AttnArgs a) {
    constexpr int KSTEPS = DH / 32, DT = DH / 16;
    constexpr int RQ = NTQ * 16;
    constexpr int OWN = (RQ * (DH / 4) + 255) / 256;                  // merged output elements (float4) per thread
    __shared__ float sm[4][RQ], sl[4][RQ];
    __shared__ float so[4][RQ][DH + 4];
    const int h = blockIdx.y, b = blockIdx.z / a.n_rblocks, rb = blockIdx.z % a.n_rblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int slot = a.batch_slots[b];
    const int T = a.T[slot];
    const int lo_from = (KVS && a.lo_from != nullptr) ? a.lo_from[slot] : 0;
    const int m = a.m, j0 = rb * RQ;
    if (j0 >= m) return;
    const int m_blk = (m - j0 < RQ) ? m - j0 : RQ;
    const int kv_len = T + j0 + m_blk;                               // positions the block's last row can see
    const int c0 = blockIdx.x * ATTN_WALK_CHUNKS;
    if (c0 * ATTN_CHUNK >= kv_len) return;                           // uniform for the workgroup
    const int c_need = (kv_len + ATTN_CHUNK - 1) / ATTN_CHUNK;
    const int c1 = c0 + ATTN_WALK_CHUNKS < c_need ? c0 + ATTN_WALK_CHUNKS : c_need;
    int c_lo = KVS ? lo_from / ATTN_CHUNK : c1;                      // chunks below c_lo: imported bf16 cache, single plane
    c_lo = c_lo < c0 ? c0 : (c_lo > c1 ? c1 : c_lo);
    const int d_model = a.H * DH;
    const size_t head_base = ((size_t)slot * a.H + h) * (size_t)a.max_seq * DH;
    const bf16_t *kh = (const bf16_t *)a.Khi + head_base; const uint8_t *kl = (const uint8_t *)a.Klo + head_base;
    const bf16_t *vh = (const bf16_t *)a.Vhi + head_base; const uint8_t *vl = (const uint8_t *)a.Vlo + head_base;

    // the block's query rows (both planes) stay on chip for the whole walk: in registers for one row
    // tile; for two, as MFMA operands in LDS (in the merge buffer, which is not needed before the end)
    constexpr bool QLDS = NTQ > 1;
    u32x4 qh[QLDS ? 1 : NTQ][KSTEPS], ql[QLDS ? 1 : NTQ][KSTEPS];
    u32x4 *qs = (u32x4 *)&so[0][0][0];                               // [NTQ][2 planes][KSTEPS][64 lanes]
    int rpos[NTQ];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        const int j = j0 + q * 16 + n;
        const bool valid = j < m;
        rpos[q] = valid ? T + j : -1;
        const int r = b * m + (valid ? j : j0);
        if (!QLDS) {
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const size_t off = xtile_off(r, h * DH + s * 32 + g * 8, d_model / 32);
                qh[q][s] = *(const u32x4 *)((const bf16_t *)a.Qhi + off);
                ql[q][s] = *(const u32x4 *)((const bf16_t *)a.Qlo + off);
            }
        } else {
            for (int s = wave; s < KSTEPS; s += 4) {                 // (the four waves share the staging)
                const size_t off = xtile_off(r, h * DH + s * 32 + g * 8, d_model / 32);
                qs[((q * 2 + 0) * KSTEPS + s) * 64 + lane] = *(const u32x4 *)((const bf16_t *)a.Qhi + off);
                qs[((q * 2 + 1) * KSTEPS + s) * 64 + lane] = *(const u32x4 *)((const bf16_t *)a.Qlo + off);
            }
        }
    }
    if (QLDS) __syncthreads();
    f32x4 o[NTQ][DT];
    float Mw[NTQ], Lw[NTQ];                                          // row n's running max; the lane's share of its running sum
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        Mw[q] = LLMA_NEG_INF; Lw[q] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[q][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    // one chunk of the wave; LO: the chunk has lo planes (a constant per call site, so that every load
    // of the chunk is unconditional)
    auto chunk = [&](int c, auto lo_tag) {
        constexpr bool LO = decltype(lo_tag)::value;
        const int key0 = c * ATTN_CHUNK + wave * 32;
        if (key0 >= kv_len) return;                                  // uniform for the wave: no row sees these positions
        u32x4 ka[2][KSTEPS], va[DT];
        u32x2 kb[2][KSTEPS], vb[DT];                     // lo planes: one byte per element
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const size_t off = (size_t)(key0 / 16 + t) * (16 * DH) + s * 512 + lane * 8;
                ka[t][s] = *(const u32x4 *)(kh + off);
                if (LO) kb[t][s] = *(const u32x2 *)(kl + off);
            }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const size_t off = (size_t)(key0 / 32) * (32 * DH) + dt * 512 + lane * 8;
            va[dt] = *(const u32x4 *)(vh + off);
            if (LO) vb[dt] = *(const u32x2 *)(vl + off);
        }
        __builtin_amdgcn_sched_barrier(0);                           // all of the chunk's blocks are in flight before the first is used
#pragma unroll
        for (int q = 0; q < NTQ; ++q) {
            if (j0 + q * 16 >= m) continue;                          // a row tile past the block's rows (uniform)
            float sv[8];
            float mx = LLMA_NEG_INF;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    const u32x4 q_hi = QLDS ? qs[((q * 2 + 0) * KSTEPS + s) * 64 + lane] : qh[QLDS ? 0 : q][s];
                    const u32x4 q_lo = QLDS ? qs[((q * 2 + 1) * KSTEPS + s) * 64 + lane] : ql[QLDS ? 0 : q][s];
                    acc = mfma16x16x32(ka[t][s], q_hi, acc);
                    acc = mfma16x16x32(ka[t][s], q_lo, acc);
                    if (LO) acc = mfma16x16x32(lo8_operand(kb[t][s]), q_hi, acc);
                }
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int key = key0 + t * 16 + 4 * g + r4;
                    float v = acc[r4] * a.scale;
                    v = (key > rpos[q]) ? LLMA_NEG_INF : v;
                    sv[t * 4 + r4] = v;
                    mx = fmaxf(mx, v);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float Mn = fmaxf(Mw[q], mx);
            const float s_old = (Mw[q] == LLMA_NEG_INF) ? 0.f : __expf(Mw[q] - Mn);     // (Mn = -inf only if both are)
            float p[8], lsum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = (Mn == LLMA_NEG_INF) ? 0.f : __expf(sv[i] - Mn);
                lsum += p[i];
            }
            Lw[q] = Lw[q] * s_old + lsum;
            Mw[q] = Mn;
            u32x2 h0, l0, h1, l1;
            split4(p, h0, l0);
            split4(p + 4, h1, l1);
            const u32x4 ph = (u32x4){h0[0], h0[1], h1[0], h1[1]};
            const u32x4 pl = (u32x4){l0[0], l0[1], l1[0], l1[1]};
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                f32x4 od = o[q][dt] * s_old;
                od = mfma16x16x32(va[dt], ph, od);
                od = mfma16x16x32(va[dt], pl, od);
                if (LO) od = mfma16x16x32(lo8_operand(vb[dt]), ph, od);
                o[q][dt] = od;
            }
        }
    };
    for (int c = c0; c < c_lo; ++c) chunk(c, std::false_type{});
    if (KVS)
        for (int c = c_lo; c < c1; ++c) chunk(c, std::true_type{});

    // publish the waves' states, merge them in wave order, write the walk's partial
    if (QLDS) __syncthreads();                                       // every wave is done with the staged query rows
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        float lsum = Lw[q];
        lsum += __shfl_xor(lsum, 16);
        lsum += __shfl_xor(lsum, 32);
        if (g == 0) { sm[wave][q * 16 + n] = Mw[q]; sl[wave][q * 16 + n] = lsum; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) *(f32x4 *)&so[wave][q * 16 + n][dt * 16 + 4 * g] = o[q][dt];
    }
    __syncthreads();
    const size_t pbase = (((size_t)b * a.H + h) * a.n_chunks + blockIdx.x) * ((size_t)a.n_rblocks * RQ) + j0;
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
        const int idx = threadIdx.x + 256 * i;
        if (idx < m_blk * (DH / 4)) {
            const int j = idx / (DH / 4), d4 = idx % (DH / 4);
            float Mc = LLMA_NEG_INF;
#pragma unroll
            for (int w = 0; w < 4; ++w) Mc = fmaxf(Mc, sm[w][j]);
            f32x4 accc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float mw = sm[w][j];
                const float sc = (mw == LLMA_NEG_INF) ? 0.f : __expf(mw - Mc);
                accc += *(const f32x4 *)&so[w][j][d4 * 4] * sc;
            }
            *(f32x4 *)(a.po + (pbase + j) * DH + d4 * 4) = accc;
        }
    }
    if (threadIdx.x < m_blk) {
        const int j = threadIdx.x;
        float Mc = LLMA_NEG_INF, Lc = 0.f;
        for (int w = 0; w < 4; ++w) Mc = fmaxf(Mc, sm[w][j]);
        for (int w = 0; w < 4; ++w) {
            const float mw = sm[w][j];
            Lc += (mw == LLMA_NEG_INF) ? 0.f : sl[w][j] * __expf(mw - Mc);
        }
        a.pm[pbase + j] = Mc;
        a.pl[pbase + j] = Lc;
    }
}

// merges the chunk partials of one (row, head): out = sum_c e^{m_c - M} O_c / sum_c e^{m_c - M} l_c,
// over the chunks that contain positions <= the row's own, in chunk order; writes hi/lo tiled planes.
// One thread per 4 output features; the partials of 16 chunks are in flight at a time.
template <int DH>
__global__ void attn_combine_bf16_kernel(AttnArgs a, int rq) {
    constexpr int CB = 16;                             // chunks per load batch
    const int r = blockIdx.x, h = blockIdx.y;
    const int b = r / a.m, j = r % a.m;
    const int slot = a.slot_const >= 0 ? a.slot_const : a.batch_slots[b];
    // live-row count and sequence length: requested before the partials, used after them (one
    // round trip to memory for all three instead of three in a row)
    const int live_last = a.rows_live != nullptr ? *a.rows_live : a.m;
    const int T = a.T[slot];
    loads_stay_above();
    const int d4 = threadIdx.x;                        // features 4 d4 .. +3
    const size_t base = ((size_t)b * a.H + h) * a.n_chunks;
    // the first batch of partials is requested before the row's position is known: every launched
    // chunk has storage, and what a chunk past the row's last one holds is dropped below
    float mv[CB], lv[CB];
    f32x4 ov[CB];
    auto fetch = [&](int c0) {
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            const int c = (c0 + u < a.n_chunks) ? c0 + u : a.n_chunks - 1;
            mv[u] = a.pm[(base + c) * rq + j];
            lv[u] = a.pl[(base + c) * rq + j];
            ov[u] = (*(const f32x4 *)(a.po + ((base + c) * rq + j) * DH + d4 * 4));
        }
    };
    fetch(0);
    loads_stay_above();
    if (j > live_last) return;                         // padding row of a generation step (its partials are stale: dropped)
    const int pos = T + j;
    const int nc = pos / a.part_span + 1;
    // running (max, sum, O) over the chunks in chunk order
    float M = LLMA_NEG_INF, L = 0.f;
    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < nc; c0 += CB) {
        if (c0 > 0) fetch(c0);
        float Mb = M;
#pragma unroll
        for (int u = 0; u < CB; ++u)
            if (c0 + u < nc) Mb = fmaxf(Mb, mv[u]);
        const float rs = (M == LLMA_NEG_INF) ? 0.f : __expf(M - Mb);
        L *= rs;
        acc *= rs;
        M = Mb;
#pragma unroll
        for (int u = 0; u < CB; ++u)
            if (c0 + u < nc) {
                const float w = (mv[u] == LLMA_NEG_INF) ? 0.f : __expf(mv[u] - M);
                L += w * lv[u];
                acc += ov[u] * w;
            }
    }
    float v[4] = {acc[0] / L, acc[1] / L, acc[2] / L, acc[3] / L};
    u32x2 hi, lo;
    split4(v, hi, lo);
    const size_t o = xtile_off(r, h * DH + d4 * 4, a.out_KSp);
    *(u32x2 *)((bf16_t *)a.out_hi + o) = hi;
    *(u32x2 *)((bf16_t *)a.out_lo + o) = lo;
}

// ---------------------------------------------------------------------------------------------
// Prompt-pass attention (more than 48 rows of one sequence): a workgroup owns 32 query rows of one
// head and walks over all 128-position chunks its rows can see; wave w takes positions
// 32 w .. 32 w + 31 of every chunk and keeps its own running (max, sum, O) over them (online
// softmax, no synchronisation inside the walk), the next chunk's K/V blocks are requested while the
// current one is multiplied; at the end the four waves merge through LDS in wave order and the
// normalised rows go straight to the hi/lo planes -- no partials, no combine kernel.  Row blocks
// are numbered from the end of the prompt (longest walks start first).
// ---------------------------------------------------------------------------------------------
template <int DH, bool KVS>
__global__ __launch_bounds__(256) void attn_prompt_bf16_kernel(AttnArgs a) {
    constexpr int KSTEPS = DH / 32, DT = DH / 16, NTQ = 2, RQ = NTQ * 16;
    __shared__ float sm[4][RQ], sl[4][RQ];
    __shared__ float so[4][RQ][DH + 4];
    const int rb = gridDim.x - 1 - blockIdx.x, h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int slot = a.slot_const;
    const int m = a.m, j0 = rb * RQ;
    const int m_blk = (m - j0 < RQ) ? m - j0 : RQ;
    const int d_model = a.H * DH;
    const size_t head_base = ((size_t)slot * a.H + h) * (size_t)a.max_seq * DH;
    const bf16_t *kh = (const bf16_t *)a.Khi + head_base; const uint8_t *kl = (const uint8_t *)a.Klo + head_base;
    const bf16_t *vh = (const bf16_t *)a.Vhi + head_base; const uint8_t *vl = (const uint8_t *)a.Vlo + head_base;
    const int T = a.T[slot];
    const int kv_len = T + j0 + m_blk;                  // positions the block's last row can see
    const int n_ch = (kv_len + ATTN_CHUNK - 1) / ATTN_CHUNK;

    u32x4 qh[NTQ][KSTEPS], ql[NTQ][KSTEPS];
    int rpos[NTQ];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        const int j = j0 + q * 16 + n;
        rpos[q] = j < m ? T + j : -1;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const size_t off = xtile_off(j < m ? j : 0, h * DH + s * 32 + g * 8, d_model / 32);
            qh[q][s] = *(const u32x4 *)((const bf16_t *)a.Qhi + off);
            ql[q][s] = *(const u32x4 *)((const bf16_t *)a.Qlo + off);
        }
    }
    auto fetch = [&](int c, u32x4 (&ka)[2][KSTEPS], u32x2 (&kb)[2][KSTEPS], u32x4 (&va)[DT], u32x2 (&vb)[DT]) {
        const int key0 = c * ATTN_CHUNK + wave * 32;    // below the rounded capacity for every launched chunk
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const size_t off = (size_t)(key0 / 16 + t) * (16 * DH) + s * 512 + lane * 8;
                ka[t][s] = *(const u32x4 *)(kh + off);
                if (KVS) kb[t][s] = *(const u32x2 *)(kl + off);
            }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const size_t off = (size_t)(key0 / 32) * (32 * DH) + dt * 512 + lane * 8;
            va[dt] = *(const u32x4 *)(vh + off);
            if (KVS) vb[dt] = *(const u32x2 *)(vl + off);
        }
    };
    float mrow[NTQ], lrow[NTQ];
    f32x4 o[NTQ][DT];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        mrow[q] = LLMA_NEG_INF;
        lrow[q] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[q][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    auto consume = [&](int c, u32x4 (&ka)[2][KSTEPS], u32x2 (&kb)[2][KSTEPS], u32x4 (&va)[DT], u32x2 (&vb)[DT]) {
        const int key0 = c * ATTN_CHUNK + wave * 32;
        if (key0 >= kv_len) return;                     // uniform for the wave
#pragma unroll
        for (int q = 0; q < NTQ; ++q) {
            float sv[8];
            float mx = LLMA_NEG_INF;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    acc = mfma16x16x32(ka[t][s], qh[q][s], acc);
                    acc = mfma16x16x32(ka[t][s], ql[q][s], acc);
                    if (KVS) acc = mfma16x16x32(lo8_operand(kb[t][s]), qh[q][s], acc);
                }
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int key = key0 + t * 16 + 4 * g + r4;
                    float v = acc[r4] * a.scale;
                    v = (key > rpos[q]) ? LLMA_NEG_INF : v;
                    sv[t * 4 + r4] = v;
                    mx = fmaxf(mx, v);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(mrow[q], mx);
            const float alpha = (mrow[q] == LLMA_NEG_INF) ? 0.f : __expf(mrow[q] - m_new);   // m_new finite then
            float psum = 0.f;
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = (m_new == LLMA_NEG_INF) ? 0.f : __expf(sv[i] - m_new);
                psum += p[i];
            }
            lrow[q] = lrow[q] * alpha + psum;           // this lane's 8 keys; lanes are added at the end
            mrow[q] = m_new;
            u32x2 h0, l0, h1, l1;
            split4(p, h0, l0);
            split4(p + 4, h1, l1);
            const u32x4 ph = (u32x4){h0[0], h0[1], h1[0], h1[1]};
            const u32x4 pl = (u32x4){l0[0], l0[1], l1[0], l1[1]};
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[q][dt] *= alpha;
                o[q][dt] = mfma16x16x32(va[dt], ph, o[q][dt]);
                o[q][dt] = mfma16x16x32(va[dt], pl, o[q][dt]);
                if (KVS) o[q][dt] = mfma16x16x32(lo8_operand(vb[dt]), ph, o[q][dt]);
            }
        }
    };
    u32x4 kaA[2][KSTEPS], vaA[DT], kaB[2][KSTEPS], vaB[DT];
    u32x2 kbA[2][KSTEPS], vbA[DT], kbB[2][KSTEPS], vbB[DT];
    fetch(0, kaA, kbA, vaA, vbA);
    for (int c = 0; c < n_ch; c += 2) {
        if (c + 1 < n_ch) fetch(c + 1, kaB, kbB, vaB, vbB);
        consume(c, kaA, kbA, vaA, vbA);
        if (c + 1 >= n_ch) break;
        if (c + 2 < n_ch) fetch(c + 2, kaA, kbA, vaA, vbA);
        consume(c + 1, kaB, kbB, vaB, vbB);
    }
    // ---- merge the four waves in wave order, normalise, write the hi/lo planes
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        float l = lrow[q];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (g == 0) { sm[wave][q * 16 + n] = mrow[q]; sl[wave][q * 16 + n] = l; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) *(f32x4 *)&so[wave][q * 16 + n][dt * 16 + 4 * g] = o[q][dt];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < m_blk * (DH / 4); idx += 256) {
        const int j = idx / (DH / 4), d4 = idx % (DH / 4);
        float M = LLMA_NEG_INF;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sm[w][j]);
        f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = sm[w][j];
            const float sc = (mw == LLMA_NEG_INF) ? 0.f : __expf(mw - M);
            acc += *(const f32x4 *)&so[w][j][d4 * 4] * sc;
            L += sl[w][j] * sc;
        }
        float v[4] = {acc[0] / L, acc[1] / L, acc[2] / L, acc[3] / L};
        u32x2 hi, lo;
        split4(v, hi, lo);
        const size_t off = xtile_off(j0 + j, h * DH + d4 * 4, a.out_KSp);
        *(u32x2 *)((bf16_t *)a.out_hi + off) = hi;
        *(u32x2 *)((bf16_t *)a.out_lo + off) = lo;
    }
}

template <int DH, bool KVS>
static void launch_attn_dh(const AttnArgs &a0, hipStream_t st) {
    // up to 48 rows per workgroup; longer row lists (prompt processing) are cut into row blocks
    AttnArgs a = a0;
    if (a.n_seqs == 1 && a.m > 48 && a.slot_const >= 0) {           // prompt pass
        hipLaunchKernelGGL((attn_prompt_bf16_kernel<DH, KVS>), dim3((a.m + 31) / 32, a.H), dim3(256), 0, st, a);
        return;
    }
    const int ntq = a.m > 32 ? 3 : (a.m + 15) / 16;
    a.n_rblocks = (a.m + ntq * 16 - 1) / (ntq * 16);
    a.part_span = ATTN_CHUNK;
    if (a.rows_live == nullptr && a.slot_const < 0 && a.n_seqs * a.m > 48 && a.m <= ATTN_COMPACT_ROWS) {     // wide batched step
        a.n_chunks = (a.n_chunks + ATTN_WALK_CHUNKS - 1) / ATTN_WALK_CHUNKS;
        a.part_span = ATTN_CHUNK * ATTN_WALK_CHUNKS;
        dim3 wgrid(a.n_chunks, a.H, a.n_seqs * a.n_rblocks);
        if (ntq == 1) hipLaunchKernelGGL((attn_walk_wave_bf16_kernel<DH, 1, KVS>), wgrid, dim3(256), 0, st, a);
        else if (ntq == 2) hipLaunchKernelGGL((attn_walk_wave_bf16_kernel<DH, 2, KVS>), wgrid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((attn_walk_bf16_kernel<DH, 3, KVS>), wgrid, dim3(256), 0, st, a);
        hipLaunchKernelGGL((attn_combine_bf16_kernel<DH>), dim3(a.n_seqs * a.m, a.H), dim3(DH / 4), 0, st, a, a.n_rblocks * ntq * 16);
        return;
    }
    dim3 grid(a.n_chunks, a.H, a.n_seqs * a.n_rblocks);
    if (a.rows_live != nullptr) {                      // generation step of one sequence: padding rows known on the device
        if (ntq == 1) hipLaunchKernelGGL((attn_bf16_kernel<DH, 1, KVS, true>), grid, dim3(256), 0, st, a);
        else if (ntq == 2) hipLaunchKernelGGL((attn_bf16_kernel<DH, 2, KVS, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((attn_bf16_kernel<DH, 3, KVS, true>), grid, dim3(256), 0, st, a);
    } else if (KVS && a.slot_const < 0 && a.lo_from != nullptr) {   // several sequences: their caches may have been imported
        if (ntq == 1) hipLaunchKernelGGL((attn_bf16_kernel<DH, 1, KVS, false, true>), grid, dim3(256), 0, st, a);
        else if (ntq == 2) hipLaunchKernelGGL((attn_bf16_kernel<DH, 2, KVS, false, true>), grid, dim3(256), 0, st, a);
        else if (a.m <= ATTN_COMPACT_ROWS) hipLaunchKernelGGL((attn_bf16_kernel<DH, 3, KVS, false, true, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((attn_bf16_kernel<DH, 3, KVS, false, true>), grid, dim3(256), 0, st, a);
    } else if (ntq == 1) hipLaunchKernelGGL((attn_bf16_kernel<DH, 1, KVS, false>), grid, dim3(256), 0, st, a);
    else if (ntq == 2) hipLaunchKernelGGL((attn_bf16_kernel<DH, 2, KVS, false>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_bf16_kernel<DH, 3, KVS, false>), grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL((attn_combine_bf16_kernel<DH>), dim3(a.n_seqs * a.m, a.H), dim3(DH / 4), 0, st, a, a.n_rblocks * ntq * 16);
}

void launch_attn_bf16(const AttnArgs &a, hipStream_t st) {
    const bool kvs = a.Klo != nullptr;
    if (a.dh == 128) { if (kvs) launch_attn_dh<128, true>(a, st); else launch_attn_dh<128, false>(a, st); }
    else { if (kvs) launch_attn_dh<64, true>(a, st); else launch_attn_dh<64, false>(a, st); }
}
