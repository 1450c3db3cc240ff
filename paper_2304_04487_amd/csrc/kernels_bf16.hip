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
#include "common.h"
#include "kernels.h"

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
                                      bf16_t *__restrict__ kh, bf16_t *__restrict__ kl,
                                      bf16_t *__restrict__ vh, bf16_t *__restrict__ vl,
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
                       (bf16_t *)kh, (bf16_t *)kl, (bf16_t *)vh, (bf16_t *)vl, H, len, dh, max_seq);
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
// The K axis is cut into S slices.  A workgroup belongs to one slice: it copies that slice of
// the activations (hi and lo planes, already in B-operand order) into LDS once, then each of its
// 4 waves walks over feature tiles, streaming the slice's KSS weight blocks of a tile straight
// from HBM into MFMA A operands (non-temporal, 1 KiB per wave-load) and taking B operands from
// LDS.  D[i][n] = sum_k A[i][k] B[k][n] with i = feature, n = activation row, so lane l ends
// with features 4(l/16)..+3 of row l%16.  Each (tile, slice) partial goes to a scratch buffer;
// the wave that draws the last ticket of a tile adds the S partials in slice order (so the sum
// does not depend on arrival order) and runs the fused epilogue.  S, KSS and the tile walk
// depend on the matrix shape only.
template <int NT, int EPI, bool SPLIT>
__global__ __launch_bounds__(256) void gemm_slicek_bf16(GemmArgs a) {
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    constexpr int U = (TILES == 2) ? 4 : 8;
    constexpr int PL = SPLIT ? 2 : 1;
    extern __shared__ u32x4 xs[];                  // [PL][NT][KSS][64], then rstd[16*NT] floats
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GemmPlan &p = a.plan;
    const int S = p.S, KSS = p.KSS, KSp = p.KSp;
    const int s = blockIdx.x % S, g = blockIdx.x / S;
    const int ks0 = s * KSS;
    float *rstd_s = (float *)(xs + (size_t)PL * NT * KSS * 64);

    // ---- activations of this slice -> LDS
    {
        const int per_plane = NT * KSS * 64;       // 16-byte pieces
        for (int i = threadIdx.x; i < per_plane; i += 256) {
            const int t = i / (KSS * 64), rem = i % (KSS * 64);
            const size_t src = ((size_t)t * KSp + ks0) * 64 + rem;
            xs[i] = ((const u32x4 *)a.Xhi)[src];
            if (SPLIT) xs[per_plane + i] = ((const u32x4 *)a.Xlo)[src];
        }
    }
    // ---- rstd of the rows from the producer's per-tile sums of squares: thread (row, i) adds
    //      tiles i, i+16, ... then the 16 threads of a row are combined by butterfly
    if (EPI != EPI_RESID) {
        const int row = threadIdx.x >> 4, i = threadIdx.x & 15;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int r = t * 16 + row;
            float ss = 0.f;
            if (r < a.rows)
                for (int j = i; j < a.ssq_tiles; j += 16) ss += a.ssq_in[(size_t)r * a.ssq_tiles + j];
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) ss += __shfl_xor(ss, off);
            if (i == 0) rstd_s[r] = 1.0f / sqrtf(ss / (float)(a.ssq_tiles * 16) + a.eps);
        }
    }
    __syncthreads();

    const int stride = p.G * 4;
    for (int task = g * 4 + wave; task < p.tasks; task += stride) {
        const u32x4 *wp[TILES];
        wp[0] = (const u32x4 *)a.W + ((size_t)task * KSp + ks0) * 64 + lane;
        if (TILES == 2) wp[1] = (const u32x4 *)a.W + ((size_t)(task + p.tasks) * KSp + ks0) * 64 + lane;
        f32x4 acc[TILES][NT];
#pragma unroll
        for (int i = 0; i < TILES; ++i)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[i][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        int k = 0;
        for (; k + U <= KSS; k += U) {
            u32x4 av[TILES][U];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < TILES; ++i) av[i][u] = __builtin_nontemporal_load(wp[i] + (k + u) * 64);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const u32x4 bh = xs[(t * KSS + k + u) * 64 + lane];
#pragma unroll
                    for (int i = 0; i < TILES; ++i) acc[i][t] = mfma16x16x32(av[i][u], bh, acc[i][t]);
                    if (SPLIT) {
                        const u32x4 bl = xs[((NT + t) * KSS + k + u) * 64 + lane];
#pragma unroll
                        for (int i = 0; i < TILES; ++i) acc[i][t] = mfma16x16x32(av[i][u], bl, acc[i][t]);
                    }
                }
        }
        for (; k < KSS; ++k) {
            u32x4 av[TILES];
#pragma unroll
            for (int i = 0; i < TILES; ++i) av[i] = __builtin_nontemporal_load(wp[i] + k * 64);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const u32x4 bh = xs[(t * KSS + k) * 64 + lane];
#pragma unroll
                for (int i = 0; i < TILES; ++i) acc[i][t] = mfma16x16x32(av[i], bh, acc[i][t]);
                if (SPLIT) {
                    const u32x4 bl = xs[((NT + t) * KSS + k) * 64 + lane];
#pragma unroll
                    for (int i = 0; i < TILES; ++i) acc[i][t] = mfma16x16x32(av[i], bl, acc[i][t]);
                }
            }
        }

        // ---- (tile, slice) partial -> scratch; last ticket of the tile adds them in slice order
        if (S > 1) {
            f32x4 *pp = (f32x4 *)a.partial + ((size_t)task * S + s) * (TILES * NT * 64) + lane;
#pragma unroll
            for (int i = 0; i < TILES; ++i)
#pragma unroll
                for (int t = 0; t < NT; ++t) pp[(i * NT + t) * 64] = acc[i][t];
            __threadfence();
            int tk = 0;
            if (lane == 0) tk = atomicAdd(a.ticket + task, 1);
            tk = __shfl(tk, 0);
            if (tk != S - 1) continue;
            __threadfence();
            const f32x4 *pq = (const f32x4 *)a.partial + (size_t)task * S * (TILES * NT * 64) + lane;
#pragma unroll
            for (int i = 0; i < TILES; ++i)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    f32x4 sum = pq[(i * NT + t) * 64];
                    for (int s2 = 1; s2 < S; ++s2) sum += pq[((size_t)s2 * TILES * NT + i * NT + t) * 64];
                    acc[i][t] = sum;
                }
            if (lane == 0) a.ticket[task] = 0;
        }

        // ---- epilogue: lane holds features 16 task + 4 g4 .. +3 of row 16 t + n
        const int n = lane & 15, g4 = lane >> 4;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int row = t * 16 + n;
            const bool live = row < a.rows;
            const int f0 = task * 16 + g4 * 4;
            if (EPI == EPI_RESID) {
                float hn[4], x[4];
                float ss = 0.f;
                if (live) {
                    f32x4 *hp = (f32x4 *)(a.out + (size_t)row * p.N + f0);
                    const f32x4 hv = *hp + acc[0][t];
                    *hp = hv;
                    const f32x4 gv = *(const f32x4 *)(a.gain + f0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) { hn[r] = hv[r]; ss += hn[r] * hn[r]; x[r] = hn[r] * gv[r]; }
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
                const int pos = live ? a.row_pos[row] : 0;
                const int slot = live ? a.row_slot[row] : 0;
                const size_t head_base = ((size_t)slot * a.H + head) * (size_t)a.max_seq * a.dh;
                if (sec < 2) {
                    const int half = a.dh / 2;
                    const int i0 = 8 * j + (g4 & 1) * 4;
                    float pr[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) pr[r] = __shfl_xor(v[r], 32);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float c = a.cs[((size_t)pos * half + i0 + r) * 2], sn = a.cs[((size_t)pos * half + i0 + r) * 2 + 1];
                        o4[r] = (g4 < 2) ? (v[r] * c - pr[r] * sn) : (v[r] * c + pr[r] * sn);
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
                            if (a.k_lo) *(u32x2 *)((bf16_t *)a.k_lo + o) = lo;
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
                        if (a.v_lo) ((bf16_t *)a.v_lo)[o] = lo;
                    }
                }
            }
        }
    }
}

template <int NT, int EPI>
static void launch_gemm_nt_epi(const GemmArgs &a, hipStream_t st) {
    const GemmPlan &p = a.plan;
    const int planes = a.split ? 2 : 1;
    const size_t lds = (size_t)planes * NT * p.KSS * 1024 + 64 * sizeof(float);
    dim3 grid(p.S * p.G), block(256);
    if (a.split) {
        static bool attr_done = false;
        if (!attr_done) { (void)hipFuncSetAttribute((const void *)gemm_slicek_bf16<NT, EPI, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); attr_done = true; }
        hipLaunchKernelGGL((gemm_slicek_bf16<NT, EPI, true>), grid, block, lds, st, a);
    } else {
        static bool attr_done = false;
        if (!attr_done) { (void)hipFuncSetAttribute((const void *)gemm_slicek_bf16<NT, EPI, false>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); attr_done = true; }
        hipLaunchKernelGGL((gemm_slicek_bf16<NT, EPI, false>), grid, block, lds, st, a);
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

// LDS bytes one workgroup needs for nt row tiles
size_t gemm_bf16_lds_bytes(const GemmPlan &p, int nt, int split) { return (size_t)(split ? 2 : 1) * nt * p.KSS * 1024 + 256; }

// rows are processed in blocks of whole 16-row tiles: as many tiles per launch (<= 3) as the
// activation slice leaves room for in LDS; weights are re-streamed per block
void launch_gemm_bf16(const GemmArgs &a0, hipStream_t st) {
    const GemmPlan &p = a0.plan;
    int nt_max = 3;
    while (nt_max > 1 && gemm_bf16_lds_bytes(p, nt_max, a0.split) > 150 * 1024) --nt_max;
    const int block_rows = nt_max * 16;
    for (int r0 = 0; r0 < a0.rows; r0 += block_rows) {
        GemmArgs a = a0;
        const int rows = a0.rows - r0 < block_rows ? a0.rows - r0 : block_rows;
        const int t0 = r0 / 16;
        a.rows = rows;
        a.Xhi = (const bf16_t *)a0.Xhi + (size_t)t0 * p.KSp * 512;
        a.Xlo = a0.Xlo ? (const bf16_t *)a0.Xlo + (size_t)t0 * p.KSp * 512 : nullptr;
        if (a0.ssq_in) a.ssq_in = a0.ssq_in + (size_t)r0 * a0.ssq_tiles;
        if (a0.out) a.out = a0.out + (size_t)r0 * p.N;
        if (a0.nx_hi) { a.nx_hi = (bf16_t *)a0.nx_hi + (size_t)t0 * a0.nx_KSp * 512; a.nx_lo = (bf16_t *)a0.nx_lo + (size_t)t0 * a0.nx_KSp * 512; }
        if (a0.ssq_out) a.ssq_out = a0.ssq_out + (size_t)r0 * (p.N / 16);
        if (a0.act_hi) { a.act_hi = (bf16_t *)a0.act_hi + (size_t)t0 * a0.act_KSp * 512; a.act_lo = (bf16_t *)a0.act_lo + (size_t)t0 * a0.act_KSp * 512; }
        if (a0.pval) { a.pval = a0.pval + (size_t)r0 * a0.n_part; a.pidx = a0.pidx + (size_t)r0 * a0.n_part; }
        if (a0.row_pos) { a.row_pos = a0.row_pos + r0; a.row_slot = a0.row_slot + r0; }
        if (a0.q_hi) { a.q_hi = (bf16_t *)a0.q_hi + (size_t)t0 * (a0.H * a0.dh / 32) * 512; a.q_lo = (bf16_t *)a0.q_lo + (size_t)t0 * (a0.H * a0.dh / 32) * 512; }
        if (rows <= 16) launch_gemm_nt<1>(a, st);
        else if (rows <= 32) launch_gemm_nt<2>(a, st);
        else launch_gemm_nt<3>(a, st);
    }
}

// how a [N][K] matrix is cut: slices of ~16 k-steps (padding K up if needed), ~2048-4096 waves
GemmPlan make_gemm_plan(int N, int K, int tiles_per_task) {
    GemmPlan p;
    p.N = N; p.K = K;
    const int KS = K / 32;
    int best_kss = 16, best_pad = 1 << 30;
    if (KS <= 24) { best_kss = KS; best_pad = 0; }
    else if (KS % 16 == 0) { best_kss = 16; best_pad = 0; }
    else
        for (int kss = 24; kss >= 12; --kss) {
            const int s = (KS + kss - 1) / kss, pad = s * kss - KS;
            if (pad < best_pad) { best_pad = pad; best_kss = kss; }
        }
    p.KSS = best_kss;
    p.S = (KS + best_kss - 1) / best_kss;
    p.KSp = p.S * p.KSS;
    p.tasks = N / 16;
    // tiles per wave so that S * G * 4 waves is about 2048..4096
    int waves_per_slice = 3072 / p.S;
    if (waves_per_slice < 4) waves_per_slice = 4;
    int tpw = (p.tasks + waves_per_slice - 1) / waves_per_slice;
    if (tpw < 1) tpw = 1;
    if (tiles_per_task == 2 && tpw > 2) tpw = (tpw + 1) / 2;
    p.G = (p.tasks + 4 * tpw - 1) / (4 * tpw);
    return p;
}

// =============================================================================================
// causal attention of m <= 16*NTQ query rows of one sequence over its KV cache
// =============================================================================================
// grid = (chunks of ATTN_CHUNK key positions, heads, sequences); 4 waves per workgroup, wave w
// owns the 64 positions [64 w, 64 w + 64) of the chunk as two groups of 32.  Per group:
// S^T = K_tile . Q^T (MFMA, keys on the A side so the cache is read as whole 1 KiB blocks; with
// hi/lo planes S = Khi.qhi + Khi.qlo + Klo.qhi), scale, causal mask by absolute position,
// online softmax per query row, O^T += V^T . P^T (again hi/lo).  The four waves' (max, sum, O)
// are merged in wave order, and the chunk's partial is written for the combine kernel.  Which
// keys a row sees, and in which order they are reduced, is a function of absolute positions only.
template <int DH, int NTQ, bool KVS>
__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnArgs a) {
    constexpr int KSTEPS = DH / 32;   // MFMA k-steps of a q.k dot product
    constexpr int DT = DH / 16;       // 16-feature tiles of the head dimension
    constexpr int RQ = NTQ * 16;
    __shared__ float sm[4][RQ], sl[4][RQ];
    __shared__ float so[RQ][DH + 4];

    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int slot = a.batch_slots[b];
    const int T = a.T[slot];
    const int m = a.m;
    const int kv_len = T + m;
    const int chunk0 = c * ATTN_CHUNK;
    if (chunk0 >= kv_len) return;                       // uniform for the workgroup
    const int d_model = a.H * DH;

    u32x4 qh[NTQ][KSTEPS], ql[NTQ][KSTEPS];
    int rpos[NTQ];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        const int j = q * 16 + n;
        const bool valid = j < m;
        rpos[q] = valid ? T + j : -1;
        const int r = b * m + (valid ? j : 0);
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const size_t o = xtile_off(r, h * DH + s * 32 + g * 8, d_model / 32);
            qh[q][s] = *(const u32x4 *)((const bf16_t *)a.Qhi + o);
            ql[q][s] = *(const u32x4 *)((const bf16_t *)a.Qlo + o);
        }
    }

    float mrow[NTQ], lrow[NTQ];
    f32x4 o[NTQ][DT];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        mrow[q] = LLMA_NEG_INF;
        lrow[q] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[q][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    const size_t head_base = ((size_t)slot * a.H + h) * (size_t)a.max_seq * DH;
    const bf16_t *kh = (const bf16_t *)a.Khi + head_base, *kl = (const bf16_t *)a.Klo + head_base;
    const bf16_t *vh = (const bf16_t *)a.Vhi + head_base, *vl = (const bf16_t *)a.Vlo + head_base;

#pragma unroll 1
    for (int gi = 0; gi < 2; ++gi) {
        const int key0 = chunk0 + (wave * 2 + gi) * 32;
        if (key0 >= kv_len) break;                      // uniform for the wave
        f32x4 s2[NTQ][2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            u32x4 ka[KSTEPS], kb[KSTEPS];
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const size_t off = (size_t)(key0 / 16 + t) * (16 * DH) + s * 512 + lane * 8;
                ka[s] = *(const u32x4 *)(kh + off);
                if (KVS) kb[s] = *(const u32x4 *)(kl + off);
            }
#pragma unroll
            for (int q = 0; q < NTQ; ++q) {
                f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    acc = mfma16x16x32(ka[s], qh[q][s], acc);
                    acc = mfma16x16x32(ka[s], ql[q][s], acc);
                    if (KVS) acc = mfma16x16x32(kb[s], qh[q][s], acc);
                }
                s2[q][t] = acc;
            }
        }
        u32x4 ph[NTQ], pl[NTQ];
#pragma unroll
        for (int q = 0; q < NTQ; ++q) {
            float sv[8];
            float mx = LLMA_NEG_INF;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int key = key0 + t * 16 + 4 * g + r;
                    float v = s2[q][t][r] * a.scale;
                    v = (key > rpos[q]) ? LLMA_NEG_INF : v;
                    sv[t * 4 + r] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float mnew = fmaxf(mrow[q], mx);
            float alpha = 1.f, psum = 0.f;
            float p[8];
            if (mnew == LLMA_NEG_INF) {
#pragma unroll
                for (int i = 0; i < 8; ++i) p[i] = 0.f;
            } else {
                alpha = __expf(mrow[q] - mnew);          // exp(-inf) = 0 on the first visible group
#pragma unroll
                for (int i = 0; i < 8; ++i) { p[i] = __expf(sv[i] - mnew); psum += p[i]; }
            }
            lrow[q] = lrow[q] * alpha + psum;
            mrow[q] = mnew;
            u32x2 h0, l0, h1, l1;
            split4(p, h0, l0);
            split4(p + 4, h1, l1);
            ph[q] = (u32x4){h0[0], h0[1], h1[0], h1[1]};
            pl[q] = (u32x4){l0[0], l0[1], l1[0], l1[1]};
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[q][dt] = o[q][dt] * alpha;
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const size_t off = (size_t)(key0 / 32) * (32 * DH) + dt * 512 + lane * 8;
            const u32x4 va = *(const u32x4 *)(vh + off);
            u32x4 vb;
            if (KVS) vb = *(const u32x4 *)(vl + off);
#pragma unroll
            for (int q = 0; q < NTQ; ++q) {
                o[q][dt] = mfma16x16x32(va, ph[q], o[q][dt]);
                o[q][dt] = mfma16x16x32(va, pl[q], o[q][dt]);
                if (KVS) o[q][dt] = mfma16x16x32(vb, ph[q], o[q][dt]);
            }
        }
    }

    // ---- merge the four waves in wave order ----
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        float l = lrow[q];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        lrow[q] = l;
        if (g == 0) { sm[wave][q * 16 + n] = mrow[q]; sl[wave][q * 16 + n] = l; }
    }
    __syncthreads();
    float scale_w[NTQ];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        float M = LLMA_NEG_INF;
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sm[w][q * 16 + n]);
        scale_w[q] = (mrow[q] == LLMA_NEG_INF) ? 0.f : __expf(mrow[q] - M);
    }
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int q = 0; q < NTQ; ++q)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    f32x4 v = o[q][dt] * scale_w[q];
                    f32x4 *p = (f32x4 *)&so[q * 16 + n][dt * 16 + 4 * g];
                    if (w == 0) *p = v; else *p = *p + v;
                }
        }
        __syncthreads();
    }
    // ---- write the chunk partial: rows j < m ----
    const size_t pbase = (((size_t)b * a.H + h) * a.n_chunks + c) * RQ;
    for (int idx = threadIdx.x; idx < m * DH; idx += 256) {
        int j = idx / DH, d = idx % DH;
        a.po[(pbase + j) * DH + d] = so[j][d];
    }
    if (threadIdx.x < m) {
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

// merges the chunk partials of one (row, head): out = sum_c e^{m_c - M} O_c / sum_c e^{m_c - M} l_c,
// over the chunks that contain positions <= the row's own, in chunk order; writes hi/lo tiled planes
template <int DH>
__global__ void attn_combine_bf16_kernel(AttnArgs a, int rq) {
    const int r = blockIdx.x, h = blockIdx.y;
    const int b = r / a.m, j = r % a.m;
    const int slot = a.batch_slots[b];
    const int pos = a.T[slot] + j;
    const int nc = pos / ATTN_CHUNK + 1;
    const int d = threadIdx.x;
    const size_t base = ((size_t)b * a.H + h) * a.n_chunks;
    float M = LLMA_NEG_INF;
    for (int c = 0; c < nc; ++c) M = fmaxf(M, a.pm[(base + c) * rq + j]);
    float L = 0.f, acc = 0.f;
    for (int c = 0; c < nc; ++c) {
        float w = __expf(a.pm[(base + c) * rq + j] - M);
        L += w * a.pl[(base + c) * rq + j];
        acc += w * a.po[((base + c) * rq + j) * DH + d];
    }
    float v = acc / L;
    bf16_t hi, lo;
    split_bf16(v, hi, lo);
    const size_t o = xtile_off(r, h * DH + d, a.out_KSp);
    ((bf16_t *)a.out_hi)[o] = hi;
    ((bf16_t *)a.out_lo)[o] = lo;
}

template <int DH, bool KVS>
static void launch_attn_dh(const AttnArgs &a, hipStream_t st) {
    const int ntq = (a.m + 15) / 16;
    dim3 grid(a.n_chunks, a.H, a.n_seqs);
    if (ntq == 1) hipLaunchKernelGGL((attn_bf16_kernel<DH, 1, KVS>), grid, dim3(256), 0, st, a);
    else if (ntq == 2) hipLaunchKernelGGL((attn_bf16_kernel<DH, 2, KVS>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_bf16_kernel<DH, 3, KVS>), grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL((attn_combine_bf16_kernel<DH>), dim3(a.n_seqs * a.m, a.H), dim3(DH), 0, st, a, ntq * 16);
}

void launch_attn_bf16(const AttnArgs &a, hipStream_t st) {
    const bool kvs = a.Klo != nullptr;
    if (a.dh == 128) { if (kvs) launch_attn_dh<128, true>(a, st); else launch_attn_dh<128, false>(a, st); }
    else { if (kvs) launch_attn_dh<64, true>(a, st); else launch_attn_dh<64, false>(a, st); }
}
