// bf16 kernels of the verification forward (paper: Eq. 3 -- one causal forward over the
// pending token plus k copied tokens): weight re-tiling, the skinny weight-streaming GEMM
// with its fused epilogues, and causal attention of a few query rows over a long KV cache.
//
// Everything here is HBM-bound at the row counts of a decoding step (1 + k <= 33 rows):
// the kernels are organised around streaming each weight / KV byte exactly once with
// fully coalesced 16-byte-per-lane loads, and use the MFMA unit only because it consumes
// those registers directly.  Reduction orders are fixed by the matrix shapes and by
// absolute key positions, never by the number of rows in the step, so row j of a k-row
// step is bit-identical to the same token processed in a one-row step.
#include "common.h"
#include "kernels.h"

// =============================================================================================
// weight re-tiling: row-major [N][K] bf16 -> 1 KiB MFMA A-operand blocks (see common.h)
// =============================================================================================
__global__ void pack_weight_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int N, int K) {
    // one thread per 16-byte piece of the destination
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)N * K / 8;
    if (idx >= total) return;
    int KS = K / 32;
    int lane = (int)(idx & 63);
    size_t blk = idx >> 6;
    int ks = (int)(blk % KS);
    size_t ft = blk / KS;
    size_t row = ft * 16 + (lane & 15);
    size_t col = (size_t)ks * 32 + (size_t)(lane >> 4) * 8;
    dst[idx] = src[(row * K + col) / 8];
}

void launch_pack_weight(const void *src, void *dst, int N, int K, hipStream_t st) {
    size_t total = (size_t)N * K / 8;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(pack_weight_kernel, dim3(blocks), dim3(256), 0, st, (const u32x4 *)src, (u32x4 *)dst, N, K);
}

// plain [H][len][dh] bf16 -> tiled K / V cache of one (slot, layer)
__global__ void kv_import_bf16_kernel(const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                      bf16_t *__restrict__ kc, bf16_t *__restrict__ vc,
                                      int H, int len, int dh, int max_seq) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)H * len * dh;
    if (idx >= total) return;
    int c = (int)(idx % dh);
    int pos = (int)((idx / dh) % len);
    int h = (int)(idx / ((size_t)dh * len));
    size_t base = (size_t)h * max_seq * dh;
    kc[base + kcache_off(pos, c, dh)] = k[idx];
    vc[base + vcache_off(pos, c, dh)] = v[idx];
}

void launch_kv_import_bf16(const void *k, const void *v, void *kc, void *vc, int H, int len, int dh,
                           int max_seq, hipStream_t st) {
    size_t total = (size_t)H * len * dh;
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(kv_import_bf16_kernel, dim3(blocks), dim3(256), 0, st, (const bf16_t *)k,
                       (const bf16_t *)v, (bf16_t *)kc, (bf16_t *)vc, H, len, dh, max_seq);
}

// =============================================================================================
// skinny GEMM  Y[rows][N] = X[rows][K] . W[N][K]^T,  rows <= 16*NT
// =============================================================================================
// One workgroup per 16-feature tile of W (SWIGLU: per pair of gate/up tiles).  Its waves split
// the K axis into contiguous ranges, each wave streams its range of 1 KiB weight blocks
// straight into MFMA A operands, B operands (activations, hi and optionally lo part) come
// from L2.  D[i][n] = sum_k A[i][k] B[k][n] with i = feature, n = activation row, so lane l
// ends with features 4(l/16)..+3 of row l%16.  The waves' partial sums are added in wave
// order through LDS; the number of waves depends on (N, K) only.
template <int NT, int EPI, bool SPLIT>
__global__ __launch_bounds__(1024) void gemm_skinny_bf16(GemmArgs a) {
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    constexpr int U = (NT == 1) ? 4 : 2;
    extern __shared__ f32x4 red[];                 // [waves][TILES][NT][64]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    const int ft = blockIdx.x;
    const int K = a.K, KS = K >> 5;
    const int ks0 = (int)(((long)KS * wave) / waves);
    const int ks1 = (int)(((long)KS * (wave + 1)) / waves);

    const u32x4 *wp[TILES];
    wp[0] = (const u32x4 *)a.W + ((size_t)ft * KS + ks0) * 64 + lane;
    if (TILES == 2) wp[1] = (const u32x4 *)a.W + ((size_t)(ft + a.N / 16) * KS + ks0) * 64 + lane;

    const bf16_t *xh[NT], *xl[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        size_t off = (size_t)(t * 16 + (lane & 15)) * K + (size_t)(lane >> 4) * 8 + (size_t)ks0 * 32;
        xh[t] = (const bf16_t *)a.Xhi + off;
        xl[t] = (const bf16_t *)a.Xlo + off;
    }

    f32x4 acc[TILES][NT];
#pragma unroll
    for (int i = 0; i < TILES; ++i)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[i][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    int ks = ks0;
    for (; ks + U <= ks1; ks += U) {
        u32x4 av[TILES][U], bh[NT][U], bl[NT][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < TILES; ++i) av[i][u] = __builtin_nontemporal_load(wp[i] + u * 64);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                bh[t][u] = *(const u32x4 *)(xh[t] + u * 32);
                if (SPLIT) bl[t][u] = *(const u32x4 *)(xl[t] + u * 32);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < TILES; ++i) {
                    acc[i][t] = mfma16x16x32(av[i][u], bh[t][u], acc[i][t]);
                    if (SPLIT) acc[i][t] = mfma16x16x32(av[i][u], bl[t][u], acc[i][t]);
                }
#pragma unroll
        for (int i = 0; i < TILES; ++i) wp[i] += U * 64;
#pragma unroll
        for (int t = 0; t < NT; ++t) { xh[t] += U * 32; xl[t] += U * 32; }
    }
    for (; ks < ks1; ++ks) {
        u32x4 av[TILES];
#pragma unroll
        for (int i = 0; i < TILES; ++i) av[i] = __builtin_nontemporal_load(wp[i]);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            u32x4 b = *(const u32x4 *)xh[t];
#pragma unroll
            for (int i = 0; i < TILES; ++i) acc[i][t] = mfma16x16x32(av[i], b, acc[i][t]);
            if (SPLIT) {
                u32x4 b2 = *(const u32x4 *)xl[t];
#pragma unroll
                for (int i = 0; i < TILES; ++i) acc[i][t] = mfma16x16x32(av[i], b2, acc[i][t]);
            }
        }
#pragma unroll
        for (int i = 0; i < TILES; ++i) wp[i] += 64;
#pragma unroll
        for (int t = 0; t < NT; ++t) { xh[t] += 32; xl[t] += 32; }
    }

    // ---- cross-wave reduction in wave order ----
#pragma unroll
    for (int i = 0; i < TILES; ++i)
#pragma unroll
        for (int t = 0; t < NT; ++t) red[((wave * TILES + i) * NT + t) * 64 + lane] = acc[i][t];
    __syncthreads();
    for (int t = wave; t < NT; t += waves) {
    f32x4 s[TILES];
#pragma unroll
    for (int i = 0; i < TILES; ++i) {
        s[i] = red[((0 * TILES + i) * NT + t) * 64 + lane];
        for (int w = 1; w < waves; ++w) s[i] += red[((w * TILES + i) * NT + t) * 64 + lane];
    }

    // ---- epilogue: lane holds features f0..f0+3 of row ----
    const int row = t * 16 + (lane & 15);
    const int f0 = ft * 16 + (lane >> 4) * 4;
    if (EPI == EPI_STORE) {
        if (row < a.rows) *(f32x4 *)(a.out + (size_t)row * a.N + f0) = s[0];
    } else if (EPI == EPI_RESID) {
        if (row < a.rows) {
            f32x4 *p = (f32x4 *)(a.out + (size_t)row * a.N + f0);
            *p = *p + s[0];
        }
    } else if (EPI == EPI_SWIGLU) {
        if (row < a.rows) {
            bf16_t hi[4], lo[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float g = s[0][r], u = s[1][r];
                float v = g / (1.0f + __expf(-g)) * u;
                split_bf16(v, hi[r], lo[r]);
            }
            u32x2 ph = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
            u32x2 pl = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
            *(u32x2 *)((bf16_t *)a.act_hi + (size_t)row * a.N + f0) = ph;
            *(u32x2 *)((bf16_t *)a.act_lo + (size_t)row * a.N + f0) = pl;
        }
    } else {  // EPI_LMHEAD: logits of 16 vocabulary entries per row -> (max, arg max) partial
        if (a.out != nullptr && row < a.rows) *(f32x4 *)(a.out + (size_t)row * a.N + f0) = s[0];
        float bv = s[0][0];
        int bi = f0;
#pragma unroll
        for (int r = 1; r < 4; ++r)
            if (s[0][r] > bv) { bv = s[0][r]; bi = f0 + r; }
#pragma unroll
        for (int sh = 16; sh <= 32; sh <<= 1) {
            float ov = __shfl_xor(bv, sh);
            int oi = __shfl_xor(bi, sh);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if ((lane >> 4) == 0 && row < a.rows) {
            a.pval[(size_t)row * a.n_part + ft] = bv;
            a.pidx[(size_t)row * a.n_part + ft] = bi;
        }
    }
    }  // row tiles
}

// number of waves that split K inside a workgroup: enough to put >= ~3000 waves in flight,
// at least 4 k-steps per wave; a function of the matrix shape only.
static int gemm_waves(int n_wg, int KS) {
    int w = 2;
    while (w < 16 && n_wg * w < 3072 && KS / (w * 2) >= 4) w *= 2;
    return w;
}

template <int NT, int EPI>
static void launch_gemm_nt_epi(const GemmArgs &a, hipStream_t st) {
    const int tiles = (EPI == EPI_SWIGLU) ? 2 : 1;
    const int n_wg = a.N / 16;
    const int waves = gemm_waves(n_wg, a.K / 32);
    const size_t lds = (size_t)waves * tiles * NT * 64 * sizeof(f32x4);
    if (a.split)
        hipLaunchKernelGGL((gemm_skinny_bf16<NT, EPI, true>), dim3(n_wg), dim3(waves * 64), lds, st, a);
    else
        hipLaunchKernelGGL((gemm_skinny_bf16<NT, EPI, false>), dim3(n_wg), dim3(waves * 64), lds, st, a);
}

template <int NT>
static void launch_gemm_nt(const GemmArgs &a, hipStream_t st) {
    switch (a.epi) {
        case EPI_STORE: launch_gemm_nt_epi<NT, EPI_STORE>(a, st); break;
        case EPI_RESID: launch_gemm_nt_epi<NT, EPI_RESID>(a, st); break;
        case EPI_SWIGLU: launch_gemm_nt_epi<NT, EPI_SWIGLU>(a, st); break;
        default: launch_gemm_nt_epi<NT, EPI_LMHEAD>(a, st); break;
    }
}

// rows <= 48 per launch; more rows are processed in blocks of 48 (weights re-streamed per block)
void launch_gemm_bf16(const GemmArgs &a0, hipStream_t st) {
    for (int r0 = 0; r0 < a0.rows; r0 += 48) {
        GemmArgs a = a0;
        int rows = a0.rows - r0 < 48 ? a0.rows - r0 : 48;
        a.rows = rows;
        a.Xhi = (const bf16_t *)a0.Xhi + (size_t)r0 * a0.K;
        a.Xlo = (const bf16_t *)a0.Xlo + (size_t)r0 * a0.K;
        if (a0.out) a.out = a0.out + (size_t)r0 * a0.N;
        if (a0.act_hi) a.act_hi = (bf16_t *)a0.act_hi + (size_t)r0 * a0.N;
        if (a0.act_lo) a.act_lo = (bf16_t *)a0.act_lo + (size_t)r0 * a0.N;
        if (a0.pval) { a.pval = a0.pval + (size_t)r0 * a0.n_part; a.pidx = a0.pidx + (size_t)r0 * a0.n_part; }
        if (rows <= 16) launch_gemm_nt<1>(a, st);
        else if (rows <= 32) launch_gemm_nt<2>(a, st);
        else launch_gemm_nt<3>(a, st);
    }
}

// =============================================================================================
// causal attention of m <= 16*NTQ query rows of one sequence over its KV cache
// =============================================================================================
// grid = (chunks of ATTN_CHUNK key positions, heads, sequences); 4 waves per workgroup, wave w
// owns the 64 positions [64 w, 64 w + 64) of the chunk as two groups of 32.  Per group:
// S^T = K_tile . Q^T (MFMA, keys on the A side so the cache is read as whole 1 KiB blocks),
// scale, causal mask by absolute position, online softmax per query row, O^T += V^T . P^T.
// The four waves' (max, sum, O) are merged in wave order, and the chunk's partial is written
// for the combine kernel.  Which keys a row sees, and in which order they are reduced, is a
// function of absolute positions only.
template <int DH, int NTQ>
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

    u32x4 qb[NTQ][KSTEPS];
    int rpos[NTQ];
#pragma unroll
    for (int q = 0; q < NTQ; ++q) {
        int j = q * 16 + n;
        bool valid = j < m;
        rpos[q] = valid ? T + j : -1;
        const bf16_t *qp = (const bf16_t *)a.Q + (size_t)(b * m + (valid ? j : 0)) * d_model + h * DH + g * 8;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) qb[q][s] = *(const u32x4 *)(qp + s * 32);
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
    const bf16_t *kbase = (const bf16_t *)a.Kc + head_base;
    const bf16_t *vbase = (const bf16_t *)a.Vc + head_base;

#pragma unroll 1
    for (int gi = 0; gi < 2; ++gi) {
        const int key0 = chunk0 + (wave * 2 + gi) * 32;
        if (key0 >= kv_len) break;                      // uniform for the wave
        u32x4 ka[2][KSTEPS], va[DT];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s)
                ka[t][s] = *(const u32x4 *)(kbase + (size_t)(key0 / 16 + t) * (16 * DH) + s * 512 + lane * 8);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            va[dt] = *(const u32x4 *)(vbase + (size_t)(key0 / 32) * (32 * DH) + dt * 512 + lane * 8);

#pragma unroll
        for (int q = 0; q < NTQ; ++q) {
            f32x4 s2[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                s2[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) s2[t] = mfma16x16x32(ka[t][s], qb[q][s], s2[t]);
            }
            float sv[8];
            float mx = LLMA_NEG_INF;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    int key = key0 + t * 16 + 4 * g + r;
                    float v = s2[t][r] * a.scale;
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
            u32x4 pb;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                pb[i] = (uint32_t)f32_to_bf16(p[2 * i]) | ((uint32_t)f32_to_bf16(p[2 * i + 1]) << 16);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[q][dt] = o[q][dt] * alpha;
                o[q][dt] = mfma16x16x32(va[dt], pb, o[q][dt]);
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
// over the chunks that contain positions <= the row's own, in chunk order.
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
    size_t o = (size_t)r * (a.H * DH) + h * DH + d;
    ((bf16_t *)a.out_hi)[o] = hi;
    ((bf16_t *)a.out_lo)[o] = lo;
}

template <int DH>
static void launch_attn_dh(const AttnArgs &a, hipStream_t st) {
    const int ntq = (a.m + 15) / 16;
    dim3 grid(a.n_chunks, a.H, a.n_seqs);
    if (ntq == 1) hipLaunchKernelGGL((attn_bf16_kernel<DH, 1>), grid, dim3(256), 0, st, a);
    else if (ntq == 2) hipLaunchKernelGGL((attn_bf16_kernel<DH, 2>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_bf16_kernel<DH, 3>), grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL((attn_combine_bf16_kernel<DH>), dim3(a.n_seqs * a.m, a.H), dim3(DH), 0, st, a, ntq * 16);
}

void launch_attn_bf16(const AttnArgs &a, hipStream_t st) {
    if (a.dh == 128) launch_attn_dh<128>(a, st);
    else launch_attn_dh<64>(a, st);
}
