// fp32 path of the verification forward (paper: Eq. 3): plain vector-ALU kernels for models
// whose weights are fp32 (the tiny parity configuration).  Launch-bound by nature; written for
// exactness and for the same row-count invariance as the bf16 path: every output element is
// reduced in an order that depends on the matrix shape / absolute key positions only.
#include "common.h"
#include "kernels.h"

__global__ void kv_import_f32_kernel(const float *__restrict__ k, const float *__restrict__ v,
                                     float *__restrict__ kc, float *__restrict__ vc, int H, int len, int dh, int max_seq) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)H * len * dh;
    if (idx >= total) return;
    int c = (int)(idx % dh);
    int pos = (int)((idx / dh) % len);
    int h = (int)(idx / ((size_t)dh * len));
    size_t o = ((size_t)h * max_seq + pos) * dh + c;
    kc[o] = k[idx];
    vc[o] = v[idx];
}
void launch_kv_import_f32(const void *k, const void *v, void *kc, void *vc, int H, int len, int dh,
                          int max_seq, hipStream_t st) {
    size_t total = (size_t)H * len * dh;
    hipLaunchKernelGGL(kv_import_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const float *)k, (const float *)v, (float *)kc, (float *)vc, H, len, dh, max_seq);
}

// One wavefront per output feature; lanes stride the reduction axis, 8 rows at a time in
// registers, butterfly reduction across the wavefront.
template <int EPI>
__global__ __launch_bounds__(64) void gemm_f32_kernel(GemmArgs a) {
    const int n = blockIdx.x, lane = threadIdx.x;
    const int K = a.K;
    const float *W = (const float *)a.W + (size_t)n * K;
    const float *Wu = (const float *)a.W + (size_t)(n + a.N) * K;       // SWIGLU: the up row
    const float *X = (const float *)a.Xhi;
    for (int r0 = 0; r0 < a.rows; r0 += 8) {
        float acc[8], accu[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) { acc[r] = 0.f; accu[r] = 0.f; }
        for (int k = lane; k < K; k += 64) {
            const float w = W[k];
            const float wu = (EPI == EPI_SWIGLU) ? Wu[k] : 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                if (r0 + r < a.rows) {
                    const float x = X[(size_t)(r0 + r) * K + k];
                    acc[r] = fmaf(w, x, acc[r]);
                    if (EPI == EPI_SWIGLU) accu[r] = fmaf(wu, x, accu[r]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                acc[r] += __shfl_xor(acc[r], off);
                if (EPI == EPI_SWIGLU) accu[r] += __shfl_xor(accu[r], off);
            }
        }
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int row = r0 + r;
                if (row >= a.rows) break;
                if (EPI == EPI_STORE) a.out[(size_t)row * a.N + n] = acc[r];
                else if (EPI == EPI_RESID) a.out[(size_t)row * a.N + n] += acc[r];
                else if (EPI == EPI_SWIGLU) {
                    const float g = acc[r];
                    ((float *)a.act_hi)[(size_t)row * a.N + n] = g / (1.0f + expf(-g)) * accu[r];
                } else {
                    if (a.out) a.out[(size_t)row * a.N + n] = acc[r];
                    a.pval[(size_t)row * a.n_part + n] = acc[r];
                    a.pidx[(size_t)row * a.n_part + n] = n;
                }
            }
        }
    }
}
void launch_gemm_f32(const GemmArgs &a, hipStream_t st) {
    dim3 grid(a.N), block(64);
    switch (a.epi) {
        case EPI_STORE: hipLaunchKernelGGL((gemm_f32_kernel<EPI_STORE>), grid, block, 0, st, a); break;
        case EPI_RESID: hipLaunchKernelGGL((gemm_f32_kernel<EPI_RESID>), grid, block, 0, st, a); break;
        case EPI_SWIGLU: hipLaunchKernelGGL((gemm_f32_kernel<EPI_SWIGLU>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((gemm_f32_kernel<EPI_LMHEAD>), grid, block, 0, st, a); break;
    }
}

// One wavefront per (row, head): lane l owns keys l, l+64, ... <= the row's position with its own
// online softmax; the 64 lane states are merged by butterfly.  Which lane owns which key is a
// function of the absolute key position only.
template <int DH>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnArgs a) {
    __shared__ float qs[DH];
    const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int b = r / a.m, j = r % a.m;
    const int slot = a.batch_slots[b];
    const int pos = a.T[slot] + j;
    const int d_model = a.H * DH;
    const float *q = (const float *)a.Qhi + (size_t)r * d_model + h * DH;
    for (int c = lane; c < DH; c += 64) qs[c] = q[c];
    __syncthreads();
    const size_t head_base = ((size_t)slot * a.H + h) * (size_t)a.max_seq * DH;
    const float *kc = (const float *)a.Khi + head_base, *vc = (const float *)a.Vhi + head_base;
    float mx = LLMA_NEG_INF, l = 0.f, acc[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = 0.f;
    for (int key = lane; key <= pos; key += 64) {
        const float *kr = kc + (size_t)key * DH, *vr = vc + (size_t)key * DH;
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < DH; ++c) s = fmaf(qs[c], kr[c], s);
        s *= a.scale;
        const float mnew = fmaxf(mx, s);
        const float alpha = expf(mx - mnew);          // 0 on the first key
        const float p = expf(s - mnew);
        l = l * alpha + p;
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] = acc[c] * alpha + p * vr[c];
        mx = mnew;
    }
    float M = mx;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float sc = (mx == LLMA_NEG_INF) ? 0.f : expf(mx - M);
    float L = l * sc;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) L += __shfl_xor(L, off);
    float *out = (float *)a.out_hi + (size_t)r * d_model + h * DH;
#pragma unroll
    for (int c = 0; c < DH; ++c) {
        float v = acc[c] * sc;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) out[c] = v / L;
    }
}
void launch_attn_f32(const AttnArgs &a, hipStream_t st) {
    dim3 grid(a.n_seqs * a.m, a.H), block(64);
    if (a.dh == 32) hipLaunchKernelGGL((attn_f32_kernel<32>), grid, block, 0, st, a);
    else if (a.dh == 64) hipLaunchKernelGGL((attn_f32_kernel<64>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((attn_f32_kernel<128>), grid, block, 0, st, a);
}
