// Small kernels around the GEMMs and attention: row set-up, the fp32 path's embedding gather /
// RMSNorm / RoPE + KV append, the vocabulary arg max with the prefix-accept / KV-truncate decision
// (paper: Algorithm 1, the compare loop after the verification forward), and the n-gram
// trigger scan over the reference (paper: Method, the match that starts a copy).
#include "common.h"
#include "kernels.h"

// ---------------------------------------------------------------------------------------------
// row set-up
// ---------------------------------------------------------------------------------------------
// one workgroup per row; also copies the row's rotary (cos, sin) pairs out of the position table
__global__ void setup_step_rows_kernel(StepState s, int m, int max_k, const float *cs, int half) {
    const int idx = blockIdx.x;
    const int b = idx / m, j = idx % m;
    const int slot = s.batch_slots[b];
    const int pos = s.T[slot] + j;
    if (threadIdx.x == 0) {
        int tok;
        if (j == 0) tok = s.pending[slot];
        else tok = (j - 1 < s.keff[b]) ? s.draft[b * max_k + j - 1] : 0;   // rows past keff are padding
        s.row_tok[idx] = tok;
        s.row_pos[idx] = pos;
        s.row_slot[idx] = slot;
    }
    for (int i = threadIdx.x; i < 2 * half; i += blockDim.x) s.row_cs[(size_t)idx * 2 * half + i] = cs[(size_t)pos * 2 * half + i];
}
void launch_setup_step_rows(const StepState &s, int n_seqs, int m, int max_k, const float *cs, int half, hipStream_t st) {
    hipLaunchKernelGGL(setup_step_rows_kernel, dim3(n_seqs * m), dim3(64), 0, st, s, m, max_k, cs, half);
}

__global__ void setup_prefill_rows_kernel(StepState s, const int *prompt, const int *base, int slot, const float *cs, int half) {
    const int j = blockIdx.x;
    const int pos = s.T[slot] + j;
    if (threadIdx.x == 0) {
        s.row_tok[j] = prompt[pos - *base];
        s.row_pos[j] = pos;
        s.row_slot[j] = slot;
        if (j == 0) s.batch_slots[0] = slot;
    }
    for (int i = threadIdx.x; i < 2 * half; i += blockDim.x) s.row_cs[(size_t)j * 2 * half + i] = cs[(size_t)pos * 2 * half + i];
}
void launch_setup_prefill_rows(const StepState &s, const int *prompt_dev, const int *base_dev, int m, int slot,
                               const float *cs, int half, hipStream_t st) {
    hipLaunchKernelGGL(setup_prefill_rows_kernel, dim3(m), dim3(64), 0, st, s, prompt_dev, base_dev, slot, cs, half);
}

__global__ void advance_T_kernel(StepState s, int slot, int by) { s.T[slot] += by; }
void launch_advance_T(const StepState &s, int slot, int by, hipStream_t st) {
    hipLaunchKernelGGL(advance_T_kernel, dim3(1), dim3(1), 0, st, s, slot, by);
}

// ---------------------------------------------------------------------------------------------
// fp32 path: embedding gather, RMSNorm, RoPE + KV append as separate small kernels
// ---------------------------------------------------------------------------------------------
__global__ void embed_f32_kernel(const float *embed, const int *row_tok, float *h, int d) {
    int r = blockIdx.x;
    size_t base = (size_t)row_tok[r] * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) h[(size_t)r * d + c] = embed[base + c];
}
void launch_embed_f32(const float *embed, const int *row_tok, float *h, int R, int d, hipStream_t st) {
    hipLaunchKernelGGL(embed_f32_kernel, dim3(R), dim3(256), 0, st, embed, row_tok, h, d);
}

// one workgroup per row; fixed summation order (thread-strided, butterfly, wave order)
__global__ __launch_bounds__(256) void rmsnorm_f32_kernel(const float *__restrict__ h, const float *__restrict__ g, float eps,
                                                          float *__restrict__ out, int d) {
    __shared__ float part[4];
    const int r = blockIdx.x;
    const float *x = h + (size_t)r * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) ss += x[c] * x[c];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = ((part[0] + part[1]) + part[2]) + part[3];
    float rstd = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256) out[(size_t)r * d + c] = x[c] * rstd * g[c];
}
void launch_rmsnorm_f32(const float *h, const float *g, float eps, float *out, int R, int d, hipStream_t st) {
    hipLaunchKernelGGL(rmsnorm_f32_kernel, dim3(R), dim3(256), 0, st, h, g, eps, out, d);
}

// grid (rows, heads), head_dim/2 threads: thread i rotates the pair (i, i + head_dim/2) of q and k
// by angle pos * theta^(-2i/head_dim) (table built on the host)
__global__ void rope_kv_f32_kernel(const float *__restrict__ qkv, StepState s, const float *__restrict__ cs,
                                   float *q_out, float *kc, float *vc, int H, int dh, int max_seq) {
    const int r = blockIdx.x, hh = blockIdx.y, i = threadIdx.x;
    const int half = dh >> 1, d = H * dh;
    const int pos = s.row_pos[r], slot = s.row_slot[r];
    const float c = cs[((size_t)pos * half + i) * 2], sn = cs[((size_t)pos * half + i) * 2 + 1];
    const float *row = qkv + (size_t)r * 3 * d;
    const float q1 = row[hh * dh + i], q2 = row[hh * dh + i + half];
    const float k1 = row[d + hh * dh + i], k2 = row[d + hh * dh + i + half];
    const float v1 = row[2 * d + hh * dh + i], v2 = row[2 * d + hh * dh + i + half];
    const size_t head_base = ((size_t)slot * H + hh) * (size_t)max_seq * dh;
    float *q = q_out + (size_t)r * d + hh * dh;
    q[i] = q1 * c - q2 * sn;
    q[i + half] = q2 * c + q1 * sn;
    float *kp = kc + head_base + (size_t)pos * dh, *vp = vc + head_base + (size_t)pos * dh;
    kp[i] = k1 * c - k2 * sn;
    kp[i + half] = k2 * c + k1 * sn;
    vp[i] = v1;
    vp[i + half] = v2;
}
void launch_rope_kv_f32(const float *qkv, const StepState &s, const float *cs_table, float *q_out, float *kc, float *vc,
                        int R, int H, int dh, int max_seq, hipStream_t st) {
    hipLaunchKernelGGL(rope_kv_f32_kernel, dim3(R, H), dim3(dh / 2), 0, st, qkv, s, cs_table, q_out, kc, vc, H, dh, max_seq);
}

// ---------------------------------------------------------------------------------------------
// vocabulary arg max (lowest id on exact ties) + prefix accept + KV truncate
// ---------------------------------------------------------------------------------------------
// One workgroup per sequence.  o_j = arg max of row j for j = 0..keff; a = longest prefix with
// o_i == draft_i; the step emits o_0..o_a, the cache keeps the rows of the pending token and
// of the a accepted drafts (T += a + 1; rows beyond are overwritten by the next step), and
// o_a becomes the pending token.
__global__ __launch_bounds__(256) void argmax_accept_kernel(const float *__restrict__ pval, const int *__restrict__ pidx,
                                                            int n_part, StepState s, int m, int max_k, int vocab, const GenState *gen) {
    __shared__ int o[40];
    const int b = blockIdx.x;
    if (gen != nullptr) gen += b;                                // llma_generate: one GenState per sequence of the batch
    if (gen != nullptr && *gen->n_out >= gen->max_new) return;   // a finished sequence / a step enqueued past the end: leave all state alone
    const int keff = s.keff[b];
    // one row per wave at a time: wave w reduces rows w, w + 4, ... over the per-tile partials
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = wave; j <= keff; j += 4) {
        const size_t r = (size_t)b * m + j;
        float bv = LLMA_NEG_INF;
        int bi = 0x7fffffff;
        for (int t0 = lane; t0 < n_part; t0 += 64 * 8) {      // 8 partials per lane in flight
            float v[8];
            int id[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = t0 + 64 * u;
                v[u] = t < n_part ? pval[r * n_part + t] : LLMA_NEG_INF;
                id[u] = t < n_part ? pidx[r * n_part + t] : 0x7fffffff;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (v[u] > bv || (v[u] == bv && id[u] < bi)) { bv = v[u]; bi = id[u]; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            float ov = __shfl_xor(bv, off);
            int oi = __shfl_xor(bi, off);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        // a row without any comparable logit (all NaN: reachable through imported caches or weights that
        // hold non-finite values) must still yield a token id the next step's embedding gather can use
        if ((unsigned)bi >= (unsigned)vocab) bi = 0;
        if (lane == 0) { o[j] = bi; s.otok[r] = bi; }
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    int a = 0;
    while (a < keff && o[a] == s.draft[b * max_k + a]) ++a;
    const int slot = s.batch_slots[b];
    s.nacc[b] = a;
    s.next[b] = o[a];
    for (int j = 0; j <= a; ++j) s.emit[b * (max_k + 1) + j] = o[j];
    s.T[slot] += a + 1;
    s.pending[slot] = o[a];
    if (gen != nullptr) {
        int i = *gen->n_out, st = *gen->n_steps;
        for (int j = 0; j <= a; ++j) gen->y[i + j] = o[j];
        gen->trace[st * 4 + 0] = 1 + keff;
        gen->trace[st * 4 + 1] = a + 1;
        gen->trace[st * 4 + 2] = keff > 0 ? gen->cur[0] : -1;
        gen->trace[st * 4 + 3] = keff > 0 ? gen->cur[1] : -1;
        *gen->n_out = i + a + 1;
        *gen->n_steps = st + 1;
    }
}
void launch_argmax_accept(const float *pval, const int *pidx, int n_part, const StepState &s, int n_seqs, int m,
                          int max_k, int vocab, const GenState *gen, hipStream_t st) {
    hipLaunchKernelGGL(argmax_accept_kernel, dim3(n_seqs), dim3(256), 0, st, pval, pidx, n_part, s, m, max_k, vocab, gen);
}

// ---------------------------------------------------------------------------------------------
// trigger: wavefront-parallel scan of the reference for the n-token tail of y
// ---------------------------------------------------------------------------------------------
// Flat position p is a candidate when it lies at least n tokens into its document and the n
// tokens before it equal the tail of y; its score is how far that agreement extends backwards
// (bounded by the document start and by the start of y).  The best candidate maximises
// (score, then smallest flat position) -- flat order is (document, position) order.
__device__ __forceinline__ unsigned long long scan_reference(const int *y, int i, const int *ref, const int *doc_offsets,
                                                             const int *ref_doc, int ref_len, int n) {
    unsigned long long best = 0ull;
    if (i >= n) {
        // first pass, eight positions per thread in flight: does the token before p equal the last
        // token of y?  (necessary for a match; nearly all positions stop here)
        const int last = y[i - 1];
        for (int p0 = threadIdx.x; p0 < ref_len; p0 += blockDim.x * 8) {
            int prev[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + u * blockDim.x;
                prev[u] = (p >= 1 && p < ref_len) ? ref[p - 1] : -1;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + u * blockDim.x;
                if (prev[u] != last || p >= ref_len) continue;      // (token ids are >= 0)
                const int pos = p - doc_offsets[ref_doc[p]];
                if (pos < n) continue;
                bool ok = true;
                for (int t = 1; t < n; ++t)
                    if (ref[p - 1 - t] != y[i - 1 - t]) { ok = false; break; }
                if (!ok) continue;
                int score = n;
                while (score < pos && score < i && ref[p - 1 - score] == y[i - 1 - score]) ++score;
                unsigned long long key = ((unsigned long long)score << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)p);
                best = key > best ? key : best;
            }
        }
    }
    // wave, then workgroup maximum
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned long long o = __shfl_xor(best, off);
        best = o > best ? o : best;
    }
    __shared__ unsigned long long wbest[16];
    if ((threadIdx.x & 63) == 0) wbest[threadIdx.x >> 6] = best;
    __syncthreads();
    const int waves = blockDim.x >> 6;
    best = wbest[0];
    for (int w = 1; w < waves; ++w) best = wbest[w] > best ? wbest[w] : best;
    return best;
}

__global__ __launch_bounds__(256) void trigger_kernel(const GenState *gp, StepState s, int max_k) {
    const int b = blockIdx.x;                                    // one workgroup per sequence of the batch
    const GenState G = gp[b];
    const int i = *G.n_out;
    unsigned long long best = 0ull;
    if (G.ref_len > 0 && G.k > 0 && i < G.max_new)
        best = scan_reference(G.y, i, G.ref, G.doc_offsets, G.ref_doc, G.ref_len, G.n);
    int keff = 0, p = 0;
    if (best != 0ull) {
        p = (int)(0xFFFFFFFFu - (unsigned)(best & 0xFFFFFFFFull));
        const int doc = G.ref_doc[p];
        const int left_in_doc = G.doc_offsets[doc + 1] - p;
        const int budget = G.max_new - i - 1;
        keff = G.k < left_in_doc ? G.k : left_in_doc;
        keff = keff < budget ? keff : budget;
        keff = keff < 0 ? 0 : keff;
        if (threadIdx.x == 0) { G.cur[0] = doc; G.cur[1] = p - G.doc_offsets[doc]; }
    }
    if (threadIdx.x == 0) s.keff[b] = keff;
    for (int j = threadIdx.x; j < keff; j += blockDim.x) s.draft[b * max_k + j] = G.ref[p + j];
}
void launch_trigger(const GenState *gen_dev, const StepState &s, int n_seqs, int max_k, hipStream_t st) {
    hipLaunchKernelGGL(trigger_kernel, dim3(n_seqs), dim3(256), 0, st, gen_dev, s, max_k);
}

// check_offsets (callers whose document list lives in device memory, where the host cannot look):
// the list must start at 0, never decrease and end at ref_len; otherwise result = (-1, -1, -1) and
// nothing is scanned (the scan's backward walk relies on positions inside their documents).
__global__ __launch_bounds__(256) void trigger_plain_kernel(const int *y, int y_len, const int *ref, const int *doc_offsets,
                                                            const int *ref_doc, int ref_len, int n_docs, int n, int *result,
                                                            int check_offsets) {
    if (ref_len <= 0 || n_docs <= 0) {
        if (threadIdx.x == 0) { result[0] = 0; result[1] = -1; result[2] = -1; }
        return;
    }
    if (check_offsets) {
        int bad = 0;
        for (int j = threadIdx.x; j < n_docs; j += blockDim.x) bad |= doc_offsets[j + 1] < doc_offsets[j];
        if (threadIdx.x == 0) bad |= (doc_offsets[0] != 0) | (doc_offsets[n_docs] != ref_len);
        if (__syncthreads_or(bad)) {
            if (threadIdx.x == 0) { result[0] = -1; result[1] = -1; result[2] = -1; }
            return;
        }
    }
    unsigned long long best = scan_reference(y, y_len, ref, doc_offsets, ref_doc, ref_len, n);
    if (threadIdx.x != 0) return;
    if (best == 0ull) { result[0] = 0; result[1] = -1; result[2] = -1; return; }
    int p = (int)(0xFFFFFFFFu - (unsigned)(best & 0xFFFFFFFFull));
    int doc = ref_doc[p];
    result[0] = 1; result[1] = doc; result[2] = p - doc_offsets[doc];
}
void launch_trigger_plain(const int *y, int y_len, const int *ref, const int *doc_offsets, const int *ref_doc,
                          int ref_len, int n_docs, int n, int *result, bool check_offsets, hipStream_t st) {
    hipLaunchKernelGGL(trigger_plain_kernel, dim3(1), dim3(256), 0, st, y, y_len, ref, doc_offsets, ref_doc, ref_len, n_docs, n,
                       result, check_offsets ? 1 : 0);
}

// ref_doc[p] = the document that contains flat position p (doc_offsets non-decreasing)
__global__ void fill_ref_doc_kernel(const int *doc_offsets, int n_docs, int *ref_doc, int ref_len) {
    int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= ref_len) return;
    int lo = 0, hi = n_docs;              // largest j with doc_offsets[j] <= p
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (doc_offsets[mid] <= p) lo = mid; else hi = mid;
    }
    ref_doc[p] = lo;
}
void launch_fill_ref_doc(const int *doc_offsets, int n_docs, int *ref_doc, int ref_len, hipStream_t st) {
    if (ref_len <= 0) return;
    hipLaunchKernelGGL(fill_ref_doc_kernel, dim3((ref_len + 255) / 256), dim3(256), 0, st, doc_offsets, n_docs, ref_doc, ref_len);
}
