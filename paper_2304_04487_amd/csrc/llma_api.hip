// C ABI of the library (include/llma.h) and the host orchestration of a decoding step:
// which kernels run in which order for the verification forward (paper: Eq. 3), the accept /
// truncate decision and the LLMA loop (paper: Algorithm 1).  All arithmetic of the method runs
// in the kernels; this file validates arguments, owns device memory and enqueues launches.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <array>
#include <map>
#include <string>
#include <utility>
#include <vector>

#include "../../include/llma.h"
#include "common.h"
#include "kernels.h"

static thread_local std::string g_err;      // errors of calls that have no context
void llma_set_error_text(const char *text) { g_err = text ? text : ""; }   // for the library's other source files

#define PREFILL_ROWS_F32 48      // fp32 path: prompt rows per pass
#define PREFILL_ROWS_MAX 2048    // bf16 path: prompt rows per pass (whole prompt when it fits)

struct EventPair { hipEvent_t a, b; };

enum StepKind { STEP_PREFILL = 0, STEP_VERIFY = 1, STEP_GEN = 2 };

// what a captured step graph was recorded for: (kind, sequences, rows per sequence, attention chunks, slot)
typedef std::array<int, 5> GraphKey;
struct GraphSlot { int seen = 0; hipGraphExec_t exec = nullptr; };

struct llma_ctx {
    llma_model_cfg cfg;
    hipStream_t st = nullptr;          // the caller's stream: everything is ordered on it
    hipStream_t run_st = nullptr;      // where the launchers enqueue: st, or cap_st while capturing
    hipStream_t cap_st = nullptr;      // private stream used only to capture step graphs
    std::map<GraphKey, GraphSlot> graphs;
    int *pin_counts = nullptr;         // pinned host ints the decoding loop's output counts are copied into
    hipEvent_t cnt_ev[2] = {nullptr, nullptr};
    bool bf16 = false;
    std::vector<void *> allocs;
    int64_t dev_bytes = 0;
    std::string err;

    // weights (owned copies; bf16 matrices re-tiled)
    void *embed = nullptr, *lm_head = nullptr;
    float *final_norm = nullptr;
    std::vector<void *> wqkv, wo, wgu, wd;
    std::vector<float *> n1, n2;
    // KV cache per layer: [max_batch][H][seq_cap][dh]; bf16 with kv_split: a second (lo) plane.
    // seq_cap = max_seq rounded up to whole attention chunks, so a chunk's block loads never leave the allocation
    int seq_cap = 0;
    std::vector<void *> kc, vc, kc_lo, vc_lo;
    float *cs_table = nullptr;
    bool kv_split = false;

    // scratch for up to Rmax rows.  bf16: x/q/att/act are tiled hi/lo planes; fp32: row-major in *_hi
    int Rmax = 0;
    float *h = nullptr, *qkv = nullptr;
    void *xhi = nullptr, *xlo = nullptr, *q = nullptr, *q_lo = nullptr, *att_hi = nullptr, *att_lo = nullptr, *act_hi = nullptr, *act_lo = nullptr;
    float *po = nullptr, *pm = nullptr, *pl = nullptr;
    const int *rows_live = nullptr;    // set per step: device count of live rows - 1 (generation, one sequence) or null
    float *part = nullptr;             // split-K partial sums (contexts whose steps can exceed 48 rows)
    int nc_max = 0;
    // bf16 GEMM work division, per-tile sums of squares of the residual rows, rstd of prompt rows
    GemmPlan plan_qkv{}, plan_o{}, plan_gu{}, plan_down{}, plan_lm{};
    float *ssq = nullptr, *rstd = nullptr;
    int Pmax = 0;                      // prompt rows processed per pass
    float *pval = nullptr;
    int *pidx = nullptr;
    int n_part = 0;

    StepState s{};
    GenState *gen_dev = nullptr;
    int *gen_prompt = nullptr, *gen_ref = nullptr, *gen_doc_offsets = nullptr, *gen_ref_doc = nullptr;
    int *gen_y = nullptr, *gen_trace = nullptr;   // [sequence of the batch][max_new + 64] tokens, x 4 trace words
    int *gen_counters = nullptr;                  // n_out[max_batch], n_steps[max_batch], cur[max_batch][2], prefill base
    int cap_prompt = 0, cap_ref = 0, cap_refdoc = 0, cap_docs = 0, cap_y = 0, cap_trace = 0;

    std::vector<int> T_host, pending_host;
    // Caches imported as bf16 values have all-zero lo planes: positions below lo_from[slot] (device
    // ints, host mirror) need no lo reads.  It is set when all layers of a slot have been imported
    // with one length and nothing was computed on the slot in between (imp_len records the lengths
    // since then, -1 = none); steps only ever write at positions >= T >= lo_from, reset clears it.
    std::vector<int> lo_from_host, imp_len;
    int *lo_from = nullptr;
    float *logits_dump = nullptr;
    int dump_rows = 0;
    int opt_split = 1, opt_timing = 0, opt_graph = 1;
    std::vector<EventPair> events;
};

static int fail(llma_ctx *c, int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    g_err = buf;
    return code;
}
#define HIP_TRY(c, expr)                                                                             \
    do {                                                                                             \
        hipError_t e_ = (expr);                                                                      \
        if (e_ != hipSuccess)                                                                        \
            return fail((c), e_ == hipErrorOutOfMemory ? LLMA_E_NOMEM : LLMA_E_HIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                                      \
    } while (0)

static int dev_alloc(llma_ctx *c, void **p, size_t bytes) {
    if (bytes == 0) bytes = 16;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) return fail(c, LLMA_E_NOMEM, "hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(e));
    c->allocs.push_back(*p);
    c->dev_bytes += (int64_t)bytes;
    return LLMA_OK;
}
#define ALLOC(c, ptr, bytes)                                         \
    do {                                                             \
        int rc_ = dev_alloc((c), (void **)&(ptr), (size_t)(bytes));  \
        if (rc_ != LLMA_OK) return rc_;                              \
    } while (0)

static void dev_free_one(llma_ctx *c, void *p) {
    if (!p) return;
    for (size_t i = 0; i < c->allocs.size(); ++i)
        if (c->allocs[i] == p) { c->allocs.erase(c->allocs.begin() + i); break; }
    (void)hipFree(p);
}

// ------------------------------------------------------------------------------------------------
// create / destroy
// ------------------------------------------------------------------------------------------------
static int check_cfg(const llma_model_cfg *g) {
    if (g->n_layers < 1 || g->d_model < 1 || g->n_heads < 1 || g->head_dim < 1 || g->d_ffn < 1 || g->vocab < 1)
        return fail(nullptr, LLMA_E_INVAL, "model dimensions must be positive");
    if (g->n_heads * g->head_dim != g->d_model) return fail(nullptr, LLMA_E_INVAL, "n_heads * head_dim != d_model");
    if (g->max_seq < 2 || g->max_batch < 1 || g->max_k < 0 || g->max_k > 32)
        return fail(nullptr, LLMA_E_INVAL, "need max_seq >= 2, max_batch >= 1, 0 <= max_k <= 32");
    if (g->dtype == LLMA_DTYPE_BF16) {
        if (g->d_model % 32 || g->d_ffn % 32 || g->vocab % 16)
            return fail(nullptr, LLMA_E_INVAL, "bf16 needs d_model %% 32 == 0, d_ffn %% 32 == 0, vocab %% 16 == 0");
        if (g->head_dim != 64 && g->head_dim != 128) return fail(nullptr, LLMA_E_INVAL, "bf16 needs head_dim 64 or 128");
    } else if (g->dtype == LLMA_DTYPE_F32) {
        if (g->head_dim != 32 && g->head_dim != 64 && g->head_dim != 128)
            return fail(nullptr, LLMA_E_INVAL, "fp32 needs head_dim 32, 64 or 128");
        if (g->d_model % 4) return fail(nullptr, LLMA_E_INVAL, "fp32 needs d_model %% 4 == 0");
    } else {
        return fail(nullptr, LLMA_E_INVAL, "unknown dtype %d", g->dtype);
    }
    if (!(g->rms_eps >= 0.f) || !(g->rope_theta > 0.f)) return fail(nullptr, LLMA_E_INVAL, "bad rms_eps / rope_theta");
    return LLMA_OK;
}

// copies one matrix into context-owned memory: fp32 as is, bf16 re-tiled (N rows, K padded to KSp k-steps)
static int take_matrix(llma_ctx *c, void **dst, const void *src, int N, int K, int KSp, int rope_dh) {
    if (c->bf16) {
        ALLOC(c, *dst, (size_t)(N / 16) * KSp * 1024);
        launch_pack_weight(src, *dst, N, K, KSp, rope_dh, c->cfg.d_model, c->st);
    } else {
        size_t bytes = (size_t)N * K * 4;
        ALLOC(c, *dst, bytes);
        HIP_TRY(c, hipMemcpyAsync(*dst, src, bytes, hipMemcpyDeviceToDevice, c->st));
    }
    return LLMA_OK;
}

static int autotune_tilek(llma_ctx *c);
static int create_impl(llma_ctx *c, const llma_weights *w) {
    const llma_model_cfg &g = c->cfg;
    const int L = g.n_layers, d = g.d_model, F = g.d_ffn, V = g.vocab, H = g.n_heads, dh = g.head_dim;
    const size_t es = c->bf16 ? 2 : 4;
    if (c->bf16) {
        c->plan_qkv = make_gemm_plan(3 * d, d, 1);
        c->plan_o = make_gemm_plan(d, d, 1);
        c->plan_gu = make_gemm_plan(F, d, 2);
        c->plan_down = make_gemm_plan(d, F, 1);
        c->plan_lm = make_gemm_plan(V, d, 1);
    }
    // ---- weights
    ALLOC(c, c->embed, (size_t)V * d * es);
    HIP_TRY(c, hipMemcpyAsync(c->embed, w->embed, (size_t)V * d * es, hipMemcpyDeviceToDevice, c->st));
    int rc = take_matrix(c, &c->lm_head, w->lm_head, V, d, c->plan_lm.KSp, 0);
    if (rc) return rc;
    ALLOC(c, c->final_norm, d * 4);
    HIP_TRY(c, hipMemcpyAsync(c->final_norm, w->final_norm, d * 4, hipMemcpyDeviceToDevice, c->st));
    c->wqkv.assign(L, nullptr); c->wo.assign(L, nullptr); c->wgu.assign(L, nullptr); c->wd.assign(L, nullptr);
    c->n1.assign(L, nullptr); c->n2.assign(L, nullptr);
    c->kc.assign(L, nullptr); c->vc.assign(L, nullptr); c->kc_lo.assign(L, nullptr); c->vc_lo.assign(L, nullptr);
    for (int l = 0; l < L; ++l) {
        if (!w->wqkv[l] || !w->wo[l] || !w->wgu[l] || !w->wdown[l] || !w->norm1[l] || !w->norm2[l])
            return fail(c, LLMA_E_INVAL, "null weight pointer in layer %d", l);
        if ((rc = take_matrix(c, &c->wqkv[l], w->wqkv[l], 3 * d, d, c->plan_qkv.KSp, dh))) return rc;
        if ((rc = take_matrix(c, &c->wo[l], w->wo[l], d, d, c->plan_o.KSp, 0))) return rc;
        if ((rc = take_matrix(c, &c->wgu[l], w->wgu[l], 2 * F, d, c->plan_gu.KSp, 0))) return rc;
        if ((rc = take_matrix(c, &c->wd[l], w->wdown[l], d, F, c->plan_down.KSp, 0))) return rc;
        ALLOC(c, c->n1[l], d * 4);
        ALLOC(c, c->n2[l], d * 4);
        HIP_TRY(c, hipMemcpyAsync(c->n1[l], w->norm1[l], d * 4, hipMemcpyDeviceToDevice, c->st));
        HIP_TRY(c, hipMemcpyAsync(c->n2[l], w->norm2[l], d * 4, hipMemcpyDeviceToDevice, c->st));
    }
    // ---- KV cache, zero-filled so that never-written positions hold finite values
    c->seq_cap = (g.max_seq + ATTN_CHUNK - 1) / ATTN_CHUNK * ATTN_CHUNK;
    const size_t kv_bytes = (size_t)g.max_batch * H * c->seq_cap * dh * es;
    for (int l = 0; l < L; ++l) {
        ALLOC(c, c->kc[l], kv_bytes);
        ALLOC(c, c->vc[l], kv_bytes);
        HIP_TRY(c, hipMemsetAsync(c->kc[l], 0, kv_bytes, c->st));
        HIP_TRY(c, hipMemsetAsync(c->vc[l], 0, kv_bytes, c->st));
        if (c->kv_split) {
            ALLOC(c, c->kc_lo[l], kv_bytes / 2);                  // lo planes: one byte per element
            ALLOC(c, c->vc_lo[l], kv_bytes / 2);
            HIP_TRY(c, hipMemsetAsync(c->kc_lo[l], 0, kv_bytes / 2, c->st));
            HIP_TRY(c, hipMemsetAsync(c->vc_lo[l], 0, kv_bytes / 2, c->st));
        }
    }
    // ---- rotary table: cos/sin(pos * theta^(-2i/dh)) in double, stored fp32
    {
        const int half = dh / 2;
        std::vector<float> cs((size_t)g.max_seq * half * 2);
        for (int i = 0; i < half; ++i) {
            const double inv = pow((double)g.rope_theta, -2.0 * i / (double)dh);
            for (int p = 0; p < g.max_seq; ++p) {
                const double ang = (double)p * inv;
                cs[((size_t)p * half + i) * 2] = (float)cos(ang);
                cs[((size_t)p * half + i) * 2 + 1] = (float)sin(ang);
            }
        }
        ALLOC(c, c->cs_table, cs.size() * 4);
        HIP_TRY(c, hipMemcpy(c->cs_table, cs.data(), cs.size() * 4, hipMemcpyHostToDevice));
    }
    // ---- scratch
    const int m_max = g.max_k + 1;
    c->Rmax = g.max_batch * m_max;
    c->Pmax = c->bf16 ? (g.max_seq < PREFILL_ROWS_MAX ? g.max_seq : PREFILL_ROWS_MAX) : PREFILL_ROWS_F32;
    if (c->Rmax < c->Pmax) c->Rmax = c->Pmax;
    const size_t Rp = ((size_t)c->Rmax + 127) / 128 * 128 + 48;  // slack: the GEMMs read whole row tiles / row blocks
    std::vector<std::pair<void *, size_t>> zero;
    auto zalloc = [&](void **p, size_t bytes) -> int { int r = dev_alloc(c, p, bytes); if (r == LLMA_OK) zero.push_back({*p, bytes}); return r; };
    if ((rc = zalloc((void **)&c->h, Rp * d * 4))) return rc;
    if (c->bf16) {
        const size_t Tt = Rp / 16;                                // row tiles
        const size_t x_bytes = Tt * c->plan_qkv.KSp * 1024, q_bytes = Tt * (d / 32) * 1024, act_bytes = Tt * c->plan_down.KSp * 1024;
        if ((rc = zalloc(&c->xhi, x_bytes)) || (rc = zalloc(&c->xlo, x_bytes)) || (rc = zalloc(&c->q, q_bytes)) ||
            (rc = zalloc(&c->q_lo, q_bytes)) || (rc = zalloc(&c->att_hi, x_bytes)) || (rc = zalloc(&c->att_lo, x_bytes)) ||
            (rc = zalloc(&c->act_hi, act_bytes)) || (rc = zalloc(&c->act_lo, act_bytes)))
            return rc;
        if ((rc = zalloc((void **)&c->ssq, Rp * (d / 16) * 4))) return rc;
        if ((rc = zalloc((void **)&c->rstd, Rp * 4))) return rc;
        c->nc_max = c->seq_cap / ATTN_CHUNK;
        // attention partials: [sequences][heads][chunks][rows], up to 48 rows per sequence (longer
        // prompt passes run the walking kernel, which has no partials)
        const size_t np = (size_t)g.max_batch * H * c->nc_max * 48;
        // partial sums of the split-K GEMM of batched steps (more than 48 rows in a step)
        const int step_rows = g.max_batch * (g.max_k + 1);
        if (step_rows > 48) {
            size_t tiles = 0;
            for (const GemmPlan *pl : {&c->plan_qkv, &c->plan_o, &c->plan_gu, &c->plan_down, &c->plan_lm}) {
                const size_t t = (size_t)pl->n_split * pl->tasks * (pl == &c->plan_gu ? 2 : 1);
                tiles = t > tiles ? t : tiles;
            }
            ALLOC(c, c->part, tiles * ((step_rows + 15) / 16) * 1024);
        }
        ALLOC(c, c->po, np * dh * 4);
        ALLOC(c, c->pm, np * 4);
        ALLOC(c, c->pl, np * 4);
    } else {
        if ((rc = zalloc((void **)&c->qkv, Rp * 3 * d * 4)) || (rc = zalloc(&c->xhi, Rp * d * 4)) || (rc = zalloc(&c->q, Rp * d * 4)) ||
            (rc = zalloc(&c->att_hi, Rp * d * 4)) || (rc = zalloc(&c->act_hi, Rp * F * 4)))
            return rc;
    }
    for (auto &z : zero) HIP_TRY(c, hipMemsetAsync(z.first, 0, z.second, c->st));
    c->n_part = c->bf16 ? V / 16 : V;
    const size_t lm_rows = (size_t)g.max_batch * m_max;      // only decoding steps run the LM head
    ALLOC(c, c->pval, lm_rows * c->n_part * 4);
    ALLOC(c, c->pidx, lm_rows * c->n_part * 4);
    // ---- step state
    StepState &s = c->s;
    ALLOC(c, s.row_tok, Rp * 4);
    ALLOC(c, s.row_pos, Rp * 4);
    ALLOC(c, s.row_slot, Rp * 4);
    ALLOC(c, s.row_cs, Rp * dh * 4);
    HIP_TRY(c, hipMemsetAsync(s.row_cs, 0, Rp * dh * 4, c->st));
    ALLOC(c, s.T, g.max_batch * 4);
    ALLOC(c, s.pending, g.max_batch * 4);
    ALLOC(c, s.batch_slots, g.max_batch * 4);
    ALLOC(c, s.keff, g.max_batch * 4);
    ALLOC(c, s.draft, (size_t)g.max_batch * (g.max_k + 1) * 4);
    ALLOC(c, s.nacc, g.max_batch * 4);
    ALLOC(c, s.next, g.max_batch * 4);
    ALLOC(c, s.emit, (size_t)g.max_batch * m_max * 4);
    ALLOC(c, s.otok, Rp * 4);
    HIP_TRY(c, hipMemsetAsync(s.T, 0, g.max_batch * 4, c->st));
    HIP_TRY(c, hipMemsetAsync(s.pending, 0xFF, g.max_batch * 4, c->st));
    HIP_TRY(c, hipMemsetAsync(s.keff, 0, g.max_batch * 4, c->st));
    HIP_TRY(c, hipMemsetAsync(s.row_pos, 0, Rp * 4, c->st));
    HIP_TRY(c, hipMemsetAsync(s.row_slot, 0, Rp * 4, c->st));
    ALLOC(c, c->gen_dev, sizeof(GenState) * g.max_batch);
    ALLOC(c, c->gen_counters, (size_t)(4 * g.max_batch + 4) * 4);
    c->T_host.assign(g.max_batch, 0);
    c->pending_host.assign(g.max_batch, -1);
    c->lo_from_host.assign(g.max_batch, 0);
    c->imp_len.assign((size_t)g.max_batch * g.n_layers, -1);
    ALLOC(c, c->lo_from, g.max_batch * 4);
    HIP_TRY(c, hipMemsetAsync(c->lo_from, 0, g.max_batch * 4, c->st));
    HIP_TRY(c, hipStreamCreateWithFlags(&c->cap_st, hipStreamNonBlocking));
    HIP_TRY(c, hipHostMalloc((void **)&c->pin_counts, (size_t)2 * g.max_batch * sizeof(int), hipHostMallocDefault));
    HIP_TRY(c, hipEventCreateWithFlags(&c->cnt_ev[0], hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->cnt_ev[1], hipEventDisableTiming));
    HIP_TRY(c, hipStreamSynchronize(c->st));
    HIP_TRY(c, hipGetLastError());
    return autotune_tilek(c);
}

// ------------------------------------------------------------------------------------------------
// decoding-step GEMM arguments outside a forward (tuning, timing): matrix `which` of layer `layer`
// (0 QKV, 1 O, 2 gate/up, 3 down, 4 LM head) over `rows` rows of whatever the scratch planes hold
// ------------------------------------------------------------------------------------------------
static GemmArgs step_gemm_args(llma_ctx *c, int which, int layer, int rows) {
    const llma_model_cfg &g = c->cfg;
    GemmArgs ga{};
    ga.rows = rows; ga.split = c->opt_split; ga.eps = g.rms_eps; ga.rstd_in = c->rstd;
    ga.ssq_tiles = g.d_model / 16; ga.H = g.n_heads; ga.dh = g.head_dim; ga.max_seq = c->seq_cap; ga.nx_KSp = c->plan_qkv.KSp;
    switch (which) {
        case 0:
            ga.W = c->wqkv[layer]; ga.plan = c->plan_qkv; ga.Xhi = c->xhi; ga.Xlo = c->xlo; ga.epi = EPI_QKV; ga.ssq_in = c->ssq;
            ga.row_pos = c->s.row_pos; ga.row_slot = c->s.row_slot; ga.row_cs = c->s.row_cs; ga.q_hi = c->q; ga.q_lo = c->q_lo;
            ga.k_hi = c->kc[layer]; ga.k_lo = c->kc_lo[layer]; ga.v_hi = c->vc[layer]; ga.v_lo = c->vc_lo[layer];
            break;
        case 1:
            ga.W = c->wo[layer]; ga.plan = c->plan_o; ga.Xhi = c->att_hi; ga.Xlo = c->att_lo; ga.epi = EPI_RESID; ga.out = c->h;
            ga.gain = c->n2[layer]; ga.nx_hi = c->xhi; ga.nx_lo = c->xlo; ga.ssq_out = c->ssq;
            break;
        case 2:
            ga.W = c->wgu[layer]; ga.plan = c->plan_gu; ga.Xhi = c->xhi; ga.Xlo = c->xlo; ga.epi = EPI_SWIGLU; ga.ssq_in = c->ssq;
            ga.act_hi = c->act_hi; ga.act_lo = c->act_lo; ga.act_KSp = c->plan_down.KSp;
            break;
        case 3:
            ga.W = c->wd[layer]; ga.plan = c->plan_down; ga.Xhi = c->act_hi; ga.Xlo = c->act_lo; ga.epi = EPI_RESID; ga.out = c->h;
            ga.gain = c->n1[layer]; ga.nx_hi = c->xhi; ga.nx_lo = c->xlo; ga.ssq_out = c->ssq;
            break;
        default:
            ga.W = c->lm_head; ga.plan = c->plan_lm; ga.Xhi = c->xhi; ga.Xlo = c->xlo; ga.epi = EPI_LMHEAD; ga.ssq_in = c->ssq;
            ga.out = nullptr; ga.pval = c->pval; ga.pidx = c->pidx; ga.n_part = c->n_part;
            break;
    }
    return ga;
}

// How many feature tiles a workgroup of the decoding GEMM takes is pure work division (a tile's sums are
// the same for any value), and which value streams a matrix fastest depends on how its tile count falls
// on the device's compute units (7B: one tile per workgroup for the 256-tile O / down matrices; 13B, 320
// tiles: two, 35.6 -> 27.0 us for down; QKV 960 tiles: four, 34.0 -> 26.1 us).  So it is measured: every
// admissible value, for 1 / 17 / 33 rows (one, two, three row tiles), on the context's own matrices and
// zeroed scratch, a few dozen launches each; a value has to beat the default by 5 % to replace it.
static int autotune_tilek(llma_ctx *c) {
    if (!c->bf16 || getenv("LLMA_NO_AUTOTUNE") != nullptr) return LLMA_OK;
    const llma_model_cfg &g = c->cfg;
    GemmPlan *plans[5] = {&c->plan_qkv, &c->plan_o, &c->plan_gu, &c->plan_down, &c->plan_lm};
    if (const char *forced = getenv("LLMA_TILEK_FT")) {       // tests: this many tiles per workgroup wherever the kernel admits it
        const int ft = atoi(forced);
        for (GemmPlan *p : plans)
            for (int nt = 1; nt <= 3; ++nt)
                if (tilek_ft_valid(*p, nt, ft)) p->tk_ft[nt - 1] = ft;
        return LLMA_OK;
    }
    const int step_rows = g.max_batch * (g.max_k + 1);
    hipEvent_t e0, e1;
    HIP_TRY(c, hipEventCreate(&e0));
    HIP_TRY(c, hipEventCreate(&e1));
    const int reps = g.n_layers < 8 ? 16 : (2 * g.n_layers < 48 ? 2 * g.n_layers : 48);
    for (int which = 0; which < 5; ++which)
        for (int nt = 1; nt <= 3; ++nt) {
            const int rows = nt == 1 ? 1 : 16 * (nt - 1) + 1;
            if (rows > step_rows || rows > 48) continue;                  // this context never launches that many row tiles
            GemmPlan &p = *plans[which];
            const int dflt = p.tk_ft[nt - 1];
            // mean launch time of this matrix at `rows` rows with FT = ft
            auto time_ft = [&](int ft, float *us) -> int {
                p.tk_ft[nt - 1] = ft;
                float ms = 0.f;
                for (int pass = 0; pass < 2; ++pass) {                    // pass 0 warms up
                    const int n = pass ? reps : 3;
                    HIP_TRY(c, hipEventRecord(e0, c->st));
                    for (int r = 0; r < n; ++r) {
                        GemmArgs ga = step_gemm_args(c, which, r % g.n_layers, rows);
                        if (!launch_gemm_bf16(ga, c->st)) return fail(c, LLMA_E_INVAL, "autotune: launch refused");
                    }
                    HIP_TRY(c, hipEventRecord(e1, c->st));
                    HIP_TRY(c, hipEventSynchronize(e1));
                    HIP_TRY(c, hipEventElapsedTime(&ms, e0, e1));
                }
                *us = ms * 1e3f / reps;
                return LLMA_OK;
            };
            float best_us = 0.f, dflt_us = 0.f;
            int best = dflt;
            for (int ft = 1; ft <= 4; ++ft) {
                if (!tilek_ft_valid(p, nt, ft)) continue;
                float us = 0.f;
                if (int rc = time_ft(ft, &us)) return rc;
                if (ft == dflt) dflt_us = us;
                if (best_us == 0.f || us < best_us) { best_us = us; best = ft; }
            }
            // A candidate replaces the default only if it wins by 5 % twice: in the sweep and again
            // head to head (default first, candidate second), so that one disturbed measurement
            // -- clocks still ramping, another process on the card -- cannot pick a slower shape.
            bool adopt = best != dflt && dflt_us > 0.f && best_us < 0.95f * dflt_us;
            if (adopt) {
                float d2 = 0.f, b2 = 0.f;
                if (int rc = time_ft(dflt, &d2)) return rc;
                if (int rc = time_ft(best, &b2)) return rc;
                adopt = b2 < 0.95f * d2;
            }
            p.tk_ft[nt - 1] = adopt ? best : dflt;
        }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    HIP_TRY(c, hipGetLastError());
    return LLMA_OK;
}

extern "C" int llma_create(const llma_model_cfg *cfg, const llma_weights *w, void *hip_stream, llma_ctx **out) {
    if (!cfg || !w || !out) return fail(nullptr, LLMA_E_INVAL, "llma_create: null argument");
    *out = nullptr;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!w->embed || !w->lm_head || !w->final_norm || !w->wqkv || !w->wo || !w->wgu || !w->wdown || !w->norm1 || !w->norm2)
        return fail(nullptr, LLMA_E_INVAL, "llma_create: null weight pointer");
    llma_ctx *c = new (std::nothrow) llma_ctx();
    if (!c) return fail(nullptr, LLMA_E_NOMEM, "llma_create: host allocation failed");
    c->cfg = *cfg;
    c->st = (hipStream_t)hip_stream;
    c->run_st = c->st;
    c->bf16 = cfg->dtype == LLMA_DTYPE_BF16;
    c->kv_split = c->bf16 && cfg->kv_split != 0;
    rc = create_impl(c, w);
    if (rc) {
        std::string e = c->err;
        llma_destroy(c);
        g_err = e;
        return rc;
    }
    *out = c;
    return LLMA_OK;
}

extern "C" int llma_destroy(llma_ctx *c) {
    if (!c) return LLMA_OK;
    (void)hipStreamSynchronize(c->st);
    for (auto &g : c->graphs) if (g.second.exec) (void)hipGraphExecDestroy(g.second.exec);
    if (c->cap_st) (void)hipStreamDestroy(c->cap_st);
    if (c->pin_counts) (void)hipHostFree(c->pin_counts);
    for (int i = 0; i < 2; ++i) if (c->cnt_ev[i]) (void)hipEventDestroy(c->cnt_ev[i]);
    for (auto &e : c->events) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    for (void *p : c->allocs) (void)hipFree(p);
    delete c;
    return LLMA_OK;
}

extern "C" const char *llma_last_error(const llma_ctx *c) { return c ? c->err.c_str() : g_err.c_str(); }
extern "C" int64_t llma_device_bytes(const llma_ctx *c) { return c ? c->dev_bytes : 0; }

extern "C" int llma_describe(const llma_ctx *c, char *buf, int32_t cap) {
    if (!c || !buf || cap < 1) return LLMA_E_INVAL;
    if (!c->bf16) { snprintf(buf, (size_t)cap, "fp32 path (plain vector-ALU kernels, nothing tuned)"); return LLMA_OK; }
    const GemmPlan *pl[5] = {&c->plan_qkv, &c->plan_o, &c->plan_gu, &c->plan_down, &c->plan_lm};
    const char *nm[5] = {"qkv", "o", "gate_up", "down", "lm_head"};
    int n = snprintf(buf, (size_t)cap, "decoding GEMM, feature tiles per workgroup at 1/2/3 row tiles (K slices):");
    for (int i = 0; i < 5 && n > 0 && n < cap; ++i)
        n += snprintf(buf + n, (size_t)(cap - n), " %s %d/%d/%d (%d)", nm[i], pl[i]->tk_ft[0], pl[i]->tk_ft[1], pl[i]->tk_ft[2], pl[i]->tk_waves);
    return LLMA_OK;
}

// ------------------------------------------------------------------------------------------------
// the forward over the rows described by ctx->s.row_* (paper: Eq. 3)
// ------------------------------------------------------------------------------------------------
static int forward_f32(llma_ctx *c, int n_seqs, int m, bool lm_head) {
    const llma_model_cfg &g = c->cfg;
    const int d = g.d_model, F = g.d_ffn, V = g.vocab, H = g.n_heads, dh = g.head_dim, L = g.n_layers;
    const int R = n_seqs * m;
    hipStream_t st = c->run_st;
    launch_embed_f32((const float *)c->embed, c->s.row_tok, c->h, R, d, st);
    GemmArgs ga{};
    ga.rows = R;
    AttnArgs aa{};
    aa.Qhi = c->q; aa.T = c->s.T; aa.batch_slots = c->s.batch_slots; aa.slot_const = -1; aa.n_seqs = n_seqs; aa.m = m; aa.H = H; aa.dh = dh;
    aa.max_seq = c->seq_cap; aa.scale = 1.0f / sqrtf((float)dh); aa.out_hi = c->att_hi;
    for (int l = 0; l < L; ++l) {
        launch_rmsnorm_f32(c->h, c->n1[l], g.rms_eps, (float *)c->xhi, R, d, st);
        ga.W = c->wqkv[l]; ga.Xhi = c->xhi; ga.N = 3 * d; ga.K = d; ga.epi = EPI_STORE; ga.out = c->qkv;
        launch_gemm_f32(ga, st);
        launch_rope_kv_f32(c->qkv, c->s, c->cs_table, (float *)c->q, (float *)c->kc[l], (float *)c->vc[l], R, H, dh, c->seq_cap, st);
        aa.Khi = c->kc[l]; aa.Vhi = c->vc[l];
        launch_attn_f32(aa, st);
        ga.W = c->wo[l]; ga.Xhi = c->att_hi; ga.N = d; ga.K = d; ga.epi = EPI_RESID; ga.out = c->h;
        launch_gemm_f32(ga, st);
        launch_rmsnorm_f32(c->h, c->n2[l], g.rms_eps, (float *)c->xhi, R, d, st);
        ga.W = c->wgu[l]; ga.Xhi = c->xhi; ga.N = F; ga.K = d; ga.epi = EPI_SWIGLU; ga.out = nullptr; ga.act_hi = c->act_hi;
        launch_gemm_f32(ga, st);
        ga.W = c->wd[l]; ga.Xhi = c->act_hi; ga.N = d; ga.K = F; ga.epi = EPI_RESID; ga.out = c->h; ga.act_hi = nullptr;
        launch_gemm_f32(ga, st);
    }
    if (lm_head) {
        launch_rmsnorm_f32(c->h, c->final_norm, g.rms_eps, (float *)c->xhi, R, d, st);
        ga.W = c->lm_head; ga.Xhi = c->xhi; ga.N = V; ga.K = d; ga.epi = EPI_LMHEAD;
        ga.out = c->logits_dump; ga.pval = c->pval; ga.pidx = c->pidx; ga.n_part = c->n_part;
        launch_gemm_f32(ga, st);
    }
    HIP_TRY(c, hipGetLastError());
    return LLMA_OK;
}

// bf16: per layer  QKV GEMM (+RMSNorm scale, RoPE, KV append) -> attention -> O GEMM (+residual,
// next-norm input) -> gate/up GEMM (+RMSNorm scale, SwiGLU) -> down GEMM (+residual, next-norm input)
static int forward_bf16(llma_ctx *c, int n_seqs, int m, int n_chunks, bool lm_head, int slot) {
    const llma_model_cfg &g = c->cfg;
    const int d = g.d_model, H = g.n_heads, dh = g.head_dim, L = g.n_layers;
    const int R = n_seqs * m;
    hipStream_t st = c->run_st;
    const int ksp_d = c->plan_qkv.KSp;          // k-steps per row tile of every activation plane that feeds a K = d GEMM
    launch_embed_prep_bf16(c->embed, c->s.row_tok, c->n1[0], c->h, c->xhi, c->xlo, c->ssq, R, d, ksp_d, st);
    GemmArgs base{};
    base.rows = R; base.split = c->opt_split; base.eps = g.rms_eps;
    base.rows_live = c->rows_live;                         // llma_generate, one sequence: the trigger's draft count (device)
    // prompt passes (no LM head) and batched steps of more than 48 rows use the panel GEMM (weights
    // streamed once for all rows); the steps in its split-K form, because a few hundred rows alone make
    // too few workgroups to fill the chip.  Steps of up to 48 rows use the tile-K GEMM.
    const bool panel = !lm_head || R > 48;
    bool refused = false;
    auto tilek_gemm = [&](GemmArgs &ga) { refused = !launch_gemm_bf16(ga, st) || refused; };
    auto panel_gemm = [&](GemmArgs &ga) {
        if (lm_head && ga.plan.n_split > 1) { ga.ksplit = ga.plan.n_split; ga.part = c->part; }
        launch_gemm_panel_bf16(ga, st);
    };
    // panel GEMM whose epilogue scales by the rows' rstd: the split-K form computes it in an extra
    // workgroup of its first kernel (its finishing kernel is the reader), otherwise a launch of its own
    auto panel_norm_gemm = [&](GemmArgs &ga) {
        if (lm_head && ga.plan.n_split > 1) ga.rstd_out = c->rstd;
        else launch_rstd_rows(c->ssq, d / 16, g.rms_eps, c->rstd, R, st);
        panel_gemm(ga);
    };
    base.rstd_in = c->rstd;
    base.ssq_tiles = d / 16; base.H = H; base.dh = dh; base.max_seq = c->seq_cap; base.nx_KSp = ksp_d;
    AttnArgs aa{};
    aa.Qhi = c->q; aa.Qlo = c->q_lo; aa.T = c->s.T; aa.batch_slots = c->s.batch_slots; aa.slot_const = n_seqs == 1 ? slot : -1; aa.n_seqs = n_seqs; aa.m = m; aa.H = H; aa.dh = dh;
    aa.rows_live = c->rows_live;
    aa.lo_from = c->kv_split ? c->lo_from : nullptr;
    aa.max_seq = c->seq_cap; aa.n_chunks = n_chunks; aa.scale = 1.0f / sqrtf((float)dh);
    aa.po = c->po; aa.pm = c->pm; aa.pl = c->pl; aa.out_hi = c->att_hi; aa.out_lo = c->att_lo; aa.out_KSp = ksp_d;
    for (int l = 0; l < L; ++l) {
        GemmArgs ga = base;
        ga.W = c->wqkv[l]; ga.plan = c->plan_qkv; ga.Xhi = c->xhi; ga.Xlo = c->xlo; ga.epi = EPI_QKV; ga.ssq_in = c->ssq;
        ga.row_pos = c->s.row_pos; ga.row_slot = c->s.row_slot; ga.row_cs = c->s.row_cs; ga.q_hi = c->q; ga.q_lo = c->q_lo;
        ga.k_hi = c->kc[l]; ga.k_lo = c->kc_lo[l]; ga.v_hi = c->vc[l]; ga.v_lo = c->vc_lo[l];
        if (panel) panel_norm_gemm(ga);
        else tilek_gemm(ga);
        aa.Khi = c->kc[l]; aa.Klo = c->kc_lo[l]; aa.Vhi = c->vc[l]; aa.Vlo = c->vc_lo[l];
        launch_attn_bf16(aa, st);
        ga = base;
        ga.W = c->wo[l]; ga.plan = c->plan_o; ga.Xhi = c->att_hi; ga.Xlo = c->att_lo; ga.epi = EPI_RESID; ga.out = c->h;
        ga.gain = c->n2[l]; ga.nx_hi = c->xhi; ga.nx_lo = c->xlo; ga.ssq_out = c->ssq;
        if (panel) panel_gemm(ga); else tilek_gemm(ga);
        ga = base;
        ga.W = c->wgu[l]; ga.plan = c->plan_gu; ga.Xhi = c->xhi; ga.Xlo = c->xlo; ga.epi = EPI_SWIGLU; ga.ssq_in = c->ssq;
        ga.act_hi = c->act_hi; ga.act_lo = c->act_lo; ga.act_KSp = c->plan_down.KSp;
        if (panel) {
            panel_norm_gemm(ga);
        } else if (c->opt_timing) {
            EventPair ep;
            HIP_TRY(c, hipEventCreate(&ep.a));
            HIP_TRY(c, hipEventCreate(&ep.b));
            HIP_TRY(c, hipEventRecord(ep.a, st));
            tilek_gemm(ga);
            HIP_TRY(c, hipEventRecord(ep.b, st));
            c->events.push_back(ep);
        } else {
            tilek_gemm(ga);
        }
        ga = base;
        ga.W = c->wd[l]; ga.plan = c->plan_down; ga.Xhi = c->act_hi; ga.Xlo = c->act_lo; ga.epi = EPI_RESID; ga.out = c->h;
        ga.gain = (l + 1 < L) ? c->n1[l + 1] : c->final_norm; ga.nx_hi = c->xhi; ga.nx_lo = c->xlo; ga.ssq_out = c->ssq;
        if (panel) panel_gemm(ga); else tilek_gemm(ga);
    }
    if (lm_head) {
        GemmArgs ga = base;
        ga.W = c->lm_head; ga.plan = c->plan_lm; ga.Xhi = c->xhi; ga.Xlo = c->xlo; ga.epi = EPI_LMHEAD; ga.ssq_in = c->ssq;
        ga.out = c->logits_dump; ga.pval = c->pval; ga.pidx = c->pidx; ga.n_part = c->n_part;
        if (panel) panel_norm_gemm(ga);
        else tilek_gemm(ga);
    }
    if (refused) return fail(c, LLMA_E_INVAL, "forward: a step of %d rows reached the decoding-step GEMM (1..48 rows)", R);
    HIP_TRY(c, hipGetLastError());
    return LLMA_OK;
}

static int forward(llma_ctx *c, int n_seqs, int m, int n_chunks, bool lm_head, int slot) {
    return c->bf16 ? forward_bf16(c, n_seqs, m, n_chunks, lm_head, slot) : forward_f32(c, n_seqs, m, lm_head);
}

// One step = row set-up + forward + bookkeeping, always the same launches for a given
// (kind, rows, attention chunk count, slot): the second time a shape is seen its launches are
// captured into a HIP graph and from then on replayed.  All per-step data (tokens, positions,
// cache lengths, drafts) lives in device memory, so a replay needs no new arguments.
static int step_body(llma_ctx *c, int kind, int n_seqs, int m, int n_chunks, int slot) {
    hipStream_t st = c->run_st;
    const int mk = c->cfg.max_k;
    c->rows_live = nullptr;
    if (kind == STEP_PREFILL) {
        launch_setup_prefill_rows(c->s, c->gen_prompt, c->gen_counters + 4 * c->cfg.max_batch, m, slot, c->cs_table, c->cfg.head_dim / 2, st);
        int rc = forward(c, 1, m, n_chunks, false, slot);
        if (rc) return rc;
        launch_advance_T(c->s, slot, m, st);
        return LLMA_OK;
    }
    c->rows_live = (kind == STEP_GEN && n_seqs == 1) ? c->s.keff : nullptr;
    if (kind == STEP_GEN) launch_trigger(c->gen_dev, c->s, n_seqs, mk, st);
    launch_setup_step_rows(c->s, n_seqs, m, mk, c->cs_table, c->cfg.head_dim / 2, st);
    int rc = forward(c, n_seqs, m, n_chunks, true, slot);
    if (rc) return rc;
    launch_argmax_accept(c->pval, c->pidx, c->n_part, c->s, n_seqs, m, mk, c->cfg.vocab, kind == STEP_GEN ? c->gen_dev : nullptr, st);
    return LLMA_OK;
}

static void drop_graphs(llma_ctx *c) {
    (void)hipStreamSynchronize(c->st);
    for (auto &g : c->graphs) if (g.second.exec) (void)hipGraphExecDestroy(g.second.exec);
    c->graphs.clear();
}

static int run_step(llma_ctx *c, int kind, int n_seqs, int m, int t_max, int slot) {
    // attention chunks launched: enough for the longest sequence.  A launched chunk streams its K/V
    // blocks before it knows whether it lies past the sequence's end, so the count is rounded up
    // (fewer distinct launch shapes, i.e. graphs) only by a few percent: to whole buckets of 1, 4 or
    // 16 chunks for up to 32, 128 or more chunks
    int n_chunks = (t_max + m + ATTN_CHUNK - 1) / ATTN_CHUNK;
    const int bucket = n_chunks <= 32 ? 1 : (n_chunks <= 128 ? 4 : 16);
    n_chunks = (n_chunks + bucket - 1) / bucket * bucket;
    if (c->bf16 && n_chunks > c->nc_max) n_chunks = c->nc_max;
    c->run_st = c->st;
    if (!c->opt_graph || c->opt_timing || c->graphs.size() > 256) return step_body(c, kind, n_seqs, m, n_chunks, slot);
    const GraphKey key = {kind, n_seqs, m, n_chunks, slot};     // every field that shapes a launch or is baked into one
    GraphSlot &gs = c->graphs[key];
    if (gs.exec == nullptr) {
        if (gs.seen++ == 0) return step_body(c, kind, n_seqs, m, n_chunks, slot);   // first time eagerly
        hipGraph_t graph = nullptr;
        if (hipStreamBeginCapture(c->cap_st, hipStreamCaptureModeRelaxed) != hipSuccess) { c->opt_graph = 0; return step_body(c, kind, n_seqs, m, n_chunks, slot); }
        c->run_st = c->cap_st;
        int rc = step_body(c, kind, n_seqs, m, n_chunks, slot);
        c->run_st = c->st;
        hipError_t e = hipStreamEndCapture(c->cap_st, &graph);
        if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
        if (e != hipSuccess || graph == nullptr) return fail(c, LLMA_E_HIP, "graph capture failed: %s", hipGetErrorString(e));
        e = hipGraphInstantiate(&gs.exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e != hipSuccess) { gs.exec = nullptr; return fail(c, LLMA_E_HIP, "hipGraphInstantiate: %s", hipGetErrorString(e)); }
    }
    HIP_TRY(c, hipGraphLaunch(gs.exec, c->st));
    return LLMA_OK;
}

// ------------------------------------------------------------------------------------------------
// sequence state
// ------------------------------------------------------------------------------------------------
static int check_slot(llma_ctx *c, int seq, const char *who) {
    if (!c) return fail(nullptr, LLMA_E_INVAL, "%s: null context", who);
    if (seq < 0 || seq >= c->cfg.max_batch) return fail(c, LLMA_E_RANGE, "%s: slot %d outside [0,%d)", who, seq, c->cfg.max_batch);
    return LLMA_OK;
}
static int push_state(llma_ctx *c, int seq) {       // host mirror -> device
    HIP_TRY(c, hipMemcpyAsync(c->s.T + seq, &c->T_host[seq], 4, hipMemcpyHostToDevice, c->st));
    HIP_TRY(c, hipMemcpyAsync(c->s.pending + seq, &c->pending_host[seq], 4, hipMemcpyHostToDevice, c->st));
    HIP_TRY(c, hipMemcpyAsync(c->lo_from + seq, &c->lo_from_host[seq], 4, hipMemcpyHostToDevice, c->st));
    HIP_TRY(c, hipStreamSynchronize(c->st));
    return LLMA_OK;
}
// something is about to be computed on the slot: the record of imported lengths no longer describes a pure import
static void forget_imports(llma_ctx *c, int seq) {
    for (int l = 0; l < c->cfg.n_layers; ++l) c->imp_len[(size_t)seq * c->cfg.n_layers + l] = -1;
}

extern "C" int llma_reset(llma_ctx *c, int32_t seq) {
    int rc = check_slot(c, seq, "llma_reset");
    if (rc) return rc;
    c->T_host[seq] = 0;
    c->pending_host[seq] = -1;
    c->lo_from_host[seq] = 0;
    forget_imports(c, seq);
    return push_state(c, seq);
}

extern "C" int llma_get_state(llma_ctx *c, int32_t seq, int32_t *T, int32_t *pending) {
    int rc = check_slot(c, seq, "llma_get_state");
    if (rc) return rc;
    int t = 0, p = -1;
    HIP_TRY(c, hipMemcpyAsync(&t, c->s.T + seq, 4, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipMemcpyAsync(&p, c->s.pending + seq, 4, hipMemcpyDeviceToHost, c->st));
    HIP_TRY(c, hipStreamSynchronize(c->st));
    if (T) *T = t;
    if (pending) *pending = p;
    return LLMA_OK;
}

extern "C" int llma_truncate(llma_ctx *c, int32_t seq, int32_t new_len) {
    int rc = check_slot(c, seq, "llma_truncate");
    if (rc) return rc;
    if (new_len < 0 || new_len > c->T_host[seq])
        return fail(c, LLMA_E_RANGE, "llma_truncate: new length %d outside [0, T = %d]", new_len, c->T_host[seq]);
    c->T_host[seq] = new_len;
    if (c->lo_from_host[seq] > new_len) c->lo_from_host[seq] = new_len;    // rows written from here on have lo planes
    return push_state(c, seq);
}

extern "C" int llma_set_pending(llma_ctx *c, int32_t seq, int32_t token) {
    int rc = check_slot(c, seq, "llma_set_pending");
    if (rc) return rc;
    if (token < 0 || token >= c->cfg.vocab) return fail(c, LLMA_E_RANGE, "llma_set_pending: token %d outside [0,%d)", token, c->cfg.vocab);
    c->pending_host[seq] = token;
    return push_state(c, seq);
}

extern "C" int llma_kv_import(llma_ctx *c, int32_t seq, int32_t layer, const void *k, const void *v, int32_t len) {
    int rc = check_slot(c, seq, "llma_kv_import");
    if (rc) return rc;
    if (!k || !v) return fail(c, LLMA_E_INVAL, "llma_kv_import: null pointer");
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, LLMA_E_RANGE, "llma_kv_import: layer %d", layer);
    if (len < 0 || len > c->cfg.max_seq) return fail(c, LLMA_E_RANGE, "llma_kv_import: len %d > max_seq %d", len, c->cfg.max_seq);
    const llma_model_cfg &g = c->cfg;
    const size_t es = c->bf16 ? 2 : 4;
    const size_t slot_off = (size_t)seq * g.n_heads * c->seq_cap * g.head_dim * es;
    void *kc = (char *)c->kc[layer] + slot_off, *vc = (char *)c->vc[layer] + slot_off;
    void *kl = c->kv_split ? (char *)c->kc_lo[layer] + slot_off / 2 : nullptr, *vl = c->kv_split ? (char *)c->vc_lo[layer] + slot_off / 2 : nullptr;
    if (len > 0) {
        if (c->bf16) launch_kv_import_bf16(k, v, kc, kl, vc, vl, g.n_heads, len, g.head_dim, c->seq_cap, c->st);
        else launch_kv_import_f32(k, v, kc, vc, g.n_heads, len, g.head_dim, c->seq_cap, c->st);
    }
    HIP_TRY(c, hipGetLastError());
    c->imp_len[(size_t)seq * g.n_layers + layer] = len;
    if (layer == g.n_layers - 1) {
        c->T_host[seq] = len;
        bool all = c->kv_split != 0;
        for (int l = 0; l < g.n_layers; ++l) all = all && c->imp_len[(size_t)seq * g.n_layers + l] == len;
        c->lo_from_host[seq] = all ? len : 0;
        return push_state(c, seq);
    }
    return LLMA_OK;
}

static int check_tokens(llma_ctx *c, const int32_t *t, int n, const char *who) {
    for (int i = 0; i < n; ++i)
        if (t[i] < 0 || t[i] >= c->cfg.vocab) return fail(c, LLMA_E_RANGE, "%s: token[%d] = %d outside [0,%d)", who, i, t[i], c->cfg.vocab);
    return LLMA_OK;
}

// feeds prompt_dev[0..len-1) in chunks; rows only write KV, no LM head
// feeds gen_prompt[0..n_feed) in chunks on top of the slot's cache; rows only write KV, no LM head
static int prefill_rows(llma_ctx *c, int seq, int n_feed) {
    // the chunk's tokens are gen_prompt[T - base ..]: base = T at the start of the prompt
    HIP_TRY(c, hipMemcpyAsync(c->gen_counters + 4 * c->cfg.max_batch, &c->T_host[seq], 4, hipMemcpyHostToDevice, c->st));
    HIP_TRY(c, hipStreamSynchronize(c->st));
    for (int off = 0; off < n_feed; off += c->Pmax) {
        const int m = n_feed - off < c->Pmax ? n_feed - off : c->Pmax;
        int rc = run_step(c, STEP_PREFILL, 1, m, c->T_host[seq], seq);
        if (rc) return rc;
        c->T_host[seq] += m;
    }
    return LLMA_OK;
}

static int ensure_cap(llma_ctx *c, int **buf, int *cap, int need) {
    if (need <= *cap) return LLMA_OK;
    drop_graphs(c);                                   // captured launches hold the old pointer
    if (*buf) { dev_free_one(c, *buf); *buf = nullptr; *cap = 0; }
    int ncap = need + need / 2 + 64;
    ALLOC(c, *buf, (size_t)ncap * 4);
    *cap = ncap;
    return LLMA_OK;
}

extern "C" int llma_prefill(llma_ctx *c, int32_t seq, const int32_t *prompt, int32_t len) {
    int rc = check_slot(c, seq, "llma_prefill");
    if (rc) return rc;
    if (!prompt || len < 1) return fail(c, LLMA_E_INVAL, "llma_prefill: need a prompt of at least one token");
    if (c->T_host[seq] + len > c->cfg.max_seq)
        return fail(c, LLMA_E_RANGE, "llma_prefill: T %d + len %d > max_seq %d", c->T_host[seq], len, c->cfg.max_seq);
    if ((rc = check_tokens(c, prompt, len, "llma_prefill"))) return rc;
    if ((rc = ensure_cap(c, &c->gen_prompt, &c->cap_prompt, len))) return rc;
    HIP_TRY(c, hipMemcpyAsync(c->gen_prompt, prompt, (size_t)len * 4, hipMemcpyHostToDevice, c->st));
    forget_imports(c, seq);
    if ((rc = prefill_rows(c, seq, len - 1))) return rc;
    c->pending_host[seq] = prompt[len - 1];
    HIP_TRY(c, hipMemcpyAsync(c->s.pending + seq, &c->pending_host[seq], 4, hipMemcpyHostToDevice, c->st));
    HIP_TRY(c, hipStreamSynchronize(c->st));
    return LLMA_OK;
}

// ------------------------------------------------------------------------------------------------
// llma_find_trigger (stateless)
// ------------------------------------------------------------------------------------------------
extern "C" int llma_find_trigger(const int32_t *y, int32_t y_len, const int32_t *ref, const int32_t *doc_offsets,
                                 int32_t n_docs, int32_t n, int32_t *doc_out, int32_t *pos_out) {
    if (!doc_out || !pos_out || !doc_offsets || n_docs < 0 || y_len < 0 || (!y && y_len > 0))
        return fail(nullptr, LLMA_E_INVAL, "llma_find_trigger: null pointer or negative count");
    if (n < 1) return fail(nullptr, LLMA_E_INVAL, "llma_find_trigger: n must be >= 1");
    for (int j = 0; j < n_docs; ++j)
        if (doc_offsets[j + 1] < doc_offsets[j] || doc_offsets[0] != 0)
            return fail(nullptr, LLMA_E_INVAL, "llma_find_trigger: doc_offsets must start at 0 and be non-decreasing");
    *doc_out = -1;
    *pos_out = -1;
    const int ref_len = n_docs > 0 ? doc_offsets[n_docs] : 0;
    if (ref_len > 0 && !ref) return fail(nullptr, LLMA_E_INVAL, "llma_find_trigger: null reference");
    if (ref_len == 0 || y_len < n) return 0;
    // device scratch for this call: [y | ref | doc_offsets | result(4)] copied in at once, then ref_doc
    const size_t n_in = (size_t)y_len + (size_t)ref_len + (size_t)(n_docs + 1) + 4;
    std::vector<int> stage(n_in);
    memcpy(stage.data(), y, (size_t)y_len * 4);
    memcpy(stage.data() + y_len, ref, (size_t)ref_len * 4);
    memcpy(stage.data() + y_len + ref_len, doc_offsets, (size_t)(n_docs + 1) * 4);
    int *buf = nullptr;
    hipError_t e = hipMalloc((void **)&buf, (n_in + (size_t)ref_len) * 4);
    if (e != hipSuccess) return fail(nullptr, LLMA_E_NOMEM, "llma_find_trigger: hipMalloc: %s", hipGetErrorString(e));
    int *dy = buf, *dref = dy + y_len, *doff = dref + ref_len, *dres = doff + n_docs + 1, *ddoc = dres + 4;
    int res[3] = {0, -1, -1};
    e = hipMemcpy(buf, stage.data(), n_in * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        launch_fill_ref_doc(doff, n_docs, ddoc, ref_len, nullptr);
        launch_trigger_plain(dy, y_len, dref, doff, ddoc, ref_len, n_docs, n, dres, false, nullptr);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpy(res, dres, 12, hipMemcpyDeviceToHost);
    (void)hipFree(buf);
    if (e != hipSuccess) return fail(nullptr, LLMA_E_HIP, "llma_find_trigger: %s", hipGetErrorString(e));
    if (res[0]) { *doc_out = res[1]; *pos_out = res[2]; }
    return res[0];
}

// ------------------------------------------------------------------------------------------------
// verify step
// ------------------------------------------------------------------------------------------------
extern "C" int llma_verify_step_batch(llma_ctx *c, int32_t n_seqs, const int32_t *seqs, const int32_t *drafts, int32_t k,
                                      int32_t *n_accepted, int32_t *next_token, int32_t *emitted) {
    if (!c) return fail(nullptr, LLMA_E_INVAL, "llma_verify_step: null context");
    const llma_model_cfg &g = c->cfg;
    if (!seqs || n_seqs < 1 || n_seqs > g.max_batch) return fail(c, LLMA_E_INVAL, "llma_verify_step: bad slot list");
    if (k < 0 || k > g.max_k) return fail(c, LLMA_E_RANGE, "llma_verify_step: k %d outside [0, max_k %d]", k, g.max_k);
    if (k > 0 && !drafts) return fail(c, LLMA_E_INVAL, "llma_verify_step: null drafts with k > 0");
    int t_max = 0;
    for (int b = 0; b < n_seqs; ++b) {
        int rc = check_slot(c, seqs[b], "llma_verify_step");
        if (rc) return rc;
        for (int b2 = 0; b2 < b; ++b2)
            if (seqs[b2] == seqs[b]) return fail(c, LLMA_E_INVAL, "llma_verify_step: slot %d listed twice", seqs[b]);
        if (c->pending_host[seqs[b]] < 0) return fail(c, LLMA_E_STATE, "llma_verify_step: slot %d has no pending token", seqs[b]);
        if (c->T_host[seqs[b]] + k + 1 > g.max_seq)
            return fail(c, LLMA_E_RANGE, "llma_verify_step: T %d + k + 1 > max_seq %d", c->T_host[seqs[b]], g.max_seq);
        if (c->T_host[seqs[b]] > t_max) t_max = c->T_host[seqs[b]];
    }
    if (k > 0) {
        int rc = check_tokens(c, drafts, n_seqs * k, "llma_verify_step(draft)");
        if (rc) return rc;
    }
    if (c->logits_dump && n_seqs * (k + 1) > c->dump_rows)
        return fail(c, LLMA_E_RANGE, "llma_verify_step: logits dump holds %d rows, step has %d", c->dump_rows, n_seqs * (k + 1));
    const int m = k + 1, mk = g.max_k;
    hipStream_t st = c->st;
    std::vector<int> keff(n_seqs, k), dr((size_t)n_seqs * (mk > 0 ? mk : 1), 0);
    for (int b = 0; b < n_seqs; ++b)
        for (int j = 0; j < k; ++j) dr[(size_t)b * mk + j] = drafts[(size_t)b * k + j];
    HIP_TRY(c, hipMemcpyAsync(c->s.batch_slots, seqs, (size_t)n_seqs * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(c, hipMemcpyAsync(c->s.keff, keff.data(), (size_t)n_seqs * 4, hipMemcpyHostToDevice, st));
    if (k > 0) HIP_TRY(c, hipMemcpyAsync(c->s.draft, dr.data(), (size_t)n_seqs * mk * 4, hipMemcpyHostToDevice, st));
    for (int b = 0; b < n_seqs; ++b) forget_imports(c, seqs[b]);
    int rc = run_step(c, STEP_VERIFY, n_seqs, m, t_max, n_seqs == 1 ? seqs[0] : 0);
    if (rc) return rc;
    std::vector<int> nacc(n_seqs), nxt(n_seqs), em((size_t)n_seqs * (mk + 1));
    HIP_TRY(c, hipMemcpyAsync(nacc.data(), c->s.nacc, (size_t)n_seqs * 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(c, hipMemcpyAsync(nxt.data(), c->s.next, (size_t)n_seqs * 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(c, hipMemcpyAsync(em.data(), c->s.emit, (size_t)n_seqs * (mk + 1) * 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(c, hipStreamSynchronize(st));
    HIP_TRY(c, hipGetLastError());
    for (int b = 0; b < n_seqs; ++b) {
        bool ok = nacc[b] >= 0 && nacc[b] <= k && nxt[b] >= 0 && nxt[b] < g.vocab;
        for (int j = 0; ok && j <= nacc[b]; ++j) ok = em[(size_t)b * (mk + 1) + j] >= 0 && em[(size_t)b * (mk + 1) + j] < g.vocab;
        if (!ok) return fail(c, LLMA_E_HIP, "llma_verify_step: device returned accepted count %d / token %d outside their ranges for slot %d", nacc[b], nxt[b], seqs[b]);
    }
    for (int b = 0; b < n_seqs; ++b) {
        c->T_host[seqs[b]] += nacc[b] + 1;
        c->pending_host[seqs[b]] = nxt[b];
        if (n_accepted) n_accepted[b] = nacc[b];
        if (next_token) next_token[b] = nxt[b];
        if (emitted)
            for (int j = 0; j <= nacc[b]; ++j) emitted[(size_t)b * (k + 1) + j] = em[(size_t)b * (mk + 1) + j];
    }
    return LLMA_OK;
}

extern "C" int llma_verify_step(llma_ctx *c, int32_t seq, const int32_t *draft, int32_t k, int32_t *n_accepted,
                                int32_t *next_token, int32_t *emitted) {
    return llma_verify_step_batch(c, 1, &seq, draft, k, n_accepted, next_token, emitted);
}

// ------------------------------------------------------------------------------------------------
// llma_generate (paper: Algorithm 1)
// ------------------------------------------------------------------------------------------------
extern "C" int llma_generate_batch(llma_ctx *c, int32_t n_seqs, const int32_t *seqs, const int32_t *prompts,
                                   const int32_t *prompt_offsets, const int32_t *refs, const int32_t *doc_offsets,
                                   const int32_t *n_docs, int32_t n, int32_t k, int32_t max_new, int32_t *out_tokens,
                                   int32_t *n_out, llma_step_rec *trace, int32_t *n_steps) {
    if (!c) return fail(nullptr, LLMA_E_INVAL, "llma_generate: null context");
    const llma_model_cfg &g = c->cfg;
    if (!seqs || n_seqs < 1 || n_seqs > g.max_batch) return fail(c, LLMA_E_INVAL, "llma_generate: bad slot list (1..max_batch %d slots)", g.max_batch);
    if (!prompts || !prompt_offsets || !out_tokens || !n_out || max_new < 1) return fail(c, LLMA_E_INVAL, "llma_generate: null / empty argument");
    if (n < 1) return fail(c, LLMA_E_INVAL, "llma_generate: n must be >= 1");
    if (k < 0 || k > g.max_k) return fail(c, LLMA_E_RANGE, "llma_generate: k %d outside [0, max_k %d]", k, g.max_k);
    if (prompt_offsets[0] != 0) return fail(c, LLMA_E_INVAL, "llma_generate: prompt_offsets[0] != 0");
    int rc;
    // per sequence: where its reference tokens and its document list start in the concatenated inputs
    std::vector<int> ref_start(n_seqs + 1, 0), docs_start(n_seqs + 1, 0);
    int max_prompt = 0;
    for (int b = 0; b < n_seqs; ++b) {
        if ((rc = check_slot(c, seqs[b], "llma_generate"))) return rc;
        for (int b2 = 0; b2 < b; ++b2)
            if (seqs[b2] == seqs[b]) return fail(c, LLMA_E_INVAL, "llma_generate: slot %d listed twice", seqs[b]);
        const int plen = prompt_offsets[b + 1] - prompt_offsets[b];
        if (plen < 1) return fail(c, LLMA_E_INVAL, "llma_generate: sequence %d has an empty prompt", b);
        if ((long)plen + max_new + k > g.max_seq)
            return fail(c, LLMA_E_RANGE, "llma_generate: prompt %d + max_new %d + k %d > max_seq %d", plen, max_new, k, g.max_seq);
        max_prompt = plen > max_prompt ? plen : max_prompt;
        const int nd = n_docs ? n_docs[b] : 0;
        if (nd < 0 || (nd > 0 && !doc_offsets)) return fail(c, LLMA_E_INVAL, "llma_generate: bad documents");
        int rlen = 0;
        if (nd > 0) {
            const int32_t *dof = doc_offsets + docs_start[b];
            if (dof[0] != 0) return fail(c, LLMA_E_INVAL, "llma_generate: doc_offsets[0] != 0");
            for (int j = 0; j < nd; ++j)
                if (dof[j + 1] < dof[j]) return fail(c, LLMA_E_INVAL, "llma_generate: doc_offsets decrease at %d", j);
            rlen = dof[nd];
            if (rlen > 0 && !refs) return fail(c, LLMA_E_INVAL, "llma_generate: null reference");
        }
        ref_start[b + 1] = ref_start[b] + rlen;
        docs_start[b + 1] = docs_start[b] + (doc_offsets ? nd + 1 : 0);
    }
    const int total_prompt = prompt_offsets[n_seqs], total_ref = ref_start[n_seqs];
    if ((rc = check_tokens(c, prompts, total_prompt, "llma_generate(prompt)"))) return rc;
    if (total_ref && (rc = check_tokens(c, refs, total_ref, "llma_generate(ref)"))) return rc;
    if (c->logits_dump && n_seqs * (k + 1) > c->dump_rows) return fail(c, LLMA_E_RANGE, "llma_generate: logits dump too small");

    hipStream_t st = c->st;
    const int ystride = max_new + 64;                       // per-sequence output / trace rows on the device
    if ((rc = ensure_cap(c, &c->gen_prompt, &c->cap_prompt, max_prompt))) return rc;
    if ((rc = ensure_cap(c, &c->gen_ref, &c->cap_ref, total_ref))) return rc;
    if ((rc = ensure_cap(c, &c->gen_ref_doc, &c->cap_refdoc, total_ref))) return rc;
    if ((rc = ensure_cap(c, &c->gen_doc_offsets, &c->cap_docs, docs_start[n_seqs] + n_seqs))) return rc;
    if ((rc = ensure_cap(c, &c->gen_y, &c->cap_y, n_seqs * ystride))) return rc;
    if ((rc = ensure_cap(c, &c->gen_trace, &c->cap_trace, 4 * n_seqs * ystride))) return rc;
    if (total_ref) HIP_TRY(c, hipMemcpyAsync(c->gen_ref, refs, (size_t)total_ref * 4, hipMemcpyHostToDevice, st));
    // device document lists: every sequence gets one (a sequence without reference: the single entry 0)
    std::vector<int> dof_host, dof_at(n_seqs);
    for (int b = 0; b < n_seqs; ++b) {
        const int nd = n_docs ? n_docs[b] : 0;
        dof_at[b] = (int)dof_host.size();
        if (nd > 0) dof_host.insert(dof_host.end(), doc_offsets + docs_start[b], doc_offsets + docs_start[b] + nd + 1);
        else dof_host.push_back(0);
    }
    HIP_TRY(c, hipMemcpyAsync(c->gen_doc_offsets, dof_host.data(), dof_host.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(c, hipMemsetAsync(c->gen_counters, 0, (size_t)(4 * g.max_batch + 4) * 4, st));
    std::vector<GenState> G(n_seqs);
    int *const cnt_out = c->gen_counters, *const cnt_steps = c->gen_counters + g.max_batch, *const cnt_cur = c->gen_counters + 2 * g.max_batch;
    for (int b = 0; b < n_seqs; ++b) {
        const int nd = n_docs ? n_docs[b] : 0, rlen = ref_start[b + 1] - ref_start[b];
        if (rlen) launch_fill_ref_doc(c->gen_doc_offsets + dof_at[b], nd, c->gen_ref_doc + ref_start[b], rlen, st);
        GenState &s = G[b];
        s.y = c->gen_y + (size_t)b * ystride; s.trace = c->gen_trace + (size_t)4 * b * ystride;
        s.n_out = cnt_out + b; s.n_steps = cnt_steps + b; s.cur = cnt_cur + 2 * b;
        s.ref = c->gen_ref + ref_start[b]; s.doc_offsets = c->gen_doc_offsets + dof_at[b]; s.ref_doc = c->gen_ref_doc + ref_start[b];
        s.ref_len = rlen; s.n_docs = nd; s.n = n; s.k = k; s.max_new = max_new; s.prompt = c->gen_prompt;
    }
    HIP_TRY(c, hipMemcpyAsync(c->gen_dev, G.data(), sizeof(GenState) * n_seqs, hipMemcpyHostToDevice, st));
    HIP_TRY(c, hipStreamSynchronize(st));     // the host staging buffers may go out of scope / change

    // ---- x: reset each slot, feed prompt[0..len-2], prompt[len-1] becomes the pending token
    std::vector<int> T0(n_seqs);
    for (int b = 0; b < n_seqs; ++b) {
        const int seq = seqs[b], plen = prompt_offsets[b + 1] - prompt_offsets[b];
        const int32_t *prompt = prompts + prompt_offsets[b];
        HIP_TRY(c, hipMemcpyAsync(c->gen_prompt, prompt, (size_t)plen * 4, hipMemcpyHostToDevice, st));
        c->T_host[seq] = 0;
        c->pending_host[seq] = prompt[plen - 1];
        c->lo_from_host[seq] = 0;
        forget_imports(c, seq);
        if ((rc = push_state(c, seq))) return rc;
        if ((rc = prefill_rows(c, seq, plen - 1))) return rc;
        HIP_TRY(c, hipStreamSynchronize(st));                   // gen_prompt is reused by the next sequence
        T0[b] = c->T_host[seq];
    }

    // ---- the decoding loop: trigger -> rows -> forward -> accept, all on the device, all sequences of
    //      the batch in one step (k + 1 rows each; a sequence that has its max_new tokens idles: its
    //      trigger copies nothing and the accept kernel leaves its state alone).  The host only reads
    //      the output counts back to know when to stop, and it does so one step late: step s+1 is
    //      already enqueued when the counts of step s are awaited, so the GPU never waits for the host.
    const int m = k + 1;
    HIP_TRY(c, hipMemcpyAsync(c->s.batch_slots, seqs, (size_t)n_seqs * 4, hipMemcpyHostToDevice, st));
    std::vector<int> produced(n_seqs, 0);
    int steps = 0, enq = 0;
    auto enqueue = [&]() -> int {
        // cache length bound for the attention grid: every enqueued step adds at most m positions
        int t_max = 0;
        for (int b = 0; b < n_seqs; ++b) t_max = T0[b] + produced[b] > t_max ? T0[b] + produced[b] : t_max;
        int r = run_step(c, STEP_GEN, n_seqs, m, t_max + 2 * m, n_seqs == 1 ? seqs[0] : 0);
        if (r) return r;
        HIP_TRY(c, hipMemcpyAsync(c->pin_counts + (size_t)(enq & 1) * g.max_batch, cnt_out, (size_t)n_seqs * 4, hipMemcpyDeviceToHost, st));
        HIP_TRY(c, hipEventRecord(c->cnt_ev[enq & 1], st));
        ++enq;
        return LLMA_OK;
    };
    if ((rc = enqueue())) return rc;
    while (true) {
        if ((rc = enqueue())) return rc;                        // one step ahead
        HIP_TRY(c, hipEventSynchronize(c->cnt_ev[steps & 1]));
        bool done = true;
        for (int b = 0; b < n_seqs; ++b) {
            const int now = c->pin_counts[(size_t)(steps & 1) * g.max_batch + b];
            if (now > max_new || now < produced[b] || (now == produced[b] && produced[b] < max_new))
                return fail(c, LLMA_E_HIP, "llma_generate: device output count of sequence %d went %d -> %d", b, produced[b], now);
            produced[b] = now;
            done = done && now >= max_new;
        }
        ++steps;
        if (done) break;
    }
    HIP_TRY(c, hipStreamSynchronize(st));                       // drains the step that ran ahead
    std::vector<int> nst(n_seqs);
    HIP_TRY(c, hipMemcpyAsync(nst.data(), cnt_steps, (size_t)n_seqs * 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(c, hipStreamSynchronize(st));
    for (int b = 0; b < n_seqs; ++b) {
        const int seq = seqs[b];
        c->T_host[seq] = T0[b] + produced[b];
        HIP_TRY(c, hipMemcpyAsync(out_tokens + (size_t)b * max_new, c->gen_y + (size_t)b * ystride, (size_t)max_new * 4, hipMemcpyDeviceToHost, st));
        if (trace) HIP_TRY(c, hipMemcpyAsync(trace + (size_t)b * max_new, c->gen_trace + (size_t)4 * b * ystride, (size_t)nst[b] * sizeof(llma_step_rec), hipMemcpyDeviceToHost, st));
        HIP_TRY(c, hipMemcpyAsync(&c->pending_host[seq], c->s.pending + seq, 4, hipMemcpyDeviceToHost, st));
        n_out[b] = produced[b];
        if (n_steps) n_steps[b] = nst[b];
    }
    HIP_TRY(c, hipStreamSynchronize(st));
    return LLMA_OK;
}

extern "C" int llma_generate(llma_ctx *c, int32_t seq, const int32_t *prompt, int32_t prompt_len, const int32_t *ref,
                             const int32_t *doc_offsets, int32_t n_docs, int32_t n, int32_t k, int32_t max_new,
                             int32_t *out_tokens, int32_t *n_out, llma_step_rec *trace, int32_t *n_steps) {
    if (!c) return fail(nullptr, LLMA_E_INVAL, "llma_generate: null context");
    if (prompt_len < 1) return fail(c, LLMA_E_INVAL, "llma_generate: null / empty argument");
    if (n_docs < 0 || (n_docs > 0 && !doc_offsets)) return fail(c, LLMA_E_INVAL, "llma_generate: bad documents");
    const int32_t poff[2] = {0, prompt_len};
    return llma_generate_batch(c, 1, &seq, prompt, poff, ref, doc_offsets, &n_docs, n, k, max_new, out_tokens, n_out, trace, n_steps);
}

// ------------------------------------------------------------------------------------------------
// inspection / options
// ------------------------------------------------------------------------------------------------
extern "C" int llma_set_logits_dump(llma_ctx *c, float *dev_buf, int32_t capacity_rows) {
    if (!c) return fail(nullptr, LLMA_E_INVAL, "llma_set_logits_dump: null context");
    if (dev_buf && capacity_rows < 1) return fail(c, LLMA_E_INVAL, "llma_set_logits_dump: capacity_rows < 1");
    drop_graphs(c);
    c->logits_dump = dev_buf;
    c->dump_rows = dev_buf ? capacity_rows : 0;
    return LLMA_OK;
}

extern "C" int llma_set_option(llma_ctx *c, int32_t option, int32_t value) {
    if (!c) return fail(nullptr, LLMA_E_INVAL, "llma_set_option: null context");
    switch (option) {
        case LLMA_OPT_ACT_SPLIT: drop_graphs(c); c->opt_split = value ? 1 : 0; return LLMA_OK;
        case LLMA_OPT_KERNEL_TIMING: c->opt_timing = value ? 1 : 0; return LLMA_OK;
        case LLMA_OPT_USE_GRAPH: c->opt_graph = value ? 1 : 0; return LLMA_OK;
        default: return fail(c, LLMA_E_INVAL, "llma_set_option: unknown option %d", option);
    }
}

extern "C" int llma_time_step_gemm(llma_ctx *c, int32_t which, int32_t rows, int32_t reps, double *mean_us) {
    if (!c || !mean_us) return fail(c, LLMA_E_INVAL, "llma_time_step_gemm: null argument");
    if (c->cfg.dtype != LLMA_DTYPE_BF16) return fail(c, LLMA_E_INVAL, "llma_time_step_gemm: bf16 models only");
    if (which < 0 || which > 4) return fail(c, LLMA_E_RANGE, "llma_time_step_gemm: matrix %d (0 QKV, 1 O, 2 gate/up, 3 down, 4 LM head)", which);
    if (rows < 1 || rows > c->cfg.max_batch * (c->cfg.max_k + 1) || reps < 1 || reps > 100000)
        return fail(c, LLMA_E_RANGE, "llma_time_step_gemm: rows %d (1..max_batch (max_k + 1) = %d) or reps %d (1..100000) out of range",
                    rows, c->cfg.max_batch * (c->cfg.max_k + 1), reps);
    const llma_model_cfg &g = c->cfg;
    HIP_TRY(c, hipStreamSynchronize(c->st));
    if (which == 0) {           // the QKV epilogue appends K and V at (row_slot, row_pos): slot 0, position 0 for every row
        HIP_TRY(c, hipMemsetAsync(c->s.row_pos, 0, sizeof(int32_t) * rows, c->st));
        HIP_TRY(c, hipMemsetAsync(c->s.row_slot, 0, sizeof(int32_t) * rows, c->st));
    }
    hipEvent_t e0, e1;
    HIP_TRY(c, hipEventCreate(&e0));
    HIP_TRY(c, hipEventCreate(&e1));
    for (int pass = 0; pass < 2; ++pass) {              // pass 0 warms up (first-launch set-up of the kernel)
        const int n = pass ? reps : (reps < g.n_layers ? reps : g.n_layers);
        HIP_TRY(c, hipEventRecord(e0, c->st));
        for (int r = 0; r < n; ++r) {
            GemmArgs ga = step_gemm_args(c, which, r % g.n_layers, rows);
            if (rows > 48) {                            // the step's own choice: panel kernel, split-K form
                if (ga.plan.n_split > 1) { ga.ksplit = ga.plan.n_split; ga.part = c->part; if (ga.epi != EPI_RESID) ga.rstd_out = c->rstd; }
                launch_gemm_panel_bf16(ga, c->st);
            } else if (!launch_gemm_bf16(ga, c->st)) {
                return fail(c, LLMA_E_RANGE, "llma_time_step_gemm: launch refused for %d rows", rows);
            }
        }
        HIP_TRY(c, hipEventRecord(e1, c->st));
        HIP_TRY(c, hipEventSynchronize(e1));
    }
    HIP_TRY(c, hipGetLastError());
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *mean_us = (double)ms * 1e3 / reps;
    return LLMA_OK;
}

extern "C" int llma_time_ffn_gemm(llma_ctx *c, int32_t rows, int32_t reps, double *mean_us) {
    if (rows > 48) return fail(c, LLMA_E_RANGE, "llma_time_ffn_gemm: rows %d outside 1..48", rows);
    return llma_time_step_gemm(c, 2, rows, reps, mean_us);
}

extern "C" int llma_get_kernel_timing(llma_ctx *c, int64_t *launches, double *total_ms) {
    if (!c || !launches || !total_ms) return fail(c, LLMA_E_INVAL, "llma_get_kernel_timing: null argument");
    HIP_TRY(c, hipStreamSynchronize(c->st));
    double tot = 0.0;
    for (auto &e : c->events) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, e.a, e.b));
        tot += ms;
        (void)hipEventDestroy(e.a);
        (void)hipEventDestroy(e.b);
    }
    *launches = (int64_t)c->events.size();
    *total_ms = tot;
    c->events.clear();
    return LLMA_OK;
}
