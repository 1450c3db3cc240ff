/* llma.h -- C ABI of the MI355X (gfx950) implementation of LLMA decoding
 * ("Inference with Reference: Lossless Acceleration of Large Language Models").
 *
 * The library runs greedy decoding of a LLaMA-style decoder (RMSNorm, RoPE, causal
 * attention over a KV cache, SwiGLU FFN, untied LM head) in which each decoding step
 * may verify k tokens copied from a reference document in ONE forward pass
 * (paper: Method, "LLMA: Inference with Reference", Eq. 3 and Algorithm 1).
 *
 * Conventions
 *  - Every function returns LLMA_OK (0) or a positive count on success and a negative
 *    LLMA_E_* code on failure; nothing throws or aborts across this boundary.  After a
 *    failure llma_last_error() gives a text.  Argument errors (INVAL/RANGE) are detected
 *    before any device work and leave the context unchanged.
 *  - "host" / "device" on a pointer says where the memory lives.  The caller owns every
 *    buffer it passes.  The library copies (and re-tiles) the weights in llma_create, so
 *    the caller may free its weight buffers once llma_create has returned.
 *  - Token ids are int32 in [0, vocab).  Sequence slots are 0 .. max_batch-1; each slot has
 *    its own KV cache of max_seq positions, its own length T and its own pending token
 *    (the last context token, emitted or given but not yet fed through the model).
 *  - All device work is enqueued on the hipStream_t given to llma_create.  Calls that
 *    return results through host pointers synchronise that stream before returning.
 *  - A context is not thread-safe: one call at a time.
 */
#ifndef LLMA_H
#define LLMA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LLMA_OK        0
#define LLMA_E_INVAL  (-1)   /* null pointer, bad enum, shape the kernels do not support  */
#define LLMA_E_RANGE  (-2)   /* k > max_k, cache overflow, token id outside [0,vocab) ... */
#define LLMA_E_NOMEM  (-3)   /* device or host allocation failed                         */
#define LLMA_E_HIP    (-4)   /* a HIP runtime call failed                                */
#define LLMA_E_STATE  (-5)   /* call not valid in the slot's current state (no pending token) */

#define LLMA_DTYPE_F32  0    /* fp32 weights, fp32 arithmetic, fp32 KV cache */
#define LLMA_DTYPE_BF16 1    /* bf16 weights and KV cache, bf16 MFMA with fp32 accumulation,
                                fp32 residual stream / softmax / logits */

typedef struct llma_ctx llma_ctx;           /* opaque; owns re-tiled weights, KV cache, scratch */

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int32_t max_seq;       /* KV positions per slot; a step with rows m needs T + m <= max_seq */
    int32_t max_batch;     /* number of sequence slots                                      */
    int32_t max_k;         /* largest copy length k accepted by the step functions (<= 32)  */
    int32_t dtype;         /* LLMA_DTYPE_*                                                  */
    int32_t kv_split;      /* bf16 only: 1 = keep K and V as a bf16 hi plane plus an 8-bit lo plane
                              (the residual x - hi as fp8 e4m3 of 256 times it: 1.5 x the cache
                              bytes, 12 significand bits), 0 = one bf16 plane.  Ignored for fp32 */
    float   rms_eps;       /* RMSNorm(x; g) = g * x / sqrt(mean(x^2) + rms_eps)              */
    float   rope_theta;    /* rotary base: feature i pairs with i + head_dim/2, angle
                              pos * rope_theta^(-2i/head_dim)                               */
} llma_model_cfg;
/* bf16 requires d_model % 32 == 0, d_ffn % 32 == 0, vocab % 16 == 0, head_dim in {64,128},
 * n_heads * head_dim == d_model.  fp32 requires head_dim in {32,64,128}. */

/* Weights: DEVICE pointers to row-major [out_features, in_features] matrices of the
 * configured dtype (bf16 = 16-bit patterns); gains are fp32 on the DEVICE.  The arrays of
 * per-layer pointers themselves live on the HOST (n_layers entries each).
 *   embed [vocab,d]  lm_head [vocab,d]  final_norm [d]
 *   wqkv [3d,d] (q rows, k rows, v rows; head h = rows h*head_dim..)   wo [d,d]
 *   wgu [2*d_ffn,d] (gate rows then up rows)   wdown [d,d_ffn]   norm1 [d]  norm2 [d] */
typedef struct {
    const void *embed, *lm_head;
    const float *final_norm;
    const void *const *wqkv, *const *wo, *const *wgu, *const *wdown;
    const float *const *norm1, *const *norm2;
} llma_weights;

/* One decoding step as LLMA executed it: rows fed through the model (1 + copied tokens),
 * tokens emitted (1 + accepted copies), and the trigger (document index and position of
 * the first copied token inside that document), doc = pos = -1 when nothing was copied.
 * (Paper: Algorithm 2 records (inputs, outputs) per step the same way.) */
typedef struct { int32_t rows_in, emitted, doc, pos; } llma_step_rec;

/* --- lifetime ------------------------------------------------------------------------ */
/* Builds a context on the current HIP device.  cfg, w: host structs.  hip_stream: a
 * hipStream_t (NULL = the default stream).  *out receives the context.  Errors: INVAL
 * (null / unsupported shape), NOMEM, HIP. */
int llma_create(const llma_model_cfg *cfg, const llma_weights *w, void *hip_stream, llma_ctx **out);
int llma_destroy(llma_ctx *ctx);
/* Text of the last error on this context (or of the last failed llma_create / stateless
 * call when ctx is NULL).  Never NULL; valid until the next call on the same thread. */
const char *llma_last_error(const llma_ctx *ctx);

/* --- sequence state ------------------------------------------------------------------ */
/* Empties slot `seq`: T = 0, no pending token. */
int llma_reset(llma_ctx *ctx, int32_t seq);
/* Prompt processing (paper: the x of LLM(x, y)).  prompt: HOST int32[len], len >= 1.
 * Feeds prompt[0..len-2] through the model on top of the slot's current cache (T += len-1)
 * and makes prompt[len-1] the pending token, so the next step's first output is the first
 * generated token y_0.  Errors: RANGE if T + len - 1 + 1 > max_seq or a token id is out of range. */
int llma_prefill(llma_ctx *ctx, int32_t seq, const int32_t *prompt, int32_t len);
/* Reads the slot's state into HOST ints (either pointer may be NULL). pending = -1 if none. */
int llma_get_state(llma_ctx *ctx, int32_t seq, int32_t *T, int32_t *pending);
/* KV truncate on request (the operation every step ends with, paper: the rows of rejected copies
 * are dropped): keeps the first new_len positions of slot `seq`, 0 <= new_len <= T, and leaves
 * the pending token as it is.  The dropped rows stay in memory and are overwritten by later
 * steps.  Used by the verify-step microbenchmark to return to the same cache length before every
 * timed step.  Errors: RANGE (new_len outside [0, T]). */
int llma_truncate(llma_ctx *ctx, int32_t seq, int32_t new_len);
/* Sets the pending token of a slot (HOST value), e.g. after llma_kv_import. */
int llma_set_pending(llma_ctx *ctx, int32_t seq, int32_t token);
/* Replaces layer `layer` of slot `seq`'s KV cache by caller data and sets T = len once the
 * last layer has been imported.  k, v: DEVICE pointers, plain layout [n_heads, len,
 * head_dim] in the configured dtype; keys are taken as already rotated.  Used to start
 * the verify-step microbenchmark from a given cache without running a prefill.  With
 * kv_split the imported values fill the hi planes exactly and the lo planes with zeros;
 * when all layers of a slot have been imported with one len (and nothing was computed on
 * the slot in between), batched steps do not read the lo planes below that position. */
int llma_kv_import(llma_ctx *ctx, int32_t seq, int32_t layer, const void *k, const void *v, int32_t len);

/* --- the three calls of the method ---------------------------------------------------- */
/* Trigger (paper: Method, the n-gram match step of Algorithm 1).  Stateless; all
 * pointers HOST; the scan itself runs on the current HIP device.
 *   y[0..y_len): output tokens generated so far.  ref: the documents' tokens, flat;
 *   doc_offsets int32[n_docs+1], non-decreasing, doc j = ref[doc_offsets[j] .. doc_offsets[j+1]).
 * A candidate is (doc, pos) with n <= pos < len(doc) and doc[pos-n..pos) == y[y_len-n..y_len):
 * the tail occurs inside ONE document and at least doc[pos] is left to copy.  Among
 * candidates the longest agreement between the text before pos and the end of y wins,
 * then the smallest doc, then the smallest pos.  Returns 1 and fills *doc_out, *pos_out;
 * returns 0 (outputs -1) when there is no candidate, y_len < n, or n_docs == 0;
 * INVAL for null pointers / n < 1 / decreasing offsets. */
int llma_find_trigger(const int32_t *y, int32_t y_len,
                      const int32_t *ref, const int32_t *doc_offsets, int32_t n_docs,
                      int32_t n, int32_t *doc_out, int32_t *pos_out);

/* The same scan for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  It calls no hipMalloc / hipFree / other
 * allocating routine and copies nothing between host and device: inputs and the result are
 * DEVICE memory of the caller, the work is enqueued on hip_stream (a hipStream_t, NULL = default
 * stream) and the call returns without synchronising.
 *   y_dev int32[y_len], ref_dev int32[ref_len], doc_offsets_dev int32[n_docs+1] as above;
 *   result_dev int32[3] receives (matched, doc, pos): (1, doc, pos), (0, -1, -1) when nothing
 *   matches, or (LLMA_E_INVAL, -1, -1) when the kernel finds that doc_offsets does not start at 0,
 *   decreases somewhere or does not end at ref_len (the host cannot read device memory to check).
 * The one buffer the scan needs beyond inputs and outputs (the document index of every reference
 * position) is a static device array of LLMA_TRIGGER_STATIC_MAX_REF ints (4 MiB) that every GPU
 * the library runs on holds until the process ends; ref_len beyond it returns LLMA_E_RANGE (use
 * llma_find_trigger).  All calls on one GPU share that array: calls that overlap in time on
 * the same GPU (different streams or threads) race and must be serialised by the caller; calls
 * one after the other on a stream are fine (every entry a call reads it has written first).
 * Returns LLMA_OK once the work is enqueued; INVAL (null pointer, negative count, n < 1), RANGE, HIP. */
#define LLMA_TRIGGER_STATIC_MAX_REF (1 << 20)
int llma_find_trigger_static(const int32_t *y_dev, int32_t y_len, const int32_t *ref_dev, int32_t ref_len,
                             const int32_t *doc_offsets_dev, int32_t n_docs, int32_t n,
                             int32_t *result_dev, void *hip_stream);

/* One verification step (paper: Eq. 3 and the draft-comparison loop of Algorithm 1) for slot `seq`.
 * draft: HOST int32[k], the copied tokens d_pos..d_pos+k-1; 0 <= k <= max_k; k = 0 is a
 * plain greedy step (Eq. 2).  The rows [pending, draft[0..k)] go through the model at
 * positions T..T+k in one causal forward, giving o_0..o_k (vocabulary arg max per row,
 * lowest id on exact ties).  a = the largest j <= k with o_i == draft[i] for all i < j.
 * Outputs (HOST, each may be NULL): *n_accepted = a; emitted[0..a] = o_0..o_a (capacity
 * k+1); *next_token = o_a.  Side effects: KV rows of the pending token and of the a
 * accepted drafts are kept, rows of rejected drafts are dropped (T += a+1), pending = o_a.
 * Errors: STATE (no pending token), RANGE (k > max_k, T + k + 1 > max_seq, bad token id). */
int llma_verify_step(llma_ctx *ctx, int32_t seq, const int32_t *draft, int32_t k,
                     int32_t *n_accepted, int32_t *next_token, int32_t *emitted);

/* The same step for n_seqs slots at once (one pass over the weights for all of them).
 * seqs: HOST int32[n_seqs], distinct slots; drafts: HOST int32[n_seqs*k]; outputs HOST
 * n_accepted[n_seqs], next_token[n_seqs], emitted[n_seqs*(k+1)] (any may be NULL). */
int llma_verify_step_batch(llma_ctx *ctx, int32_t n_seqs, const int32_t *seqs,
                           const int32_t *drafts, int32_t k,
                           int32_t *n_accepted, int32_t *next_token, int32_t *emitted);

/* LLMA decoding (paper: Algorithm 1) of exactly max_new tokens for slot `seq`: reset,
 * prefill, then steps; each step runs the trigger on the device against the reference
 * and feeds 1 + k_eff rows, k_eff = min(k, tokens left in the matched document, max_new -
 * generated - 1), or one row when nothing matches, fewer than n tokens were generated, or
 * k_eff = 0.  The reference is given separately from the prompt (it need not be part of
 * it).  All pointers HOST.  out_tokens: capacity max_new; *n_out receives max_new.
 * trace (may be NULL): capacity max_new records; *n_steps (may be NULL) receives the
 * number of steps.  Needs prompt_len + max_new + k <= max_seq.  n_docs may be 0 (plain
 * greedy).  Errors: INVAL, RANGE. */
int llma_generate(llma_ctx *ctx, int32_t seq, const int32_t *prompt, int32_t prompt_len,
                  const int32_t *ref, const int32_t *doc_offsets, int32_t n_docs,
                  int32_t n, int32_t k, int32_t max_new,
                  int32_t *out_tokens, int32_t *n_out,
                  llma_step_rec *trace, int32_t *n_steps);

/* The same decoding for n_seqs sequences at once (next step after the paper's batch-1
 * set-up; every sequence follows Algorithm 1 on its own prompt and its own reference, the
 * sequences share each pass over the weights).  Every step feeds k + 1 rows per sequence:
 * a sequence's trigger decides how many of them are drafts (its trace records 1 + k_eff), a
 * sequence that already has its max_new tokens idles.  All pointers HOST.
 *   seqs            int32[n_seqs], distinct slots (each is reset)
 *   prompts         the prompts back to back; prompt_offsets int32[n_seqs + 1], [0] = 0
 *   refs            the references back to back (may be NULL if all are empty)
 *   doc_offsets     the sequences' document-offset lists back to back, sequence b contributing
 *                   n_docs[b] + 1 entries that start at 0 (relative to its own reference); may be
 *                   NULL if n_docs is NULL or all zero
 *   n_docs          int32[n_seqs] (NULL = no references: plain greedy)
 *   out_tokens      int32[n_seqs * max_new], row b = sequence b; n_out int32[n_seqs]
 *   trace           n_seqs * max_new records, row b = sequence b (may be NULL); n_steps
 *                   int32[n_seqs] (may be NULL)
 * Needs n_seqs <= max_batch and prompt length + max_new + k <= max_seq for every sequence.
 * The tokens of a sequence are those the single-sequence call produces for it (bit for bit
 * while n_seqs * (k + 1) <= 48; larger steps run a different GEMM whose sums are taken in
 * another order, so a near-tie of two logits may then resolve differently).
 * Errors: INVAL, RANGE; on error before the first launch the context is unchanged. */
int llma_generate_batch(llma_ctx *ctx, int32_t n_seqs, const int32_t *seqs,
                        const int32_t *prompts, const int32_t *prompt_offsets,
                        const int32_t *refs, const int32_t *doc_offsets, const int32_t *n_docs,
                        int32_t n, int32_t k, int32_t max_new,
                        int32_t *out_tokens, int32_t *n_out,
                        llma_step_rec *trace, int32_t *n_steps);

/* --- inspection / measurement --------------------------------------------------------- */
/* When dev_buf != NULL every later forward also writes its rows' logits, fp32
 * [rows, vocab] row-major, to this DEVICE buffer (capacity_rows >= rows of the largest
 * step, else RANGE at step time).  NULL switches the dump off.  For parity tests. */
int llma_set_logits_dump(llma_ctx *ctx, float *dev_buf, int32_t capacity_rows);

#define LLMA_OPT_ACT_SPLIT   1  /* bf16 only: feed activations to the MFMA GEMMs as the sum of
                                   two bf16 numbers (hi + lo) -- doubles the (free, memory-bound)
                                   MFMA work, removes the activation rounding error. default 1 */
#define LLMA_OPT_KERNEL_TIMING 2 /* bracket every launch of the FFN gate/up GEMM (the kernel
                                   that streams the most bytes) with HIP events. default 0 */
#define LLMA_OPT_USE_GRAPH   3  /* replay captured HIP graphs for the per-step kernel sequence. default 1 */
int llma_set_option(llma_ctx *ctx, int32_t option, int32_t value);
/* Sums the event pairs recorded since the last call: *launches = number of gate/up GEMM
 * launches, *total_ms = their summed duration.  Synchronises the stream. */
int llma_get_kernel_timing(llma_ctx *ctx, int64_t *launches, double *total_ms);
/* Mean duration in microseconds of the FFN gate/up GEMM of a decoding step with `rows` rows
 * (1..48): `reps` launches back to back on the context's stream, cycling through the layers'
 * own matrices (so every launch streams its weights from HBM), one event pair around all of
 * them.  The activations are whatever the context's scratch holds; outputs go to scratch.
 * bf16 models only.  Synchronises the stream.  For the roofline figure of the benchmark. */
int llma_time_ffn_gemm(llma_ctx *ctx, int32_t rows, int32_t reps, double *mean_us);
/* The same measurement for any weight matrix of a layer and any step size the context admits:
 * which = 0 QKV, 1 attention output, 2 FFN gate/up, 3 FFN down, 4 LM head; rows = 1 ..
 * max_batch * (max_k + 1).  Launches what a step of that many rows launches for the matrix
 * (up to 48 rows the decoding GEMM, above that the panel GEMM in its split-K form together
 * with its finishing kernel).  which = 0 appends K / V rows to sequence slot 0 at position 0
 * and every call overwrites the context's activation scratch: llma_reset the context before
 * decoding with it again.  Synchronises the stream. */
int llma_time_step_gemm(llma_ctx *ctx, int32_t which, int32_t rows, int32_t reps, double *mean_us);
/* One line of text about what the context tuned at creation (the work division of the decoding
 * GEMMs, which llma_create picks by timing; it changes no result).  buf: HOST, cap bytes. */
int llma_describe(const llma_ctx *ctx, char *buf, int32_t cap);
/* Device bytes the context holds (weights, KV cache, scratch). */
int64_t llma_device_bytes(const llma_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* LLMA_H */
