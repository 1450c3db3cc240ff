// Host-side launchers of the HIP kernels (each enqueues on the given stream and returns).
#pragma once
#include "common.h"

// ---- bf16 path (kernels_bf16.hip)
GemmPlan make_gemm_plan(int N, int K, int tiles_per_task);
bool tilek_ft_valid(const GemmPlan &p, int nt, int ft);     // can the decoding GEMM run ft feature tiles per workgroup at nt row tiles?
int tilek_ft_default(const GemmPlan &p, int nt);
void launch_pack_weight(const void *src, void *dst, int N, int K, int KSp, int rope_dh, int d, hipStream_t st);
void launch_kv_import_bf16(const void *k, const void *v, void *kh, void *kl, void *vh, void *vl, int H, int len, int dh,
                           int max_seq, hipStream_t st);
void launch_embed_prep_bf16(const void *embed, const int *row_tok, const float *gain, float *h, void *nx_hi, void *nx_lo,
                            float *ssq_out, int R, int d, int KSp, hipStream_t st);
bool launch_gemm_bf16(const GemmArgs &a, hipStream_t st);   // false (nothing launched) unless 1 <= rows <= 48
void launch_gemm_panel_bf16(const GemmArgs &a, hipStream_t st);
void launch_rstd_rows(const float *ssq, int ssq_tiles, float eps, float *rstd, int rows, hipStream_t st);
void launch_attn_bf16(const AttnArgs &a, hipStream_t st);

// ---- fp32 path (kernels_f32.hip)
void launch_kv_import_f32(const void *k, const void *v, void *kc, void *vc, int H, int len, int dh,
                          int max_seq, hipStream_t st);
void launch_gemm_f32(const GemmArgs &a, hipStream_t st);
void launch_attn_f32(const AttnArgs &a, hipStream_t st);

// ---- shared small kernels (kernels_misc.hip)
struct StepState {            // device pointers describing the rows of the step in flight
    int *row_tok, *row_pos, *row_slot;   // [R]
    float *row_cs;                       // [R][head_dim/2][2] (cos, sin) of each row's position
    int *T, *pending;                    // [max_batch]
    int *batch_slots;                    // [n_seqs]
    int *keff;                           // [n_seqs] drafts actually used per sequence
    int *draft;                          // [n_seqs][max_k]
    int *nacc, *next, *emit;             // results: [n_seqs], [n_seqs], [n_seqs][max_k+1]
    int *otok;                           // [R] arg max per row
};
struct GenState {             // device-resident state of llma_generate, one per sequence of the batch
    int *y; int *n_out; int *n_steps; int *trace;  // y[max_new], trace[max_new][4]
    int *cur;                            // [2] (doc, pos) of the trigger of the step in flight
    const int *ref; const int *doc_offsets; const int *ref_doc; int ref_len, n_docs;
    int n, k, max_new;
    const int *prompt;                   // device copy of the prompt (prefill)
};

// rows of a verify step: row (b, j) = pending[slot_b] (j = 0) or draft[b][j-1]; pos = T[slot_b] + j
void launch_setup_step_rows(const StepState &s, int n_seqs, int m, int max_k, const float *cs, int half, hipStream_t st);
// rows of a prefill chunk for one slot: tokens prompt[T[slot] - *base_dev + j], pos = T[slot] + j
void launch_setup_prefill_rows(const StepState &s, const int *prompt_dev, const int *base_dev, int m, int slot,
                               const float *cs, int half, hipStream_t st);
void launch_advance_T(const StepState &s, int slot, int by, hipStream_t st);
// fp32 path: h[r][:] = embed[row_tok[r]][:]
void launch_embed_f32(const float *embed, const int *row_tok, float *h, int R, int d, hipStream_t st);
// fp32 path: x = RMSNorm(h; g)
void launch_rmsnorm_f32(const float *h, const float *g, float eps, float *out, int R, int d, hipStream_t st);
// fp32 path: rotate q, k of every row at its position, write q, append k and v to the cache
void launch_rope_kv_f32(const float *qkv, const StepState &s, const float *cs_table, float *q_out, float *kc, float *vc,
                        int R, int H, int dh, int max_seq, hipStream_t st);
// final arg max over the per-row partials, then prefix accept + KV truncate + bookkeeping
void launch_argmax_accept(const float *pval, const int *pidx, int n_part, const StepState &s, int n_seqs, int m,
                          int max_k, int vocab, const GenState *gen /*device array [n_seqs] or null*/, hipStream_t st);
// trigger scan for each sequence being generated (gen_dev[b]); fills keff[b] / draft[b][:]
void launch_trigger(const GenState *gen_dev, const StepState &s, int n_seqs, int max_k, hipStream_t st);
// stateless trigger on device arrays (llma_find_trigger): result[0..2] = matched, doc, pos; with
// check_offsets the kernel itself validates doc_offsets and reports (-1, -1, -1) for a bad list
void launch_trigger_plain(const int *y, int y_len, const int *ref, const int *doc_offsets, const int *ref_doc,
                          int ref_len, int n_docs, int n, int *result, bool check_offsets, hipStream_t st);
void launch_fill_ref_doc(const int *doc_offsets, int n_docs, int *ref_doc, int ref_len, hipStream_t st);
