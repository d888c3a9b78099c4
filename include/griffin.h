/*
 * griffin.h -- C ABI of the MI355X (gfx950) library for GRIFFIN's feed-forward hot path
 * (arXiv 2404.01365): prompt-conditioned selection of FF neurons, compaction of the selected
 * weights, and generation through the pruned gated FF block.
 *
 * Conventions common to every entry point
 *   - Every data pointer is DEVICE memory owned by the caller unless its comment says HOST.
 *     The library never allocates, frees or synchronises; all work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream) and the call returns at once.
 *   - Arguments are validated on the host before any HIP call; a bad argument returns an error
 *     code and enqueues nothing.  A failed launch returns GRIFFIN_EHIP; griffin_last_hip_error()
 *     returns the HIP runtime's text for it.
 *   - Matrices are NEURON-MAJOR: Wg, W1 and W2 are each [n][d] with row stride `ld` elements,
 *     row j holding neuron j.  Wg and W1 are the paper's W_g and W_1 (D_FF x D, Section 3);
 *     W2 is the transpose of the paper's W_2 (D x D_FF), so that the "rows of W_1, W_g and
 *     columns of W_2" selected in Section 4.2 are the same row j of all three arrays.
 *   - dtype is the storage type of X, x, y and of all weights and biases (fp32 or bf16).
 *     Accumulation, activations, Z, the statistic s and the selection run in fp32.
 *   - d must be a multiple of 8; d, n <= 2^20; ld >= d and a multiple of 8 (16-byte rows).
 *   - A block may carry W2 a second time in the paper's own orientation (W2t, see griffin_layer).
 */
#ifndef GRIFFIN_H
#define GRIFFIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRIFFIN_OK = 0,
    GRIFFIN_EINVAL = 1,        /* null pointer, negative size, bad enum                     */
    GRIFFIN_ESHAPE = 2,        /* sizes inconsistent with each other or with the alignment  */
    GRIFFIN_EWORKSPACE = 3,    /* workspace missing or smaller than the *_workspace_bytes   */
    GRIFFIN_EUNSUPPORTED = 4,  /* valid request this build has no kernel for                */
    GRIFFIN_EHIP = 5           /* the HIP runtime refused a launch                          */
} griffin_status;

/* sigma of Eq. 2 / Eq. 3; the GLU variants named in Section 1 (SwiGLU, GEGLU, ReGLU). */
typedef enum { GRIFFIN_ACT_SILU = 0, GRIFFIN_ACT_GELU_TANH = 1, GRIFFIN_ACT_RELU = 2 } griffin_act;
typedef enum { GRIFFIN_F32 = 0, GRIFFIN_BF16 = 1 } griffin_dtype;

#define GRIFFIN_MAX_SEQS 256   /* sequences per griffin_prefill_select call      */
#define GRIFFIN_MAX_BATCH 64   /* rows per griffin_ff_decode* call               */

/*
 * One FF block (Section 3, Eq. 1-3), full (n = D_FF) or compressed (n = k, Eq. 4-5).
 * Wg == NULL selects the non-gated FF_1 of Eq. 2.  bg, b1 ([n]) and b2 ([d]) may be NULL;
 * b2 is never pruned (Eq. 5).
 */
typedef struct {
    int32_t d;        /* model width D                                  */
    int32_t n;        /* neurons held: D_FF for a full block, k for a compact one */
    int32_t dtype;    /* griffin_dtype */
    int32_t act;      /* griffin_act   */
    const void *Wg;   /* [n][d] stride ld, or NULL */
    const void *W1;   /* [n][d] stride ld */
    const void *W2;   /* [n][d] stride ld (transpose of the paper's W_2) */
    int64_t ld;       /* row stride of the three matrices, in elements */
    const void *bg;   /* [n] or NULL */
    const void *b1;   /* [n] or NULL */
    const void *b2;   /* [d] or NULL */
    const void *W2t;  /* optional second copy of W2, output-feature-major: [d][ldt], row c holding
                         W2[0..n-1][c] (this IS the paper's W_2, D x n) followed by zeros up to
                         ldt.  When a block has it, griffin_ff_decode streams it instead of W2 for
                         a single row (batch == 1), which lets every workgroup finish its own output
                         features (no partial rows); such a block may leave W2 NULL if it is only
                         ever used that way.  Every other route (batch > 1, griffin_ff_decode_multi,
                         the indexed calls, griffin_compact's source) reads the neuron-major W2 and
                         returns GRIFFIN_EUNSUPPORTED (GRIFFIN_EINVAL for griffin_compact) when it
                         is NULL.  griffin_compact fills W2t when the target block has it.  bf16
                         blocks with d a multiple of 512 only. */
    int64_t ldt;      /* row stride of W2t in elements: a multiple of 512, >= n; 0 without W2t */
} griffin_layer;

const char *griffin_status_string(int status);
const char *griffin_last_hip_error(void);   /* text of the last HIP failure on this thread */
const char *griffin_version(void);

/* k for "keep this fraction of D_FF" (Section 5 quotes FF sparsity = 1 - keep):
 * floor(keep * d_ff + 0.5) clamped to [1, d_ff]. */
int32_t griffin_k_from_fraction(int32_t d_ff, double keep);

/*
 * Prompt phase (Section 4.2, "Prompt Phase Expert Neuron Selection").
 * For n_seqs prompts packed row-wise in X, computes the FF activations Z = FF_1(X) (Eq. 3,
 * or Eq. 2 when L->Wg is NULL), scales every token row of Z to unit l2 norm (Section 4.1),
 * takes the l2 norm of every neuron's column over the tokens of each sequence (Eq. 6) and
 * returns, per sequence, the indices of the k largest entries of s.  Ties go to the lower
 * index; indices are ascending.  A token whose activations are all zero adds nothing to s.
 *
 *   X               [total_tokens][d], row stride ldx elements, L->dtype
 *   cu_seqlens_host HOST int32 [n_seqs+1]: cu[0] = 0, non-decreasing, cu[n_seqs] = total_tokens;
 *                   sequence b owns rows cu[b] .. cu[b+1]-1.  Read before the call returns.
 *   k               1 <= k <= L->n
 *   idx_out         [n_seqs][k] int32
 *   s_out           [n_seqs][L->n] fp32, or NULL
 *   Z_out           [total_tokens][L->n] fp32 with row stride ldz elements, or NULL (then Z
 *                   lives in the workspace).  Exposed because the prompt's own output uses the
 *                   full block (Section 5.1) and needs exactly this Z.
 *   workspace       at least griffin_prefill_workspace_bytes(L, total_tokens, n_seqs,
 *                   Z_out != NULL) bytes, 256-byte aligned
 * An empty sequence (length 0) selects indices 0 .. k-1 and reports s = 0.
 */
size_t griffin_prefill_workspace_bytes(const griffin_layer *L, int64_t total_tokens,
                                       int32_t n_seqs, int32_t have_z_out);
int griffin_prefill_select(const griffin_layer *L, const void *X, int64_t ldx,
                           const int32_t *cu_seqlens_host, int32_t n_seqs, int32_t k,
                           int32_t *idx_out, float *s_out, float *Z_out, int64_t ldz,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * Top-k of an arbitrary non-negative score (the selection step of Section 4.2 on its own;
 * also serves the shared-set statistic of Eq. 7 and static scores).
 *   scores [n_rows][n] fp32, all >= 0 and finite;  idx_out [n_rows][k] int32 ascending.
 */
int griffin_topk(const float *scores, int32_t n_rows, int32_t n, int32_t k, int32_t *idx_out,
                 void *stream);

/*
 * Shared selection for a batch (Section 5.3, Eq. 7): s_bar = sum_b s_b / sqrt(S_b).
 *   s [n_seqs][n] fp32 as written by griffin_prefill_select; cu_seqlens_host as above (HOST);
 *   sbar_out [n] fp32.  Sequences of length 0 are skipped.
 */
int griffin_stat_shared(const float *s, const int32_t *cu_seqlens_host, int32_t n_seqs,
                        int32_t n, float *sbar_out, void *stream);

/*
 * Static selector of the paper's magnitude baseline (Section 5.1, "Setup"): one score per neuron
 * from the weights alone, ||W1_j||_2, times ||Wg_j||_2 for GLU blocks (the paper names no norm;
 * l2 is taken).  score_out [L->n] fp32; feed it to griffin_topk.  The prompt still uses the
 * full block.
 */
int griffin_weight_norm_score(const griffin_layer *L, float *score_out, void *stream);

/*
 * Sampling-based selection (Appendix B): k_top experts by top-k of s, the other k - k_top drawn
 * from the remaining neurons without replacement with probability proportional to s_j
 * (k_top = 0: "sampling"; k_top = k/2: "top-k + sampling"; k_top = k: plain top-k).  The draw is
 * the exponential-clocks form of weighted sampling without replacement: neuron j rings at
 * e_j / s_j and the earliest rings win, decided on q_j = s_j / e_j, largest first, ties to the
 * lower index; a zero weight never beats a positive one.  The device forms q_j in single precision
 * (values above 1e38 count as 1e38), so two neurons whose quotients differ by less than a few
 * units of 1e-7 relative may swap against an exact evaluation.
 *   s [n] fp32 >= 0 (the statistic of Eq. 6, or s_bar of Eq. 7)
 *   e [n] fp32 > 0: one unit-rate exponential variate per neuron, drawn by the caller (the
 *     library draws no random numbers)
 *   idx_out [k] int32 ascending
 *   workspace griffin_select_sampled_workspace_bytes(n, k_top) bytes, 256-byte aligned
 */
size_t griffin_select_sampled_workspace_bytes(int32_t n, int32_t k_top);
int griffin_select_sampled(const float *s, const float *e, int32_t n, int32_t k, int32_t k_top,
                           int32_t *idx_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Jaccard similarity of selected sets (Section 4.1): out[a][b] = |E_a n E_b| / |E_a u E_b| for
 * every pair of the n_sets ascending index lists idx [n_sets][k] (as written by
 * griffin_prefill_select).  out [n_sets][n_sets] fp32; n_sets <= GRIFFIN_MAX_SEQS.
 */
int griffin_jaccard(const int32_t *idx, int32_t n_sets, int32_t k, float *out, void *stream);

/*
 * Compaction (Section 4.2; Eq. 4-5): C->Wg/W1/W2 row t <- L row idx[t], C->bg/b1 entry t <-
 * L entry idx[t]; b2 is not touched (the caller passes L->b2 as C->b2).  If C->W2t is given,
 * C->W2t[c][t] <- L->W2[idx[t]][c] as well (columns k .. C->ldt-1 are zeroed), and C->W2 may be
 * NULL; L->W2 is always the source.  C describes
 * caller-allocated device buffers: C->n == k, C->d == L->d, same dtype and act, C->ld >= d.
 * A matrix or bias that is NULL in L must be NULL in C.  idx [k] int32 device, each in
 * [0, L->n); the kernel clamps out-of-range entries instead of faulting.
 */
int griffin_compact(const griffin_layer *L, const int32_t *idx, int32_t k,
                    const griffin_layer *C, void *stream);

/*
 * Generation phase (Section 4.2, "Generation with Expert Neurons"; Eq. 4-5):
 *   z = sigma(Wg x + bg) * (W1 x + b1),   y = sum_j z_j W2[j][:] + b2
 * for `batch` independent rows x[b] through the ONE block C (a compact block, or a full one
 * with n = D_FF, which is Eq. 1).  x, y: [batch][d] contiguous, C->dtype.  With batch > 1 the
 * rows share one selected set (Section 5.3, Eq. 7) and the weights are streamed once per
 * four rows; five rows and more of a bf16 block with d a multiple of 512 up to 5120 take the
 * matrix cores and stream them once per sixteen rows.
 * workspace >= griffin_decode_workspace_bytes(d, n, batch) bytes, 256-byte aligned.
 */
size_t griffin_decode_workspace_bytes(int32_t d, int32_t n, int32_t batch);
int griffin_ff_decode(const griffin_layer *C, const void *x, void *y, int32_t batch,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * griffin_ff_decode for callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit for bit the same y as griffin_ff_decode, but the partial rows live
 * in a device array inside the library (8 MiB per GPU, held from the first call on that GPU until the
 * process ends) instead of a caller workspace.  The call allocates and frees nothing.
 *   - A request whose griffin_decode_workspace_bytes(C->d, C->n, batch) exceeds
 *     griffin_ff_decode_static_max_bytes() (8 MiB: one row at any width the library decodes, i.e.
 *     d <= 8192; two rows up to d = 4096) returns GRIFFIN_EWORKSPACE and enqueues nothing.
 *   - The current device must be the one `stream` belongs to (as for every entry point); the first
 *     call on a device looks the array's address up (GRIFFIN_EHIP if the runtime refuses).
 *   - All calls on one GPU share the array: calls on different streams of one GPU that may overlap
 *     race on it.  Calls on one stream are ordered and need nothing between them; the array needs
 *     no clearing (every word that is read was written by the same call).
 */
size_t griffin_ff_decode_static_max_bytes(void);
int griffin_ff_decode_static(const griffin_layer *C, const void *x, void *y, int32_t batch, void *stream);

/*
 * Per-sequence expert sets (every sample picks its own neurons, Section 4.2): row b of x goes
 * through its own compact block Cs[b].  Cs is a HOST array of `batch` HOST structs that must
 * agree in d, n, dtype, act, ld and in which optional pointers are NULL.
 */
int griffin_ff_decode_multi(const griffin_layer *Cs, int32_t batch, const void *x, void *y,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same without compact copies: row b uses neurons idx[b][0..k-1] (distinct) of the full block
 * L, read in place.  idx [batch][k] int32 device (out-of-range entries are clamped).
 * With a workspace of griffin_decode_workspace_bytes(d, L->n, batch) bytes (sized for the whole
 * block rather than for k neurons) five rows and more take ONE pass over the whole block, every row
 * dropping the neurons outside its own set: the sets of a batch cover most of the block between them,
 * so this moves far fewer bytes than a pass per row (bf16, d a multiple of 512 up to 5120).
 */
int griffin_ff_decode_indexed(const griffin_layer *L, const int32_t *idx, int32_t k,
                              int32_t batch, const void *x, void *y, void *workspace,
                              size_t workspace_bytes, void *stream);

/*
 * griffin_ff_decode_indexed for callers that decode many tokens with the same sets (Section 4.2: the
 * expert neurons are chosen at the prompt and kept for the whole generation phase).  The one-pass
 * route needs, per neuron, the rows of the batch that selected it; griffin_ff_decode_indexed derives
 * those membership words from idx at every call, here the caller builds them once:
 *   sets   griffin_index_sets_bytes(L->n, batch) bytes, device, 4-byte aligned: [ceil(batch/16)][L->n]
 *          uint32, bit b of word j of group g set iff row 16 g + b holds neuron j; written by
 *          griffin_index_sets_build(idx, k, batch, L->n, ...), valid as long as idx does not change.
 * griffin_ff_decode_indexed_sets takes the same idx as well: when the one-pass route does not apply
 * (fewer than five rows, a workspace sized for k neurons only, a shape it does not cover) the rows
 * go through the index lists exactly as in griffin_ff_decode_indexed and sets is not read.
 */
size_t griffin_index_sets_bytes(int32_t n, int32_t batch);
int griffin_index_sets_build(const int32_t *idx, int32_t k, int32_t batch, int32_t n, void *sets,
                             size_t sets_bytes, void *stream);
int griffin_ff_decode_indexed_sets(const griffin_layer *L, const int32_t *idx, int32_t k, const void *sets,
                                   int32_t batch, const void *x, void *y, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * The prompt's own output (Section 5.1: the prompt phase uses the full FF block; Eq. 1):
 *   Y = Z W_2^T + b_2  for the activations Z written by griffin_prefill_select (Z_out).
 *   Z    [total_tokens][d_ff] fp32, row stride ldz elements
 *   W2p  the paper's W_2, [d][d_ff] (row c = output feature c), row stride ldw elements, in
 *        `dtype`; this is the transpose of the neuron-major W2 of griffin_layer
 *   b2   [d] in `dtype`, or NULL
 *   Y    [total_tokens][d] in `dtype`, row stride ldy elements
 *   workspace  griffin_prompt_out_workspace_bytes(total_tokens, d_ff, d) bytes, 16-byte aligned
 *        (fp32 partial sums when the long contraction over d_ff is cut into ranges; may be 0)
 * bf16 blocks with d_ff a multiple of 8 and d a multiple of 4 run on the matrix cores (Z is
 * rounded to bf16 on the way); other shapes take a plain fp32 path (total_tokens <= 2^18).
 */
size_t griffin_prompt_out_workspace_bytes(int64_t total_tokens, int32_t d_ff, int32_t d);
int griffin_ff_prompt_out(const float *Z, int64_t ldz, int64_t total_tokens, int32_t d_ff, int32_t d,
                          int32_t dtype, const void *W2p, int64_t ldw, const void *b2, void *Y,
                          int64_t ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The whole prompt phase of one FF block in one call (Section 4.2 and Section 5.1): Z = FF_1(X)
 * is formed once and serves both the selection of the expert neurons (as griffin_prefill_select:
 * Section 4.1, Eq. 6, top-k per sequence) and the prompt's own output through the FULL block
 * (as griffin_ff_prompt_out: Y = Z W_2^T + b_2, Eq. 1).  Same results as the two calls one after
 * the other; on the matrix-core path the bf16 copy of Z that the second product reads is written
 * by the first product's own epilogue instead of by a pass over Z.
 *   L, X, ldx, cu_seqlens_host, n_seqs, k, idx_out, s_out   as in griffin_prefill_select
 *   W2p, ldw        the paper's W_2, [d][L->n] (row c = output feature c), in L->dtype, row stride
 *                   ldw elements; L->b2 is added when it is not NULL
 *   Y, ldy          [total_tokens][d] in L->dtype, row stride ldy elements
 *   workspace       griffin_prompt_phase_workspace_bytes(L, total_tokens, n_seqs) bytes, 256-byte
 *                   aligned; Z lives there (fp32 [total_tokens][L->n]) and is not returned
 */
size_t griffin_prompt_phase_workspace_bytes(const griffin_layer *L, int64_t total_tokens, int32_t n_seqs);
int griffin_prompt_phase(const griffin_layer *L, const void *W2p, int64_t ldw, const void *X, int64_t ldx,
                         const int32_t *cu_seqlens_host, int32_t n_seqs, int32_t k,
                         int32_t *idx_out, float *s_out, void *Y, int64_t ldy,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * MEASUREMENT ONLY -- not part of the method's interface and the one entry point that keeps state
 * between calls (a one-shot, per-thread note of three event handles; every other entry point is
 * stateless, apart from addresses and kernel attributes looked up once per device).  It exists so that a benchmark can time the kernels of a decode call on the stream
 * they run on (the generation phase is where the time goes, Section 5.2):
 * the next griffin_ff_decode* call made by this thread records, on that call's stream,
 * event_begin just before its weight-streaming kernel, event_mid between that kernel and the
 * small kernel that sums the partial rows, and event_end after the latter; then it forgets
 * them.  All are hipEvent_t created by the caller with timing enabled; any may be NULL.
 */
int griffin_trace_next_decode(void *event_begin, void *event_mid, void *event_end);

#ifdef __cplusplus
}
#endif
#endif /* GRIFFIN_H */
