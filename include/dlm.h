/*
 * dlm.h - C ABI of the MI355X (gfx950) hot path of DepCap block-wise diffusion-LM decoding.
 *
 * The three calls of the method, in the paper's problem statement (Sec. 3, "Two decisions in
 * block-wise inference"):
 *   dlm_step         one denoising step: the masked-diffusion transformer predicts a distribution
 *                    for every position of the active span against a cached prefix, and the
 *                    per-position statistics of Sec. 4.2 / 4.3 are reduced over the vocabulary
 *   block_boundary   DepGA-Block: how far the next block extends (Sec. 4.2, Eq. 3-4)
 *   select_parallel  CAP-Decoding: which masked positions of the block are decoded now
 *                    (Sec. 4.3, Eq. 5-6, Alg. 1), and the token write of Eq. 2
 *
 * Conventions for every function:
 *   - returns DLM_OK (0) or a negative DLM_E* code; never throws, never aborts, never synchronises
 *     the stream; when an error is returned no device memory has been written and no kernel
 *     launched.  dlm_last_error() gives a thread-local message for the last failure.
 *   - "DEVICE" pointers are HIP device memory of the current device; "host" pointers are ordinary
 *     host memory that is read completely before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is enqueued
 *     on it; outputs are valid once the caller has synchronised it.
 *   - the caller owns every buffer it passes; the library owns what *_create allocated.
 *   - dtype: DLM_F32 = IEEE binary32, DLM_BF16 = bfloat16; accumulation is always fp32.  DLM_BF16 is what the caller's
 *     weights, embeddings and logits are stored as.  Inside a pass the matrix cores are fed IEEE half: the layer weights are
 *     converted once, by dlm_model_create (exactly, except that a weight below 2^-14 in magnitude keeps an absolute error of
 *     at most 2^-25), and the activations the GEMMs and the attention read are rounded to half (11 significant bits, values
 *     beyond +-65504 saturate) instead of bfloat16 (8 bits); the residual stream is fp32.
 */
#ifndef DLM_H
#define DLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { DLM_OK = 0, DLM_EINVAL = -1, DLM_ESHAPE = -2, DLM_ECAPACITY = -3, DLM_ENOMEM = -4, DLM_EHIP = -5 };
enum { DLM_F32 = 0, DLM_BF16 = 1 };

const char* dlm_last_error(void);

/* ---- model ------------------------------------------------------------------------------- */

/* Pre-norm transformer without causal mask: RMSNorm, rotary embedding on half-split pairs
 * (i, i + head_dim/2), grouped-query attention (query head h reads kv head h / (n_q/n_kv)),
 * SwiGLU feed-forward, untied LM head, no biases.  Requirements: head_dim in {32, 64, 128};
 * n_q_heads % n_kv_heads == 0; for DLM_BF16 every matrix dimension is a multiple of 32. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, mask_id, dtype;
  float rms_eps, rope_theta;
} dlm_config;

/* DEVICE pointers to row-major [out, in] matrices of the model dtype.  The per-layer members are
 * host arrays of n_layers DEVICE pointers.  wqkv rows: Q heads, then K heads, then V heads.
 * w_gate_up rows: the d_ffn gate rows, then the d_ffn up rows. */
typedef struct {
  const void* embed;              /* [vocab, d_model] */
  const void* const* wqkv;        /* [(n_q + 2 n_kv) * head_dim, d_model] */
  const void* const* wo;          /* [d_model, n_q * head_dim] */
  const void* const* w_gate_up;   /* [2 * d_ffn, d_model] */
  const void* const* w_down;      /* [d_model, d_ffn] */
  const void* const* norm1;       /* [d_model] */
  const void* const* norm2;       /* [d_model] */
  const void* final_norm;         /* [d_model] */
  const void* lm_head;            /* [vocab, d_model] */
} dlm_weights;

typedef struct dlm_model dlm_model;
typedef struct dlm_state dlm_state;

/* Copies the weights into library-owned device memory (bf16 matrices are re-tiled for the matrix
 * cores, in IEEE half, on `stream`).  The caller may release its own tensors once `stream` has been synchronised.
 * bf16 layer matrices are kept twice where the kernel that serves passes of up to 16 to 64 rows has a
 * layout of its own for them (what all workgroups read at the same step adjacent in memory): the
 * model then takes up to twice its layer weights (30 GB for an 8B model).  A copy that does not fit
 * is left out; the environment variable DLM_W_STEPS=0, read by this call, leaves them all out
 * (results are bit-identical either way: the same products are added in the same order).
 * Errors: DLM_EINVAL (null pointer, bad dtype), DLM_ESHAPE (unsupported dimensions), DLM_ENOMEM. */
int dlm_model_create(const dlm_config* cfg, const dlm_weights* w, void* stream, dlm_model** out);
void dlm_model_destroy(dlm_model* m);

/* Decode state for up to max_seqs independent sequences ("slots"): the prefix KV cache
 * [layer][slot][max_seq_len][n_kv*head_dim] (K after the rotary embedding), the retained
 * look-ahead logits p^prev of Sec. 4.2 (two buffers of max_lookahead rows per slot) and the
 * workspaces of one pass of up to max_rows packed rows.  All slots start empty (kv_len 0).
 * Errors: DLM_EINVAL, DLM_ECAPACITY (a size is not positive, max_seqs > 32), DLM_ENOMEM. */
int dlm_state_create(const dlm_model* m, int max_seqs, int max_seq_len, int max_rows, int max_lookahead,
                     dlm_state** out);
void dlm_state_destroy(dlm_state* s);
/* Forget a slot's cache and retained logits (host bookkeeping only). */
int dlm_state_reset(dlm_state* s, int slot);
/* Cached prefix length of a slot, or a negative error code. */
int dlm_state_kv_len(const dlm_state* s, int slot);

/* ---- dlm_step ------------------------------------------------------------------------------ */

/* One packed pass over n_seqs sequences; sequence b owns rows [row_offsets[b], row_offsets[b+1])
 * of every per-row array, which are the absolute positions span_start[b], span_start[b]+1, ...
 * Each row attends (bidirectionally) to the slot's cached prefix [0, kv_len) and to all rows of
 * its own span; span_start[b] must equal the slot's kv_len.  After the pass the first
 * commit_len[b] rows join the cache (Sec. 5.2: prefix KV cached per decoded block).
 * suffix_len[b] > 0 (dual cache, Sec. 5.2, Q2): the rows also attend to the suffix_len[b] positions right
 * after the span, with the keys and values an earlier pass over those positions left in the cache
 * (every pass writes the K and V of all its rows at their positions; only the committed ones count
 * as prefix).  They are not recomputed.
 *
 * Statistics (Sec. 4.2, 4.3; natural log; the mask token's probability is forced to 0 first;
 * argmax ties go to the lowest token id) are written for every row:
 *   max_logit, lse = log sum exp, conf = max_v p(v), argmax, entropy = H(p),
 *   kl = KL(p^curr || p^prev) (Eq. 3) on the kl_count[b] rows starting at relative row
 *   kl_first[b], where p^prev is the retained distribution of the same absolute position; 0 on
 *   all other rows.
 * The logits of the save_count[b] rows starting at relative row save_first[b] are retained as the
 * slot's new p^prev (replacing the old one after this pass has read it).
 * `tokens` is device memory the host cannot inspect: an id outside [0, vocab) is read as the nearest
 * valid id (clamped), never as an address outside the embedding table.
 *
 * Errors (nothing is launched): DLM_EINVAL (null pointer, n_seqs < 1, offsets not increasing, slot
 * out of range or repeated, span_start != kv_len, commit/kl/save ranges outside the span, a kl row
 * with no retained p^prev, a suffix beyond the positions an earlier pass has covered),
 * DLM_ECAPACITY (rows > max_rows, span beyond max_seq_len, save_count > max_lookahead, n_seqs >
 * max_seqs).  DLM_EHIP: the runtime refused a launch; the state's host bookkeeping is unchanged but
 * what the kernels that did run wrote (uncommitted cache rows, activations) is unspecified. */
typedef struct {
  int32_t n_seqs;
  const int32_t* slot;         /* host [n_seqs] state slot of each sequence (NULL: 0, 1, ...)      */
  const int32_t* row_offsets;  /* host [n_seqs+1]                                                  */
  const int32_t* span_start;   /* host [n_seqs]                                                    */
  const int32_t* commit_len;   /* host [n_seqs]                                                    */
  const int32_t* kl_first;     /* host [n_seqs] (NULL with kl_count: no KL rows)                   */
  const int32_t* kl_count;     /* host [n_seqs]                                                    */
  const int32_t* save_first;   /* host [n_seqs] (NULL with save_count: nothing retained)           */
  const int32_t* save_count;   /* host [n_seqs]                                                    */
  const int32_t* tok_start;    /* host [n_seqs] index into `tokens` of the span's first row        */
  const int32_t* suffix_len;   /* host [n_seqs] (NULL: 0) cached positions after the span to attend */
  const int32_t* tokens;       /* DEVICE token ids (mask_id on undecoded slots)                    */
  void* logits;                /* DEVICE out [rows, vocab], model dtype                            */
  float* max_logit;            /* DEVICE out [rows]                                                */
  float* lse;                  /* DEVICE out [rows]                                                */
  float* entropy;              /* DEVICE out [rows]                                                */
  float* kl;                   /* DEVICE out [rows]                                                */
  float* conf;                 /* DEVICE out [rows]                                                */
  int32_t* argmax;             /* DEVICE out [rows]                                                */
} dlm_step_desc;

int dlm_step(dlm_state* s, const dlm_step_desc* d, void* stream);

/* ---- block_boundary ------------------------------------------------------------------------ */

/* DepGA-Block (Sec. 4.2).  For sequence b the candidate window is the W_b = win_len[b] positions
 * after the frontier, stored at I[win_start[b] ...], H[win_start[b] ...] (the caller sizes it:
 * W = min(L_max, L_remain), 1 <= W_b <= 256); I = last-block influence (Eq. 3), H = entropy of
 * those positions (the kl and entropy outputs of dlm_step can be passed as they are).
 * Both signals are smoothed (centred moving average of radius smooth_radius, truncated at the
 * window edges) and normalised inside the window (norm_mode 0: by the window mean, 1: by the
 * window max, 2: min-max, 3: not at all), S_k = I~_k - lambda H~_k (Eq. 4), and
 *   rule 0: the block ends immediately before the first k with S_k < 0,
 *   rule 1: before the first k whose prefix sum S_0 + ... + S_k < 0 (the cumulative form, Sec. 4.4),
 * whole window if there is none; L is clipped to [l_min, W_b] (the window wins).  cold[b] != 0:
 * first block, L = min(l_min, W_b) and the signals are not read (cold may be NULL).
 * Outputs: L_out DEVICE [n_seqs]; S_out DEVICE, indexed like I (nullable); margin_out DEVICE [n_seqs]
 * (nullable) = the smallest |decision quantity| examined up to the crossing.
 * Errors: DLM_EINVAL (null, n_seqs < 1, lambda <= 0, l_min < 1, bad mode/rule, radius < 0),
 * DLM_ECAPACITY (W_b < 1 or > 256, n_seqs > 32). */
typedef struct {
  float lambda;
  int32_t l_min, smooth_radius, norm_mode, rule;
} dlm_boundary_params;

int block_boundary(const float* I, const float* H, const int32_t* win_start, const int32_t* win_len, const int32_t* cold,
                   int n_seqs, const dlm_boundary_params* p, int32_t* L_out, float* S_out,
                   float* margin_out, void* stream);

/* ---- select_parallel ----------------------------------------------------------------------- */

/* CAP-Decoding (Sec. 4.3, Alg. 1).  The block of sequence b is the block_len[b] <= 256 rows
 * starting at row row_start[b] of logits / lse / conf / argmax, and the same positions start at
 * tokens[tok_start[b]].  A row is eligible iff its token equals mask_id.
 *   mode 0: pool = eligible rows with conf >= tau_low (Eq. 5); i, j conflict iff
 *           (logit_i[y_j] - lse_i) + (logit_j[y_i] - lse_j) > gamma (Eq. 6); phase 1 takes every
 *           pooled row with conf >= tau_high and drops their conflicts; phase 2 walks the rest by
 *           descending conf (ties: lower row first), taking a row and dropping its conflicts;
 *           if nothing was taken, the most confident eligible row alone.
 *   mode 1: every eligible row with conf >= tau_high, else the most confident one (the
 *           confidence-threshold rule of Sec. 5.1);  mode 2: the most confident one only.
 * Outputs: selected_out DEVICE uint8 [same indexing as logits rows; only block rows written];
 * n_selected_out DEVICE [n_seqs]; if apply_tokens != 0, tokens[i] = argmax[i] for the selected
 * rows (Eq. 2); margin_out DEVICE [n_seqs] (nullable) = the smallest distance of an examined
 * quantity from the threshold or neighbour that decides it.  An argmax entry outside [0, vocab) is
 * clamped into it before it indexes the logits.
 * Errors: DLM_EINVAL (null, n_seqs < 1, bad dtype/mode, tau_high < tau_low in mode 0, vocab < 2),
 * DLM_ECAPACITY (block_len < 0 or > 256, n_seqs > 32). */
typedef struct {
  float tau_low, tau_high, gamma;
  int32_t mode;
} dlm_select_params;

int select_parallel(const void* logits, int vocab, int dtype, const float* lse, const float* conf,
                    const int32_t* argmax, int32_t* tokens, const int32_t* row_start,
                    const int32_t* tok_start, const int32_t* block_len, int n_seqs, int mask_id,
                    const dlm_select_params* p, int apply_tokens, uint8_t* selected_out,
                    int32_t* n_selected_out, float* margin_out, void* stream);

/* ---- components of dlm_step, exported for isolated tests and measurement --------------------- */

/* The vocabulary reduction of dlm_step on its own.  logits DEVICE [rows, vocab]; prev (nullable)
 * DEVICE [rows, vocab] of the same dtype gives kl per row (else kl = 0); prev_lse (nullable) DEVICE
 * [rows] fp32: the log-sum-exp of each prev row as an earlier call returned it in `lse` (dlm_step
 * keeps it with the retained logits); NULL: recomputed from prev in the same pass.  Same outputs and
 * definitions as dlm_step.  workspace: DEVICE scratch of at least dlm_vocab_stats_workspace(rows)
 * bytes.  Errors: DLM_EINVAL, DLM_ECAPACITY (rows < 1, workspace too small). */
size_t dlm_vocab_stats_workspace(int rows);
int dlm_vocab_stats(const void* logits, const void* prev, const float* prev_lse, int rows, int vocab, int dtype, int mask_id,
                    float* max_logit, float* lse, float* entropy, float* kl, float* conf,
                    int32_t* argmax, void* workspace, size_t workspace_bytes, void* stream);

/* dlm_vocab_stats for callers that cannot allocate or pass a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, outputs and definitions, but the partial states live in a
 * file-scope device array of the library (4 MiB per GPU the library runs on, held until the process ends), whose address
 * is resolved once per device (at the first dlm_model_create on that device, else at the first call).  No hipMalloc,
 * hipFree or other allocating call is made.  Limit: rows <= 4096 (DLM_ECAPACITY beyond; use dlm_vocab_stats there).
 * All calls on one GPU share the array: calls that overlap on one GPU (different streams, different threads) race;
 * calls on one stream are ordered and safe.  Errors: DLM_EINVAL, DLM_ECAPACITY, DLM_EHIP (address resolution failed). */
int dlm_vocab_stats_static(const void* logits, const void* prev, const float* prev_lse, int rows, int vocab, int dtype, int mask_id,
                           float* max_logit, float* lse, float* entropy, float* kl, float* conf, int32_t* argmax,
                           void* stream);

/* y[M, N] = x[M, K] * w[N, K]^T with fp32 accumulation; all row-major DEVICE, dtype for x, w and y.
 * A test helper around the GEMM kernels of dlm_step: for DLM_BF16 it allocates scratch, re-tiles x
 * and w (dlm_step keeps both tiled) and synchronises the stream before returning; K, N multiples
 * of 32.  Errors: DLM_EINVAL, DLM_ESHAPE, DLM_ENOMEM, DLM_EHIP. */
int dlm_gemm_nt(const void* x, const void* w, void* y, int M, int N, int K, int dtype, void* stream);

/* out[A, n_q, hd] = softmax(q k^T / sqrt(hd)) v without mask; q [A, n_q, hd], k and v [T, n_kv, hd],
 * all DEVICE row-major of `dtype`; the attention kernel of dlm_step on dense operands.
 * Errors: DLM_EINVAL, DLM_ESHAPE. */
int dlm_attention(const void* q, const void* k, const void* v, void* out, int A, int T, int n_q, int n_kv,
                  int head_dim, int dtype, void* stream);

/* ---- what the GPU achieves on the resources the rooflines are drawn against -------------------
 * For callers that report measurements (bench.py): kernels that do nothing but the one thing, timed
 * with events on `stream`, which is synchronised before the call returns.
 *
 * dlm_probe_hbm_read: streams `bytes` of DEVICE memory at src `reps` times (16-byte loads, every byte
 * once per repetition; use a buffer larger than the 256 MB memory-side cache) and reports the read
 * rate in GB/s.  dlm_probe_mfma: `reps` launches of independent 16x16x32 half-precision products out of
 * registers on every SIMD, on operands of pseudo-random values (what the chip sustains then is set by
 * its power limit, below the published rate, which constant operands reach), reports TFLOP/s.
 * Errors: DLM_EINVAL, DLM_ESHAPE (fewer than 16 MiB), DLM_ENOMEM, DLM_EHIP. */
int dlm_probe_hbm_read(const void* src, size_t bytes, int reps, double* gb_per_s, void* stream);
int dlm_probe_mfma(int reps, double* tflop_per_s, void* stream);

/* Where dlm_step takes the vocabulary statistics of a bf16 model's pass that compares no row with a
 * retained distribution and retains none (kl_count and save_count all zero: the in-block passes of
 * Sec. 4.3) and has at most 64 rows.  enable != 0 (the default of a new state): from the LM-head
 * GEMM's epilogue, which leaves one online-softmax state (maximum, sum of exponentials, their
 * logit-weighted sum, lowest token id of the maximum; Sec. 4.2 entropy, Sec. 4.3 confidence and
 * prediction) per row and column group, finished by a small merge: the logits are written but
 * not read back.  enable == 0: from the streamed reduction over the written logits, as every other
 * pass does.  Both take the logits as written (rounded to the model's dtype) and leave out the mask
 * token; their results differ only in the order of the fp32 sums.  Errors: DLM_EINVAL (null state). */
int dlm_state_fuse_stats(dlm_state* s, int enable);

/* Per-kernel-class timing of dlm_step: the launches of every class whose bit is set in class_mask
 * are bracketed by HIP events on the caller's stream (0 switches the timing off; events cost queue
 * time, so bracket few classes when a class's own duration matters).  dlm_profile_read synchronises
 * those events and returns, per class c < n, the accumulated milliseconds and launch count since the
 * last reset.  Classes: 0 QKV GEMM, 1 O GEMM, 2 gate/up GEMM, 3 down GEMM, 4 LM-head GEMM,
 * 5 attention, 6 vocabulary statistics, 7 other (row tables, embedding, and for fp32 models the
 * row-wise glue). */
int dlm_profile_enable(dlm_state* s, unsigned class_mask);
int dlm_profile_read(dlm_state* s, int n, double* ms_out, int64_t* launches_out, int reset);

#ifdef __cplusplus
}
#endif
#endif
