/*
 * kvm.h -- C ABI of the Key-Value Means (KVM) attention layer hot path for AMD MI355X (gfx950).
 *
 * One KVM layer, as stated in the paper's Method section ("KVM Formulation"): every query runs
 * a single softmax over [compressed state rows || exact causal block sliding window]; after each
 * chunk the block that leaves the window is folded into the state (append the least redundant
 * tokens while the budget allows, merge the rest winner-take-all into running sums), and the
 * state is re-normalised just in time before it is read (LayerNorm on keys, stored radius on
 * values).
 *
 * Conventions
 *  - All pointers named q/k/v/gate/out/lse and every state buffer are DEVICE pointers owned by
 *    the caller; the library owns only the small host handle `kvm_state`.  Pointers inside
 *    `kvm_config` named ln_*, tau_* are DEVICE pointers too; `budget_table` is a HOST pointer
 *    that is copied at init.
 *  - Every call orders its work on the caller's stream (`void *stream` is a hipStream_t passed as
 *    a plain pointer so that this header needs no HIP header; NULL = the default stream) and
 *    returns without synchronising the host: work the caller enqueues on that stream afterwards
 *    sees all of it.  kvm_prefill_chunked and kvm_prefill_backward also use two streams the state
 *    owns (default priority, non-blocking, created at first use): part of their kernels runs there,
 *    forked from and joined back to the caller's stream by events inside the call.  Calls on one
 *    state must be issued in order on one stream (or be ordered by the caller).
 *  - Return value: KVM_OK (0) or a negative kvm_status.  Argument, state and capacity errors
 *    (KVM_ERR_ARG, KVM_ERR_STATE, KVM_ERR_CAPACITY, KVM_ERR_UNSUPPORTED, KVM_ERR_LIMIT) are detected
 *    before anything is enqueued: such a call leaves the state untouched.  KVM_ERR_HIP means a
 *    runtime call failed part-way: the streams are still joined back to the caller's, but the
 *    state's contents are undefined from then on (destroy it, or import a checkpoint).  The same
 *    code reports, on the next call on the state, that a fold kernel whose workgroups wait for
 *    each other (KVM_DEBUG_FOLD_SPLIT) ran into the time limit of such a wait.
 *  - q and k arrive already prepared (normalised, partially RoPE-rotated on the first
 *    `rope_dims` channels) as the paper states at the end of "KVM weight preparation"; the
 *    library needs `rope_dims` only to zero the rotary sub-space of memory keys.
 *  - Shapes: B batch, H_q query heads, H_kv key/value heads (H_q % H_kv == 0; a group of
 *    H_q/H_kv query heads shares one KV head's state, window, gate and LN_s), d = head_dim
 *    (64 or 128), C = chunk_len, L = n_bswa_chunks * C.  A "unit" is one (batch, KV head).
 *  - I/O dtype: KVM_F32 or KVM_BF16 for q, k, v, out, the memory keys and the normalised
 *    readout rows.  State key sums are fp64 (they feed the slot argmax, which has to be
 *    reproducible), value sums and radii fp32.
 */
#ifndef KVM_H
#define KVM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kvm_status {
  KVM_OK = 0,
  KVM_ERR_ARG = -1,         /* bad argument / unsupported shape                          */
  KVM_ERR_CAPACITY = -2,    /* the bound buffer cannot hold the rows the budget asks for */
  KVM_ERR_STATE = -3,       /* call not valid in the state's current position            */
  KVM_ERR_HIP = -4,         /* a HIP runtime call failed (see kvm_last_hip_error)        */
  KVM_ERR_UNSUPPORTED = -5, /* shape/dtype combination has no kernel                     */
  KVM_ERR_LIMIT = -6        /* beyond the fixed maximum of an allocation-free entry point */
} kvm_status;

enum { KVM_F32 = 0, KVM_BF16 = 1 };
enum { KVM_BUDGET_NONE = 0, KVM_BUDGET_FIXED = 1, KVM_BUDGET_SQRT = 2, KVM_BUDGET_TABLE = 3 };

/* Layer constants.  Budget B(e) ("We choose n_append as follows", Method section):
 *   NONE : no compressed state, the layer is pure block-sliding-window attention;
 *   FIXED: B(e) = budget_fixed;
 *   SQRT : B(e) = floor(budget_scale * ceil(sqrt(e)));
 *   TABLE: B(e) = budget_table[min(e / C - 1, len - 1)].
 * e is the end of the chunk that has just been attended. */
typedef struct kvm_config {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  int32_t rope_dims;       /* r: first r channels are rotary, zeroed in memory keys (eq. "memory key") */
  int32_t chunk_len;       /* C */
  int32_t n_bswa_chunks;   /* L = n_bswa_chunks * C ("Chunks and attention regions") */
  int32_t n_sink;          /* S: first S state rows are never merge targets ("Merge"); default 1 */
  int32_t io_dtype;        /* KVM_F32 | KVM_BF16 */
  int32_t budget_kind;
  int64_t budget_fixed;
  double budget_scale;
  const int64_t *budget_table; /* host */
  int64_t budget_table_len;
  float ln_eps;            /* LN_s epsilon; 0 selects 1e-5 */
  float norm_eps;          /* eps_norm of the value readout; 0 selects 1e-12 */
  const float *ln_gamma;   /* device [H_kv, d], 16-byte aligned, or NULL => 1 */
  const float *ln_beta;    /* device [H_kv, d], 16-byte aligned, or NULL => 0 */
  const float *tau_state;  /* device [H_q] or NULL => 1 ("Readout": per-head inverse temperatures) */
  const float *tau_bswa;   /* device [H_q] or NULL => 1 */
} kvm_config;

/* Element strides of the prefill operands; the head_dim axis is always contiguous.
 * NULL in kvm_prefill_chunked means dense [B, T, H, d] (and [B, T, H] for gate and lse). */
typedef struct kvm_strides {
  int64_t q_b, q_t, q_h;
  int64_t k_b, k_t, k_h;
  int64_t v_b, v_t, v_h;
  int64_t o_b, o_t, o_h;
  int64_t g_b, g_t, g_h;
  int64_t lse_b, lse_t, lse_h;
} kvm_strides;

typedef struct kvm_state kvm_state;

const char *kvm_strerror(int status);
/* Text of the last HIP error seen by this thread's library calls ("" if none). */
const char *kvm_last_hip_error(void);

/* Rows the state reaches after `max_tokens` tokens under the config's budget (integer replay of
 * M*(e) = max(m, min(B(e), m + C)); creation gives C).  Negative on bad config. */
int64_t kvm_state_rows_for(const kvm_config *cfg, int64_t max_tokens);

/* Bytes of device memory kvm_state_init needs to run up to `max_tokens` tokens: state sums,
 * radii, normalised readout rows, window ring and fold/decode scratch.  0 on bad config. */
size_t kvm_state_bytes(const kvm_config *cfg, int64_t max_tokens);

/* Bind an empty state (m = 0, no tokens seen) to caller memory `dev_buf` (256-byte aligned,
 * at least kvm_state_bytes(cfg, max_tokens) bytes).  Enqueues nothing.  The buffer must stay
 * alive until kvm_state_destroy; its contents need not be initialised.  What the buffer holds is
 * the layer's recurrent state as "Compressed State and BSWA Window" describes it -- the running
 * gated sums of memory keys and values and the stored radii of m rows, the last L tokens -- plus
 * the normalised readout rows of "Readout" and scratch; its row capacity follows the budget rule
 * ("We choose n_append as follows": M* = max(m, min(B(e), m + C))) replayed up to max_tokens. */
int kvm_state_init(kvm_state **out, const kvm_config *cfg, void *dev_buf, size_t bytes,
                   int64_t max_tokens);
int kvm_state_destroy(kvm_state *st);

/* Chunk-wise prefill of T more tokens (pseudocode appendix; "Chunks and attention regions").
 * The running token count must be a multiple of C on entry; T may end inside a chunk (that
 * chunk is completed by kvm_decode_step).  For each chunk: attention of its queries over the
 * current state and the window, then, if the chunk is complete and e >= L, the fold of block
 * [e - L, e - L + C).  Leaves the last L tokens in the state's window ring.
 *   q, out: [B, T, H_q, d]; k, v: [B, T, H_kv, d]; gate: [B, T, H_kv] fp32 merge gate g_t > 0
 *   or NULL (g = 1); lse: [B, T, H_q] fp32 natural-log sum of exponentials, or NULL.
 * KVM_ERR_CAPACITY if the budget over this call exceeds the bound buffer (nothing enqueued). */
int kvm_prefill_chunked(kvm_state *st, const void *q, const void *k, const void *v,
                        const float *gate, void *out, float *lse, int64_t T,
                        const kvm_strides *strides, void *stream);

/* One new token per sequence ("Readout" with a single query; "Chunks and attention regions": the
 * window is the current block so far plus the n_bswa_chunks - 1 blocks before it): append
 * (k, v, g) to the window, attend the query over state and window, and fold when this token
 * completes a chunk with e >= L.
 *   q, out: [B, H_q, d]; k, v: [B, H_kv, d]; gate: [B, H_kv] or NULL. */
int kvm_decode_step(kvm_state *st, const void *q, const void *k, const void *v,
                    const float *gate, void *out, void *stream);

/* One decode step over a ragged batch: the sequences of n_states states, each state at its own
 * position and with its own number of state rows (the "growth" budget makes rows a function of
 * the tokens seen; requests that joined at different times stand at different positions), in one
 * attention launch.  Per state the effect is that of kvm_decode_step; a state whose token
 * completes a chunk folds afterwards (its own launches).  All states must share one configuration
 * apart from batch and capacity (heads, head_dim, dtype, chunk, window, sinks, LN_s parameters,
 * temperatures: the first state's are used).
 *   q, out: [sum of batches, H_q, d]; k, v: [sum, H_kv, d]; gate: [sum, H_kv] or NULL; rows in
 *   the order of `states`, each state's sequences together.
 *   workspace: device memory, 16-byte aligned, kvm_decode_multi_workspace_bytes(sum of batches)
 *   bytes, owned by the caller; rewritten by every call (stream-ordered).
 * KVM_ERR_CAPACITY (nothing enqueued) if any state's fold would exceed its buffer; KVM_ERR_ARG on
 * mismatched configurations. */
size_t kvm_decode_multi_workspace_bytes(int64_t n_sequences);
int kvm_decode_step_multi(kvm_state *const *states, int32_t n_states, const void *q, const void *k,
                          const void *v, const float *gate, void *out, void *workspace,
                          size_t workspace_bytes, void *stream);

/* kvm_decode_step_multi for callers that cannot allocate or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus the
 * workspace, same effect, same results to the bit (the same attention and fold kernels run).  The
 * per-sequence descriptor table lives in a device array inside the library, fixed at
 * KVM_STATIC_MAX_SEQUENCES sequences per call (about 224 KiB on every GPU the library runs on,
 * held until the process ends); it is filled by a small kernel from values passed as kernel
 * arguments, so the call makes no hipMalloc / hipFree, no host-to-device copy and no host heap
 * allocation (with kvm_state_profile off).  More sequences than the maximum: KVM_ERR_LIMIT,
 * nothing enqueued (kvm_last_hip_error() says how many were asked for).  The table is rewritten
 * by every call: calls on one GPU must be ordered (one stream, or events); calls that overlap on
 * one GPU race on it. */
#define KVM_STATIC_MAX_SEQUENCES 4096
int kvm_decode_step_multi_static(kvm_state *const *states, int32_t n_states, const void *q, const void *k,
                                 const void *v, const float *gate, void *out, void *stream);

/* Fold one overflow block into the state ("Append" and "Merge"): memory keys, similarity to
 * the normalised state, append of the n_append least similar tokens, winner-take-all merge of
 * the rest into rows >= S of the updated state, refresh of the normalised readout rows.
 *   k_blk, v_blk: [B, n_tokens, H_kv, d]; gate_blk: [B, n_tokens, H_kv] or NULL;
 *   n_tokens must equal C; e = end of the chunk just attended (argument of the budget);
 *   assign_out: nullable int32 [B, H_kv, n_tokens], the row each token went to (an appended
 *   token gets its new row);  score_out: nullable fp32 [B, H_kv, n_tokens, 2] =
 *   (append score s_j of "Append", winning merge score max_i of "Merge"), NaN where not computed
 *   (the two numbers the backward pass needs to tell a row's creator from the tokens merged into it).
 * Used by the two calls above; exported for callers that keep their own window. */
int kvm_state_fold(kvm_state *st, const void *k_blk, const void *v_blk, const float *gate_blk,
                   int32_t n_tokens, int64_t e, int32_t *assign_out, float *score_out,
                   void *stream);

/* Backward pass of a whole-sequence prefill (the paper's "Speed Benchmarks" time a backward pass;
 * what it computes follows from the forward definition in "KVM Formulation" by the chain rule).
 * `st` must be the state that a kvm_prefill_chunked over exactly these T tokens, from an empty
 * state, has left -- in one call, or in several that each started on a chunk boundary, their
 * operands concatenated here (KVM_ERR_STATE when the token, fold or row counts disagree); it is
 * read, not changed.  Given dout, the
 * gradient of a scalar loss with respect to that call's out, the call writes the gradients with
 * respect to its q, k, v and gate and to the layer's LN_s parameters and temperatures.
 *   - Slot assignments are replayed as recorded: `assign` (int32 [folds, B, H_kv, C]) and `score`
 *     (fp32 [folds, B, H_kv, C, 2]) are the records that kvm_state_trace collected during the
 *     forward (the argmax is piecewise constant and gets no gradient; the append scores tell the
 *     token that created a row from tokens that merged into it in the same fold).  The roundings
 *     of the memory keys and readout rows to the I/O dtype are passed straight through.  A row's radius carries gradient to the value that created the row.
 *   - q, out, dout, dq: [B, T, H_q, d]; k, v, dk, dv: [B, T, H_kv, d] (I/O dtype, dense);
 *     gate (nullable: g = 1), dgate: [B, T, H_kv] fp32 (dgate is the gradient at g = 1 when gate is
 *     NULL; 0 for tokens that were never folded); lse: [B, T, H_q] fp32 as the forward wrote it;
 *     dgamma, dbeta: [H_kv, d] fp32; dtau_state, dtau_bswa: [H_q] fp32.  Every gradient is
 *     overwritten (sums over the batch for the parameters).  All device pointers, the caller's.
 *   - workspace: device, 256-byte aligned, kvm_backward_workspace_bytes(st, T) bytes; rewritten.
 * Work is enqueued on `stream`; the host is not blocked (with bf16 and head_dim 128 part of each
 * chunk's work runs on the state's own two streams, the ones a prefill's folds use, forked from
 * and joined to `stream` by events inside the call: later work on `stream` sees all of it).
 * Parameter gradients are summed with fp64 atomics (their last fp32 bit can differ from run to
 * run). */
typedef struct kvm_grads {
  void *dq, *dk, *dv;
  float *dgate, *dgamma, *dbeta, *dtau_state, *dtau_bswa;
} kvm_grads;
size_t kvm_backward_workspace_bytes(const kvm_state *st, int64_t T);
int kvm_prefill_backward(kvm_state *st, const void *q, const void *k, const void *v, const float *gate,
                         const void *out, const float *lse, const void *dout, const int32_t *assign,
                         const float *score, const kvm_grads *grads, int64_t T, void *workspace,
                         size_t workspace_bytes, void *stream);

/* Introspection (host values, no device work). */
int kvm_state_rows(const kvm_state *st, int64_t *m_out);          /* current m, same for all units */
int kvm_state_tokens(const kvm_state *st, int64_t *tokens_seen);
int kvm_state_capacity(const kvm_state *st, int64_t *rows_out);   /* rows the bound buffer holds */
int kvm_state_folds(const kvm_state *st, int64_t *folds_out);     /* folds done so far */
/* Which code path this state's folds take as things stand (its shape, the debug knobs):
 * 1 = a run of folds in one launch, one workgroup per unit; 2 = one kernel per fold step.
 * For reports (bench.py names the kernels it timed); both paths compute the same fold. */
int kvm_state_fold_path(const kvm_state *st, int64_t *path_out);

/* Record every later fold's assignments and scores: fold number f (0 = the creation fold of
 * this state, counted over its whole life) writes assign[f] as int32 [B, H_kv, C] and
 * score[f] as fp32 [B, H_kv, C, 2].  Folds beyond `max_folds` are not recorded.  NULLs stop it. */
int kvm_state_trace(kvm_state *st, int32_t *assign, float *score, int64_t max_folds);

/* Move the state into a larger buffer sized for `new_max_tokens` (growth scheduler: called
 * after KVM_ERR_CAPACITY; with a growing budget -- the power-law and saturating schedules of the
 * budget paragraph -- the rows a state needs are a function of the tokens it will see).  Copies
 * on `stream`; the old buffer may be freed once the stream has passed this point.  The capacity is
 * named by tokens, like kvm_state_bytes, so that caller and library size the buffer by one rule. */
int kvm_state_grow(kvm_state *st, void *new_buf, size_t new_bytes, int64_t new_max_tokens,
                   void *stream);

/* Copy the state out / in (checkpoint: the recurrent state of "Compressed State and BSWA Window"
 * is all a sequence carries from one chunk to the next).  Every pointer is nullable (skipped).
 * kvm_state_import trusts its counters: m rows, tokens_seen and folds (the number of folds done,
 * which numbers the records of kvm_state_trace) must be those of the exported state, or describe
 * a state the caller built (any m up to the capacity; tokens_seen then only has to make the next
 * fold fall where the caller wants it).  Key sums are fp64, as the library holds them.
 * Rows are dense:
 *   sK fp64 [B, H_kv, m, d], sV fp32 [B, H_kv, m, d], rho fp32 [B, H_kv, m],
 *   w fp32 [B, H_kv, m] (1 + merged gates), n int32 [B, H_kv, m] (tokens in the row),
 *   khat, vhat I/O dtype [B, H_kv, m, d] (normalised readout; export only),
 *   win_k, win_v I/O dtype [B, H_kv, L, d], win_g fp32 [B, H_kv, L]: ring, token p at p % L. */
int kvm_state_export(const kvm_state *st, double *sK, float *sV, float *rho, float *w,
                     int32_t *n, void *khat, void *vhat, void *win_k, void *win_v,
                     float *win_g, void *stream);
int kvm_state_import(kvm_state *st, const double *sK, const float *sV, const float *rho,
                     const float *w, const int32_t *n, const void *win_k, const void *win_v,
                     const float *win_g, int64_t m, int64_t tokens_seen, int64_t folds,
                     void *stream);

/* Choices the library normally makes by itself, forced for tests and comparisons (no passage of
 * the paper).  value 0 gives the choice back to the library.  Takes effect from the next call on.
 *   KVM_DEBUG_FOLD_PATH         1: a run of folds is one launch, one workgroup per unit (bf16,
 *                               head_dim 128, block lengths 64 * 2^k up to 1024), 2: one kernel
 *                               per fold step (the default)
 *   KVM_DEBUG_FOLD_WAVES        8 or 16: wavefronts of a fold workgroup on the one-launch path
 *   KVM_DEBUG_PREFILL_SCHEDULE  1: chunk by chunk on the caller's stream, folds in place,
 *                               2: folds ahead on the library's stream, attention in groups
 *   KVM_DEBUG_FOLD_CHAINS       1 or 2: fold chains side by side (kernel-per-step path)
 *   KVM_DEBUG_MERGE_COPY        1 / 2: token-centred merge with row copies on / off (same path)
 *   KVM_DEBUG_BACKWARD_PATH     1: attention adjoints on the vector ALU on every shape (it also
 *                               sizes kvm_backward_workspace_bytes: set it before asking)
 *   KVM_DEBUG_FOLD_SPLIT        1, 2, 4 or 8: workgroups that share a unit's state rows on the
 *                               one-launch path (ignored where the shape does not allow it) */
enum { KVM_DEBUG_FOLD_PATH = 0, KVM_DEBUG_FOLD_WAVES = 1, KVM_DEBUG_PREFILL_SCHEDULE = 2, KVM_DEBUG_FOLD_CHAINS = 3,
       KVM_DEBUG_MERGE_COPY = 4, KVM_DEBUG_BACKWARD_PATH = 5, KVM_DEBUG_FOLD_SPLIT = 6, KVM_DEBUG_KNOBS = 8 };
int kvm_debug_set(kvm_state *st, int knob, int value);

/* Kernel timing for benchmarks (no passage of the paper: a measurement aid).  While enabled,
 * every attention launch and every fold of this state is bracketed by HIP events recorded on
 * the call's stream.  kvm_state_profile_read waits for the recorded events, adds up the elapsed
 * milliseconds per class, returns them with the number of launches, and clears the record:
 *   ms[0], count[0]: prefill attention launches (one per chunk)
 *   ms[1], count[1]: folds (all kernels of one fold together)
 *   ms[2], count[2]: decode attention launches
 * enable = 2 additionally keeps the prefill's fold stream from overlapping its attention
 * launches, so that each kernel is timed alone (slower overall; for kernel rooflines). */
int kvm_state_profile(kvm_state *st, int enable);
int kvm_state_profile_read(kvm_state *st, double ms[3], int64_t count[3]);

/* ---- Attention weight preparation in front of the layer -------------------------------------
 * The paper's appendix "GPTAlpha-2 Attention weight preparation" (value residual, token shift,
 * LN_q / LN_k, rotary embedding on the first r channels) and the merge gate of the Method section
 * ("KVM weight preparation": g_t = 1 + ELU(x_t W_g)), applied to the "simple" q~, k~, v~ that the
 * input projections produced; its outputs are what kvm_prefill_chunked / kvm_decode_step take.
 *   v~ <- (1 - lambda) v~ + lambda v~first;  a_t = a~_t + alpha (a~_{t-1} - a~_t) for a in {q, k, v};
 *   q <- RoPE_r(LN_q(q)),  k <- RoPE_r(LN_k(k));  rotary pairs are channels (c, c + r/2),
 *   angle = position * base^(-2c/r).
 * All parameter arrays are device fp32, 16-byte aligned; NULL selects the neutral value (alpha = 0: no shift,
 * lambda = 0, gamma = 1, beta = 0).  rope_dims: 0, or an even number whose half is 8, 16, 32 or 64
 * channels (bf16) / 4 ... 64 (fp32).  d_model: width of x (a multiple of 8 for bf16, 4 for fp32). */
typedef struct kvm_prep_params {
  int32_t batch, n_q_heads, n_kv_heads, head_dim; /* d_h: 64 or 128 */
  int32_t rope_dims;                               /* r */
  int32_t io_dtype;                                /* KVM_F32 | KVM_BF16: q~, k~, v~, x and the outputs */
  int32_t d_model;                                 /* 0 when no gate is computed */
  float ln_eps;                                    /* 0 selects 1e-5 */
  double rope_base;                                /* 0 selects 10000 */
  const float *alpha_q;                            /* [H_q, d_h] */
  const float *alpha_k, *alpha_v, *lambda_v;       /* [H_kv, d_h] */
  const float *lnq_gamma, *lnq_beta;               /* [H_q, d_h] */
  const float *lnk_gamma, *lnk_beta;               /* [H_kv, d_h] */
  const float *w_gate;                             /* [d_model, H_kv] */
} kvm_prep_params;

/* Bytes of device scratch kvm_prepare_qkv needs for T tokens (the rotation table, and the merge
 * gate's weights split into two bf16 halves when the gate runs on the matrix cores); 0 on bad
 * arguments. */
size_t kvm_prepare_scratch_bytes(const kvm_prep_params *p, int64_t T);

/* Prepares T tokens at absolute positions pos0 .. pos0 + T - 1 for every sequence of the batch.
 *   q_raw [B, T, H_q, d_h], k_raw, v_raw [B, T, H_kv, d_h]: I/O dtype, contiguous, device;
 *   v_first: same shape as v_raw, or NULL (no value residual);
 *   x [B, T, d_model] I/O dtype, or NULL (no gate; then gate_out is not written);
 *   prev_q [B, H_q, d_h], prev_k, prev_v [B, H_kv, d_h]: the simple rows of the token before this
 *     call (prev_v after its own value residual), or NULL: the first token is then not shifted;
 *   q_out, k_out, v_out: shaped like the inputs, must not alias them; gate_out fp32 [B, T, H_kv];
 *   scratch: kvm_prepare_scratch_bytes(p, T) bytes, 16-byte aligned like every other pointer.
 * Work is enqueued on `stream`; the host is not blocked.  Buffers stay the caller's.
 * Errors: KVM_ERR_ARG (shapes, alignment, aliasing, missing gate arguments), KVM_ERR_HIP. */
int kvm_prepare_qkv(const kvm_prep_params *p, const void *q_raw, const void *k_raw, const void *v_raw,
                    const void *v_first, const void *x, const void *prev_q, const void *prev_k,
                    const void *prev_v, void *q_out, void *k_out, void *v_out, float *gate_out,
                    void *scratch, int64_t T, int64_t pos0, void *stream);

/* Measured peaks of the GPU, for rooflines (no passage of the paper: measurement aids).  Both
 * calls enqueue a microkernel on `stream`, wait for it (they block the host) and report its rate.
 *   kvm_measure_mfma_bf16_peak: 2048 workgroups x 4 waves issue `iters` x 4 independent
 *     32x32x16 bf16 matrix instructions on register operands; scratch: device, >= 4 bytes
 *     (never written in practice); *tflops (host) receives TFLOP/s.
 *   kvm_measure_copy_peak: copies `bytes` (a multiple of 16; src, dst device, 16-byte aligned,
 *     not overlapping) five times with 16-byte accesses; *gbs (host) receives GB/s counting
 *     bytes read plus bytes written.
 *   kvm_measure_read_peak: streams `bytes` of src five times without writing (scratch: device,
 *     >= 4 bytes, never written in practice); *gbs receives GB/s read: the yardstick for kernels
 *     that read far more than they write, such as the decode attention.
 * Errors: KVM_ERR_ARG for bad arguments, KVM_ERR_HIP when a runtime call fails. */
int kvm_measure_mfma_bf16_peak(int iters, void *scratch, double *tflops, void *stream);
int kvm_measure_copy_peak(const void *src, void *dst, size_t bytes, double *gbs, void *stream);
int kvm_measure_read_peak(const void *src, size_t bytes, void *scratch, double *gbs, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KVM_H */
