// Internal declarations shared by the host side of the KVM library and its HIP kernels.
// Nothing here is part of the public ABI (see include/kvm.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvm {

// A strided source of per-token keys, values and merge gates for all units.
// Element strides; the head_dim axis is contiguous.  Token index 0 is `k`'s first token.
struct Src {
  const void *k, *v;
  const float *g;  // nullable: g = 1
  int64_t k_b, k_h, k_t;
  int64_t v_b, v_h, v_t;
  int64_t g_b, g_h, g_t;
};

// Device views of one bound state.  U = B * H_kv units; rows are padded to Mcap.
struct Dev {
  // state proper
  double *sK;    // [U, Mcap, d] running gated sums of memory keys (fp64: feeds the argmax)
  float *sV;     // [U, Mcap, d] running gated sums of values
  float *rho;    // [U, Mcap]    radius stored at row creation
  float *w;      // [U, Mcap]    1 + sum of merged gates (diagnostic)
  int32_t *n;    // [U, Mcap]    tokens in the row (diagnostic)
  // Normalised readout, one copy ("slot") per recent state version: version v (= number of
  // folds done) lives in slot v % NS.  A fold reads the old version and writes the new one in
  // full, so attention over earlier chunks can still be running on the old slots.
  void *khat;    // [NS, U, Mcap, d] I/O dtype: LN_s(sK)
  void *vhat;    // [NS, U, Mcap, d] I/O dtype: rho * sV / max(||sV||, eps)
  int64_t slot_elems;  // U * Mcap * d
  int32_t NS;
  // window ring: token p lives in slot p % L
  void *winK, *winV;  // [U, L, d] I/O dtype
  float *winG;        // [U, L]
  // fold scratch, per overflow token
  void *kbar;        // [U, C, d] I/O dtype memory keys (the host points this at one of the
                     //           `group` blocks that a batched memkey launch fills)
  float2 *score;     // [U, C]    x = append score s_j, y = winning merge score
  int32_t *pi;       // [U, C]    row the token goes to
  int32_t *app;      // [U, C]    rank among appended tokens, or -1
  int32_t *creator;  // [U, C]    token that creates new row number a
  // parameters
  const float *gamma, *beta;          // [H_kv, d] or null
  const float *tau_state, *tau_bswa;  // [H_q] or null
  int32_t B, Hq, Hkv, U, d, r, C, L, S, Mcap;
  int32_t Ufull;  // units of the whole state (a view of part of the batch keeps the state's strides)
  float ln_eps, norm_eps;
  int32_t io;  // KVM_F32 / KVM_BF16
};


// One attention launch: the queries of up to kMaxGroup consecutive chunks (prefill), or one
// query per sequence (decode).  Chunk boundaries are absolute multiples of C.
constexpr int kMaxGroup = 16;
struct AttnArgs {
  const void *q;
  void *out;
  float *lse;  // nullable
  int64_t q_b, q_t, q_h, o_b, o_t, o_h, lse_b, lse_t, lse_h;  // q/out/lse index 0 = position s
  Src in;            // keys/values of this call: token index 0 = position t0
  int64_t t0;        // positions below t0 come from the ring
  int64_t s;         // position of the first query of the launch
  int32_t n_chunks;  // chunks covered
  int32_t nq_total;  // queries covered (all chunks but the last are full)
  int32_t put_token = 0;  // decode (rows kernel): also store the token at position s into the ring
  int32_t m[kMaxGroup];     // state rows each chunk sees
  int32_t slot[kMaxGroup];  // readout slot of that state version
};

// fold.hip
hipError_t launch_memkey(const Dev &dv, const Src &src, int n_blocks, hipStream_t st);
hipError_t launch_score(const Dev &dv, int slot, int row0, int row1, bool first_pass, hipStream_t st);
hipError_t launch_select(const Dev &dv, int m, int n_app, bool take_all, hipStream_t st);
hipError_t launch_accum(const Dev &dv, const Src &src, int m_before, int m_after, int row_begin,
                        bool do_create, bool do_merge, bool do_copy, bool check_app, int slot_old,
                        int slot_new, hipStream_t st);
// selection + creation + second scoring pass of a small append, one launch
bool append_fits(const Dev &dv, int n_app);
hipError_t launch_append(const Dev &dv, const Src &src, int m, int n_app, int slot_new, hipStream_t st);
// the merge of a small fold in a prefill: token-centred merge into slot_new + copies of untouched rows
hipError_t launch_merge_copy(const Dev &dv, const Src &src, bool check_app, int slot_old, int slot_new,
                             int m_before, hipStream_t st);
hipError_t launch_merge_inplace(const Dev &dv, const Src &src, bool check_app, int slot, hipStream_t st);
hipError_t launch_refresh(const Dev &dv, int m, int slot, hipStream_t st);
hipError_t launch_ring_copy(const Dev &dv, const Src &src, int64_t src_t0, int64_t p0, int64_t p1,
                            hipStream_t st);
// fold_fused.hip (bf16, d = 128): a run of up to kFoldMaxSteps consecutive folds in one launch,
// one workgroup per unit.  Step i folds the block whose first token is src's token s[i].tok and
// whose memory keys are in slab s[i].kbar_block of the scratch (launch_memkey), from s[i].m to
// s[i].m_after rows, reading readout slot s[i].so and writing slot s[i].sn (the same slot when
// in_place; otherwise untouched rows are copied over).  trace >= 0: the fold's assignments and
// scores also go to trace_assign / trace_score at that fold index (trace_stride = tokens of one
// fold over all units).  narrow: the 8-wave workgroup that fits beside an attention workgroup on
// a compute unit; otherwise 16 waves and the unit to itself.
constexpr int kFoldMaxSteps = 8;
constexpr int kFoldMaxSplit = 8;   // workgroups that may share a unit's rows
struct FoldStep {
  int32_t m, m_after, so, sn;
  int64_t tok;
  int32_t trace, kbar_block;
  uint32_t xnum, pad;   // number of the fold's first exchange among the unit's workgroups (split > 1)
};
struct FoldRunArgs {
  int32_t n, in_place;
  FoldStep s[kFoldMaxSteps];
  int32_t *trace_assign;
  float *trace_score;
  int64_t trace_stride;
  int32_t split;               // workgroups per unit (a power of two); 1: none of the next two is used
  unsigned long long *xtab;    // the exchange table, fold_exchange_bytes() of zeroed device memory
  int32_t *err;                // set to 1 when a wait for a sibling workgroup ran into its time limit
};
bool fold_fused_fits(const Dev &dv, int split = 1);
size_t fold_exchange_bytes(const Dev &dv, int split);
// readout rows [0, m) recomputed from the sums with the one-launch path's arithmetic
hipError_t launch_refresh16(const Dev &dv, int m, int slot, hipStream_t st);
hipError_t launch_fold_fused(const Dev &dv, const Src &src, const FoldRunArgs &run, bool narrow, hipStream_t st);
// score_mfma.hip (bf16, d = 128)
hipError_t launch_score_mfma(const Dev &dv, int slot, int row0, int row1, bool first_pass, hipStream_t st);
// attn_rows.hip
hipError_t launch_attn_rows(const Dev &dv, const AttnArgs &a, hipStream_t st);
// One decode step over sequences of several states (kvm_decode_step_multi): per sequence, where
// its arrays start (its first KV head) and where it stands.
struct SeqDesc {
  const void *khat, *vhat;  // current readout version, this sequence's first unit
  void *winK, *winV;        // window ring, this sequence's first unit
  float *winG;
  int64_t pos;              // position of the token being decoded
  int32_t m, Mcap;          // state rows now, rows per unit in the buffer
};
hipError_t launch_decode_multi(const Dev &dv, const SeqDesc *seq, int n_seq, const void *q, const void *k,
                               const void *v, const float *gate, void *out, hipStream_t st);
// attn_mfma.hip (bf16, d = 128)
hipError_t launch_attn_mfma(const Dev &dv, const AttnArgs &a, hipStream_t st);

// backward.hip: the backward pass of a whole-sequence prefill that started from an empty state.
// Dense operands: q, out, dout, dq [B, T, Hq, d]; k, v, dk, dv [B, T, Hkv, d]; gate, dgate
// [B, T, Hkv]; lse [B, T, Hq]; assign [folds, U, C].  The work arrays have the state's row
// capacity (Mcap rows per unit).
struct Bwd {
  Dev dv;  // dimensions, parameters and the final sums (sK, sV, rho) of the state after the forward
  bool on_mfma;  // attention adjoints on the matrix cores (decides the workspace layout and the launches)
  int64_t T;
  const void *q, *k, *v, *out, *dout;
  const float *gate, *lse;
  const int32_t *assign;
  const float *score;  // [folds, U, C, 2] the forward's record of (append score, merge score)
  void *dq, *dk, *dv_out;
  float *dgate, *dgamma, *dbeta, *dtau_state, *dtau_bswa;
  // workspace
  double *wsK;           // [U, Mcap, d] key sums of the version being visited
  float *wsV;            // [U, Mcap, d]
  float *dsK, *dsV;      // [U, Mcap, d] adjoints of the sums
  float *drho;           // [U, Mcap]
  void *khat, *vhat;     // [U, Mcap, d] I/O dtype: readout of the version being visited
  float *xhat;           // [U, Mcap, d] the key sums of that version, standardised (before gamma, beta)
  float *rden;           // [U, Mcap]    1 / sqrt(var + eps) of those rows
  float *dkhat, *dvhat;  // [U, Mcap, d] adjoint of that readout (one chunk's)
  // fp32 accumulators of dk, dv: [B, T, Hkv, d] (ring_rows = 0), or, on the matrix-core path, only
  // the share a token gets when its fold is undone, kept until the token's block is finished as
  // window keys: [U, ring_rows, d] with ring_rows = L + C, block number mod (n_bswa + 1)
  float *dk_acc, *dv_acc;
  int32_t ring_rows;
  float *delta;          // [B, T, Hq] sum over channels of dout * out
  float *P, *dS;         // [U, G, C, Mcap + L] probabilities and logit adjoints of one chunk
  double *par64;         // [2 * Hkv * d + 2 * Hq] fp64 accumulators of dgamma, dbeta, dtau_state, dtau_bswa
};
// one chunk of the walk: its queries, the state rows it saw, and the fold that followed it
struct BwdChunk {
  int64_t s;       // first position
  int32_t nq;      // queries
  int32_t m;       // state rows the chunk saw ( = rows before the fold that follows)
  int32_t fold;    // index of the fold that followed the chunk, or -1
  int32_t m_after; // state rows after that fold
};
// Two more streams and a few untimed events, owned by the caller, for the matrix-core path: what
// does not depend on the dq role's D, or on the state at all, runs beside the chain undo-fold ->
// dq -> dk of the state rows (see run_backward).
struct BwdStreams {
  hipStream_t side = nullptr, side2 = nullptr;  // null: everything on the one stream
  hipEvent_t fork = nullptr, dq_done = nullptr, join_state = nullptr, join_window[2] = {nullptr, nullptr};
};
hipError_t run_backward(const Bwd &a, const BwdChunk *chunks, int n_chunks, hipStream_t st, const BwdStreams &x);
// backward_mfma.hip (bf16, d = 128): one chunk's dq, dk, dv and readout adjoint on the matrix cores
bool backward_on_mfma(const Dev &dv);
enum { kRoleDQ = 0, kRoleDK = 1, kRoleDV = 2 };
enum { kSecBoth = 0, kSecWindow = 1, kSecState = 2 };
// one role of the matrix-core tile kernel over one chunk; roles dK, dV: all key workgroups, or only
// those of the chunk's own tokens (window keys), or only those of the state rows
hipError_t launch_backward_mfma(const Bwd &a, int64_t cs, int nq, int m, bool folded, int role, int section,
                                hipStream_t st);

}  // namespace kvm
