// Host side of the KVM library: the C ABI of include/kvm.h, the state handle, the growth
// schedule (integer replay of the paper's budget rule) and the per-chunk launch sequence.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/kvm.h"
#include "kvm_internal.h"

using kvm::AttnArgs;
using kvm::Dev;
using kvm::Src;

struct kvm_state {
  kvm_config cfg;
  std::vector<int64_t> table;
  Dev dv;
  void *buf = nullptr;
  size_t bytes = 0;
  int64_t m = 0, tokens = 0, folds = 0;
  int32_t *trace_assign = nullptr;
  float *trace_score = nullptr;
  int64_t trace_max = 0;
  bool mfma = false;  // bf16, d = 128, C % 64 == 0: matrix-core kernels
  bool fused = false; // folds run as one launch per run of folds (fold_fused.hip)
  // a unit's rows shared among several workgroups of that launch: the exchange table (part of the
  // state buffer), whether it has been zeroed, the next exchange number (never reused: the
  // table's entries are told apart by it), and the error word the kernel raises when a wait for a
  // sibling workgroup ran into its time limit (host memory the device can write)
  unsigned long long *xtab = nullptr;
  size_t xtab_bytes = 0;
  bool xtab_clean = false;
  uint32_t xchg = 2;
  int32_t *xerr_host = nullptr, *xerr_dev = nullptr;
  // kvm_debug_set knobs (0 = the library's own choice)
  int dbg[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int group = 1;      // chunks per attention launch in prefill; the readout has 2 * group slots
  // prefill pipeline: folds run ahead on a library-owned stream, attention follows in groups
  int64_t inplace = 0;  // folds done in place so far: version v lives in slot (v - inplace) mod NS
  static constexpr int kMaxChains = 2;
  hipStream_t fold_streams[kMaxChains] = {nullptr, nullptr};
  std::vector<hipEvent_t> sync_events;  // untimed events, reused call after call
  size_t sync_used = 0;
  // optional kernel timing: (start, stop, class) event pairs, events reused across reads
  bool profile = false;
  bool isolate = false;  // profiling aid: never let folds and attention share the chip
  struct Span {
    hipEvent_t a, b;
    int kind, count;  // count: how many launches (or folds) the bracket covers
  };
  std::vector<Span> spans;
  std::vector<hipEvent_t> free_events;
};

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char *what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return KVM_ERR_HIP;
}
#define HIP_TRY(expr)                                  \
  do {                                                 \
    hipError_t e__ = (expr);                           \
    if (e__ != hipSuccess) return hip_fail(e__, #expr); \
  } while (0)

inline size_t esize(int io) { return io == KVM_BF16 ? 2 : 4; }
inline size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

int64_t ceil_sqrt(int64_t e) {
  if (e <= 0) return 0;
  int64_t n = (int64_t)std::ceil(std::sqrt((double)e));
  while (n * n < e) ++n;
  while (n > 0 && (n - 1) * (n - 1) >= e) --n;
  return n;
}

int64_t budget_at(const kvm_config &c, const std::vector<int64_t> &table, int64_t e) {
  switch (c.budget_kind) {
    case KVM_BUDGET_FIXED: return c.budget_fixed;
    case KVM_BUDGET_SQRT: return (int64_t)std::floor(c.budget_scale * (double)ceil_sqrt(e));
    case KVM_BUDGET_TABLE: {
      if (table.empty()) return 0;
      int64_t idx = e / c.chunk_len - 1;
      if (idx < 0) idx = 0;
      if (idx >= (int64_t)table.size()) idx = (int64_t)table.size() - 1;
      return table[idx];
    }
    default: return 0;
  }
}

// Rows after folding one block at chunk end e: creation copies a whole chunk, afterwards
// M* = max(m, min(B(e), m + C)).
int64_t rows_after(const kvm_config &c, const std::vector<int64_t> &table, int64_t m, int64_t e) {
  if (c.budget_kind == KVM_BUDGET_NONE) return 0;
  if (m == 0) return c.chunk_len;
  const int64_t B = budget_at(c, table, e);
  const int64_t capped = B < m + c.chunk_len ? B : m + c.chunk_len;
  return m > capped ? m : capped;
}

bool config_ok(const kvm_config *c) {
  if (!c) return false;
  if (c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0) return false;
  if (c->n_q_heads % c->n_kv_heads) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->rope_dims < 0 || c->rope_dims > c->head_dim) return false;
  if (c->chunk_len <= 0 || c->n_bswa_chunks < 1) return false;
  if (c->n_sink < 0 || c->n_sink >= c->chunk_len) return false;
  if (c->io_dtype != KVM_F32 && c->io_dtype != KVM_BF16) return false;
  if (c->budget_kind < KVM_BUDGET_NONE || c->budget_kind > KVM_BUDGET_TABLE) return false;
  if (c->budget_kind == KVM_BUDGET_TABLE && (!c->budget_table || c->budget_table_len <= 0)) return false;
  if (c->budget_kind == KVM_BUDGET_SQRT && !(c->budget_scale >= 0.0)) return false;
  if (c->budget_kind == KVM_BUDGET_FIXED && c->budget_fixed < 0) return false;
  return true;
}

std::vector<int64_t> table_of(const kvm_config *c) {
  if (c->budget_kind == KVM_BUDGET_TABLE)
    return std::vector<int64_t>(c->budget_table, c->budget_table + c->budget_table_len);
  return {};
}

// Rows reached after running from (m, tokens) to `until` tokens.
int64_t replay_rows(const kvm_config &c, const std::vector<int64_t> &table, int64_t m, int64_t tokens,
                    int64_t until) {
  const int64_t C = c.chunk_len, L = C * c.n_bswa_chunks;
  for (int64_t e = (tokens / C + 1) * C; e <= until; e += C)
    if (e >= L) m = rows_after(c, table, m, e);
  return m;
}

int64_t capacity_rows(const kvm_config &c, const std::vector<int64_t> &table, int64_t max_tokens) {
  int64_t rows = replay_rows(c, table, 0, 0, max_tokens);
  if (rows < c.chunk_len) rows = c.chunk_len;
  return (rows + 63) / 64 * 64;
}

struct Layout {
  size_t sK, sV, rho, w, n, khat, vhat, winK, winV, winG, kbar, score, pi, app, xtab, xtab_bytes, creator, total;
};

bool use_mfma(const kvm_config &c) {
  return c.io_dtype == KVM_BF16 && c.head_dim == 128 && c.chunk_len % 64 == 0;
}
// Chunks per prefill attention launch.  The matrix-core path launches groups of chunks so that
// a launch has thousands of workgroups; the generic path launches chunk by chunk.
int group_of(const kvm_config &c) { return use_mfma(c) ? 8 : 1; }
constexpr int kClusterBelowUnits = 256;  // compute units of the chip this library is written for

Layout layout_of(const kvm_config &c, int64_t Mcap) {
  const size_t U = (size_t)c.batch * c.n_kv_heads, d = c.head_dim, C = c.chunk_len;
  const size_t L = C * c.n_bswa_chunks, es = esize(c.io_dtype), M = (size_t)Mcap;
  Layout l;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o += up256(bytes);
    return at;
  };
  l.sK = take(U * M * d * 8);
  l.sV = take(U * M * d * 4);
  l.rho = take(U * M * 4);
  l.w = take(U * M * 4);
  l.n = take(U * M * 4);
  const size_t NS = 2 * (size_t)group_of(c);
  l.khat = take(NS * U * M * d * es);
  l.vhat = take(NS * U * M * d * es);
  l.winK = take(U * L * d * es);
  l.winV = take(U * L * d * es);
  l.winG = take(U * L * 4);
  l.kbar = take((size_t)group_of(c) * U * C * d * es);
  l.score = take(U * C * 8);
  l.pi = take(U * C * 4);
  l.app = take(U * C * 4);
  // exchange table of the one-launch fold when a unit's rows are shared among workgroups: only
  // states with fewer units than the chip has compute units ever do that
  l.xtab_bytes = use_mfma(c) && U < (size_t)kClusterBelowUnits
                     ? U * 2 * (size_t)kvm::kFoldMaxSplit * 2 * C * sizeof(unsigned long long) : 0;
  l.xtab = take(l.xtab_bytes);
  l.creator = take(U * C * 4);
  l.total = o;
  return l;
}

void bind(Dev &dv, const kvm_config &c, void *buf, int64_t Mcap) {
  const Layout l = layout_of(c, Mcap);
  char *p = (char *)buf;
  dv.sK = (double *)(p + l.sK);
  dv.sV = (float *)(p + l.sV);
  dv.rho = (float *)(p + l.rho);
  dv.w = (float *)(p + l.w);
  dv.n = (int32_t *)(p + l.n);
  dv.khat = p + l.khat;
  dv.vhat = p + l.vhat;
  dv.winK = p + l.winK;
  dv.winV = p + l.winV;
  dv.winG = (float *)(p + l.winG);
  dv.kbar = p + l.kbar;
  dv.score = (float2 *)(p + l.score);
  dv.pi = (int32_t *)(p + l.pi);
  dv.app = (int32_t *)(p + l.app);
  dv.creator = (int32_t *)(p + l.creator);
  dv.gamma = c.ln_gamma;
  dv.beta = c.ln_beta;
  dv.tau_state = c.tau_state;
  dv.tau_bswa = c.tau_bswa;
  dv.B = c.batch;
  dv.Hq = c.n_q_heads;
  dv.Hkv = c.n_kv_heads;
  dv.U = c.batch * c.n_kv_heads;
  dv.Ufull = dv.U;
  dv.d = c.head_dim;
  dv.r = c.rope_dims;
  dv.C = c.chunk_len;
  dv.L = c.chunk_len * c.n_bswa_chunks;
  dv.S = c.n_sink;
  dv.Mcap = (int32_t)Mcap;
  dv.NS = 2 * group_of(c);
  dv.slot_elems = (int64_t)dv.U * Mcap * dv.d;
  dv.ln_eps = c.ln_eps > 0.f ? c.ln_eps : 1e-5f;
  dv.norm_eps = c.norm_eps > 0.f ? c.norm_eps : 1e-12f;
  dv.io = c.io_dtype;
}

Src ring_src(const kvm_state *st) {
  const Dev &dv = st->dv;
  Src s;
  s.k = dv.winK;
  s.v = dv.winV;
  s.g = dv.winG;
  s.k_b = s.v_b = (int64_t)dv.Hkv * dv.L * dv.d;
  s.k_h = s.v_h = (int64_t)dv.L * dv.d;
  s.k_t = s.v_t = dv.d;
  s.g_b = (int64_t)dv.Hkv * dv.L;
  s.g_h = dv.L;
  s.g_t = 1;
  return s;
}

// `src` with its token origin moved forward by `tok` tokens.
Src advance(const Src &s, int64_t tok, size_t es) {
  Src r = s;
  r.k = (const char *)s.k + tok * s.k_t * (int64_t)es;
  r.v = (const char *)s.v + tok * s.v_t * (int64_t)es;
  if (s.g) r.g = s.g + tok * s.g_t;
  return r;
}

// Readout slot of state version `ver` (versions are numbered by the folds done).
int slot_of(const kvm_state *st, int64_t ver) {
  const int64_t ns = st->dv.NS;
  return (int)(((ver - st->inplace) % ns + ns) % ns);
}

// Fold the C-token block whose first token is src's token 0.  e = end of the chunk just attended.
// Reads readout version `folds` and writes version folds + 1: into the next slot, with untouched
// rows copied over (prefill, where attention launches still read the older versions), or, in_place,
// over the version it read (decode and the fold entry point: nothing else is in flight).
// kbar_block >= 0: the block's memory keys were already computed into that slab of the scratch.
// The sequences [b0, b0 + nb) of a state as a state of their own: same strides, moved pointers.
Dev batch_view(const Dev &full, int b0, int nb, size_t es) {
  Dev v = full;
  const int64_t u0 = (int64_t)b0 * full.Hkv, M = full.Mcap, d = full.d, L = full.L, C = full.C;
  v.B = nb;
  v.U = nb * full.Hkv;
  v.sK += u0 * M * d;
  v.sV += u0 * M * d;
  v.rho += u0 * M;
  v.w += u0 * M;
  v.n += u0 * M;
  v.khat = (char *)full.khat + u0 * M * d * es;  // the slot stride stays the whole state's
  v.vhat = (char *)full.vhat + u0 * M * d * es;
  v.winK = (char *)full.winK + u0 * L * d * es;
  v.winV = (char *)full.winV + u0 * L * d * es;
  v.winG += u0 * L;
  v.kbar = (char *)full.kbar + u0 * C * d * es;  // the block stride stays Ufull * C * d
  v.score += u0 * C;
  v.pi += u0 * C;
  v.app += u0 * C;
  v.creator += u0 * C;
  return v;
}
Src batch_view(const Src &s, int b0, size_t es) {
  Src r = s;
  r.k = (const char *)s.k + b0 * s.k_b * (int64_t)es;
  r.v = (const char *)s.v + b0 * s.v_b * (int64_t)es;
  if (s.g) r.g = s.g + b0 * s.g_b;
  return r;
}

// The launches of one fold over the units of `dv` (the whole state or a view of part of its
// batch), from m to m_after rows, reading readout slot so and writing slot sn.
int fold_launches(const kvm_state *st, Dev dv, const Src &src, int64_t m, int64_t m_after, int so, int sn,
                  bool in_place, int kbar_block, hipStream_t stream) {
  const kvm_config &c = st->cfg;
  const int n_app = (int)(m_after - m);
  if (kbar_block < 0) {
    HIP_TRY(kvm::launch_memkey(dv, src, 1, stream));
  } else {
    dv.kbar = (char *)dv.kbar + (size_t)kbar_block * dv.Ufull * dv.C * dv.d * esize(c.io_dtype);
  }
  const bool copy = !in_place;
  if (n_app == dv.C) {
    // room for the whole block (state creation included): no scores are needed
    HIP_TRY(kvm::launch_select(dv, (int)m, n_app, true, stream));
    HIP_TRY(kvm::launch_accum(dv, src, (int)m, (int)m_after, 0, true, false, copy, false, so, sn, stream));
  } else {
    if (st->mfma)
      HIP_TRY(kvm::launch_score_mfma(dv, so, 0, (int)m, true, stream));
    else
      HIP_TRY(kvm::launch_score(dv, so, 0, (int)m, true, stream));
    if (kvm::append_fits(dv, n_app)) {
      HIP_TRY(kvm::launch_append(dv, src, (int)m, n_app, sn, stream));
    } else if (n_app > 0) {
      // new rows first, so that the remaining tokens can be scored against them too
      HIP_TRY(kvm::launch_select(dv, (int)m, n_app, false, stream));
      HIP_TRY(kvm::launch_accum(dv, src, (int)m, (int)m_after, (int)m, true, false, false, false, so, sn, stream));
      if (st->mfma)
        HIP_TRY(kvm::launch_score_mfma(dv, sn, (int)m, (int)m_after, false, stream));
      else
        HIP_TRY(kvm::launch_score(dv, sn, (int)m, (int)m_after, false, stream));
    }
    const int mc = st->dbg[KVM_DEBUG_MERGE_COPY];  // 1 / 2 force it on / off: for comparisons
    const bool small = mc ? mc == 1 : (int64_t)dv.Ufull * m_after < 64 * 1024;
    if (in_place)
      HIP_TRY(kvm::launch_merge_inplace(dv, src, n_app > 0, sn, stream));
    else if (small)
      HIP_TRY(kvm::launch_merge_copy(dv, src, n_app > 0, so, sn, (int)m, stream));
    else
      HIP_TRY(kvm::launch_accum(dv, src, (int)m, (int)m_after, 0, false, true, true, n_app > 0, so, sn, stream));
  }
  return KVM_OK;
}

// What a fold leaves for the parity tests: its assignments and scores, for the units of `dv`
// (unit u0 on of the state), into the trace buffers at fold number `fold`.
int fold_trace(const kvm_state *st, const Dev &dv, int64_t u0, int64_t fold, hipStream_t stream) {
  const size_t ntok_all = (size_t)st->dv.U * dv.C, ntok = (size_t)dv.U * dv.C, off = (size_t)u0 * dv.C;
  if (st->trace_assign && fold < st->trace_max)
    HIP_TRY(hipMemcpyAsync(st->trace_assign + fold * ntok_all + off, dv.pi, ntok * 4, hipMemcpyDeviceToDevice, stream));
  if (st->trace_score && fold < st->trace_max)
    HIP_TRY(hipMemcpyAsync(st->trace_score + (fold * ntok_all + off) * 2, dv.score, ntok * 8, hipMemcpyDeviceToDevice,
                           stream));
  return KVM_OK;
}

// The one-launch fold path (a run of folds in one kernel, one workgroup per unit; bf16, d = 128
// states whose tables fit LDS) is taken when there are at least as many units as compute units,
// so that one workgroup per unit fills the chip (measured on 256 units of the paper's benchmark
// shape: 17 % off the prefill with a growing state, 2 % with 256 rows), or when kvm_debug_set asks
// for it.  With fewer units one compute unit per unit of the state is slower than launches over
// the whole chip by more than the launch boundaries cost (64 units: 13-15 ms against 11 ms).
constexpr int kFusedMinUnits = 256;
// With fewer units a unit's rows can be shared among `split` workgroups of the launch (a power of
// two, at most kFoldMaxSplit; units x split workgroups must be resident together, one per compute
// unit): 0 = the kernel-per-step path.
int fold_split(const kvm_state *st) {
  if (!st->fused) return 0;
  const int path = st->dbg[KVM_DEBUG_FOLD_PATH];
  if (path == 2) return 0;
  const int U = st->dv.U;
  int want = st->dbg[KVM_DEBUG_FOLD_SPLIT];
  if (want == 0) {
    if (U >= kFusedMinUnits) return 1;
    if (path != 1) return 0;
    want = 1;
  }
  if (want == 1) return 1;
  const bool ok = (want == 2 || want == 4 || want == 8) && st->xtab && (int64_t)U * want <= kClusterBelowUnits &&
                  st->dv.Mcap / 64 >= want && kvm::fold_fused_fits(st->dv, want);
  return ok ? want : 1;
}
bool use_fused(const kvm_state *st) { return fold_split(st) > 0; }

__global__ __launch_bounds__(256) void zero_words_kernel(unsigned long long *p, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ull;
}

// Arguments of a one-launch run; with shared rows also what the exchange needs: the table zeroed
// once (on `stream`, ahead of the first launch that uses it) and the error word.
int fused_run(kvm_state *st, bool in_place, hipStream_t stream, kvm::FoldRunArgs *out) {
  kvm::FoldRunArgs run;
  run.n = 0;
  run.in_place = in_place ? 1 : 0;
  run.trace_assign = st->trace_assign;
  run.trace_score = st->trace_score;
  run.trace_stride = (int64_t)st->dv.U * st->dv.C;
  run.split = fold_split(st);
  run.xtab = nullptr;
  run.err = nullptr;
  if (run.split > 1) {
    if (!st->xerr_host) {
      HIP_TRY(hipHostMalloc((void **)&st->xerr_host, sizeof(int32_t), hipHostMallocMapped));
      *st->xerr_host = 0;
      HIP_TRY(hipHostGetDevicePointer((void **)&st->xerr_dev, st->xerr_host, 0));
    }
    if (!st->xtab_clean) {
      hipLaunchKernelGGL(zero_words_kernel, dim3(256), dim3(256), 0, stream, st->xtab, st->xtab_bytes / 8);
      HIP_TRY(hipGetLastError());
      st->xtab_clean = true;
    }
    run.xtab = st->xtab;
    run.err = st->xerr_dev;
  }
  *out = run;
  return KVM_OK;
}
// The exchange numbers of one fold (first scoring pass, and the second one when some but not all
// of the block is appended): consecutive, never 0 in their low 16 bits.
uint32_t take_exchanges(kvm_state *st, int64_t m, int64_t m_after) {
  const int64_t n_app = m_after - m;
  const uint32_t need = n_app == st->dv.C ? 0u : n_app > 0 ? 2u : 1u;
  if (((st->xchg & 0xffffu) == 0u) || (need == 2u && ((st->xchg + 1u) & 0xffffu) == 0u)) {
    // skip the number whose tag would be 0, keeping the parity sequence strictly alternating
    st->xchg += 2u;
  }
  const uint32_t first = st->xchg;
  st->xchg += need;
  return first;
}
int cluster_error(const kvm_state *st) {
  if (st->xerr_host && *(volatile int32_t *)st->xerr_host != 0) {
    g_hip_error = "a fold workgroup waited for a sibling workgroup past its time limit; the state is undefined";
    return KVM_ERR_HIP;
  }
  return KVM_OK;
}

int fold_block(kvm_state *st, const Src &src, int64_t e, int32_t *assign_out, float *score_out,
               hipStream_t stream, bool in_place, int kbar_block = -1) {
  const kvm_config &c = st->cfg;
  if (c.budget_kind == KVM_BUDGET_NONE) return KVM_OK;
  const int64_t m = st->m;
  const int64_t m_after = rows_after(c, st->table, m, e);
  if (m_after > st->dv.Mcap) return KVM_ERR_CAPACITY;
  const Dev &dv = st->dv;
  const int so = slot_of(st, st->folds), sn = in_place ? so : slot_of(st, st->folds + 1);
  const size_t ntok = (size_t)dv.U * dv.C;
  if (use_fused(st)) {
    kvm::FoldRunArgs run;
    const int rc_run = fused_run(st, in_place, stream, &run);
    if (rc_run != KVM_OK) return rc_run;
    run.n = 1;
    run.s[0] = {(int32_t)m, (int32_t)m_after, so, sn, 0, st->folds < st->trace_max ? (int32_t)st->folds : -1, 0,
                take_exchanges(st, m, m_after), 0u};
    HIP_TRY(kvm::launch_memkey(dv, src, 1, stream));
    // a fold of its own (decode, the fold entry point, the chunk-by-chunk schedule): the narrow
    // workgroup, two to a compute unit, unless asked otherwise (measured 3 % ahead of the wide one)
    HIP_TRY(kvm::launch_fold_fused(dv, src, run, st->dbg[KVM_DEBUG_FOLD_WAVES] != 16, stream));
  } else {
    int rc = fold_launches(st, dv, src, m, m_after, so, sn, in_place, kbar_block, stream);
    if (rc != KVM_OK) return rc;
    if (st->trace_assign && st->folds < st->trace_max)
      HIP_TRY(hipMemcpyAsync(st->trace_assign + st->folds * ntok, dv.pi, ntok * 4,
                             hipMemcpyDeviceToDevice, stream));
    if (st->trace_score && st->folds < st->trace_max)
      HIP_TRY(hipMemcpyAsync(st->trace_score + st->folds * ntok * 2, dv.score, ntok * 8,
                             hipMemcpyDeviceToDevice, stream));
  }
  if (assign_out)
    HIP_TRY(hipMemcpyAsync(assign_out, dv.pi, ntok * 4, hipMemcpyDeviceToDevice, stream));
  if (score_out)
    HIP_TRY(hipMemcpyAsync(score_out, dv.score, ntok * 8, hipMemcpyDeviceToDevice, stream));
  st->m = m_after;
  st->folds += 1;
  if (in_place) st->inplace += 1;
  return KVM_OK;
}

// An untimed event from the state's pool (for ordering between the two streams).
hipError_t next_sync_event(kvm_state *st, hipEvent_t *out) {
  if (st->sync_used == st->sync_events.size()) {
    hipEvent_t e;
    hipError_t rc = hipEventCreateWithFlags(&e, hipEventDisableTiming);
    if (rc != hipSuccess) return rc;
    st->sync_events.push_back(e);
  }
  *out = st->sync_events[st->sync_used++];
  return hipSuccess;
}

// Work arrays of the backward pass, in the order of kvm::Bwd.
struct BwdLayout {
  size_t wsK, wsV, dsK, dsV, drho, khat, vhat, xhat, rden, dkhat, dvhat, dk_acc, dv_acc, delta, P, dS, par64, total;
};
// mfma_path: the attention adjoints run on the matrix cores (bwd_on_mfma); that one flag decides
// the layout here and the launches in run_backward alike.
BwdLayout bwd_layout(const kvm_config &c, int64_t Mcap, int64_t T, bool mfma_path) {
  const size_t U = (size_t)c.batch * c.n_kv_heads, d = c.head_dim, C = c.chunk_len;
  const size_t L = C * c.n_bswa_chunks, es = esize(c.io_dtype), M = (size_t)Mcap;
  const size_t G = c.n_q_heads / c.n_kv_heads, Tn = (size_t)T;
  BwdLayout l;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o += up256(bytes);
    return at;
  };
  l.wsK = take(U * M * d * 8);
  l.wsV = take(U * M * d * 4);
  l.dsK = take(U * M * d * 4);
  l.dsV = take(U * M * d * 4);
  l.drho = take(U * M * 4);
  l.khat = take(U * M * d * es);
  l.vhat = take(U * M * d * es);
  l.xhat = take(U * M * d * 4);
  l.rden = take(U * M * 4);
  l.dkhat = take(U * M * d * 4);
  l.dvhat = take(U * M * d * 4);
  // full-size accumulators of dk, dv on the vector-ALU path; on the matrix-core path a ring of
  // one window's blocks and one more (see kvm::Bwd)
  l.dk_acc = take(U * (mfma_path ? L + C : Tn) * d * 4);
  l.dv_acc = take(U * (mfma_path ? L + C : Tn) * d * 4);
  l.delta = take((size_t)c.batch * Tn * c.n_q_heads * 4);
  // the chunk's probabilities and logit adjoints are written out only by the vector-ALU kernels
  const bool probs = !mfma_path;
  l.P = take(probs ? U * G * C * (M + L) * 4 : 0);
  l.dS = take(probs ? U * G * C * (M + L) * 4 : 0);
  l.par64 = take((2 * (size_t)c.n_kv_heads * d + 2 * (size_t)c.n_q_heads) * 8);
  l.total = o;
  return l;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// The backward's attention adjoints run on the matrix cores for the shapes those kernels are
// written and tested for, unless kvm_debug_set asked for the vector-ALU kernels.
bool bwd_on_mfma(const kvm_state *st) {
  return kvm::backward_on_mfma(st->dv) && st->dbg[KVM_DEBUG_BACKWARD_PATH] != 1;
}

// RAII bracket: records a start event now and a stop event when it goes out of scope.
struct ProfileSpan {
  kvm_state *st;
  hipStream_t stream;
  hipEvent_t a = nullptr, b = nullptr;
  int kind, count;
  ProfileSpan(kvm_state *s, int k, hipStream_t str, int n = 1) : st(s), stream(str), kind(k), count(n) {
    if (!st || !st->profile) return;
    auto get = [&]() -> hipEvent_t {
      hipEvent_t e = nullptr;
      if (!st->free_events.empty()) {
        e = st->free_events.back();
        st->free_events.pop_back();
      } else if (hipEventCreate(&e) != hipSuccess) {
        e = nullptr;
      }
      return e;
    };
    a = get();
    b = get();
    if (a && b) (void)hipEventRecord(a, stream);
  }
  ~ProfileSpan() {
    if (a && b) {
      (void)hipEventRecord(b, stream);
      st->spans.push_back({a, b, kind, count});
    }
  }
};

// ---------------------------------------------------------------------------------------------
// Allocation-free ragged decode (kvm_decode_step_multi_static): the per-sequence descriptor table
// that kvm_decode_step_multi keeps in a caller workspace lives in this file-scope device array
// instead, one copy per GPU, held until the process ends.  Host code never uses the array's name
// as an address: scratch_on_device() asks the runtime for the array's address on the current
// device once and keeps it.
constexpr int kStaticMaxSeq = 4096;   // sequences per call
constexpr int kStaticMaxDev = 64;     // devices a process can hold
static __device__ __align__(256) unsigned char scratch[kStaticMaxSeq * sizeof(kvm::SeqDesc)];

struct ScratchPtrs {
  void *ptr[kStaticMaxDev] = {};
  bool known[kStaticMaxDev] = {};
};
ScratchPtrs g_scratch;
std::mutex g_scratch_mutex;

// Address of `scratch` on the device that is current for the calling thread.
int scratch_on_device(void **out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kStaticMaxDev) return KVM_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch.known[dev]) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return KVM_ERR_HIP;
    g_scratch.ptr[dev] = p;
    g_scratch.known[dev] = true;
  }
  *out = g_scratch.ptr[dev];
  return KVM_OK;
}

// Up to kPackStates states' worth of descriptors per launch, handed over as a kernel argument
// (no host-to-device copy, no host buffer): per state where its arrays start and where it stands;
// thread i of the launch writes the descriptor of sequence pack.seq0[0] + i.
constexpr int kPackStates = 32;
struct StatePack {
  const void *khat[kPackStates], *vhat[kPackStates];  // current readout version, first unit
  void *winK[kPackStates], *winV[kPackStates];
  float *winG[kPackStates];
  int64_t pos[kPackStates];
  int32_t m[kPackStates], Mcap[kPackStates];
  int32_t seq0[kPackStates + 1];  // first sequence of each state; [n] = one past the last
  int32_t n;
};
__global__ __launch_bounds__(256) void seqdesc_fill_kernel(StatePack pk, kvm::SeqDesc *table, int Hkv, int L, int d,
                                                           int es) {
  const int s = pk.seq0[0] + blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= pk.seq0[pk.n]) return;
  int i = 0;
  while (i + 1 < pk.n && s >= pk.seq0[i + 1]) ++i;
  const int64_t u0 = (int64_t)(s - pk.seq0[i]) * Hkv;  // the sequence's first unit within its state
  kvm::SeqDesc sd;
  sd.khat = (const char *)pk.khat[i] + u0 * pk.Mcap[i] * d * es;
  sd.vhat = (const char *)pk.vhat[i] + u0 * pk.Mcap[i] * d * es;
  sd.winK = (char *)pk.winK[i] + u0 * L * d * es;
  sd.winV = (char *)pk.winV[i] + u0 * L * d * es;
  sd.winG = pk.winG[i] + u0 * L;
  sd.pos = pk.pos[i];
  sd.m = pk.m[i];
  sd.Mcap = pk.Mcap[i];
  table[s] = sd;
}

}  // namespace

extern "C" {

const char *kvm_strerror(int status) {
  switch (status) {
    case KVM_OK: return "ok";
    case KVM_ERR_ARG: return "bad argument";
    case KVM_ERR_CAPACITY: return "state buffer too small for the rows the budget asks for";
    case KVM_ERR_STATE: return "call not valid at the state's current position";
    case KVM_ERR_HIP: return "HIP runtime error";
    case KVM_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case KVM_ERR_LIMIT: return "beyond the fixed size of an allocation-free entry point's static buffer";
    default: return "unknown status";
  }
}

const char *kvm_last_hip_error(void) { return g_hip_error.c_str(); }

int64_t kvm_state_rows_for(const kvm_config *cfg, int64_t max_tokens) {
  if (!config_ok(cfg) || max_tokens < 0) return -1;
  return replay_rows(*cfg, table_of(cfg), 0, 0, max_tokens);
}

size_t kvm_state_bytes(const kvm_config *cfg, int64_t max_tokens) {
  if (!config_ok(cfg) || max_tokens < 0) return 0;
  return layout_of(*cfg, capacity_rows(*cfg, table_of(cfg), max_tokens)).total;
}

int kvm_state_init(kvm_state **out, const kvm_config *cfg, void *dev_buf, size_t bytes,
                   int64_t max_tokens) {
  if (!out || !config_ok(cfg) || !dev_buf || max_tokens < 0) return KVM_ERR_ARG;
  if (((uintptr_t)dev_buf & 255) != 0) return KVM_ERR_ARG;
  if (!aligned16(cfg->ln_gamma) || !aligned16(cfg->ln_beta)) return KVM_ERR_ARG;
  std::vector<int64_t> table = table_of(cfg);
  const int64_t Mcap = capacity_rows(*cfg, table, max_tokens);
  if (layout_of(*cfg, Mcap).total > bytes) return KVM_ERR_CAPACITY;
  kvm_state *st = new (std::nothrow) kvm_state();
  if (!st) return KVM_ERR_ARG;
  st->cfg = *cfg;
  st->table = std::move(table);
  st->cfg.budget_table = st->table.empty() ? nullptr : st->table.data();
  st->buf = dev_buf;
  st->bytes = bytes;
  bind(st->dv, st->cfg, dev_buf, Mcap);
  {
    const Layout l = layout_of(st->cfg, Mcap);
    st->xtab = l.xtab_bytes ? (unsigned long long *)((char *)dev_buf + l.xtab) : nullptr;
    st->xtab_bytes = l.xtab_bytes;
    st->xtab_clean = false;
  }
  st->mfma = use_mfma(*cfg);
  st->fused = st->mfma && kvm::fold_fused_fits(st->dv);
  st->group = group_of(*cfg);
  *out = st;
  return KVM_OK;
}

int kvm_state_destroy(kvm_state *st) {
  if (st) {
    for (auto &sp : st->spans) {
      (void)hipEventDestroy(sp.a);
      (void)hipEventDestroy(sp.b);
    }
    for (auto e : st->free_events) (void)hipEventDestroy(e);
    for (auto e : st->sync_events) (void)hipEventDestroy(e);
    for (hipStream_t fs : st->fold_streams)
      if (fs) (void)hipStreamDestroy(fs);
    if (st->xerr_host) (void)hipHostFree(st->xerr_host);
  }
  delete st;
  return KVM_OK;
}

int kvm_debug_set(kvm_state *st, int knob, int value) {
  if (!st || knob < 0 || knob >= KVM_DEBUG_KNOBS || value < 0) return KVM_ERR_ARG;
  st->dbg[knob] = value;
  return KVM_OK;
}

int kvm_state_profile(kvm_state *st, int enable) {
  if (!st) return KVM_ERR_ARG;
  st->profile = enable != 0;
  st->isolate = enable == 2;
  return KVM_OK;
}

int kvm_state_profile_read(kvm_state *st, double ms[3], int64_t count[3]) {
  if (!st || !ms || !count) return KVM_ERR_ARG;
  for (int i = 0; i < 3; ++i) {
    ms[i] = 0.0;
    count[i] = 0;
  }
  for (auto &sp : st->spans) {
    HIP_TRY(hipEventSynchronize(sp.b));
    float t = 0.f;
    HIP_TRY(hipEventElapsedTime(&t, sp.a, sp.b));
    ms[sp.kind] += t;
    count[sp.kind] += sp.count;
    st->free_events.push_back(sp.a);
    st->free_events.push_back(sp.b);
  }
  st->spans.clear();
  return KVM_OK;
}

int kvm_prefill_chunked(kvm_state *st, const void *q, const void *k, const void *v,
                        const float *gate, void *out, float *lse, int64_t T,
                        const kvm_strides *sp, void *stream_) {
  if (!st || !q || !k || !v || !out || T <= 0) return KVM_ERR_ARG;
  if (cluster_error(st) != KVM_OK) return KVM_ERR_HIP;
  hipStream_t stream = (hipStream_t)stream_;
  const kvm_config &c = st->cfg;
  const Dev &dv = st->dv;
  const int64_t C = dv.C, L = dv.L, d = dv.d;
  const size_t es = esize(c.io_dtype);
  if (st->tokens % C != 0) return KVM_ERR_STATE;
  kvm_strides s;
  if (sp) {
    s = *sp;
  } else {
    s.q_b = T * dv.Hq * d; s.q_t = dv.Hq * d; s.q_h = d;
    s.k_b = T * dv.Hkv * d; s.k_t = dv.Hkv * d; s.k_h = d;
    s.v_b = s.k_b; s.v_t = s.k_t; s.v_h = s.k_h;
    s.o_b = s.q_b; s.o_t = s.q_t; s.o_h = s.q_h;
    s.g_b = T * dv.Hkv; s.g_t = dv.Hkv; s.g_h = 1;
    s.lse_b = T * dv.Hq; s.lse_t = dv.Hq; s.lse_h = 1;
  }
  const int64_t vec = 16 / (int64_t)es;
  const int64_t strides16[] = {s.q_b, s.q_t, s.q_h, s.k_b, s.k_t, s.k_h, s.v_b, s.v_t, s.v_h, s.o_b, s.o_t, s.o_h};
  for (int64_t x : strides16)
    if (x % vec) return KVM_ERR_ARG;
  // rows of k and v are whole and apart (the tile loads count on at least d elements between tokens)
  if (s.k_t < d || s.v_t < d || s.q_t < d || s.o_t < d) return KVM_ERR_ARG;
  if (s.q_h < d || s.k_h < d || s.v_h < d || s.o_h < d) return KVM_ERR_ARG;
  // the tile loads keep a token's byte offset inside a tile in 32 bits (64 rows of a tile times
  // the stride): a token stride of up to 16 MiB is far beyond any fused-projection layout
  if (s.k_t * (int64_t)es > (int64_t)1 << 24 || s.v_t * (int64_t)es > (int64_t)1 << 24) return KVM_ERR_ARG;
  for (int64_t x : strides16)
    if (x < 0) return KVM_ERR_ARG;
  if (gate && (s.g_b < 0 || s.g_t < 0 || s.g_h < 0)) return KVM_ERR_ARG;
  // lse is written: its three strides must address B * T * H_q distinct floats
  if (lse && (s.lse_h <= 0 || s.lse_t <= 0 || s.lse_b <= 0)) return KVM_ERR_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return KVM_ERR_ARG;

  const int64_t t0 = st->tokens, t_end = t0 + T;
  if (replay_rows(c, st->table, st->m, t0, t_end) > dv.Mcap) return KVM_ERR_CAPACITY;

  Src in;
  in.k = k; in.v = v; in.g = gate;
  in.k_b = s.k_b; in.k_h = s.k_h; in.k_t = s.k_t;
  in.v_b = s.v_b; in.v_h = s.v_h; in.v_t = s.v_t;
  in.g_b = s.g_b; in.g_h = s.g_h; in.g_t = s.g_t;
  const Src ring = ring_src(st);

  // Plan.  The schedule is data independent: which state version (and how many rows) each chunk
  // sees, and which chunks are followed by a fold, is integer arithmetic.
  struct Chunk {
    int64_t s;
    int32_t nq, m;
    int64_t ver;
    bool folds;
  };
  std::vector<Chunk> plan;
  {
    int64_t m = st->m, ver = st->folds;
    for (int64_t cs = t0; cs < t_end; cs += C) {
      const int64_t ce = cs + C < t_end ? cs + C : t_end;
      Chunk ch{cs, (int32_t)(ce - cs), (int32_t)m, ver, false};
      if (ce - cs == C && ce >= L && c.budget_kind != KVM_BUDGET_NONE) {
        ch.folds = true;
        m = rows_after(c, st->table, m, ce);
        ver += 1;
      }
      plan.push_back(ch);
    }
  }
  // Two schedules.  The pipelined one below keeps a readout version per chunk, which costs a copy
  // of every untouched row's readout per fold: U * m * d * 2 elements read and written.  When the
  // state is large against the block (many units, thousands of rows, a few hundred tokens per
  // fold) that copy outweighs what the pipeline gains, and the call runs chunk by chunk on the
  // caller's stream instead: attention of a chunk, then its fold in place.
  {
    int64_t m_max = 0;
    for (const Chunk &ch : plan) m_max = ch.m > m_max ? ch.m : m_max;
    const double copy_us = (double)dv.U * (double)m_max * (double)d * (double)es * 4.0 / 4.0e6;  // at ~4 TB/s
    const int forced = st->dbg[KVM_DEBUG_PREFILL_SCHEDULE];  // 1 serial, 2 pipelined: for comparisons
    // (and a call of a few chunks has nothing to pipeline: the events would cost more than they buy)
    const bool serial = forced ? forced == 1 : (copy_us > 45.0 || plan.size() <= 4);
    if (serial) {
      for (const Chunk &ch : plan) {
        AttnArgs a;
        a.put_token = 0;
        a.q = (const char *)q + (ch.s - t0) * s.q_t * (int64_t)es;
        a.out = (char *)out + (ch.s - t0) * s.o_t * (int64_t)es;
        a.lse = lse ? lse + (ch.s - t0) * s.lse_t : nullptr;
        a.q_b = s.q_b; a.q_t = s.q_t; a.q_h = s.q_h;
        a.o_b = s.o_b; a.o_t = s.o_t; a.o_h = s.o_h;
        a.lse_b = s.lse_b; a.lse_t = s.lse_t; a.lse_h = s.lse_h;
        a.in = in;
        a.t0 = t0;
        a.s = ch.s;
        a.n_chunks = 1;
        a.nq_total = ch.nq;
        for (int i = 0; i < kvm::kMaxGroup; ++i) {
          a.m[i] = (int32_t)st->m;
          a.slot[i] = (int32_t)slot_of(st, st->folds);
        }
        {
          ProfileSpan span(st, 0, stream);
          if (st->mfma)
            HIP_TRY(kvm::launch_attn_mfma(dv, a, stream));
          else
            HIP_TRY(kvm::launch_attn_rows(dv, a, stream));
        }
        if (ch.folds) {
          const int64_t ce = ch.s + C, lo = ce - L;
          ProfileSpan span(st, 1, stream);
          const int rc = lo >= t0 ? fold_block(st, advance(in, lo - t0, es), ce, nullptr, nullptr, stream, true)
                                  : fold_block(st, advance(ring, lo % L, es), ce, nullptr, nullptr, stream, true);
          if (rc != KVM_OK) return rc;
        }
      }
      const int64_t p0 = t_end - L > t0 ? t_end - L : t0;
      HIP_TRY(kvm::launch_ring_copy(dv, in, t0, p0, t_end, stream));
      st->tokens = t_end;
      return KVM_OK;
    }
  }
  // Folds depend only on k, v, g and the previous fold, so they run ahead on their own stream,
  // each writing a fresh readout version; attention follows on the caller's stream in groups
  // of chunks, each group waiting for the last version it reads.  A slot is rewritten only
  // after the attention launch that read its previous version has finished.
  // The fold chain is a sequence of small dependent launches; when a fold moves little data the
  // chain is bound by their latencies, not by bytes, and the batch is split into two halves
  // whose chains run side by side on streams of their own (units are independent).  Two, not
  // more: with four chains the step was measured 40 % to 100 % slower, with four, eight and
  // sixteen hardware queues alike.
  int n_chains = 1;
  {
    int64_t m_max = 0;
    for (const Chunk &ch : plan) m_max = ch.m > m_max ? ch.m : m_max;
    const double fold_mb = (double)dv.U * ((double)m_max * d * es * 5.0 + (double)C * d * es * 4.0) / 1.0e6;
    if (fold_mb < 96.0 && dv.B % 2 == 0) n_chains = 2;
    const int forced = st->dbg[KVM_DEBUG_FOLD_CHAINS];  // 1 or 2: for comparisons
    if ((forced == 1 || forced == 2) && dv.B % forced == 0) n_chains = forced;
    if (use_fused(st)) n_chains = 1;  // one workgroup per unit already: nothing to split
  }
  // The one-launch folds of this schedule take the wide workgroup (16 waves, one per compute
  // unit) unless asked otherwise: measured 7 % to 11 % ahead of the narrow one beside attention.
  // With a unit's rows shared among workgroups the narrow one is the default: it is the shape that
  // fits beside an attention workgroup, and sharing is chosen where the folds are to run hidden.
  const bool narrow_folds = st->dbg[KVM_DEBUG_FOLD_WAVES] == 8 || (st->dbg[KVM_DEBUG_FOLD_WAVES] == 0 && fold_split(st) > 1);
  hipStream_t fstream[kvm_state::kMaxChains];
  Dev cdv[kvm_state::kMaxChains];
  const int cb = dv.B / n_chains;  // sequences per chain
  for (int c2 = 0; c2 < n_chains; ++c2) {
    if (!st->fold_streams[c2]) HIP_TRY(hipStreamCreateWithFlags(&st->fold_streams[c2], hipStreamNonBlocking));
    fstream[c2] = st->fold_streams[c2];
    cdv[c2] = n_chains == 1 ? dv : batch_view(dv, c2 * cb, cb, es);
  }
  // From here on work is forked onto the fold streams.  Whatever happens, the caller's stream
  // waits for them before the call returns: they may still be reading the caller's k, v and gate.
  auto forked = [&]() -> int {
  st->sync_used = 0;
  std::vector<hipEvent_t> slot_busy(dv.NS, nullptr);
  hipEvent_t ev;
  HIP_TRY(next_sync_event(st, &ev));
  HIP_TRY(hipEventRecord(ev, stream));
  for (int c2 = 0; c2 < n_chains; ++c2) HIP_TRY(hipStreamWaitEvent(fstream[c2], ev, 0));
  const int G = st->group;
  const int n_chunks = (int)plan.size();
  int next_fold = 0;                 // folds of chunks < next_fold are enqueued
  hipEvent_t last_fold_ev[kvm_state::kMaxChains] = {nullptr, nullptr};
  hipEvent_t last_att_ev = nullptr;
  auto wait_for_folds = [&]() -> int {
    for (int c2 = 0; c2 < n_chains; ++c2)
      if (last_fold_ev[c2]) HIP_TRY(hipStreamWaitEvent(stream, last_fold_ev[c2], 0));
    return KVM_OK;
  };
  auto enqueue_folds_through = [&](int last_chunk) -> int {
    if (st->isolate && last_att_ev)
      for (int c2 = 0; c2 < n_chains; ++c2) HIP_TRY(hipStreamWaitEvent(fstream[c2], last_att_ev, 0));
    while (next_fold <= last_chunk && next_fold < n_chunks) {
      if (!plan[next_fold].folds) {
        ++next_fold;
        continue;
      }
      // a run of folds whose overflow blocks are consecutive in this call's k: their memory
      // keys are computed by one launch (blocks taken from the ring go one at a time)
      const int64_t lo0 = plan[next_fold].s + C - L;
      int run = 1;
      const int run_cap = use_fused(st) && G > kvm::kFoldMaxSteps ? kvm::kFoldMaxSteps : G;
      if (lo0 >= t0)
        while (run < run_cap && next_fold + run <= last_chunk && next_fold + run < n_chunks &&
               plan[next_fold + run].folds)
          ++run;
      const bool batched = lo0 >= t0;
      // Events cost microseconds each on the queue: one bracket and one ordering event per run
      // of folds, not per fold.  The slots this run rewrites must have been read to the end:
      // one wait per distinct attention launch (usually one), ahead of the run rather than
      // between its folds.
      {
        hipEvent_t waited[2 * kvm::kMaxGroup];
        int n_waited = 0;
        for (int i = 0; i < run; ++i) {
          const int sn = slot_of(st, st->folds + 1 + i);
          hipEvent_t e = slot_busy[sn];
          slot_busy[sn] = nullptr;
          bool seen = e == nullptr;
          for (int k2 = 0; k2 < n_waited && !seen; ++k2) seen = waited[k2] == e;
          if (!seen) {
            for (int c2 = 0; c2 < n_chains; ++c2) HIP_TRY(hipStreamWaitEvent(fstream[c2], e, 0));
            waited[n_waited++] = e;
          }
        }
      }
      // rows and slots of the run's folds (integer arithmetic, the same for every chain)
      struct Step {
        int64_t m, m_after;
        int so, sn;
      };
      Step steps[kvm::kMaxGroup];
      {
        int64_t m = st->m;
        for (int i = 0; i < run; ++i) {
          const int64_t ce = plan[next_fold + i].s + C;
          steps[i].m = m;
          steps[i].m_after = rows_after(c, st->table, m, ce);
          if (steps[i].m_after > dv.Mcap) return KVM_ERR_CAPACITY;
          steps[i].so = slot_of(st, st->folds + i);
          steps[i].sn = slot_of(st, st->folds + i + 1);
          m = steps[i].m_after;
        }
      }
      if (use_fused(st)) {
        ProfileSpan span(st, 1, fstream[0], run);
        kvm::FoldRunArgs fr;
        const int rc_run = fused_run(st, false, fstream[0], &fr);
        if (rc_run != KVM_OK) return rc_run;
        fr.n = run;
        for (int i = 0; i < run; ++i) {
          const int64_t lo = plan[next_fold + i].s + C - L;
          const int64_t fold_no = st->folds + i;
          fr.s[i] = {(int32_t)steps[i].m, (int32_t)steps[i].m_after, steps[i].so, steps[i].sn,
                     batched ? lo - lo0 : 0, fold_no < st->trace_max ? (int32_t)fold_no : -1, i,
                     take_exchanges(st, steps[i].m, steps[i].m_after), 0u};
        }
        const Src fsrc = batched ? advance(in, lo0 - t0, es) : advance(ring, lo0 % L, es);
        HIP_TRY(kvm::launch_memkey(dv, fsrc, run, fstream[0]));
        HIP_TRY(kvm::launch_fold_fused(dv, fsrc, fr, narrow_folds, fstream[0]));
      } else
      for (int c2 = 0; c2 < n_chains; ++c2) {
        // the timing bracket goes on the first chain only (the chains run side by side)
        ProfileSpan span(c2 == 0 ? st : nullptr, 1, fstream[c2], run);
        const Src cin = batch_view(in, c2 * cb, es), cring = batch_view(ring, c2 * cb, es);
        if (batched) HIP_TRY(kvm::launch_memkey(cdv[c2], advance(cin, lo0 - t0, es), run, fstream[c2]));
        for (int i = 0; i < run; ++i) {
          const int64_t lo = plan[next_fold + i].s + C - L;  // first token of the overflow block
          const int rc = batched ? fold_launches(st, cdv[c2], advance(cin, lo - t0, es), steps[i].m, steps[i].m_after,
                                                 steps[i].so, steps[i].sn, false, i, fstream[c2])
                                 : fold_launches(st, cdv[c2], advance(cring, lo % L, es), steps[i].m,
                                                 steps[i].m_after, steps[i].so, steps[i].sn, false, -1, fstream[c2]);
          if (rc != KVM_OK) return rc;
          const int rt = fold_trace(st, cdv[c2], (int64_t)c2 * cb * dv.Hkv, st->folds + i, fstream[c2]);
          if (rt != KVM_OK) return rt;
        }
      }
      st->m = steps[run - 1].m_after;
      st->folds += run;
      for (int c2 = 0; c2 < n_chains; ++c2) {
        HIP_TRY(next_sync_event(st, &last_fold_ev[c2]));
        HIP_TRY(hipEventRecord(last_fold_ev[c2], fstream[c2]));
      }
      next_fold += run;
    }
    return KVM_OK;
  };
  // Groups grow: the first holds the chunks that see the state as the call found it (they wait for
  // no fold), the next ones two and four chunks, so that attention starts at once and has work
  // while the first folds of the chain run; from then on G chunks per launch.
  int first = 0;
  while (first < n_chunks && first < G && plan[first].ver == plan[0].ver) ++first;
  int gsz = first;
  for (int g0 = 0, g1 = 0; g0 < n_chunks; g0 = g1) {
    g1 = g0 + gsz < n_chunks ? g0 + gsz : n_chunks;
    gsz = g0 == 0 ? 2 : 2 * gsz;
    gsz = gsz > G ? G : gsz;
    // the last chunk of the group reads the version written by the fold after chunk g1 - 2
    int rc = enqueue_folds_through(g1 - 2);
    if (rc != KVM_OK) return rc;
    rc = wait_for_folds();
    if (rc != KVM_OK) return rc;
    AttnArgs a;
    a.put_token = 0;  // a prefill copies its last L tokens into the ring once, at the end
    const int64_t cs = plan[g0].s;
    a.q = (const char *)q + (cs - t0) * s.q_t * (int64_t)es;
    a.out = (char *)out + (cs - t0) * s.o_t * (int64_t)es;
    a.lse = lse ? lse + (cs - t0) * s.lse_t : nullptr;
    a.q_b = s.q_b; a.q_t = s.q_t; a.q_h = s.q_h;
    a.o_b = s.o_b; a.o_t = s.o_t; a.o_h = s.o_h;
    a.lse_b = s.lse_b; a.lse_t = s.lse_t; a.lse_h = s.lse_h;
    a.in = in;
    a.t0 = t0;
    a.s = cs;
    a.n_chunks = g1 - g0;
    a.nq_total = (int32_t)((g1 - 1 - g0) * C + plan[g1 - 1].nq);
    for (int i = 0; i < kvm::kMaxGroup; ++i) {
      a.m[i] = i < g1 - g0 ? plan[g0 + i].m : 0;
      a.slot[i] = i < g1 - g0 ? (int32_t)slot_of(st, plan[g0 + i].ver) : 0;
    }
    {
      ProfileSpan span(st, 0, stream);
      if (st->mfma)
        HIP_TRY(kvm::launch_attn_mfma(dv, a, stream));
      else
        HIP_TRY(kvm::launch_attn_rows(dv, a, stream));
    }
    HIP_TRY(next_sync_event(st, &ev));
    HIP_TRY(hipEventRecord(ev, stream));
    for (int i = g0; i < g1; ++i) slot_busy[slot_of(st, plan[i].ver)] = ev;
    last_att_ev = ev;
  }
  {
    int rc = enqueue_folds_through(n_chunks - 1);
    if (rc != KVM_OK) return rc;
    rc = wait_for_folds();
    if (rc != KVM_OK) return rc;
  }
  return KVM_OK;
  };
  const int rc_forked = forked();
  if (rc_forked != KVM_OK) {
    // best effort (the runtime has already failed once): join the fold streams back
    for (int c2 = 0; c2 < n_chains; ++c2) {
      hipEvent_t e = nullptr;
      if (next_sync_event(st, &e) == hipSuccess && hipEventRecord(e, fstream[c2]) == hipSuccess)
        (void)hipStreamWaitEvent(stream, e, 0);
    }
    return rc_forked;
  }
  // keep the last L tokens for the calls that follow
  const int64_t p0 = t_end - L > t0 ? t_end - L : t0;
  HIP_TRY(kvm::launch_ring_copy(dv, in, t0, p0, t_end, stream));
  st->tokens = t_end;
  return KVM_OK;
}

int kvm_decode_step(kvm_state *st, const void *q, const void *k, const void *v,
                    const float *gate, void *out, void *stream_) {
  if (!st || !q || !k || !v || !out) return KVM_ERR_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return KVM_ERR_ARG;
  if (cluster_error(st) != KVM_OK) return KVM_ERR_HIP;
  hipStream_t stream = (hipStream_t)stream_;
  const kvm_config &c = st->cfg;
  const Dev &dv = st->dv;
  const int64_t C = dv.C, L = dv.L, d = dv.d;
  const size_t es = esize(c.io_dtype);
  const int64_t u = st->tokens;
  const bool completes = (u + 1) % C == 0 && u + 1 >= L;
  if (completes && rows_after(c, st->table, st->m, u + 1) > dv.Mcap) return KVM_ERR_CAPACITY;

  Src tok;
  tok.k = k; tok.v = v; tok.g = gate;
  tok.k_b = tok.v_b = dv.Hkv * d; tok.k_h = tok.v_h = d; tok.k_t = tok.v_t = 0;
  tok.g_b = dv.Hkv; tok.g_h = 1; tok.g_t = 0;

  AttnArgs a;
  a.q = q; a.out = out; a.lse = nullptr;
  a.q_b = a.o_b = dv.Hq * d; a.q_t = a.o_t = 0; a.q_h = a.o_h = d;
  a.lse_b = a.lse_t = a.lse_h = 0;
  a.in = tok;
  a.t0 = u;           // the new token is read from the call's k, v; older ones from the ring
  a.put_token = 1;    // and stored into the ring by the same launch
  a.s = u;
  a.n_chunks = 1;
  a.nq_total = 1;
  for (int i = 0; i < kvm::kMaxGroup; ++i) {
    a.m[i] = (int32_t)st->m;
    a.slot[i] = (int32_t)slot_of(st, st->folds);
  }
  {
    ProfileSpan span(st, 2, stream);
    HIP_TRY(kvm::launch_attn_rows(dv, a, stream));
  }
  st->tokens = u + 1;
  if (completes) {
    const int64_t lo = u + 1 - L;
    ProfileSpan span(st, 1, stream);
    int rc = fold_block(st, advance(ring_src(st), lo % L, es), u + 1, nullptr, nullptr, stream, true);
    if (rc != KVM_OK) return rc;
  }
  return KVM_OK;
}

size_t kvm_decode_multi_workspace_bytes(int64_t n_sequences) {
  return n_sequences > 0 ? (size_t)n_sequences * sizeof(kvm::SeqDesc) : 0;
}

int kvm_decode_step_multi(kvm_state *const *states, int32_t n_states, const void *q, const void *k,
                          const void *v, const float *gate, void *out, void *workspace,
                          size_t workspace_bytes, void *stream_) {
  if (!states || n_states <= 0 || !q || !k || !v || !out || !workspace) return KVM_ERR_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(workspace))
    return KVM_ERR_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  const kvm_state *first = states[0];
  if (!first) return KVM_ERR_ARG;
  const kvm_config &c0 = first->cfg;
  int64_t n_seq = 0;
  for (int i = 0; i < n_states; ++i) {
    const kvm_state *st = states[i];
    if (!st) return KVM_ERR_ARG;
    for (int j = 0; j < i; ++j)
      if (states[j] == st) return KVM_ERR_ARG;  // a state takes one token per step
    const kvm_config &c = st->cfg;
    if (c.n_q_heads != c0.n_q_heads || c.n_kv_heads != c0.n_kv_heads || c.head_dim != c0.head_dim ||
        c.io_dtype != c0.io_dtype || c.chunk_len != c0.chunk_len || c.n_bswa_chunks != c0.n_bswa_chunks ||
        c.n_sink != c0.n_sink || c.rope_dims != c0.rope_dims || c.tau_state != c0.tau_state ||
        c.tau_bswa != c0.tau_bswa)
      return KVM_ERR_ARG;
    n_seq += st->dv.B;
  }
  if (workspace_bytes < kvm_decode_multi_workspace_bytes(n_seq)) return KVM_ERR_ARG;
  const int64_t C = first->dv.C, L = first->dv.L, d = first->dv.d;
  const size_t es = esize(c0.io_dtype);
  // capacity of every fold this step triggers, before anything is enqueued
  for (int i = 0; i < n_states; ++i) {
    const kvm_state *st = states[i];
    const int64_t u = st->tokens;
    if ((u + 1) % C == 0 && u + 1 >= L && rows_after(st->cfg, st->table, st->m, u + 1) > st->dv.Mcap)
      return KVM_ERR_CAPACITY;
  }
  std::vector<kvm::SeqDesc> desc((size_t)n_seq);
  size_t s = 0;
  for (int i = 0; i < n_states; ++i) {
    const kvm_state *st = states[i];
    const Dev &dv = st->dv;
    const int64_t slot = slot_of(st, st->folds);
    for (int b = 0; b < dv.B; ++b, ++s) {
      const int64_t u0 = (int64_t)b * dv.Hkv;
      kvm::SeqDesc &sd = desc[s];
      sd.khat = (const char *)dv.khat + (slot * dv.slot_elems + u0 * dv.Mcap * d) * es;
      sd.vhat = (const char *)dv.vhat + (slot * dv.slot_elems + u0 * dv.Mcap * d) * es;
      sd.winK = (char *)dv.winK + u0 * L * d * es;
      sd.winV = (char *)dv.winV + u0 * L * d * es;
      sd.winG = dv.winG + u0 * L;
      sd.pos = st->tokens;
      sd.m = (int32_t)st->m;
      sd.Mcap = dv.Mcap;
    }
  }
  // pageable source: the copy is staged before the call returns, and ordered on the stream
  HIP_TRY(hipMemcpyAsync(workspace, desc.data(), desc.size() * sizeof(kvm::SeqDesc), hipMemcpyHostToDevice,
                         stream));
  {
    ProfileSpan span(states[0], 2, stream);
    HIP_TRY(kvm::launch_decode_multi(first->dv, (const kvm::SeqDesc *)workspace, (int)n_seq, q, k, v, gate, out,
                                     stream));
  }
  for (int i = 0; i < n_states; ++i) {
    kvm_state *st = states[i];
    const int64_t u = st->tokens;
    st->tokens = u + 1;
    if ((u + 1) % C == 0 && u + 1 >= L) {
      const int64_t lo = u + 1 - L;
      ProfileSpan span(st, 1, stream);
      int rc = fold_block(st, advance(ring_src(st), lo % L, es), u + 1, nullptr, nullptr, stream, true);
      if (rc != KVM_OK) return rc;
    }
  }
  return KVM_OK;
}

int kvm_decode_step_multi_static(kvm_state *const *states, int32_t n_states, const void *q, const void *k,
                                 const void *v, const float *gate, void *out, void *stream_) {
  if (!states || n_states <= 0 || !q || !k || !v || !out) return KVM_ERR_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return KVM_ERR_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  const kvm_state *first = states[0];
  if (!first) return KVM_ERR_ARG;
  const kvm_config &c0 = first->cfg;
  int64_t n_seq = 0;
  for (int i = 0; i < n_states; ++i) {
    const kvm_state *st = states[i];
    if (!st) return KVM_ERR_ARG;
    for (int j = 0; j < i; ++j)
      if (states[j] == st) return KVM_ERR_ARG;  // a state takes one token per step
    const kvm_config &c = st->cfg;
    if (c.n_q_heads != c0.n_q_heads || c.n_kv_heads != c0.n_kv_heads || c.head_dim != c0.head_dim ||
        c.io_dtype != c0.io_dtype || c.chunk_len != c0.chunk_len || c.n_bswa_chunks != c0.n_bswa_chunks ||
        c.n_sink != c0.n_sink || c.rope_dims != c0.rope_dims || c.tau_state != c0.tau_state ||
        c.tau_bswa != c0.tau_bswa)
      return KVM_ERR_ARG;
    n_seq += st->dv.B;
  }
  if (n_seq > kStaticMaxSeq) {
    g_hip_error = "kvm_decode_step_multi_static: " + std::to_string(n_seq) + " sequences, the static table holds " +
                  std::to_string(kStaticMaxSeq);
    return KVM_ERR_LIMIT;
  }
  const int64_t C = first->dv.C, L = first->dv.L, d = first->dv.d;
  const size_t es = esize(c0.io_dtype);
  for (int i = 0; i < n_states; ++i) {
    const kvm_state *st = states[i];
    const int64_t u = st->tokens;
    if ((u + 1) % C == 0 && u + 1 >= L && rows_after(st->cfg, st->table, st->m, u + 1) > st->dv.Mcap)
      return KVM_ERR_CAPACITY;
  }
  void *table = nullptr;
  {
    const int rc = scratch_on_device(&table);
    if (rc != KVM_OK) return rc;
  }
  // the descriptor table, kPackStates states per launch
  for (int i0 = 0, seq0 = 0; i0 < n_states; i0 += kPackStates) {
    StatePack pk;
    pk.n = n_states - i0 < kPackStates ? n_states - i0 : kPackStates;
    int sq = seq0;
    for (int i = 0; i < pk.n; ++i) {
      const kvm_state *st = states[i0 + i];
      const Dev &dv = st->dv;
      const int64_t slot = slot_of(st, st->folds);
      pk.khat[i] = (const char *)dv.khat + slot * dv.slot_elems * (int64_t)es;
      pk.vhat[i] = (const char *)dv.vhat + slot * dv.slot_elems * (int64_t)es;
      pk.winK[i] = dv.winK;
      pk.winV[i] = dv.winV;
      pk.winG[i] = dv.winG;
      pk.pos[i] = st->tokens;
      pk.m[i] = (int32_t)st->m;
      pk.Mcap[i] = dv.Mcap;
      pk.seq0[i] = sq;
      sq += dv.B;
    }
    pk.seq0[pk.n] = sq;
    for (int i = pk.n + 1; i <= kPackStates; ++i) pk.seq0[i] = sq;
    const int n_here = sq - seq0;
    hipLaunchKernelGGL(seqdesc_fill_kernel, dim3((n_here + 255) / 256), dim3(256), 0, stream, pk,
                       (kvm::SeqDesc *)table, (int)first->dv.Hkv, (int)L, (int)d, (int)es);
    HIP_TRY(hipGetLastError());
    seq0 = sq;
  }
  {
    ProfileSpan span(states[0], 2, stream);
    HIP_TRY(kvm::launch_decode_multi(first->dv, (const kvm::SeqDesc *)table, (int)n_seq, q, k, v, gate, out, stream));
  }
  for (int i = 0; i < n_states; ++i) {
    kvm_state *st = states[i];
    const int64_t u = st->tokens;
    st->tokens = u + 1;
    if ((u + 1) % C == 0 && u + 1 >= L) {
      const int64_t lo = u + 1 - L;
      ProfileSpan span(st, 1, stream);
      int rc = fold_block(st, advance(ring_src(st), lo % L, es), u + 1, nullptr, nullptr, stream, true);
      if (rc != KVM_OK) return rc;
    }
  }
  return KVM_OK;
}

int kvm_state_fold(kvm_state *st, const void *k_blk, const void *v_blk, const float *gate_blk,
                   int32_t n_tokens, int64_t e, int32_t *assign_out, float *score_out,
                   void *stream_) {
  if (!st || !k_blk || !v_blk) return KVM_ERR_ARG;
  if (n_tokens != st->dv.C) return KVM_ERR_ARG;
  if (!aligned16(k_blk) || !aligned16(v_blk)) return KVM_ERR_ARG;
  if (cluster_error(st) != KVM_OK) return KVM_ERR_HIP;
  const Dev &dv = st->dv;
  Src src;
  src.k = k_blk; src.v = v_blk; src.g = gate_blk;
  src.k_b = src.v_b = (int64_t)n_tokens * dv.Hkv * dv.d;
  src.k_t = src.v_t = (int64_t)dv.Hkv * dv.d;
  src.k_h = src.v_h = dv.d;
  src.g_b = (int64_t)n_tokens * dv.Hkv; src.g_t = dv.Hkv; src.g_h = 1;
  if (st->cfg.budget_kind != KVM_BUDGET_NONE &&
      rows_after(st->cfg, st->table, st->m, e) > dv.Mcap)
    return KVM_ERR_CAPACITY;
  return fold_block(st, src, e, assign_out, score_out, (hipStream_t)stream_, true);
}

size_t kvm_backward_workspace_bytes(const kvm_state *st, int64_t T) {
  if (!st || T <= 0) return 0;
  return bwd_layout(st->cfg, st->dv.Mcap, T, bwd_on_mfma(st)).total;
}

int kvm_prefill_backward(kvm_state *st, const void *q, const void *k, const void *v, const float *gate,
                         const void *out, const float *lse, const void *dout, const int32_t *assign,
                         const float *score, const kvm_grads *grads, int64_t T, void *workspace,
                         size_t workspace_bytes, void *stream) {
  if (!st || !q || !k || !v || !out || !lse || !dout || !grads || !workspace || T <= 0) return KVM_ERR_ARG;
  if (!grads->dq || !grads->dk || !grads->dv || !grads->dgate || !grads->dgamma || !grads->dbeta ||
      !grads->dtau_state || !grads->dtau_bswa)
    return KVM_ERR_ARG;
  const kvm_config &c = st->cfg;
  const int64_t C = c.chunk_len, L = C * c.n_bswa_chunks;
  // the state must be the one a forward over exactly these T tokens, from empty, has left
  std::vector<kvm::BwdChunk> chunks;
  int64_t m = 0, folds = 0;
  for (int64_t s = 0; s < T; s += C) {
    const int64_t e = s + C < T ? s + C : T;
    kvm::BwdChunk ch;
    ch.s = s;
    ch.nq = (int32_t)(e - s);
    ch.m = (int32_t)m;
    ch.fold = -1;
    if (e == s + C && e >= L && c.budget_kind != KVM_BUDGET_NONE) {
      ch.fold = (int32_t)folds++;
      m = rows_after(c, st->table, m, e);
    }
    ch.m_after = (int32_t)m;
    chunks.push_back(ch);
  }
  if (st->tokens != T || st->folds != folds || st->m != m) return KVM_ERR_STATE;
  if (folds > 0 && (!assign || !score)) return KVM_ERR_ARG;
  const bool on_mfma = bwd_on_mfma(st);
  const BwdLayout l = bwd_layout(c, st->dv.Mcap, T, on_mfma);
  if (workspace_bytes < l.total || ((uintptr_t)workspace & 255)) return KVM_ERR_ARG;
  const void *ptrs[] = {q, k, v, out, dout, grads->dq, grads->dk, grads->dv};
  for (const void *p : ptrs)
    if (!aligned16(p)) return KVM_ERR_ARG;
  kvm::Bwd a;
  a.dv = st->dv;
  a.on_mfma = on_mfma;
  a.T = T;
  a.q = q; a.k = k; a.v = v; a.out = out; a.dout = dout;
  a.gate = gate; a.lse = lse; a.assign = assign; a.score = score;
  a.dq = grads->dq; a.dk = grads->dk; a.dv_out = grads->dv;
  a.dgate = grads->dgate; a.dgamma = grads->dgamma; a.dbeta = grads->dbeta;
  a.dtau_state = grads->dtau_state; a.dtau_bswa = grads->dtau_bswa;
  char *w = (char *)workspace;
  a.wsK = (double *)(w + l.wsK); a.wsV = (float *)(w + l.wsV);
  a.dsK = (float *)(w + l.dsK); a.dsV = (float *)(w + l.dsV); a.drho = (float *)(w + l.drho);
  a.khat = w + l.khat; a.vhat = w + l.vhat;
  a.xhat = (float *)(w + l.xhat); a.rden = (float *)(w + l.rden);
  a.dkhat = (float *)(w + l.dkhat); a.dvhat = (float *)(w + l.dvhat);
  a.dk_acc = (float *)(w + l.dk_acc); a.dv_acc = (float *)(w + l.dv_acc);
  a.delta = (float *)(w + l.delta);
  a.ring_rows = 0;
  a.P = (float *)(w + l.P); a.dS = (float *)(w + l.dS);
  a.par64 = (double *)(w + l.par64);
  kvm::BwdStreams x;
  if (on_mfma) {
    for (hipStream_t &fs : st->fold_streams)
      if (!fs) HIP_TRY(hipStreamCreateWithFlags(&fs, hipStreamNonBlocking));
    x.side = st->fold_streams[0];
    x.side2 = st->fold_streams[1];
    st->sync_used = 0;
    for (hipEvent_t *e : {&x.fork, &x.dq_done, &x.join_state, &x.join_window[0], &x.join_window[1]})
      HIP_TRY(next_sync_event(st, e));
  }
  const hipError_t e_run = kvm::run_backward(a, chunks.data(), (int)chunks.size(), (hipStream_t)stream, x);
  if (e_run != hipSuccess) {
    // the side streams may still be reading the caller's tensors: join them back (best effort)
    for (hipStream_t side : {x.side, x.side2}) {
      hipEvent_t e = nullptr;
      if (side && next_sync_event(st, &e) == hipSuccess && hipEventRecord(e, side) == hipSuccess)
        (void)hipStreamWaitEvent((hipStream_t)stream, e, 0);
    }
    return hip_fail(e_run, "kvm::run_backward");
  }
  return KVM_OK;
}

int kvm_state_rows(const kvm_state *st, int64_t *m_out) {
  if (!st || !m_out) return KVM_ERR_ARG;
  *m_out = st->m;
  return KVM_OK;
}
int kvm_state_tokens(const kvm_state *st, int64_t *tokens_seen) {
  if (!st || !tokens_seen) return KVM_ERR_ARG;
  *tokens_seen = st->tokens;
  return KVM_OK;
}
int kvm_state_capacity(const kvm_state *st, int64_t *rows_out) {
  if (!st || !rows_out) return KVM_ERR_ARG;
  *rows_out = st->dv.Mcap;
  return KVM_OK;
}
int kvm_state_fold_path(const kvm_state *st, int64_t *path_out) {
  if (!st || !path_out) return KVM_ERR_ARG;
  *path_out = use_fused(st) ? 1 : 2;
  return KVM_OK;
}
int kvm_state_folds(const kvm_state *st, int64_t *folds_out) {
  if (!st || !folds_out) return KVM_ERR_ARG;
  *folds_out = st->folds;
  return KVM_OK;
}

int kvm_state_trace(kvm_state *st, int32_t *assign, float *score, int64_t max_folds) {
  if (!st || max_folds < 0) return KVM_ERR_ARG;
  st->trace_assign = assign;
  st->trace_score = score;
  st->trace_max = (assign || score) ? max_folds : 0;
  return KVM_OK;
}

int kvm_state_grow(kvm_state *st, void *new_buf, size_t new_bytes, int64_t new_max_tokens,
                   void *stream_) {
  if (!st || !new_buf || ((uintptr_t)new_buf & 255) != 0) return KVM_ERR_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  const kvm_config &c = st->cfg;
  const int64_t Mnew = capacity_rows(c, st->table, new_max_tokens);
  if (Mnew < st->m) return KVM_ERR_CAPACITY;
  if (layout_of(c, Mnew).total > new_bytes) return KVM_ERR_CAPACITY;
  Dev nd = st->dv;
  bind(nd, c, new_buf, Mnew);
  const Dev &od = st->dv;
  const size_t U = od.U, d = od.d, es = esize(c.io_dtype), m = (size_t)st->m;
  auto copy2d = [&](void *dst, const void *src, size_t row_bytes) -> hipError_t {
    if (m == 0) return hipSuccess;
    return hipMemcpy2DAsync(dst, (size_t)Mnew * row_bytes, src, (size_t)od.Mcap * row_bytes,
                            m * row_bytes, U, hipMemcpyDeviceToDevice, stream);
  };
  HIP_TRY(copy2d(nd.sK, od.sK, d * 8));
  HIP_TRY(copy2d(nd.sV, od.sV, d * 4));
  HIP_TRY(copy2d(nd.rho, od.rho, 4));
  HIP_TRY(copy2d(nd.w, od.w, 4));
  HIP_TRY(copy2d(nd.n, od.n, 4));
  const int64_t slot = slot_of(st, st->folds);  // only the current version is live
  HIP_TRY(copy2d((char *)nd.khat + slot * nd.slot_elems * (int64_t)es,
                 (const char *)od.khat + slot * od.slot_elems * (int64_t)es, d * es));
  HIP_TRY(copy2d((char *)nd.vhat + slot * nd.slot_elems * (int64_t)es,
                 (const char *)od.vhat + slot * od.slot_elems * (int64_t)es, d * es));
  const size_t win = U * od.L * d * es;
  HIP_TRY(hipMemcpyAsync(nd.winK, od.winK, win, hipMemcpyDeviceToDevice, stream));
  HIP_TRY(hipMemcpyAsync(nd.winV, od.winV, win, hipMemcpyDeviceToDevice, stream));
  HIP_TRY(hipMemcpyAsync(nd.winG, od.winG, U * od.L * 4, hipMemcpyDeviceToDevice, stream));
  st->dv = nd;
  st->buf = new_buf;
  st->bytes = new_bytes;
  {
    const Layout l = layout_of(c, Mnew);
    st->xtab = l.xtab_bytes ? (unsigned long long *)((char *)new_buf + l.xtab) : nullptr;
    st->xtab_bytes = l.xtab_bytes;
    st->xtab_clean = false;
  }
  st->fused = st->mfma && kvm::fold_fused_fits(st->dv);
  return KVM_OK;
}

int kvm_state_export(const kvm_state *st, double *sK, float *sV, float *rho, float *w,
                     int32_t *n, void *khat, void *vhat, void *win_k, void *win_v,
                     float *win_g, void *stream_) {
  if (!st) return KVM_ERR_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  const Dev &dv = st->dv;
  const size_t U = dv.U, d = dv.d, es = esize(st->cfg.io_dtype), m = (size_t)st->m;
  auto out2d = [&](void *dst, const void *src, size_t row_bytes) -> hipError_t {
    if (!dst || m == 0) return hipSuccess;
    return hipMemcpy2DAsync(dst, m * row_bytes, src, (size_t)dv.Mcap * row_bytes, m * row_bytes, U,
                            hipMemcpyDeviceToDevice, stream);
  };
  HIP_TRY(out2d(sK, dv.sK, d * 8));
  HIP_TRY(out2d(sV, dv.sV, d * 4));
  HIP_TRY(out2d(rho, dv.rho, 4));
  HIP_TRY(out2d(w, dv.w, 4));
  HIP_TRY(out2d(n, dv.n, 4));
  const int64_t slot_off = slot_of(st, st->folds) * dv.slot_elems * (int64_t)es;
  HIP_TRY(out2d(khat, (const char *)dv.khat + slot_off, d * es));
  HIP_TRY(out2d(vhat, (const char *)dv.vhat + slot_off, d * es));
  const size_t win = U * dv.L * d * es;
  if (win_k) HIP_TRY(hipMemcpyAsync(win_k, dv.winK, win, hipMemcpyDeviceToDevice, stream));
  if (win_v) HIP_TRY(hipMemcpyAsync(win_v, dv.winV, win, hipMemcpyDeviceToDevice, stream));
  if (win_g) HIP_TRY(hipMemcpyAsync(win_g, dv.winG, U * dv.L * 4, hipMemcpyDeviceToDevice, stream));
  return KVM_OK;
}

int kvm_state_import(kvm_state *st, const double *sK, const float *sV, const float *rho,
                     const float *w, const int32_t *n, const void *win_k, const void *win_v,
                     const float *win_g, int64_t m, int64_t tokens_seen, int64_t folds,
                     void *stream_) {
  if (!st || m < 0 || tokens_seen < 0 || folds < 0) return KVM_ERR_ARG;
  if (m > 0 && (!sK || !sV || !rho)) return KVM_ERR_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  const Dev &dv = st->dv;
  if (m > dv.Mcap) return KVM_ERR_CAPACITY;
  const size_t U = dv.U, d = dv.d, es = esize(st->cfg.io_dtype), mm = (size_t)m;
  auto in2d = [&](void *dst, const void *src, size_t row_bytes) -> hipError_t {
    if (!src || mm == 0) return hipSuccess;
    return hipMemcpy2DAsync(dst, (size_t)dv.Mcap * row_bytes, src, mm * row_bytes, mm * row_bytes, U,
                            hipMemcpyDeviceToDevice, stream);
  };
  HIP_TRY(in2d(dv.sK, sK, d * 8));
  HIP_TRY(in2d(dv.sV, sV, d * 4));
  HIP_TRY(in2d(dv.rho, rho, 4));
  HIP_TRY(in2d(dv.w, w, 4));
  HIP_TRY(in2d(dv.n, n, 4));
  const size_t win = U * dv.L * d * es;
  if (win_k) HIP_TRY(hipMemcpyAsync(dv.winK, win_k, win, hipMemcpyDeviceToDevice, stream));
  if (win_v) HIP_TRY(hipMemcpyAsync(dv.winV, win_v, win, hipMemcpyDeviceToDevice, stream));
  if (win_g) HIP_TRY(hipMemcpyAsync(dv.winG, win_g, U * dv.L * 4, hipMemcpyDeviceToDevice, stream));
  if (use_fused(st))
    HIP_TRY(kvm::launch_refresh16(dv, (int)m, slot_of(st, folds), stream));
  else
    HIP_TRY(kvm::launch_refresh(dv, (int)m, slot_of(st, folds), stream));
  st->m = m;
  st->tokens = tokens_seen;
  st->folds = folds;
  return KVM_OK;
}

}  // extern "C"
