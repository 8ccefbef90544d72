// Row attention: one workgroup per (query, query head, sequence) runs the single softmax of the
// paper's "Readout" equations over [normalised state rows || visible window tokens], streaming
// keys and values once from HBM.  This is the decode kernel (one query per sequence, memory
// bound) and also serves fp32 prefill, where every query of a chunk gets its own workgroup.
//
// A key row of D elements is read by D/VEC adjacent lanes with one 16-byte load each, so a wave
// covers 64/(D/VEC) keys per step; each such lane group keeps its own online-softmax state
// (running max, sum, output fragment) and the groups are merged at the end.
#include "kvm_device.h"
#include "kvm_internal.h"

namespace kvm {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// What one workgroup needs, gathered by the kernels below: a query position of one unit and GQ
// consecutive query heads of it (GQ = 1: one head; in a decode step with grouped queries a
// workgroup takes a KV head's whole group, so that every key and value row is fetched once for
// all of its heads instead of once per head).
template <typename T>
struct RowQuery {
  const T *q, *khat, *vhat, *ring_k, *ring_v, *in_k, *in_v;  // first head's query row, this unit's arrays
  T *out;            // first head's output row
  float *lse;        // first head's slot, or null
  int64_t q_h, o_h, lse_h;  // element strides between the heads
  int64_t pos, t0;   // query position; window positions below t0 come from the ring
  int64_t in_kt, in_vt;
  int m, hq;         // state rows; first head
  // decode: the workgroup that holds a KV head's first query head also stores the new token (k,
  // v, gate at position pos, read from in_k / in_v like every key at or after t0) into its ring
  // slot; nobody reads that slot in this launch
  T *put_k, *put_v;  // ring rows of this unit, or null
  float *put_g;
  float gate;
};

template <typename T, int D, int GQ>
__device__ __forceinline__ void attn_row(const Dev &dv, const RowQuery<T> &rq) {
  constexpr int VEC = Vec16<T>::kN;
  constexpr int LPR = D / VEC;   // lanes per key row
  constexpr int RPW = 64 / LPR;  // key rows per wave step
  constexpr int KB = 4;          // rows in flight per lane group
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPR, cl = lane % LPR;
  const int64_t pos = rq.pos;
  const int64_t cs = pos / dv.C * dv.C;                      // its chunk starts here
  const int64_t wb = cs + dv.C - dv.L > 0 ? cs + dv.C - dv.L : 0;  // first window position

  if (rq.put_k && threadIdx.x < LPR) {
    const int slot = (int)(pos % dv.L);
    float x[VEC];
    Vec16<T>::load(rq.in_k + (pos - rq.t0) * rq.in_kt + threadIdx.x * VEC, x);
    Vec16<T>::store(rq.put_k + (int64_t)slot * D + threadIdx.x * VEC, x);
    Vec16<T>::load(rq.in_v + (pos - rq.t0) * rq.in_vt + threadIdx.x * VEC, x);
    Vec16<T>::store(rq.put_v + (int64_t)slot * D + threadIdx.x * VEC, x);
    if (threadIdx.x == 0) rq.put_g[slot] = rq.gate;
  }
  const float rs = kLog2e * rsqrtf((float)D);
  float qf[GQ][VEC], c_state[GQ], c_bswa[GQ];
#pragma unroll
  for (int hh = 0; hh < GQ; ++hh) {
    Vec16<T>::load(rq.q + hh * rq.q_h + cl * VEC, qf[hh]);
    c_state[hh] = (dv.tau_state ? dv.tau_state[rq.hq + hh] : 1.f) * rs;
    c_bswa[hh] = (dv.tau_bswa ? dv.tau_bswa[rq.hq + hh] : 1.f) * rs;
  }

  const int m = rq.m;
  const int total = m + (int)(pos - wb + 1);
  const T *khat = rq.khat, *vhat = rq.vhat, *ring_k = rq.ring_k, *ring_v = rq.ring_v;
  const T *in_k = rq.in_k, *in_v = rq.in_v;

  float m_run[GQ], l_run[GQ], acc[GQ][VEC];
#pragma unroll
  for (int hh = 0; hh < GQ; ++hh) {
    m_run[hh] = -INFINITY;
    l_run[hh] = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[hh][i] = 0.f;
  }

  for (int n0 = 0; n0 < total; n0 += 4 * RPW * KB) {
    float kf[KB][VEC], vf[KB][VEC];
    bool is_state[KB], on[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      const int n = n0 + (kb * 4 + wave) * RPW + sub;
      const int nc = n < total ? n : total - 1;
      const T *kp, *vp;
      if (nc < m) {
        kp = khat + (int64_t)nc * D;
        vp = vhat + (int64_t)nc * D;
      } else {
        const int64_t p = wb + (nc - m);
        if (p >= rq.t0) {
          kp = in_k + (p - rq.t0) * rq.in_kt;
          vp = in_v + (p - rq.t0) * rq.in_vt;
        } else {
          const int slot = (int)(p % dv.L);
          kp = ring_k + (int64_t)slot * D;
          vp = ring_v + (int64_t)slot * D;
        }
      }
      Vec16<T>::load(kp + cl * VEC, kf[kb]);
      Vec16<T>::load(vp + cl * VEC, vf[kb]);
      on[kb] = n < total;
      is_state[kb] = nc < m;
    }
#pragma unroll
    for (int hh = 0; hh < GQ; ++hh) {
      float t[KB];
      float m_new = m_run[hh];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) dot = fmaf(qf[hh][i], kf[kb][i], dot);
        dot = group_sum<LPR>(dot);  // over the lanes that share the key row, on the vector ALU
        t[kb] = on[kb] ? dot * (is_state[kb] ? c_state[hh] : c_bswa[hh]) : -INFINITY;
        m_new = fmaxf(m_new, t[kb]);
      }
      if (m_new != -INFINITY) {
        const float alpha = exp2f(m_run[hh] - m_new);
        l_run[hh] *= alpha;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[hh][i] *= alpha;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const float p = exp2f(t[kb] - m_new);
          l_run[hh] += p;
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[hh][i] = fmaf(p, vf[kb][i], acc[hh][i]);
        }
        m_run[hh] = m_new;
      }
    }
  }

  __shared__ float sh_m[GQ][4], sh_l[GQ][4], sh_acc[GQ][4][D];
#pragma unroll
  for (int hh = 0; hh < GQ; ++hh) {
    // merge the lane groups of this wave
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      const float m_o = __shfl_xor(m_run[hh], o, kWave);
      const float l_o = __shfl_xor(l_run[hh], o, kWave);
      const float m_n = fmaxf(m_run[hh], m_o);
      const float sa = m_n == -INFINITY ? 0.f : exp2f(m_run[hh] - m_n);
      const float sb = m_n == -INFINITY ? 0.f : exp2f(m_o - m_n);
      l_run[hh] = l_run[hh] * sa + l_o * sb;
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[hh][i] = acc[hh][i] * sa + __shfl_xor(acc[hh][i], o, kWave) * sb;
      m_run[hh] = m_n;
    }
    if (sub == 0) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) sh_acc[hh][wave][cl * VEC + i] = acc[hh][i];
      if (cl == 0) {
        sh_m[hh][wave] = m_run[hh];
        sh_l[hh][wave] = l_run[hh];
      }
    }
  }
  __syncthreads();
  // merge the four waves: wave hh % 4 finishes head hh
#pragma unroll
  for (int hh = 0; hh < GQ; ++hh) {
    if (wave == (hh & 3) && sub == 0) {
      const float mm = fmaxf(fmaxf(sh_m[hh][0], sh_m[hh][1]), fmaxf(sh_m[hh][2], sh_m[hh][3]));
      float l = 0.f, o[VEC];
#pragma unroll
      for (int i = 0; i < VEC; ++i) o[i] = 0.f;
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) {
        const float sc = exp2f(sh_m[hh][wv] - mm);  // a wave that saw no key has max -inf -> 0
        l += sh_l[hh][wv] * sc;
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] += sh_acc[hh][wv][cl * VEC + i] * sc;
      }
      const float inv = 1.f / l;
#pragma unroll
      for (int i = 0; i < VEC; ++i) o[i] *= inv;
      Vec16<T>::store(rq.out + hh * rq.o_h + cl * VEC, o);
      if (rq.lse && cl == 0) rq.lse[hh * rq.lse_h] = (mm + log2f(l)) * kLn2;
    }
  }
}

// One workgroup per (query, group of GQ query heads, sequence) of one state.
template <typename T, int D, int GQ>
__global__ __launch_bounds__(256) void attn_rows_kernel(Dev dv, AttnArgs a) {
  const int qi = blockIdx.x, hq = blockIdx.y * GQ, b = blockIdx.z;
  const int hkv = hq / (dv.Hq / dv.Hkv);
  const int u = b * dv.Hkv + hkv;
  RowQuery<T> rq;
  rq.pos = a.s + qi;
  const int ci = (int)(rq.pos / dv.C - a.s / dv.C);  // chunk of this query within the launch
  rq.q = (const T *)a.q + b * a.q_b + (int64_t)qi * a.q_t + hq * a.q_h;
  rq.out = (T *)a.out + b * a.o_b + (int64_t)qi * a.o_t + hq * a.o_h;
  rq.lse = a.lse ? a.lse + b * a.lse_b + (int64_t)qi * a.lse_t + hq * a.lse_h : nullptr;
  rq.q_h = a.q_h;
  rq.o_h = a.o_h;
  rq.lse_h = a.lse_h;
  rq.m = a.m[ci];
  rq.hq = hq;
  rq.khat = (const T *)dv.khat + a.slot[ci] * dv.slot_elems + (int64_t)u * dv.Mcap * D;
  rq.vhat = (const T *)dv.vhat + a.slot[ci] * dv.slot_elems + (int64_t)u * dv.Mcap * D;
  rq.ring_k = (const T *)dv.winK + (int64_t)u * dv.L * D;
  rq.ring_v = (const T *)dv.winV + (int64_t)u * dv.L * D;
  rq.in_k = (const T *)a.in.k + b * a.in.k_b + hkv * a.in.k_h;
  rq.in_v = (const T *)a.in.v + b * a.in.v_b + hkv * a.in.v_h;
  rq.in_kt = a.in.k_t;
  rq.in_vt = a.in.v_t;
  rq.t0 = a.t0;
  rq.put_k = rq.put_v = nullptr;
  rq.put_g = nullptr;
  rq.gate = 1.f;
  if (a.put_token && hq == hkv * (dv.Hq / dv.Hkv)) {
    rq.put_k = (T *)dv.winK + (int64_t)u * dv.L * D;
    rq.put_v = (T *)dv.winV + (int64_t)u * dv.L * D;
    rq.put_g = dv.winG + (int64_t)u * dv.L;
    rq.gate = a.in.g ? a.in.g[b * a.in.g_b + hkv * a.in.g_h + (rq.pos - a.t0) * a.in.g_t] : 1.f;
  }
  attn_row<T, D, GQ>(dv, rq);
}

// Decode over sequences that live in different states (each at its own position, with its own
// number of state rows): one workgroup per (group of GQ query heads, sequence); sequence s reads
// seq[s].  dv is the states' common configuration (heads, chunk, window, temperatures).
template <typename T, int D, int GQ>
__global__ __launch_bounds__(256) void attn_rows_multi_kernel(Dev dv, const SeqDesc *seq, const void *q,
                                                              const void *k, const void *v, const float *gate,
                                                              void *out) {
  const int hq = blockIdx.x * GQ, s = blockIdx.y;
  const int hkv = hq / (dv.Hq / dv.Hkv);
  const SeqDesc sd = seq[s];
  RowQuery<T> rq;
  rq.pos = sd.pos;
  rq.q = (const T *)q + ((int64_t)s * dv.Hq + hq) * D;
  rq.out = (T *)out + ((int64_t)s * dv.Hq + hq) * D;
  rq.lse = nullptr;
  rq.q_h = rq.o_h = D;
  rq.lse_h = 0;
  rq.m = sd.m;
  rq.hq = hq;
  rq.khat = (const T *)sd.khat + (int64_t)hkv * sd.Mcap * D;
  rq.vhat = (const T *)sd.vhat + (int64_t)hkv * sd.Mcap * D;
  rq.ring_k = (const T *)sd.winK + (int64_t)hkv * dv.L * D;
  rq.ring_v = (const T *)sd.winV + (int64_t)hkv * dv.L * D;
  // the new token is read from the call's k, v (position pos); everything older from the ring
  rq.in_k = (const T *)k + ((int64_t)s * dv.Hkv + hkv) * D;
  rq.in_v = (const T *)v + ((int64_t)s * dv.Hkv + hkv) * D;
  rq.in_kt = rq.in_vt = 0;
  rq.t0 = sd.pos;
  rq.put_k = rq.put_v = nullptr;
  rq.put_g = nullptr;
  rq.gate = 1.f;
  if (hq == hkv * (dv.Hq / dv.Hkv)) {
    rq.put_k = (T *)sd.winK + (int64_t)hkv * dv.L * D;
    rq.put_v = (T *)sd.winV + (int64_t)hkv * dv.L * D;
    rq.put_g = sd.winG + (int64_t)hkv * dv.L;
    rq.gate = gate ? gate[(int64_t)s * dv.Hkv + hkv] : 1.f;
  }
  attn_row<T, D, GQ>(dv, rq);
}

// Query heads a decode workgroup takes together: the KV head's whole group when it has 2 or 4
// heads, four of them when it has a multiple of four (so that the group's first head, whose
// workgroup stores the token, starts a workgroup either way).
int heads_together(const Dev &dv) {
  const int G = dv.Hq / dv.Hkv;
  return G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1);
}

}  // namespace

#define KVM_ROWS_DISPATCH(KERNEL, GQV, grid, ...)                                                   \
  do {                                                                                              \
    if (dv.io == 0 && dv.d == 64)                                                                   \
      hipLaunchKernelGGL((KERNEL<float, 64, GQV>), grid, dim3(256), 0, st, __VA_ARGS__);            \
    else if (dv.io == 0 && dv.d == 128)                                                             \
      hipLaunchKernelGGL((KERNEL<float, 128, GQV>), grid, dim3(256), 0, st, __VA_ARGS__);           \
    else if (dv.io == 1 && dv.d == 64)                                                              \
      hipLaunchKernelGGL((KERNEL<bf16_t, 64, GQV>), grid, dim3(256), 0, st, __VA_ARGS__);           \
    else if (dv.io == 1 && dv.d == 128)                                                             \
      hipLaunchKernelGGL((KERNEL<bf16_t, 128, GQV>), grid, dim3(256), 0, st, __VA_ARGS__);          \
    else                                                                                            \
      return hipErrorInvalidValue;                                                                  \
  } while (0)

hipError_t launch_attn_rows(const Dev &dv, const AttnArgs &a, hipStream_t st) {
  if (a.nq_total <= 0) return hipSuccess;
  // a decode step (one query per sequence) takes a KV head's query heads together; a prefill on
  // this path has queries enough to fill the GPU head by head
  const int gq = a.put_token ? heads_together(dv) : 1;
  dim3 grid(a.nq_total, dv.Hq / gq, dv.B);
  if (gq == 4)
    KVM_ROWS_DISPATCH(attn_rows_kernel, 4, grid, dv, a);
  else if (gq == 2)
    KVM_ROWS_DISPATCH(attn_rows_kernel, 2, grid, dv, a);
  else
    KVM_ROWS_DISPATCH(attn_rows_kernel, 1, grid, dv, a);
  return hipGetLastError();
}

hipError_t launch_decode_multi(const Dev &dv, const SeqDesc *seq, int n_seq, const void *q, const void *k,
                               const void *v, const float *gate, void *out, hipStream_t st) {
  if (n_seq <= 0) return hipSuccess;
  const int gq = heads_together(dv);
  dim3 agrid(dv.Hq / gq, n_seq);
  if (gq == 4)
    KVM_ROWS_DISPATCH(attn_rows_multi_kernel, 4, agrid, dv, seq, q, k, v, gate, out);
  else if (gq == 2)
    KVM_ROWS_DISPATCH(attn_rows_multi_kernel, 2, agrid, dv, seq, q, k, v, gate, out);
  else
    KVM_ROWS_DISPATCH(attn_rows_multi_kernel, 1, agrid, dv, seq, q, k, v, gate, out);
  return hipGetLastError();
}

}  // namespace kvm
