// Backward pass of a whole-sequence prefill (the paper's "Speed Benchmarks" time one; what it
// computes follows from the forward definition in "KVM Formulation" by the chain rule).
//
// The walk goes over the chunks in reverse.  For a chunk: first the fold that followed it is
// undone (its tokens receive the adjoint of the rows they went to -- gated for merged tokens,
// ungated plus the radius term for the tokens that created a row -- and are subtracted from the
// running sums again, which turns the sums back into the version the chunk saw); then the
// chunk's attention is differentiated against that version's readout and its window; then the
// readout's adjoint goes through LN_s and through the radius normalisation into the adjoint of
// the sums.  Slot assignments are replayed from the forward's record (the argmax is piecewise
// constant); the roundings of the materialised vectors are passed straight through.
//
// This file holds the kernels for every dtype and head size (vector ALU, fp32 accumulation, the
// chunk's probabilities and logit adjoints written out once and read by the two contraction
// kernels) and the walk itself.
#include <stdlib.h>

#include "kvm_device.h"
#include "kvm_internal.h"

namespace kvm {

namespace {

template <typename T, int D>
__device__ __forceinline__ void load_row(const T *p, int lane, float (&f)[D / 64]) {
#pragma unroll
  for (int c = 0; c < D / 64; ++c) f[c] = Io<T>::load(p + lane * (D / 64) + c);
}

// delta[row] = sum over channels of dout * out ("Readout": the softmax's own term of the chain rule)
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const void *out_, const void *dout_, float *delta,
                                                        int64_t rows) {
  const T *out = (const T *)out_, *dout = (const T *)dout_;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  float a[D / 64], b[D / 64];
  load_row<T, D>(out + row * D, lane, a);
  load_row<T, D>(dout + row * D, lane, b);
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < D / 64; ++c) s += a[c] * b[c];
  s = wave_sum(s);
  if (lane == 0) delta[row] = s;
}

// The LN_s parameter gradients of a workgroup's rows: summed over its four waves in LDS, then one
// fp64 atomic per channel (dgamma at par64[h * D + ch], dbeta behind all the dgammas).
constexpr int kRowsPerWave = 16;
template <int D, int kWaves>
__device__ __forceinline__ void block_param_add(const Bwd &a, int h, const float (&dga)[D / 64],
                                                const float (&dbe)[D / 64], float (*red)[kWaves][D]) {
  constexpr int CPL = D / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    red[0][wave][lane * CPL + c] = dga[c];
    red[1][wave][lane * CPL + c] = dbe[c];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * D; i += 64 * kWaves) {
    const int which = i / D, ch = i % D;
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) sum += red[which][w][ch];
    if (sum != 0.f) atomicAdd(a.par64 + (which * a.dv.Hkv + h) * D + ch, (double)sum);
  }
}

// Undo fold number `fold` (block [lo, lo + C)).  A wave takes kUnfoldRows consecutive rows of the
// state after the fold (one: the tokens of a row are a chain of dependent loads, and rows in
// parallel hide it better than rows in turn): it scans the block's recorded targets (64 tokens
// per ballot) and handles the tokens bound for its row -- they all read the row's adjoint, which
// is loaded once, and the merged ones are taken out of the row's sums again in registers, so
// that nothing needs an atomic.  A token bound for a row of this fold's own making either
// created that row or merged into it afterwards: the forward appends the tokens with the
// smallest (append score, position) keys, so among the tokens bound for one new row the creator
// is the one with the smallest key.
constexpr int kUnfoldRows = 16;  // at most
constexpr int kUnfoldWaves = 4;  // waves per workgroup (16 measured slower: the workgroup waits for its slowest row)

template <typename T, int D>
__global__ __launch_bounds__(64 * kUnfoldWaves) void bwd_unfold_kernel(Bwd a, int fold, int64_t lo, int m_before,
                                                                     int m_after, int rows_per_wave) {
  constexpr int CPL = D / 64;
  __shared__ float red[2][kUnfoldWaves][D];
  const Dev &dv = a.dv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u = blockIdx.y, b = u / dv.Hkv, h = u % dv.Hkv;
  const int C = dv.C;
  const int row_first = (blockIdx.x * kUnfoldWaves + wave) * rows_per_wave;
  const int64_t base = ((int64_t)fold * dv.U + u) * C;
  float dga_sum[CPL] = {}, dbe_sum[CPL] = {};
  float gam[CPL], bet[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    gam[c] = dv.gamma ? dv.gamma[h * D + lane * CPL + c] : 1.f;
    bet[c] = dv.beta ? dv.beta[h * D + lane * CPL + c] : 0.f;
  }
  int tg[8];
  auto load_targets = [&](int j0) {
#pragma unroll
    for (int bk = 0; bk < 8; ++bk) {
      const int j = j0 + 64 * bk + lane;
      tg[bk] = j < C ? a.assign[base + j] : -1;
    }
  };
  if (row_first < m_after) load_targets(0);
  for (int rr = 0; rr < rows_per_wave; ++rr) {
    const int row = row_first + rr;
    if (row >= m_after) break;
    const bool fresh = row >= m_before;  // a row this fold created: it ends here
    const int64_t ro = ((int64_t)u * dv.Mcap + row) * D;
    int creator = -1;
    if (fresh) {
      float best = 0.f;
      for (int j0 = 0; j0 < C; j0 += 512) {
        if (C > 512) load_targets(j0);
#pragma unroll
        for (int bk = 0; bk < 8; ++bk) {
          uint64_t hits = __builtin_amdgcn_ballot_w64(tg[bk] == row);
          while (hits) {
            const int j = j0 + 64 * bk + __builtin_ctzll(hits);
            hits &= hits - 1;
            const float sj = a.score[2 * (base + j)];
            if (creator < 0 || sj < best) {  // positions ascend: equal scores keep the earlier token
              best = sj;
              creator = j;
            }
          }
        }
      }
    }
    bool loaded = false;
    float dsk[CPL], dsv[CPL], sv[CPL], dr = 0.f;
    double sk[CPL];
    for (int j0 = 0; j0 < C; j0 += 512) {
      if (C > 512) load_targets(j0);
#pragma unroll
      for (int bk = 0; bk < 8; ++bk) {
        uint64_t hits = __builtin_amdgcn_ballot_w64(tg[bk] == row);
        while (hits) {
          const int j = j0 + 64 * bk + __builtin_ctzll(hits);
          hits &= hits - 1;
          if (!loaded) {
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
              dsk[c] = a.dsK[ro + lane * CPL + c];
              dsv[c] = a.dsV[ro + lane * CPL + c];
              sk[c] = fresh ? 0.0 : a.wsK[ro + lane * CPL + c];
              sv[c] = fresh ? 0.f : a.wsV[ro + lane * CPL + c];
            }
            dr = a.drho[(int64_t)u * dv.Mcap + row];
            loaded = true;
          }
          const int64_t tok = ((int64_t)b * a.T + lo + j) * dv.Hkv + h;
          // where the token's share goes: its row of the full accumulators, or of the ring
          const int64_t acc_row =
              a.ring_rows ? (int64_t)u * a.ring_rows + (int)((lo / C) % (a.ring_rows / C)) * C + j : tok;
          float kf[CPL], vf[CPL];
          load_row<T, D>((const T *)a.k + tok * D, lane, kf);
          load_row<T, D>((const T *)a.v + tok * D, lane, vf);
          const float g = a.gate ? a.gate[tok] : 1.f;
          // memory key of the token as the forward made it: LN_s in fp64 over the key with its
          // rotary channels zeroed, rounded to the I/O dtype
          double x[CPL], s = 0.0;
#pragma unroll
          for (int c = 0; c < CPL; ++c) {
            x[c] = lane * CPL + c < dv.r ? 0.0 : (double)kf[c];
            s += x[c];
          }
          const double mean = wave_sum(s) / (double)D;
          double qq = 0.0;
#pragma unroll
          for (int c = 0; c < CPL; ++c) qq += (x[c] - mean) * (x[c] - mean);
          const double rden = 1.0 / sqrt(wave_sum(qq) / (double)D + (double)dv.ln_eps);
          float xhat[CPL], kbar[CPL], dkbar[CPL], dvt[CPL];
#pragma unroll
          for (int c = 0; c < CPL; ++c) {
            const double xh = (x[c] - mean) * rden;
            xhat[c] = (float)xh;
            kbar[c] = Io<T>::round_from(xh * (double)gam[c] + (double)bet[c]);
          }
          float dg = 0.f;
          if (j == creator) {
            // a new row is the ungated memory key and value; its radius is the value's length
            float nn = 0.f;
#pragma unroll
            for (int c = 0; c < CPL; ++c) nn += vf[c] * vf[c];
            const float nv = sqrtf(wave_sum(nn));
            const float drn = nv > 0.f ? dr / nv : 0.f;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
              dkbar[c] = dsk[c];
              dvt[c] = dsv[c] + drn * vf[c];
            }
          } else {
            float dot = 0.f;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
              dkbar[c] = g * dsk[c];
              dvt[c] = g * dsv[c];
              dot += dsk[c] * kbar[c] + dsv[c] * vf[c];
              // back to the version before the fold: the token leaves its row's sums again
              sk[c] -= (double)g * (double)kbar[c];
              sv[c] -= g * vf[c];
            }
            dg = wave_sum(dot);
          }
          if (lane == 0) a.dgate[tok] = dg;
          // through LN_s of the memory key
          float s1 = 0.f, s2 = 0.f;
#pragma unroll
          for (int c = 0; c < CPL; ++c) {
            s1 += dkbar[c] * gam[c];
            s2 += dkbar[c] * gam[c] * xhat[c];
          }
          const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
#pragma unroll
          for (int c = 0; c < CPL; ++c) {
            const int ch = lane * CPL + c;
            const float dkz = (dkbar[c] * gam[c] - m1 - xhat[c] * m2) * (float)rden;
            // plain stores: walking backwards, a token's fold is undone before any chunk that had
            // the token in its window is visited, so this is the first contribution it receives
            a.dk_acc[acc_row * D + ch] = ch >= dv.r ? dkz : 0.f;
            a.dv_acc[acc_row * D + ch] = dvt[c];
            dga_sum[c] += dkbar[c] * xhat[c];
            dbe_sum[c] += dkbar[c];
          }
        }
      }
    }
    if (loaded && !fresh) {
      // the row as the earlier version had it: its sums, and its readout as the forward made it
      // (rows that the fold left alone keep the readout they have)
      double sm = 0.0;
      float nn = 0.f;
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        a.wsK[ro + lane * CPL + c] = sk[c];
        a.wsV[ro + lane * CPL + c] = sv[c];
        sm += sk[c];
        nn += sv[c] * sv[c];
      }
      const double mean = wave_sum(sm) / (double)D;
      double qq = 0.0;
#pragma unroll
      for (int c = 0; c < CPL; ++c) qq += (sk[c] - mean) * (sk[c] - mean);
      const double rden = 1.0 / sqrt(wave_sum(qq) / (double)D + (double)dv.ln_eps);
      const float vs = dv.rho[(int64_t)u * dv.Mcap + row] / fmaxf(sqrtf(wave_sum(nn)), dv.norm_eps);
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        const int ch = lane * CPL + c;
        Io<T>::store((T *)a.khat + ro + ch, Io<T>::round_from((sk[c] - mean) * rden * (double)gam[c] + (double)bet[c]));
        Io<T>::store((T *)a.vhat + ro + ch, sv[c] * vs);
        a.xhat[ro + ch] = (float)((sk[c] - mean) * rden);
      }
      if (lane == 0) a.rden[(int64_t)u * dv.Mcap + row] = (float)rden;
    }
  }
  block_param_add<D, kUnfoldWaves>(a, h, dga_sum, dbe_sum, red);
}

// Readout of the visited version: rows [0, m) of every unit, as the forward computes it.
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_readout_kernel(Bwd a, int m) {
  constexpr int CPL = D / 64;
  const Dev &dv = a.dv;
  const int lane = threadIdx.x & 63;
  const int u = blockIdx.y, h = u % dv.Hkv;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= m) return;
  const int64_t ro = ((int64_t)u * dv.Mcap + row) * D;
  double sk[CPL], s = 0.0;
  float sv[CPL], nn = 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    sk[c] = a.wsK[ro + lane * CPL + c];
    sv[c] = a.wsV[ro + lane * CPL + c];
    s += sk[c];
    nn += sv[c] * sv[c];
  }
  const double mean = wave_sum(s) / (double)D;
  double qq = 0.0;
#pragma unroll
  for (int c = 0; c < CPL; ++c) qq += (sk[c] - mean) * (sk[c] - mean);
  const double rden = 1.0 / sqrt(wave_sum(qq) / (double)D + (double)dv.ln_eps);
  const float vs = dv.rho[(int64_t)u * dv.Mcap + row] / fmaxf(sqrtf(wave_sum(nn)), dv.norm_eps);
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane * CPL + c;
    const double g_ = dv.gamma ? (double)dv.gamma[h * D + ch] : 1.0;
    const double b_ = dv.beta ? (double)dv.beta[h * D + ch] : 0.0;
    Io<T>::store((T *)a.khat + ro + ch, Io<T>::round_from((sk[c] - mean) * rden * g_ + b_));
    Io<T>::store((T *)a.vhat + ro + ch, sv[c] * vs);
    a.xhat[ro + ch] = (float)((sk[c] - mean) * rden);
  }
  if (lane == 0) a.rden[(int64_t)u * dv.Mcap + row] = (float)rden;
}

// Adjoint of the readout into the adjoint of the sums: rows [0, m).
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_readout_adjoint_kernel(Bwd a, int m) {
  constexpr int CPL = D / 64;
  __shared__ float red[2][4][D];
  const Dev &dv = a.dv;
  const int lane = threadIdx.x & 63;
  const int u = blockIdx.y, h = u % dv.Hkv;
  float dga_sum[CPL] = {}, dbe_sum[CPL] = {};
  for (int jj = 0; jj < kRowsPerWave; ++jj) {
  const int row = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kRowsPerWave + jj;
  if (row >= m) break;
  const int64_t ro = ((int64_t)u * dv.Mcap + row) * D;
  double sk[CPL], s = 0.0;
  float sv[CPL], dkh[CPL], dvh[CPL], nn = 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    sk[c] = a.wsK[ro + lane * CPL + c];
    sv[c] = a.wsV[ro + lane * CPL + c];
    dkh[c] = a.dkhat[ro + lane * CPL + c];
    dvh[c] = a.dvhat[ro + lane * CPL + c];
    s += sk[c];
    nn += sv[c] * sv[c];
  }
  const double mean = wave_sum(s) / (double)D;
  double qq = 0.0;
#pragma unroll
  for (int c = 0; c < CPL; ++c) qq += (sk[c] - mean) * (sk[c] - mean);
  const double rden = 1.0 / sqrt(wave_sum(qq) / (double)D + (double)dv.ln_eps);
  float xhat[CPL], ga[CPL], s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane * CPL + c;
    xhat[c] = (float)((sk[c] - mean) * rden);
    ga[c] = dv.gamma ? dv.gamma[h * D + ch] : 1.f;
    s1 += dkh[c] * ga[c];
    s2 += dkh[c] * ga[c] * xhat[c];
  }
  const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
  // value readout: rho * sV / max(|sV|, eps)
  const float nrm = sqrtf(wave_sum(nn));
  const float den = fmaxf(nrm, dv.norm_eps);
  const float rho = dv.rho[(int64_t)u * dv.Mcap + row];
  float dot = 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c) dot += dvh[c] * sv[c];
  dot = wave_sum(dot) / den;  // dvhat . unit vector
  const float back = nrm > dv.norm_eps ? rho * dot / (den * den) : 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane * CPL + c;
    a.dsK[ro + ch] += (dkh[c] * ga[c] - m1 - xhat[c] * m2) * (float)rden;
    a.dsV[ro + ch] += rho / den * dvh[c] - back * sv[c];
    dga_sum[c] += dkh[c] * xhat[c];
    dbe_sum[c] += dkh[c];
  }
  if (lane == 0) a.drho[(int64_t)u * dv.Mcap + row] += dot;
  }
  block_param_add<D, 4>(a, h, dga_sum, dbe_sum, red);
}

// One chunk's keys: state rows [0, m) of the visited version, then window positions [wb, s + nq).
struct ChunkArgs {
  int64_t s, wb;
  int32_t nq, m, nk, ld;  // nk = m + window keys; ld = row pitch of P and dS
};

template <typename T, int D>
__device__ __forceinline__ void key_of(const Bwd &a, const ChunkArgs &c, int u, int b, int h, int j,
                                       const T *&key, const T *&val, int64_t &pos) {
  const Dev &dv = a.dv;
  if (j < c.m) {
    const int64_t ro = ((int64_t)u * dv.Mcap + j) * D;
    key = (const T *)a.khat + ro;
    val = (const T *)a.vhat + ro;
    pos = -1;
  } else {
    pos = c.wb + (j - c.m);
    const int64_t tok = ((int64_t)b * a.T + pos) * dv.Hkv + h;
    key = (const T *)a.k + tok * D;
    val = (const T *)a.v + tok * D;
  }
}

// P and dS of one (query, head): a wave per key in turn.
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_probs_kernel(Bwd a, ChunkArgs c) {
  constexpr int CPL = D / 64;
  const Dev &dv = a.dv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x, g = blockIdx.y, u = blockIdx.z;
  const int G = dv.Hq / dv.Hkv, b = u / dv.Hkv, h = u % dv.Hkv, hq = h * G + g;
  const int64_t t = c.s + i;
  const int64_t qrow = ((int64_t)b * a.T + t) * dv.Hq + hq;
  float qf[CPL], df[CPL];
  load_row<T, D>((const T *)a.q + qrow * D, lane, qf);
  load_row<T, D>((const T *)a.dout + qrow * D, lane, df);
  const float lse = a.lse[qrow], delta = a.delta[qrow];
  const float ts = dv.tau_state ? dv.tau_state[hq] : 1.f, tb = dv.tau_bswa ? dv.tau_bswa[hq] : 1.f;
  const float scale = rsqrtf((float)D);
  const int64_t prow = (((int64_t)u * G + g) * dv.C + i) * c.ld;
  float acc_s = 0.f, acc_b = 0.f;
  for (int j = wave; j < c.nk; j += 4) {
    const T *key, *val;
    int64_t pos;
    key_of<T, D>(a, c, u, b, h, j, key, val, pos);
    float kf[CPL], vf[CPL];
    load_row<T, D>(key, lane, kf);
    load_row<T, D>(val, lane, vf);
    float d1 = 0.f, d2 = 0.f;
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) {
      d1 += qf[cc] * kf[cc];
      d2 += df[cc] * vf[cc];
    }
    const float raw = wave_sum(d1) * scale;
    const float dp = wave_sum(d2);
    const bool state = j < c.m;
    const float p = (state || pos <= t) ? __expf((state ? ts : tb) * raw - lse) : 0.f;
    const float ds = p * (dp - delta);
    if (lane == 0) {
      a.P[prow + j] = p;
      a.dS[prow + j] = ds;
    }
    if (state) acc_s += ds * raw; else acc_b += ds * raw;
  }
  if (lane == 0) {
    atomicAdd(a.par64 + 2 * dv.Hkv * D + hq, (double)acc_s);
    atomicAdd(a.par64 + 2 * dv.Hkv * D + dv.Hq + hq, (double)acc_b);
  }
}

// dq of one (query, head): sum over keys of dS * tau * scale * key.
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dq_kernel(Bwd a, ChunkArgs c) {
  constexpr int CPL = D / 64;
  __shared__ float red[4][D];
  const Dev &dv = a.dv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x, g = blockIdx.y, u = blockIdx.z;
  const int G = dv.Hq / dv.Hkv, b = u / dv.Hkv, h = u % dv.Hkv, hq = h * G + g;
  const int64_t qrow = ((int64_t)b * a.T + c.s + i) * dv.Hq + hq;
  const float ts = dv.tau_state ? dv.tau_state[hq] : 1.f, tb = dv.tau_bswa ? dv.tau_bswa[hq] : 1.f;
  const int64_t prow = (((int64_t)u * G + g) * dv.C + i) * c.ld;
  float acc[CPL] = {};
  for (int j = wave; j < c.nk; j += 4) {
    const T *key, *val;
    int64_t pos;
    key_of<T, D>(a, c, u, b, h, j, key, val, pos);
    float kf[CPL];
    load_row<T, D>(key, lane, kf);
    const float coef = a.dS[prow + j] * (j < c.m ? ts : tb);
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) acc[cc] += coef * kf[cc];
  }
#pragma unroll
  for (int cc = 0; cc < CPL; ++cc) red[wave][lane * CPL + cc] = acc[cc];
  __syncthreads();
  if (wave == 0) {
    const float scale = rsqrtf((float)D);
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) {
      const int ch = lane * CPL + cc;
      Io<T>::store((T *)a.dq + qrow * D + ch, (red[0][ch] + red[1][ch] + red[2][ch] + red[3][ch]) * scale);
    }
  }
}

// Adjoint of one key and its value: sums over the chunk's queries and the group's heads.
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_dkv_kernel(Bwd a, ChunkArgs c) {
  constexpr int CPL = D / 64;
  __shared__ float red[2][4][D];
  const Dev &dv = a.dv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x, u = blockIdx.y;
  const int G = dv.Hq / dv.Hkv, b = u / dv.Hkv, h = u % dv.Hkv;
  const bool state = j < c.m;
  float ak[CPL] = {}, av[CPL] = {};
  for (int p = wave; p < G * c.nq; p += 4) {
    const int g = p / c.nq, i = p % c.nq, hq = h * G + g;
    const int64_t qrow = ((int64_t)b * a.T + c.s + i) * dv.Hq + hq;
    const int64_t at = (((int64_t)u * G + g) * dv.C + i) * c.ld + j;
    const float tau = state ? (dv.tau_state ? dv.tau_state[hq] : 1.f) : (dv.tau_bswa ? dv.tau_bswa[hq] : 1.f);
    const float ds = a.dS[at] * tau, pr = a.P[at];
    float qf[CPL], df[CPL];
    load_row<T, D>((const T *)a.q + qrow * D, lane, qf);
    load_row<T, D>((const T *)a.dout + qrow * D, lane, df);
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) {
      ak[cc] += ds * qf[cc];
      av[cc] += pr * df[cc];
    }
  }
#pragma unroll
  for (int cc = 0; cc < CPL; ++cc) {
    red[0][wave][lane * CPL + cc] = ak[cc];
    red[1][wave][lane * CPL + cc] = av[cc];
  }
  __syncthreads();
  if (wave == 0) {
    const float scale = rsqrtf((float)D);
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) {
      const int ch = lane * CPL + cc;
      const float dk = (red[0][0][ch] + red[0][1][ch] + red[0][2][ch] + red[0][3][ch]) * scale;
      const float dvv = red[1][0][ch] + red[1][1][ch] + red[1][2][ch] + red[1][3][ch];
      if (state) {
        const int64_t ro = ((int64_t)u * dv.Mcap + j) * D;
        a.dkhat[ro + ch] = dk;
        a.dvhat[ro + ch] = dvv;
      } else {
        const int64_t tok = ((int64_t)b * a.T + c.wb + (j - c.m)) * dv.Hkv + h;
        a.dk_acc[tok * D + ch] += dk;
        a.dv_acc[tok * D + ch] += dvv;
      }
    }
  }
}

// the parameter gradients leave their fp64 accumulators: [dgamma | dbeta | dtau_state | dtau_bswa]
__global__ __launch_bounds__(256) void bwd_params_kernel(Bwd a) {
  const int n_ln = a.dv.Hkv * a.dv.d, i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_ln) {
    a.dgamma[i] = (float)a.par64[i];
    a.dbeta[i] = (float)a.par64[n_ln + i];
  }
  if (i < a.dv.Hq) {
    a.dtau_state[i] = (float)a.par64[2 * n_ln + i];
    a.dtau_bswa[i] = (float)a.par64[2 * n_ln + a.dv.Hq + i];
  }
}

// fp32 accumulators to the I/O dtype, eight elements per thread (n is a multiple of 64)
template <typename T>
__global__ __launch_bounds__(256) void bwd_cast_kernel(const float *src, T *dst, int64_t n) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
  const float4 x = *reinterpret_cast<const float4 *>(src + i), y = *reinterpret_cast<const float4 *>(src + i + 4);
  if constexpr (sizeof(T) == 4) {
    *reinterpret_cast<float4 *>((float *)dst + i) = x;
    *reinterpret_cast<float4 *>((float *)dst + i + 4) = y;
  } else {
    *reinterpret_cast<uint4 *>((uint16_t *)dst + i) =
        make_uint4(pack_bf16(x.x, x.y), pack_bf16(x.z, x.w), pack_bf16(y.x, y.y), pack_bf16(y.z, y.w));
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_zero_floats_kernel(float *p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// Zero fill with a kernel of the library's own (a caller may capture the call in a graph, where
// memset nodes are best avoided): n4 pieces of 16 bytes.
__global__ __launch_bounds__(256) void bwd_zero_kernel(uint4 *p, int64_t n4) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) p[i] = make_uint4(0u, 0u, 0u, 0u);
}
hipError_t zero_fill(void *p, size_t bytes, hipStream_t st) {
  const int64_t n4 = (int64_t)((bytes + 15) / 16);  // the work arrays are padded to 256 bytes
  if (n4 == 0) return hipSuccess;
  const int64_t want = (n4 + 255) / 256;
  const unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
  hipLaunchKernelGGL(bwd_zero_kernel, dim3(blocks), dim3(256), 0, st, (uint4 *)p, n4);
  return hipGetLastError();
}

#define BWD_DISPATCH(dv, KERNEL, grid, block, st, ...)                                    \
  do {                                                                                    \
    if ((dv).io == 0 && (dv).d == 64)                                                     \
      hipLaunchKernelGGL((KERNEL<float, 64>), grid, block, 0, st, __VA_ARGS__);           \
    else if ((dv).io == 0 && (dv).d == 128)                                               \
      hipLaunchKernelGGL((KERNEL<float, 128>), grid, block, 0, st, __VA_ARGS__);          \
    else if ((dv).io == 1 && (dv).d == 64)                                                \
      hipLaunchKernelGGL((KERNEL<bf16_t, 64>), grid, block, 0, st, __VA_ARGS__);          \
    else if ((dv).io == 1 && (dv).d == 128)                                               \
      hipLaunchKernelGGL((KERNEL<bf16_t, 128>), grid, block, 0, st, __VA_ARGS__);         \
    else                                                                                  \
      return hipErrorInvalidValue;                                                        \
    if (hipError_t e_ = hipGetLastError(); e_ != hipSuccess) return e_;                   \
  } while (0)

#define BWD_TRY(expr)                        \
  do {                                       \
    if (hipError_t e_ = (expr); e_ != hipSuccess) return e_; \
  } while (0)

}  // namespace

hipError_t run_backward(const Bwd &a_in, const BwdChunk *chunks, int n_chunks, hipStream_t st, const BwdStreams &x) {
  const Dev &dv = a_in.dv;
  const int G = dv.Hq / dv.Hkv, D = dv.d;
  const bool on_mfma = a_in.on_mfma;  // decided once by the caller, who sized the workspace by it
  Bwd a = a_in;
  // On the matrix-core path a token's dk, dv are finished when its block has been the window keys
  // of a launch; until then only what the token got when its fold was undone is kept, for the
  // blocks of one window.  Elsewhere dk, dv are summed in full-size fp32 accumulators.
  a.ring_rows = on_mfma ? dv.L + dv.C : 0;
  const int64_t state_elems = (int64_t)dv.U * dv.Mcap * D;
  const int64_t kv_elems = (int64_t)dv.B * a.T * dv.Hkv * D;
  const int64_t q_rows = (int64_t)dv.B * a.T * dv.Hq;
  // everything that is accumulated starts at zero; the sums start as the forward left them
  BWD_TRY(zero_fill(a.dsK, state_elems * 4, st));
  BWD_TRY(zero_fill(a.dsV, state_elems * 4, st));
  BWD_TRY(zero_fill(a.drho, (size_t)dv.U * dv.Mcap * 4, st));
  if (!on_mfma) {
    BWD_TRY(zero_fill(a.dk_acc, kv_elems * 4, st));
    BWD_TRY(zero_fill(a.dv_acc, kv_elems * 4, st));
  }
  BWD_TRY(zero_fill(a.par64, (size_t)(2 * dv.Hkv * D + 2 * dv.Hq) * 8, st));
  // dgate is the caller's tensor: its size need not be a multiple of 16 bytes
  BWD_DISPATCH(dv, bwd_zero_floats_kernel, dim3((unsigned)(((int64_t)dv.B * a.T * dv.Hkv + 255) / 256)), dim3(256), st,
               a.dgate, (int64_t)dv.B * a.T * dv.Hkv);
  if (dv.sK) {
    BWD_TRY(hipMemcpyAsync(a.wsK, dv.sK, state_elems * 8, hipMemcpyDeviceToDevice, st));
    BWD_TRY(hipMemcpyAsync(a.wsV, dv.sV, state_elems * 4, hipMemcpyDeviceToDevice, st));
  }

  // the readout of the last version; undoing a fold then rewrites the rows it touched
  if (n_chunks > 0 && chunks[n_chunks - 1].m_after > 0) {
    const int m_end = chunks[n_chunks - 1].m_after;
    BWD_DISPATCH(dv, bwd_readout_kernel, dim3((m_end + 3) / 4, dv.U), dim3(256), st, a, m_end);
  }
  // D = dout . out per query (the matrix-core dq kernel computes it for its own queries)
  if (!on_mfma)
    BWD_DISPATCH(dv, bwd_delta_kernel, dim3((unsigned)((q_rows + 3) / 4)), dim3(256), st, a.out, a.dout, a.delta, q_rows);
  // Matrix-core path, three streams.  The caller's carries the chain that the state imposes:
  // undo the fold, dq (which also forms D), dk of the state rows.  dv of the state rows needs the
  // undone fold only and runs on `side`.  dk and dv of the chunk's own tokens (window keys) need D
  // and nothing of the state: they run on `side2` and may still be running while the next chunk
  // of the walk is on the other two, which is what fills the chip while a fold is undone.  The
  // ring holds one block more than a window so that the fold undone then writes another slot than
  // they read; they must be done before the fold after that.
  const bool use_side = on_mfma && x.side && x.side2 && x.fork && x.dq_done && x.join_state && x.join_window[0] &&
                        x.join_window[1];
  bool state_busy = false, window_busy[2] = {false, false};
  for (int ci = n_chunks - 1; ci >= 0; --ci) {
    const BwdChunk &ch = chunks[ci];
    if (state_busy) {  // the fold about to be undone reads the value adjoints the dv role adds to
      BWD_TRY(hipStreamWaitEvent(st, x.join_state, 0));
      state_busy = false;
    }
    if (window_busy[ci & 1]) {  // ... and writes the ring slot that the window keys of chunk ci + 2 read
      BWD_TRY(hipStreamWaitEvent(st, x.join_window[ci & 1], 0));
      window_busy[ci & 1] = false;
    }
    if (ch.fold >= 0) {
      // rows per wave: so many that the launch is about one resident round of waves (8 per SIMD,
      // 8192 on the chip) -- a wave's rows share one scan of the block's targets, and more waves
      // than fit at once only queue up behind the scan of the first
      int rpw = (int)((int64_t)dv.U * ch.m_after / 8192);
      rpw = rpw < 1 ? 1 : (rpw > kUnfoldRows ? kUnfoldRows : rpw);
      BWD_DISPATCH(dv, bwd_unfold_kernel, dim3((ch.m_after + kUnfoldWaves * rpw - 1) / (kUnfoldWaves * rpw), dv.U),
                   dim3(64 * kUnfoldWaves), st, a, ch.fold, ch.s + ch.nq - dv.L, ch.m, ch.m_after, rpw);
    }
    const int64_t c0 = ch.s / dv.C * dv.C;
    ChunkArgs c;
    c.s = ch.s;
    c.wb = c0 + dv.C - dv.L > 0 ? c0 + dv.C - dv.L : 0;
    c.nq = ch.nq;
    c.m = ch.m;
    c.nk = ch.m + (int)(ch.s + ch.nq - c.wb);
    c.ld = dv.Mcap + dv.L;
    if (on_mfma) {
      // the chunk's own block was folded after the last chunk that had it in its window
      const int cj = ci + dv.L / dv.C - 1;
      const bool folded = cj < n_chunks && chunks[cj].fold >= 0;
      if (use_side) {
        BWD_TRY(hipEventRecord(x.fork, st));
        BWD_TRY(hipStreamWaitEvent(x.side, x.fork, 0));
        BWD_TRY(launch_backward_mfma(a, ch.s, ch.nq, ch.m, folded, kRoleDV, kSecState, x.side));
        BWD_TRY(hipEventRecord(x.join_state, x.side));
        state_busy = true;
        // (behind it on the same stream, so that the wait for the next chunk's join_state, one
        // fold before the ring slot is rewritten, also covers it)
        BWD_TRY(launch_backward_mfma(a, ch.s, ch.nq, ch.m, folded, kRoleDV, kSecWindow, x.side));
        BWD_TRY(launch_backward_mfma(a, ch.s, ch.nq, ch.m, folded, kRoleDQ, kSecBoth, st));
        BWD_TRY(hipEventRecord(x.dq_done, st));
        BWD_TRY(hipStreamWaitEvent(x.side2, x.dq_done, 0));
        BWD_TRY(launch_backward_mfma(a, ch.s, ch.nq, ch.m, folded, kRoleDK, kSecWindow, x.side2));
        BWD_TRY(hipEventRecord(x.join_window[ci & 1], x.side2));
        window_busy[ci & 1] = true;
        BWD_TRY(launch_backward_mfma(a, ch.s, ch.nq, ch.m, folded, kRoleDK, kSecState, st));
      } else {
        for (int role : {kRoleDQ, kRoleDK, kRoleDV})
          BWD_TRY(launch_backward_mfma(a, ch.s, ch.nq, ch.m, folded, role, kSecBoth, st));
      }
    } else {
      BWD_DISPATCH(dv, bwd_probs_kernel, dim3(ch.nq, G, dv.U), dim3(256), st, a, c);
      BWD_DISPATCH(dv, bwd_dq_kernel, dim3(ch.nq, G, dv.U), dim3(256), st, a, c);
      BWD_DISPATCH(dv, bwd_dkv_kernel, dim3(c.nk, dv.U), dim3(256), st, a, c);
    }
    if (ch.m > 0 && !on_mfma)  // (the matrix-core kernels do this in their epilogues)
      BWD_DISPATCH(dv, bwd_readout_adjoint_kernel, dim3((ch.m + 4 * kRowsPerWave - 1) / (4 * kRowsPerWave), dv.U),
                   dim3(256), st, a, ch.m);
  }
  if (state_busy) {  // the last launch on that stream is a dv role of window keys
    BWD_TRY(hipEventRecord(x.join_state, x.side));
    BWD_TRY(hipStreamWaitEvent(st, x.join_state, 0));
  }
  for (int i = 0; i < 2; ++i)
    if (window_busy[i]) BWD_TRY(hipStreamWaitEvent(st, x.join_window[i], 0));
  {
    const int n = dv.Hkv * D > dv.Hq ? dv.Hkv * D : dv.Hq;
    hipLaunchKernelGGL(bwd_params_kernel, dim3((n + 255) / 256), dim3(256), 0, st, a);
  }
  if (on_mfma) return hipGetLastError();  // dk, dv went out finished
  const unsigned cast_blocks = (unsigned)((kv_elems / 8 + 255) / 256);
  if (dv.io == 0) {
    hipLaunchKernelGGL((bwd_cast_kernel<float>), dim3(cast_blocks), dim3(256), 0, st, a.dk_acc, (float *)a.dk, kv_elems);
    hipLaunchKernelGGL((bwd_cast_kernel<float>), dim3(cast_blocks), dim3(256), 0, st, a.dv_acc, (float *)a.dv_out, kv_elems);
  } else {
    hipLaunchKernelGGL((bwd_cast_kernel<bf16_t>), dim3(cast_blocks), dim3(256), 0, st, a.dk_acc, (bf16_t *)a.dk, kv_elems);
    hipLaunchKernelGGL((bwd_cast_kernel<bf16_t>), dim3(cast_blocks), dim3(256), 0, st, a.dv_acc, (bf16_t *)a.dv_out, kv_elems);
  }
  return hipGetLastError();
}

}  // namespace kvm
