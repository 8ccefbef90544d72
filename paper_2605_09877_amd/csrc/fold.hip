// Fold of one overflow block into the compressed state (sections "KVM weight preparation",
// "Append", "Merge" and the readout equations of the paper's Method section), as wavefront
// kernels: one 64-lane wave owns one token or one state row and reduces over head_dim.
//
//   memkey : k-bar_j = LN_s(k_j with the rotary channels zeroed), materialised in the I/O dtype
//   score  : s_j = max_i k-bar_j . s-hat^K_i and pi(j) = argmax_{i >= S}   (generic, fp64 dot)
//   select : the n_append smallest s_j become new rows, in position order
//   accum  : new rows are created, each row finds the tokens that merge into it and adds them in
//            position order,
//            touched rows get their normalised readout (LN_s on keys, stored radius on values)
//
// Everything that decides an integer (LN_s of keys, the key sums) is computed in fp64 so that
// the decision can be reproduced on a CPU; values and radii are fp32.
#include <type_traits>

#include "kvm_device.h"
#include "kvm_internal.h"

namespace kvm {

namespace {

// An unsigned type of the given size in bytes.
template <int kBytes>
struct PieceOf;
template <>
struct PieceOf<4> { using type = uint32_t; };
template <>
struct PieceOf<8> { using type = uint2; };
template <>
struct PieceOf<16> { using type = uint4; };

template <typename T, int D>
__device__ __forceinline__ void write_readout(const Dev &dv, int slot, int u, int h, int row,
                                              const double (&sk)[D / 64], const float (&sv)[D / 64],
                                              float rho, int lane, float *khat_copy = nullptr) {
  constexpr int CPL = D / 64;
  double s = 0.0;
#pragma unroll
  for (int c = 0; c < CPL; ++c) s += sk[c];
  const double mean = wave_sum(s) / (double)D;
  double q = 0.0;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const double dl = sk[c] - mean;
    q += dl * dl;
  }
  // one fp64 reciprocal per row; (x - mean) * rden differs from (x - mean) / den by an ulp of
  // fp64 at most, far below what the rounding to the I/O dtype can see
  const double rden = 1.0 / sqrt(wave_sum(q) / (double)D + (double)dv.ln_eps);
  float nn = 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c) nn += sv[c] * sv[c];
  const float nrm = sqrtf(wave_sum(nn));
  const float vs = rho / fmaxf(nrm, dv.norm_eps);
  T *kh = (T *)dv.khat + slot * dv.slot_elems + ((int64_t)u * dv.Mcap + row) * D;
  T *vh = (T *)dv.vhat + slot * dv.slot_elems + ((int64_t)u * dv.Mcap + row) * D;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane * CPL + c;
    const double ga = dv.gamma ? (double)dv.gamma[h * D + ch] : 1.0;
    const double be = dv.beta ? (double)dv.beta[h * D + ch] : 0.0;
    const double y = (sk[c] - mean) * rden * ga + be;
    Io<T>::store(kh + ch, Io<T>::round_from(y));
    Io<T>::store(vh + ch, sv[c] * vs);
    if (khat_copy) khat_copy[ch] = Io<T>::round_from(y);  // the stored value, for a reader in the same workgroup
  }
}

// ------------------------------------------------------------------ memory keys
// Covers n_blocks consecutive C-token blocks of `src`; block i goes to the i-th [U, C, d] slab
// after dv.kbar (memory keys depend on k alone, so a prefill computes them a group at a time).
// A token takes D / kN adjacent lanes, 16 bytes of channels each, so a wave handles several tokens.
constexpr int kMemkeyTok = 4;  // tokens per lane group, their loads in flight together
template <typename T, int D>
__global__ __launch_bounds__(256) void memkey_kernel(Dev dv, Src src, int n_blocks) {
  constexpr int VEC = Vec16<T>::kN;
  constexpr int LPT = D / VEC;   // lanes per token
  constexpr int TPW = 64 / LPT;  // tokens per wave and round
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPT, cl = lane % LPT;
  const int u = blockIdx.y, b = u / dv.Hkv, h = u % dv.Hkv;
  const int n_tok = dv.C * n_blocks;
  const int j0 = (blockIdx.x * 4 + wave) * TPW * kMemkeyTok + sub;
  float raw[kMemkeyTok][VEC];
#pragma unroll
  for (int t = 0; t < kMemkeyTok; ++t) {
    const int j = j0 + t * TPW;
    const int jc = j < n_tok ? j : n_tok - 1;  // lanes past the end repeat the last token, store nothing
    const T *krow = (const T *)src.k + b * src.k_b + h * src.k_h + (int64_t)jc * src.k_t;
    Vec16<T>::load(krow + cl * VEC, raw[t]);
  }
  double ga[VEC], be[VEC];
#pragma unroll
  for (int c = 0; c < VEC; ++c) {
    const int ch = cl * VEC + c;
    ga[c] = dv.gamma ? (double)dv.gamma[h * D + ch] : 1.0;
    be[c] = dv.beta ? (double)dv.beta[h * D + ch] : 0.0;
  }
#pragma unroll
  for (int t = 0; t < kMemkeyTok; ++t) {
    const int j = j0 + t * TPW;
    double x[VEC];
    double s = 0.0;
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      x[c] = cl * VEC + c < dv.r ? 0.0 : (double)raw[t][c];
      s += x[c];
    }
    const double mean = group_sum<LPT>(s) / (double)D;
    double q = 0.0;
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
      const double dl = x[c] - mean;
      q += dl * dl;
    }
    const double rden = 1.0 / sqrt(group_sum<LPT>(q) / (double)D + (double)dv.ln_eps);
    float y[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) y[c] = Io<T>::round_from((x[c] - mean) * rden * ga[c] + be[c]);
    if (j < n_tok) {
      T *out = (T *)dv.kbar + ((int64_t)(j / dv.C) * dv.Ufull * dv.C + (int64_t)u * dv.C + j % dv.C) * D;
      Vec16<T>::store(out + cl * VEC, y);
    }
  }
}

// ------------------------------------------------------------------ similarity + winners (generic)
// One wave per token; lanes stride over state rows [row0, row1); each dot product is an fp64 sum
// of the I/O-dtype operands.  first_pass: rows are the pre-append state, writes s_j (all rows)
// and the best eligible row.  Otherwise rows are the ones appended in this fold and only tokens
// that were not appended themselves may move to them (strictly larger score only).
template <typename T, int D>
__global__ __launch_bounds__(256) void score_kernel(Dev dv, int slot, int row0, int row1, int first_pass) {
  __shared__ double kb[4][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u = blockIdx.y;
  const int j = blockIdx.x * 4 + wave;
  const int64_t tj = (int64_t)u * dv.C + j;
  const bool active = j < dv.C && (first_pass || dv.app[tj] < 0);
  if (active) {
    const T *kbar = (const T *)dv.kbar + tj * D;
    for (int c = lane; c < D; c += 64) kb[wave][c] = (double)Io<T>::load(kbar + c);
  }
  __syncthreads();
  if (!active) return;
  double best_all = -INFINITY, best = -INFINITY;
  int best_i = 0x7fffffff;
  const T *kh = (const T *)dv.khat + slot * dv.slot_elems + (int64_t)u * dv.Mcap * D;
  for (int i = row0 + lane; i < row1; i += 64) {
    const T *row = kh + (int64_t)i * D;
    double acc = 0.0;
    for (int c = 0; c < D; ++c) acc += kb[wave][c] * (double)Io<T>::load(row + c);
    best_all = acc > best_all ? acc : best_all;
    if (i >= dv.S && acc > best) {
      best = acc;
      best_i = i;
    }
  }
  best_all = wave_max(best_all);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double ob = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(best_i, o, kWave);
    if (ob > best || (ob == best && oi < best_i)) {
      best = ob;
      best_i = oi;
    }
  }
  if (lane == 0) {
    if (first_pass) {
      dv.score[tj] = make_float2((float)best_all, (float)best);
      dv.pi[tj] = best_i;
      dv.app[tj] = -1;
    } else if (best_i != 0x7fffffff && (float)best > dv.score[tj].y) {
      // compare in the stored (fp32) precision so both passes rank alike
      dv.score[tj].y = (float)best;
      dv.pi[tj] = best_i;
    }
  }
}

// ------------------------------------------------------------------ append selection
// One workgroup per unit.  take_all: every token becomes a row, in order (state creation, or a
// budget with room for the whole block).
__global__ __launch_bounds__(256) void select_kernel(Dev dv, int m, int n_app, int take_all) {
  extern __shared__ float sh[];  // C scores, then C flags
  float *sc = sh;
  int *flag = (int *)(sh + dv.C);
  const int u = blockIdx.x, C = dv.C;
  const int64_t base = (int64_t)u * C;
  if (take_all) {
    const float qnan = __uint_as_float(0x7fc00000u);
    for (int j = threadIdx.x; j < C; j += blockDim.x) {
      dv.app[base + j] = j;
      dv.pi[base + j] = m + j;
      dv.creator[base + j] = j;
      dv.score[base + j] = make_float2(qnan, qnan);
    }
    return;
  }
  for (int j = threadIdx.x; j < C; j += blockDim.x) sc[j] = dv.score[base + j].x;
  __syncthreads();
  for (int j = threadIdx.x; j < C; j += blockDim.x) {
    const float sj = sc[j];
    int rank = 0;
    for (int t = 0; t < C; ++t) {
      const float st = sc[t];
      rank += (st < sj || (st == sj && t < j)) ? 1 : 0;
    }
    flag[j] = rank < n_app ? 1 : 0;
  }
  __syncthreads();
  for (int j = threadIdx.x; j < C; j += blockDim.x) {
    if (flag[j]) {
      int a = 0;
      for (int t = 0; t < j; ++t) a += flag[t];
      dv.app[base + j] = a;
      dv.pi[base + j] = m + a;
      dv.creator[base + a] = j;
      dv.score[base + j].y = __uint_as_float(0x7fc00000u);
    } else {
      dv.app[base + j] = -1;
    }
  }
}

// ------------------------------------------------------------------ a small append in one launch
// A fold that appends only a few rows (n_app <= kAppendMax) does its selection, the creation of
// the new rows and the second scoring pass (the block's other tokens against the new rows) here,
// one workgroup per unit, instead of in three dependent launches: each of those is a few
// microseconds of work behind ten of latency, and a growing state appends at almost every fold.
//   1. selection as in select_kernel;
//   2. a wave per new row: sums, radius, readout into slot_new (as accum_kernel's creation);
//   3. a lane per remaining token: its dot products with the new rows' normalised keys (staged
//      in LDS), summed in fp64 over the I/O-dtype operands; a strictly larger score moves the
//      token to the new row, the lowest row winning ties, compared in the stored fp32 precision
//      as in score_kernel's second pass.
constexpr int kAppendMax = 16;

template <typename T, int D>
__global__ __launch_bounds__(256) void append_kernel(Dev dv, Src src, int m, int n_app, int slot_new) {
  // C sort keys (8 bytes each), kAppendMax creators, 4 wave counts, n_app x D new keys
  extern __shared__ __attribute__((aligned(16))) unsigned long long sh64[];
  const int C = dv.C;
  unsigned long long *key = sh64;
  int *cr = (int *)(sh64 + C);
  int *wcnt = cr + kAppendMax;
  float *kn = (float *)(wcnt + 4);
  const int u = blockIdx.x, b = u / dv.Hkv, h = u % dv.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t base = (int64_t)u * C;
  const T *vsrc = (const T *)src.v + b * src.v_b + h * src.v_h;
  const T *kbar = (const T *)dv.kbar + base * D;
  constexpr int VEC = Vec16<T>::kN, NCH = D / VEC;

  // The (score, position) order as one unsigned 64-bit order: the float's bits made monotonic
  // (sign flipped for positives, all bits for negatives) above the token index.
  for (int j = threadIdx.x; j < C; j += blockDim.x) {
    uint32_t f = __float_as_uint(dv.score[base + j].x);
    f = f == 0x80000000u ? 0u : f;  // -0 and +0 are one score
    const uint32_t mono = (f & 0x80000000u) ? ~f : (f | 0x80000000u);
    key[j] = ((unsigned long long)mono << 32) | (uint32_t)j;
  }
  __syncthreads();
  {  // a thread per token: the host sends only blocks of at most 256 tokens here
    const int j = threadIdx.x;
    const bool on = j < C;
    // the second pass's operand: the token's whole memory key, asked for before anything else
    // waits (the rows of 64 tokens are 64 separate cache lines per load)
    uint4 raw[NCH];
    if (on) {
#pragma unroll
      for (int q = 0; q < NCH; ++q) raw[q] = *reinterpret_cast<const uint4 *>(kbar + (int64_t)j * D + q * VEC);
    }
    // rank of a token = how many precede it; the n_app first are taken
    bool take = false;
    if (on) {
      const unsigned long long kj = key[j];
      int rank = 0;
      for (int t = 0; t < C; t += 2) {
        const ulonglong2 k2 = *reinterpret_cast<const ulonglong2 *>(key + t);
        rank += k2.x < kj ? 1 : 0;
        rank += k2.y < kj ? 1 : 0;
      }
      take = rank < n_app;
    }
    // position of a taken token among the taken ones, in token order: ballot within the wave,
    // wave counts through LDS
    const uint64_t bal = __builtin_amdgcn_ballot_w64(take);
    if (lane == 0) wcnt[wave] = __builtin_popcountll(bal);
    __syncthreads();
    int a = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) a += wcnt[w];
    if (on) {
      if (take) {
        dv.app[base + j] = a;
        dv.pi[base + j] = m + a;
        dv.creator[base + a] = j;
        cr[a] = j;
        dv.score[base + j].y = __uint_as_float(0x7fc00000u);
      } else {
        dv.app[base + j] = -1;
      }
    }
    __syncthreads();

    // creation: a wave per new row, two rows of a wave in flight together
    constexpr int CPL = D / 64;
    for (int a0 = wave; a0 < n_app; a0 += 8) {
      double sk[2][CPL];
      float sv[2][CPL];
      float nn[2] = {0.f, 0.f};
      const bool two = a0 + 4 < n_app;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        if (r == 1 && !two) break;
        const int j0c = cr[a0 + 4 * r];
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
          const int ch = lane * CPL + c;
          sk[r][c] = (double)Io<T>::load(kbar + (int64_t)j0c * D + ch);
          sv[r][c] = Io<T>::load(vsrc + (int64_t)j0c * src.v_t + ch);
          nn[r] += sv[r][c] * sv[r][c];
        }
      }
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        if (r == 1 && !two) break;
        const int an = a0 + 4 * r, row = m + an;
        const int64_t ro = (int64_t)u * dv.Mcap + row;
        const float rho = sqrtf(wave_sum(nn[r]));
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
          dv.sK[ro * D + lane * CPL + c] = sk[r][c];
          dv.sV[ro * D + lane * CPL + c] = sv[r][c];
        }
        if (lane == 0) {
          dv.rho[ro] = rho;
          dv.w[ro] = 1.f;
          dv.n[ro] = 1;
        }
        write_readout<T, D>(dv, slot_new, u, h, row, sk[r], sv[r], rho, lane, kn + an * D);
      }
    }
    __syncthreads();  // the new rows' normalised keys are in LDS

    // second pass: this lane's token against the new rows, eight at a time.  bf16 operands: the
    // products are exact in fp32 and so is most of the sum; fp32 operands take the fp64 sum the
    // generic scoring kernel takes.
    using Acc = typename std::conditional<std::is_same<T, float>::value, double, float>::type;
    if (on && !take) {
      Acc best = -INFINITY;
      int best_a = 0;
      for (int a0 = 0; a0 < n_app; a0 += 8) {
        Acc acc[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = (Acc)0;
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
          float x[VEC];
          unpack16<T>(raw[q], x);
#pragma unroll
          for (int an = 0; an < 8; ++an)
            if (a0 + an < n_app) {
#pragma unroll
              for (int e = 0; e < VEC; e += 4) {
                const float4 k4 = *reinterpret_cast<const float4 *>(kn + (a0 + an) * D + q * VEC + e);
                acc[an] += (Acc)x[e] * (Acc)k4.x;
                acc[an] += (Acc)x[e + 1] * (Acc)k4.y;
                acc[an] += (Acc)x[e + 2] * (Acc)k4.z;
                acc[an] += (Acc)x[e + 3] * (Acc)k4.w;
              }
            }
        }
#pragma unroll
        for (int an = 0; an < 8; ++an)
          if (a0 + an < n_app && acc[an] > best) {
            best = acc[an];
            best_a = a0 + an;
          }
      }
      if (m + best_a >= dv.S && (float)best > dv.score[base + j].y) {
        dv.score[base + j].y = (float)best;
        dv.pi[base + j] = m + best_a;
      }
    }
  }
}

// ------------------------------------------------------------------ create + merge + readout refresh
// A wave takes kAccumRows consecutive rows of [row_begin, m_after) of the updated state, one
// after the other.  do_create: rows >=
// m_before are created from their creator token; do_merge: the tokens whose target is this row
// are added in ascending position; do_copy: an untouched row's readout is copied to the new state
// version.  A fold that appends only part of the block runs create first (so the new rows have
// a normalised key to score against), then the second scoring pass, then merge.
constexpr int kAccumRows = 4;  // consecutive rows per wave: they share one scan of the targets

template <typename T, int D>
__global__ __launch_bounds__(256) void accum_kernel(Dev dv, Src src, int m_before, int m_after,
                                                    int row_begin, int do_create, int do_merge,
                                                    int do_copy, int check_app, int slot_old,
                                                    int slot_new) {
  constexpr int CPL = D / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u = blockIdx.y, b = u / dv.Hkv, h = u % dv.Hkv;
  const int row_first = row_begin + (blockIdx.x * 4 + wave) * kAccumRows;
  if (row_first >= m_after) return;
  const int C = dv.C;
  const int64_t base = (int64_t)u * C;
  const T *vsrc = (const T *)src.v + b * src.v_b + h * src.v_h;
  const float *gsrc = src.g ? src.g + b * src.g_b + h * src.g_h : nullptr;
  const T *kbar = (const T *)dv.kbar + base * D;

  // Most rows of a fold are not touched and only need their readout copied to the new state
  // version: those copies are requested first, so that they travel while the targets are
  // scanned.  The wave moves a row's k-hat and v-hat (2 * D elements) as 64 equal pieces.
  using Piece = typename PieceOf<2 * D * (int)sizeof(T) / 64>::type;
  Piece piece[kAccumRows] = {};
  if (do_copy) {
#pragma unroll
    for (int rr = 0; rr < kAccumRows; ++rr) {
      const int row = row_first + rr;
      if (row < m_before && row < m_after) {
        const int64_t eo = (slot_old * dv.slot_elems + ((int64_t)u * dv.Mcap + row) * D) * (int64_t)sizeof(T);
        const char *from = (lane < 32 ? (const char *)dv.khat : (const char *)dv.vhat) + eo;
        piece[rr] = reinterpret_cast<const Piece *>(from)[lane & 31];
      }
    }
  }
  // The block's merge targets, 64 tokens per register (blocks longer than 512 tokens take
  // further rounds below).  check_app: tokens appended in this fold carry their own new row in
  // pi and do not merge.
  int tg[8];
  auto load_targets = [&](int j0) {
#pragma unroll
    for (int bk = 0; bk < 8; ++bk) {
      const int j = j0 + 64 * bk + lane;
      tg[bk] = j < C ? dv.pi[base + j] : -1;
    }
    if (check_app) {
#pragma unroll
      for (int bk = 0; bk < 8; ++bk) {
        const int j = j0 + 64 * bk + lane;
        if (j < C && dv.app[base + j] >= 0) tg[bk] = -1;
      }
    }
  };
  if (do_merge) load_targets(0);

#pragma unroll
  for (int rr = 0; rr < kAccumRows; ++rr) {
    const int row = row_first + rr;
    if (row >= m_after) break;
    const int64_t ro = (int64_t)u * dv.Mcap + row;
    double sk[CPL];
    float sv[CPL];
    float rho = 0.f, w = 0.f;
    int n = 0;
    bool loaded = false;
    if (do_create && row >= m_before) {
      const int j0 = dv.creator[base + (row - m_before)];
      float nn = 0.f;
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        const int ch = lane * CPL + c;
        sk[c] = (double)Io<T>::load(kbar + (int64_t)j0 * D + ch);
        sv[c] = Io<T>::load(vsrc + (int64_t)j0 * src.v_t + ch);
        nn += sv[c] * sv[c];
      }
      rho = sqrtf(wave_sum(nn));
      w = 1.f;
      n = 1;
      loaded = true;
    }
    if (do_merge && row >= dv.S) {
      // the tokens that merge into this row, in ascending position: 64 tokens per ballot
      for (int j0 = 0; j0 < C; j0 += 512) {
        if (C > 512) load_targets(j0);
#pragma unroll
        for (int bk = 0; bk < 8; ++bk) {
          uint64_t hits = __builtin_amdgcn_ballot_w64(tg[bk] == row);
          while (hits) {
            const int t = j0 + 64 * bk + __builtin_ctzll(hits);
            hits &= hits - 1;
            if (!loaded) {
#pragma unroll
              for (int c = 0; c < CPL; ++c) {
                sk[c] = dv.sK[ro * D + lane * CPL + c];
                sv[c] = dv.sV[ro * D + lane * CPL + c];
              }
              rho = dv.rho[ro];
              w = dv.w[ro];
              n = dv.n[ro];
              loaded = true;
            }
            const float g = gsrc ? gsrc[(int64_t)t * src.g_t] : 1.f;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
              const int ch = lane * CPL + c;
              sk[c] = fma((double)g, (double)Io<T>::load(kbar + (int64_t)t * D + ch), sk[c]);
              sv[c] = fmaf(g, Io<T>::load(vsrc + (int64_t)t * src.v_t + ch), sv[c]);
            }
            w += g;
            n += 1;
          }
        }
      }
    }
    if (!loaded) {
      // untouched row: the sums stay; the new state version gets the copy of its readout
      if (do_copy && row < m_before) {
        const int64_t eo = (slot_new * dv.slot_elems + ro * D) * (int64_t)sizeof(T);
        char *to = (lane < 32 ? (char *)dv.khat : (char *)dv.vhat) + eo;
        reinterpret_cast<Piece *>(to)[lane & 31] = piece[rr];
      }
      continue;
    }
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
      dv.sK[ro * D + lane * CPL + c] = sk[c];
      dv.sV[ro * D + lane * CPL + c] = sv[c];
    }
    if (lane == 0) {
      dv.rho[ro] = rho;
      dv.w[ro] = w;
      dv.n[ro] = n;
    }
    write_readout<T, D>(dv, slot_new, u, h, row, sk, sv, rho, lane);
  }
}

// The merge pass of a fold done in place (nothing else reads the readout meanwhile, so untouched
// rows need no work at all): one wave per token.  The earliest token of each target row does the
// row: it adds every token with that target, in ascending position, and rewrites the row's
// readout; the other waves leave at once.
template <typename T, int D>
__device__ __forceinline__ void merge_token_wave(const Dev &dv, const Src &src, int check_app, int slot, int blk,
                                                 int u) {
  constexpr int CPL = D / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = u / dv.Hkv, h = u % dv.Hkv;
  const int C = dv.C;
  const int j = blk * 4 + wave;
  if (j >= C) return;
  const int64_t base = (int64_t)u * C;
  const int row = dv.pi[base + j];
  if (row < dv.S || row == 0x7fffffff) return;
  if (check_app && dv.app[base + j] >= 0) return;
  const T *vsrc = (const T *)src.v + b * src.v_b + h * src.v_h;
  const float *gsrc = src.g ? src.g + b * src.g_b + h * src.g_h : nullptr;
  const T *kbar = (const T *)dv.kbar + base * D;
  int tg[8];
  auto load_targets = [&](int j0) {
#pragma unroll
    for (int bk = 0; bk < 8; ++bk) {
      const int t = j0 + 64 * bk + lane;
      tg[bk] = t < C ? dv.pi[base + t] : -1;
    }
    if (check_app) {
#pragma unroll
      for (int bk = 0; bk < 8; ++bk) {
        const int t = j0 + 64 * bk + lane;
        if (t < C && dv.app[base + t] >= 0) tg[bk] = -1;
      }
    }
  };
  // The row's sums are requested before it is known whether this wave is the one that does the
  // row: in decode-sized folds (few tokens, many rows) it almost always is, and the loads then
  // travel together with the scan of the targets.
  const int64_t ro = (int64_t)u * dv.Mcap + row;
  double sk[CPL];
  float sv[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    sk[c] = dv.sK[ro * D + lane * CPL + c];
    sv[c] = dv.sV[ro * D + lane * CPL + c];
  }
  const float rho = dv.rho[ro];
  float w = dv.w[ro];
  int n = dv.n[ro];
  // is an earlier token bound for the same row?
  for (int j0 = 0; j0 <= j; j0 += 512) {
    load_targets(j0);
#pragma unroll
    for (int bk = 0; bk < 8; ++bk) {
      const int t0 = j0 + 64 * bk;
      uint64_t hits = __builtin_amdgcn_ballot_w64(tg[bk] == row);
      if (t0 + 64 > j) hits &= t0 > j ? 0ull : ((1ull << (j - t0)) - 1ull);
      if (hits) return;
    }
  }
  for (int j0 = j / 512 * 512; j0 < C; j0 += 512) {
    if (C > 512) load_targets(j0);
#pragma unroll
    for (int bk = 0; bk < 8; ++bk) {
      uint64_t hits = __builtin_amdgcn_ballot_w64(tg[bk] == row);
      while (hits) {
        const int t = j0 + 64 * bk + __builtin_ctzll(hits);
        hits &= hits - 1;
        const float g = gsrc ? gsrc[(int64_t)t * src.g_t] : 1.f;
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
          const int ch = lane * CPL + c;
          sk[c] = fma((double)g, (double)Io<T>::load(kbar + (int64_t)t * D + ch), sk[c]);
          sv[c] = fmaf(g, Io<T>::load(vsrc + (int64_t)t * src.v_t + ch), sv[c]);
        }
        w += g;
        n += 1;
      }
    }
  }
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    dv.sK[ro * D + lane * CPL + c] = sk[c];
    dv.sV[ro * D + lane * CPL + c] = sv[c];
  }
  if (lane == 0) {
    dv.w[ro] = w;
    dv.n[ro] = n;
  }
  write_readout<T, D>(dv, slot, u, h, row, sk, sv, rho, lane);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void merge_inplace_kernel(Dev dv, Src src, int check_app, int slot) {
  merge_token_wave<T, D>(dv, src, check_app, slot, blockIdx.x, blockIdx.y);
}

// The same merge for a prefill's small folds, where the new state version lives in another slot:
// the token waves above write the touched rows' readout into slot_new, and further workgroups of
// the same launch copy the readout of the rows no token goes to (a wave takes kCopyRows rows,
// asks for their readout, scans the block's targets, stores the copies of the untouched ones).
// Against accum_kernel, which walks rows and finds each row's tokens, a touched row here starts
// from its token: one wave per touched row and a short chain of dependent loads, which is what
// counts when the whole launch is a few thousand waves; accum_kernel moves the bytes of a large
// state faster.
constexpr int kCopyRows = 4;
template <typename T, int D>
__device__ __forceinline__ void copy_untouched_wave(const Dev &dv, int check_app, int slot_old, int slot_new,
                                                    int m_before, int blk, int u) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row_first = (blk * 4 + wave) * kCopyRows;
  if (row_first >= m_before) return;
  const int C = dv.C;
  const int64_t base = (int64_t)u * C;
  using Piece = typename PieceOf<2 * D * (int)sizeof(T) / 64>::type;
  Piece piece[kCopyRows] = {};
#pragma unroll
  for (int rr = 0; rr < kCopyRows; ++rr) {
    const int row = row_first + rr;
    if (row < m_before) {
      const int64_t eo = (slot_old * dv.slot_elems + ((int64_t)u * dv.Mcap + row) * D) * (int64_t)sizeof(T);
      const char *from = (lane < 32 ? (const char *)dv.khat : (const char *)dv.vhat) + eo;
      piece[rr] = reinterpret_cast<const Piece *>(from)[lane & 31];
    }
  }
  bool touched[kCopyRows] = {};
  for (int j0 = 0; j0 < C; j0 += 64) {
    const int j = j0 + lane;
    int tg = j < C ? dv.pi[base + j] : -1;
    if (check_app && j < C && dv.app[base + j] >= 0) tg = -1;
#pragma unroll
    for (int rr = 0; rr < kCopyRows; ++rr)
      touched[rr] = touched[rr] || __builtin_amdgcn_ballot_w64(tg == row_first + rr) != 0;
  }
#pragma unroll
  for (int rr = 0; rr < kCopyRows; ++rr) {
    const int row = row_first + rr;
    if (row < m_before && (!touched[rr] || row < dv.S)) {  // sinks take no merges
      const int64_t eo = (slot_new * dv.slot_elems + ((int64_t)u * dv.Mcap + row) * D) * (int64_t)sizeof(T);
      char *to = (lane < 32 ? (char *)dv.khat : (char *)dv.vhat) + eo;
      reinterpret_cast<Piece *>(to)[lane & 31] = piece[rr];
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void merge_copy_kernel(Dev dv, Src src, int check_app, int slot_old, int slot_new,
                                                         int m_before, int n_tok_blocks) {
  if ((int)blockIdx.x < n_tok_blocks)
    merge_token_wave<T, D>(dv, src, check_app, slot_new, blockIdx.x, blockIdx.y);
  else
    copy_untouched_wave<T, D>(dv, check_app, slot_old, slot_new, m_before, blockIdx.x - n_tok_blocks, blockIdx.y);
}

// Recompute the normalised readout of rows [0, m) from the stored sums (after an import).
template <typename T, int D>
__global__ __launch_bounds__(256) void refresh_kernel(Dev dv, int m, int slot) {
  constexpr int CPL = D / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u = blockIdx.y, h = u % dv.Hkv;
  const int row = blockIdx.x * 4 + wave;
  if (row >= m) return;
  const int64_t ro = (int64_t)u * dv.Mcap + row;
  double sk[CPL];
  float sv[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    sk[c] = dv.sK[ro * D + lane * CPL + c];
    sv[c] = dv.sV[ro * D + lane * CPL + c];
  }
  write_readout<T, D>(dv, slot, u, h, row, sk, sv, dv.rho[ro], lane);
}

// Copy positions [p0, p1) of a token source (its token 0 is position src_t0) into the ring.
template <typename T>
__global__ __launch_bounds__(64) void ring_copy_kernel(Dev dv, Src src, int64_t src_t0, int64_t p0) {
  const int u = blockIdx.y, b = u / dv.Hkv, h = u % dv.Hkv;
  const int64_t p = p0 + blockIdx.x;
  const int64_t t = p - src_t0;
  const int slot = (int)(p % dv.L);
  const T *ks = (const T *)src.k + b * src.k_b + h * src.k_h + t * src.k_t;
  const T *vs = (const T *)src.v + b * src.v_b + h * src.v_h + t * src.v_t;
  T *kd = (T *)dv.winK + ((int64_t)u * dv.L + slot) * dv.d;
  T *vd = (T *)dv.winV + ((int64_t)u * dv.L + slot) * dv.d;
  for (int c = threadIdx.x; c < dv.d; c += 64) {
    kd[c] = ks[c];
    vd[c] = vs[c];
  }
  if (threadIdx.x == 0)
    dv.winG[(int64_t)u * dv.L + slot] = src.g ? src.g[b * src.g_b + h * src.g_h + t * src.g_t] : 1.f;
}

#define KVM_DISPATCH(dv, KERNEL, grid, block, shmem, st, ...)                                   \
  do {                                                                                          \
    if ((dv).io == 0 && (dv).d == 64)                                                           \
      hipLaunchKernelGGL((KERNEL<float, 64>), grid, block, shmem, st, __VA_ARGS__);             \
    else if ((dv).io == 0 && (dv).d == 128)                                                     \
      hipLaunchKernelGGL((KERNEL<float, 128>), grid, block, shmem, st, __VA_ARGS__);            \
    else if ((dv).io == 1 && (dv).d == 64)                                                      \
      hipLaunchKernelGGL((KERNEL<bf16_t, 64>), grid, block, shmem, st, __VA_ARGS__);            \
    else if ((dv).io == 1 && (dv).d == 128)                                                     \
      hipLaunchKernelGGL((KERNEL<bf16_t, 128>), grid, block, shmem, st, __VA_ARGS__);           \
    else                                                                                        \
      return hipErrorInvalidValue;                                                              \
  } while (0)

}  // namespace

hipError_t launch_memkey(const Dev &dv, const Src &src, int n_blocks, hipStream_t st) {
  const int per_wg = kMemkeyTok * 4 * 64 / (dv.d * (dv.io == 0 ? 4 : 2) / 16);  // tokens per workgroup
  dim3 grid((dv.C * n_blocks + per_wg - 1) / per_wg, dv.U);
  KVM_DISPATCH(dv, memkey_kernel, grid, dim3(256), 0, st, dv, src, n_blocks);
  return hipGetLastError();
}

hipError_t launch_score(const Dev &dv, int slot, int row0, int row1, bool first_pass, hipStream_t st) {
  dim3 grid((dv.C + 3) / 4, dv.U);
  KVM_DISPATCH(dv, score_kernel, grid, dim3(256), 0, st, dv, slot, row0, row1, first_pass ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_select(const Dev &dv, int m, int n_app, bool take_all, hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(dv.U), dim3(256), (size_t)dv.C * 8, st, dv, m, n_app,
                     take_all ? 1 : 0);
  return hipGetLastError();
}

bool append_fits(const Dev &dv, int n_app) {
  return n_app > 0 && n_app <= kAppendMax && dv.C % 2 == 0 && dv.C <= 256;
}

hipError_t launch_append(const Dev &dv, const Src &src, int m, int n_app, int slot_new, hipStream_t st) {
  const size_t lds = (size_t)dv.C * 8 + (kAppendMax + 4) * 4 + (size_t)n_app * dv.d * 4;
  KVM_DISPATCH(dv, append_kernel, dim3(dv.U), dim3(256), lds, st, dv, src, m, n_app, slot_new);
  return hipGetLastError();
}

hipError_t launch_accum(const Dev &dv, const Src &src, int m_before, int m_after, int row_begin,
                        bool do_create, bool do_merge, bool do_copy, bool check_app, int slot_old,
                        int slot_new, hipStream_t st) {
  if (m_after <= row_begin) return hipSuccess;
  dim3 grid((m_after - row_begin + 4 * kAccumRows - 1) / (4 * kAccumRows), dv.U);
  KVM_DISPATCH(dv, accum_kernel, grid, dim3(256), 0, st, dv, src, m_before, m_after, row_begin,
               do_create ? 1 : 0, do_merge ? 1 : 0, do_copy ? 1 : 0, check_app ? 1 : 0, slot_old, slot_new);
  return hipGetLastError();
}

hipError_t launch_merge_inplace(const Dev &dv, const Src &src, bool check_app, int slot, hipStream_t st) {
  dim3 grid((dv.C + 3) / 4, dv.U);
  KVM_DISPATCH(dv, merge_inplace_kernel, grid, dim3(256), 0, st, dv, src, check_app ? 1 : 0, slot);
  return hipGetLastError();
}

hipError_t launch_merge_copy(const Dev &dv, const Src &src, bool check_app, int slot_old, int slot_new,
                             int m_before, hipStream_t st) {
  const int n_tok_blocks = (dv.C + 3) / 4, n_row_blocks = (m_before + 4 * kCopyRows - 1) / (4 * kCopyRows);
  dim3 grid(n_tok_blocks + n_row_blocks, dv.U);
  KVM_DISPATCH(dv, merge_copy_kernel, grid, dim3(256), 0, st, dv, src, check_app ? 1 : 0, slot_old, slot_new,
               m_before, n_tok_blocks);
  return hipGetLastError();
}

hipError_t launch_refresh(const Dev &dv, int m, int slot, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  dim3 grid((m + 3) / 4, dv.U);
  KVM_DISPATCH(dv, refresh_kernel, grid, dim3(256), 0, st, dv, m, slot);
  return hipGetLastError();
}

hipError_t launch_ring_copy(const Dev &dv, const Src &src, int64_t src_t0, int64_t p0, int64_t p1,
                            hipStream_t st) {
  if (p1 <= p0) return hipSuccess;
  dim3 grid((unsigned)(p1 - p0), dv.U);
  if (dv.io == 0)
    hipLaunchKernelGGL(ring_copy_kernel<float>, grid, dim3(64), 0, st, dv, src, src_t0, p0);
  else
    hipLaunchKernelGGL(ring_copy_kernel<bf16_t>, grid, dim3(64), 0, st, dv, src, src_t0, p0);
  return hipGetLastError();
}

}  // namespace kvm
