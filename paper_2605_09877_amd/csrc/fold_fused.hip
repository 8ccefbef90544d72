// A run of folds in one launch, one workgroup per (sequence, KV head) unit (bf16, head_dim 128).
//
// A fold (sections "KVM weight preparation", "Append", "Merge" and the readout equations of the
// paper's Method section) is a chain of small dependent steps: memory keys, similarity of the block
// to the normalised state, selection of the tokens to append, creation of their rows, similarity of
// the remaining tokens to the new rows, winner-take-all accumulation, readout refresh.  Units are
// independent of each other, and consecutive folds of one unit depend on each other through that
// unit's state alone, so one workgroup can walk a unit through all of a run's folds with workgroup
// barriers between the steps: no launch boundaries inside the chain and none between its folds,
// and a workgroup per unit leaves the rest of the chip to the attention launches that run beside
// it.  Per fold:
//   1. memory keys k-bar = LN_s(zero_r(k)) in fp64, kept in registers as matrix-core operands by
//      the wave that owns the 32 tokens (and written once to scratch for step 5);
//   2. D[row, token] = K-hat_tile . K-bar^T on the matrix cores, state rows streaming HBM/L2 ->
//      LDS in 64-row tiles: append score s_j = max over all rows, merge target = argmax over rows
//      >= S (a lane owns a token and scans rows in ascending order: ties keep the lowest row);
//   3. when the budget has room for some of the block: the n_append smallest (s_j, j) are taken
//      (ranks by counting), their rows are created (step 5) and step 2 runs again over the new
//      rows for the tokens that were not taken (a strictly larger score moves a token);
//   4. tokens are ordered by (target row, creator first, position) by counting, which gives every
//      touched row its tokens in the order in which they are added;
//   5. 16 lanes per touched row (8 channels each): sums read (or created from the creator token),
//      tokens added in ascending position, sums written, readout row (LN_s in fp64 on keys, stored
//      radius on values) written into the new state version; rows nothing was added to are copied
//      to the new version (prefill) or left alone (in place).
// Integer decisions rest on fp64 LN_s and fp64 key sums, as everywhere in this library.
#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr int kNoRow = 0x7fffffff;
constexpr int kTileBytes = kTileElems * 2;   // 16 KiB
constexpr int kTileBufs = 4;                  // two stages of two tiles
constexpr uint32_t kOrdBits = 11;             // (row << 11) | order within the row; C <= 1024

__device__ __forceinline__ bool beats(float sa, int ia, float sb, int ib) {
  return sa > sb || (sa == sb && ia < ib);
}

// LDS layout of one workgroup (bytes from the start of dynamic shared memory).
struct FoldLds {
  uint32_t tiles;    // kTileBufs tiles of K-hat; between score passes also scratch for sort keys
  uint32_t app;      // float [C]  append score s_j
  uint32_t best;     // float [C]  winning merge score
  uint32_t pi;       // int   [C]  target row
  uint32_t rank;     // int   [C]  rank among the appended tokens, or -1
  uint32_t sorted;   // u16   [C]  tokens ordered by (row, creator first, position)
  uint32_t seg;      // u16   [C]  positions in `sorted` where a row's tokens start
  uint32_t merge;    // float/int [3][NW * 32] partial winners of waves that share tokens
  uint32_t masks;    // u64   [C / 64] taken-token masks
  uint32_t counters; // int   [4]
  uint32_t bitmap;   // u32   [Mcap / 32] rows that receive tokens in this fold
  uint32_t total;
};
__host__ __device__ inline FoldLds fold_lds(int C, int Mcap, int NW) {
  FoldLds l;
  uint32_t o = 0;
  auto take = [&](uint32_t bytes) {
    const uint32_t at = o;
    o += (bytes + 15u) & ~15u;
    return at;
  };
  l.tiles = take(kTileBufs * kTileBytes);
  l.app = take(4u * C);
  l.best = take(4u * C);
  l.pi = take(4u * C);
  l.rank = take(4u * C);
  l.sorted = take(2u * C);
  l.seg = take(2u * C);
  l.merge = take(3u * 4u * NW * 32);
  l.masks = take(8u * ((C + 63) / 64));
  l.counters = take(16);
  l.bitmap = take(4u * ((Mcap + 31) / 32));
  l.total = o;
  return l;
}

template <int NW>
struct Ctx {
  const Dev &dv;
  unsigned char *smem;
  FoldLds l;
  int u, tid, lane, wave;
  __device__ float *s_app() const { return (float *)(smem + l.app); }
  __device__ float *s_best() const { return (float *)(smem + l.best); }
  __device__ int *s_pi() const { return (int *)(smem + l.pi); }
  __device__ int *s_rank() const { return (int *)(smem + l.rank); }
  __device__ uint16_t *s_sorted() const { return (uint16_t *)(smem + l.sorted); }
  __device__ uint16_t *s_seg() const { return (uint16_t *)(smem + l.seg); }
  __device__ int *s_cnt() const { return (int *)(smem + l.counters); }
  __device__ uint32_t *s_bitmap() const { return (uint32_t *)(smem + l.bitmap); }
  __device__ unsigned long long *s_masks() const { return (unsigned long long *)(smem + l.masks); }
};

// ------------------------------------------------------------------------------------------------
// Step 1: the memory keys of the wave's 32 tokens as B operands (lane = 32 g + i holds token i,
// channels 16 ks + 8 g .. + 7 for ks = 0..7), computed from k in fp64.  `store`: also written to
// the unit's scratch block for the accumulation step.
__device__ __forceinline__ void memory_keys(const Dev &dv, const uint16_t *krow, int h, bool store,
                                            uint16_t *kbar_row, int lane, bf16x8 (&kreg)[8]) {
  constexpr int D = kHeadDim;
  const int g = lane >> 5;
  float x[64];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const uint4 raw = *reinterpret_cast<const uint4 *>(krow + 16 * ks + 8 * g);
    float f[8];
    unpack16<bf16_t>(raw, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[8 * ks + e] = (16 * ks + 8 * g + e) < dv.r ? 0.f : f[e];
  }
  double s = 0.0;
#pragma unroll
  for (int c = 0; c < 64; ++c) s += (double)x[c];
  const double mean = swap_sum<true>(s) / (double)D;   // with the lane that holds the other 64 channels
  double q = 0.0;
#pragma unroll
  for (int c = 0; c < 64; ++c) {
    const double dl = (double)x[c] - mean;
    q += dl * dl;
  }
  const double rden = 1.0 / sqrt(swap_sum<true>(q) / (double)D + (double)dv.ln_eps);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const int ch0 = 16 * ks + 8 * g;
    float ga[8], be[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      ga[e] = 1.f;
      be[e] = 0.f;
    }
    if (dv.gamma) {
      const float4 a0 = *reinterpret_cast<const float4 *>(dv.gamma + h * D + ch0);
      const float4 a1 = *reinterpret_cast<const float4 *>(dv.gamma + h * D + ch0 + 4);
      ga[0] = a0.x; ga[1] = a0.y; ga[2] = a0.z; ga[3] = a0.w;
      ga[4] = a1.x; ga[5] = a1.y; ga[6] = a1.z; ga[7] = a1.w;
    }
    if (dv.beta) {
      const float4 a0 = *reinterpret_cast<const float4 *>(dv.beta + h * D + ch0);
      const float4 a1 = *reinterpret_cast<const float4 *>(dv.beta + h * D + ch0 + 4);
      be[0] = a0.x; be[1] = a0.y; be[2] = a0.z; be[3] = a0.w;
      be[4] = a1.x; be[5] = a1.y; be[6] = a1.z; be[7] = a1.w;
    }
    Frag8 f;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const double y0 = ((double)x[8 * ks + e] - mean) * rden * (double)ga[e] + (double)be[e];
      const double y1 = ((double)x[8 * ks + e + 1] - mean) * rden * (double)ga[e + 1] + (double)be[e + 1];
      f.w[e >> 1] = (uint32_t)float_to_bf16_bits((float)y0) | ((uint32_t)float_to_bf16_bits((float)y1) << 16);
    }
    kreg[ks] = f.v;
    if (store) *reinterpret_cast<uint4 *>(kbar_row + ch0) = f.q;
  }
}

// ------------------------------------------------------------------------------------------------
// Step 2: one pass of the block's tokens over state rows [row0, row1) of readout version `slot`.
// first: rows are the state before the append; every token gets s_j and its best row >= S.
// Otherwise rows are the ones created in this fold; a token that was not taken moves to one of
// them when that score is strictly larger than its stored best.
template <int NW>
__device__ __forceinline__ void score_pass(const Ctx<NW> &cx, const Src &src, int64_t tok, int slot, int row0,
                                           int row1, bool first, uint16_t *kbar_blk) {
  constexpr int D = kHeadDim;
  const Dev &dv = cx.dv;
  const int lane = cx.lane, wave = cx.wave, u = cx.u;
  const int g = lane >> 5, l32 = lane & 31;
  const int b = u / dv.Hkv, h = u % dv.Hkv;
  const int C = dv.C, TG = C / 32;
  const int n_tiles = (row1 - row0 + kTileKeys - 1) / kTileKeys;
  const int n_stages = (n_tiles + 1) / 2;
  uint16_t *Ks = (uint16_t *)(cx.smem + cx.l.tiles);
  const uint32_t ks_addr = lds_addr_of(Ks);
  const char *khat = (const char *)dv.khat + (slot * dv.slot_elems + ((int64_t)u * dv.Mcap + row0) * D) * 2;
  uint32_t koff[8];
  ktile_offsets(lane, koff);
  // this wave's share of a tile's sixteen 1-KiB loads: pieces wave, wave + NW, ...; the chunk
  // permutation of a piece depends on (piece % 4) = (wave % 4)
  const DmaLane dl = dma_lane(lane);
  const int wq = wave & 3;
  const uint32_t kcol = wq == 0 ? dl.kcol[0] : wq == 1 ? dl.kcol[1] : wq == 2 ? dl.kcol[2] : dl.kcol[3];
  auto issue_stage = [&](int sg) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int t = 2 * sg + i;
      if (t < n_tiles) {
        const int base = t * kTileKeys, valid = row1 - row0 - base;
        const uint32_t buf = ks_addr + (uint32_t)(2 * (sg & 1) + i) * kTileBytes;
#pragma unroll
        for (int n = 0; n < 16 / NW; ++n) {
          const int bi = wave + NW * n;
          int r = 4 * bi + (int)dl.rl;
          r = r < valid ? r : valid - 1;   // rows past the end repeat the last one (masked below)
          dma16(khat + (uint32_t)base * (D * 2), (uint32_t)r * (D * 2) + kcol, buf + (uint32_t)bi * 1024u);
        }
      }
    }
  };
  float *x_all = (float *)(cx.smem + cx.l.merge), *x_best = x_all + NW * 32;
  int *x_idx = (int *)(x_best + NW * 32);

  for (int g0 = 0; g0 < TG; g0 += NW) {
    const int Gp = TG - g0 < NW ? TG - g0 : NW;   // token groups in this round
    const int wpg = NW / Gp;                      // waves that share a group's tokens (they split the tiles)
    const int gi = wave / wpg, sub = wave % wpg;
    const bool active = gi < Gp;
    const int j = (g0 + (active ? gi : 0)) * 32 + l32;
    if (n_stages > 0) issue_stage(0);
    bf16x8 kreg[8];
    if (active) {
      if (first) {
        const uint16_t *krow = (const uint16_t *)src.k + b * src.k_b + h * src.k_h + (tok + j) * src.k_t;
        memory_keys(dv, krow, h, sub == 0, kbar_blk + (int64_t)j * D, lane, kreg);
      } else {
        const uint16_t *krow = kbar_blk + (int64_t)j * D;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          Frag8 f;
          f.q = *reinterpret_cast<const uint4 *>(krow + 16 * ks + 8 * g);
          kreg[ks] = f.v;
        }
      }
    }
    float best_all = -INFINITY, best = -INFINITY;
    int best_i = kNoRow;
    for (int sg = 0; sg < n_stages; ++sg) {
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      if (sg + 1 < n_stages) issue_stage(sg + 1);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int t = 2 * sg + i;
        if (!active || t >= n_tiles || (t % wpg) != sub) continue;
        const uint16_t *Kt = Ks + (2 * (sg & 1) + i) * kTileElems;
#pragma unroll
        for (int rh = 0; rh < 2; ++rh) {
          // two accumulation chains (channels 0..63 and 64..127)
          f32x16 acc0, acc1;
          {
            bf16x8 kf[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) kf[q] = ktile_frag(Kt, koff, rh, q);
            const f32x16 zero = {0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
              acc0 = mfma32(kf[ks], kreg[ks], ks == 0 ? zero : acc0);
              acc1 = mfma32(kf[ks + 4], kreg[ks + 4], ks == 0 ? zero : acc1);
            }
          }
          const int base = row0 + t * kTileKeys + 32 * rh;
          if (base >= row1) continue;
          const bool edge = base < dv.S || base + 32 > row1;
          if (edge) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int i2 = base + mfma_row(v, g);
              const float sc = acc0[v] + acc1[v];
              if (i2 < row1) {
                best_all = fmaxf(best_all, sc);
                if (i2 >= dv.S && sc > best) {
                  best = sc;
                  best_i = i2;
                }
              }
            }
          } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const float sc = acc0[v] + acc1[v];
              if (sc > best) {
                best = sc;
                best_i = base + mfma_row(v, g);
              }
            }
          }
        }
      }
    }
    best_all = fmaxf(best_all, best);
    {
      // the other lane half holds the other rows of the same token
      const float ob = __shfl_xor(best, 32, kWave);
      const int oi = __shfl_xor(best_i, 32, kWave);
      const float oa = __shfl_xor(best_all, 32, kWave);
      if (beats(ob, oi, best, best_i)) {
        best = ob;
        best_i = oi;
      }
      best_all = fmaxf(best_all, oa);
    }
    // the waves that share the tokens, through LDS
    if (wpg > 1) {
      if (active && sub != 0 && g == 0) {
        const int xi = wave * 32 + l32;
        x_all[xi] = best_all;
        x_best[xi] = best;
        x_idx[xi] = best_i;
      }
      __syncthreads();
      if (active && sub == 0 && g == 0) {
        for (int o = 1; o < wpg; ++o) {
          const int xi = (wave + o) * 32 + l32;
          best_all = fmaxf(best_all, x_all[xi]);
          if (beats(x_best[xi], x_idx[xi], best, best_i)) {
            best = x_best[xi];
            best_i = x_idx[xi];
          }
        }
      }
    }
    if (active && sub == 0 && g == 0) {
      if (first) {
        cx.s_app()[j] = best_all;
        cx.s_best()[j] = best;
        cx.s_pi()[j] = best_i;
        cx.s_rank()[j] = -1;
      } else if (cx.s_rank()[j] < 0 && best_i != kNoRow && best > cx.s_best()[j]) {
        cx.s_best()[j] = best;
        cx.s_pi()[j] = best_i;
      }
    }
    __syncthreads();   // tile buffers and the merge scratch are free again
  }
}

// ------------------------------------------------------------------------------------------------
// Step 3: the n_app tokens with the smallest (s_j, position) are taken; a taken token's rank among
// the taken ones, in position order, is the new row it creates.
template <int NW>
__device__ __forceinline__ void select_tokens(const Ctx<NW> &cx, int m, int n_app) {
  constexpr int NT = 64 * NW;
  const int C = cx.dv.C, tid = cx.tid, lane = cx.lane;
  unsigned long long *key = (unsigned long long *)(cx.smem + cx.l.tiles);   // [C], tiles are idle here
  for (int j = tid; j < C; j += NT) {
    uint32_t f = __float_as_uint(cx.s_app()[j]);
    f = f == 0x80000000u ? 0u : f;   // -0 and +0 are one score
    const uint32_t mono = (f & 0x80000000u) ? ~f : (f | 0x80000000u);
    key[j] = ((unsigned long long)mono << 32) | (uint32_t)j;
  }
  __syncthreads();
  for (int j0 = 0; j0 < C; j0 += NT) {   // C is a multiple of 64: whole waves
    const int j = j0 + tid;
    bool take = false;
    if (j < C) {
      const unsigned long long kj = key[j];
      int rank = 0;
      for (int t = 0; t < C; t += 2) {
        const ulonglong2 k2 = *reinterpret_cast<const ulonglong2 *>(key + t);
        rank += k2.x < kj ? 1 : 0;
        rank += k2.y < kj ? 1 : 0;
      }
      take = rank < n_app;
    }
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(take);
    if (lane == 0 && j < C) cx.s_masks()[j >> 6] = bal;
  }
  __syncthreads();
  for (int j = tid; j < C; j += NT) {
    const int wj = j >> 6, lj = j & 63;
    const unsigned long long mine = cx.s_masks()[wj];
    if ((mine >> lj) & 1ull) {
      int a = __builtin_popcountll(mine & ((1ull << lj) - 1ull));
      for (int w2 = 0; w2 < wj; ++w2) a += __builtin_popcountll(cx.s_masks()[w2]);
      cx.s_rank()[j] = a;
      cx.s_pi()[j] = m + a;
      cx.s_best()[j] = __uint_as_float(0x7fc00000u);
    } else {
      cx.s_rank()[j] = -1;
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// Step 4: tokens ordered by (row, creator first, position); where each row's run of tokens starts;
// which of the rows below m receive tokens.  identity: every token creates its own row, in
// position order (nothing to sort).  Returns the number of runs.
template <int NW>
__device__ __forceinline__ int order_tokens(const Ctx<NW> &cx, int m, bool identity) {
  constexpr int NT = 64 * NW;
  const int C = cx.dv.C, tid = cx.tid, lane = cx.lane;
  uint32_t *key = (uint32_t *)(cx.smem + cx.l.tiles);   // [C]
  int *cnt = cx.s_cnt();
  if (tid == 0) cnt[0] = 0;
  if (identity) {
    // every token creates its own row, in position order
    for (int j = tid; j < C; j += NT) {
      cx.s_sorted()[j] = (uint16_t)j;
      cx.s_seg()[j] = (uint16_t)j;
    }
    __syncthreads();
    return C;
  }
  for (int j = tid; j < C; j += NT) {
    const int row = cx.s_pi()[j];
    const uint32_t ord = cx.s_rank()[j] >= 0 ? 0u : (uint32_t)(j + 1);
    key[j] = row == kNoRow ? (0xffffffffu - (uint32_t)(C - 1 - j)) : (((uint32_t)row << kOrdBits) | ord);
  }
  __syncthreads();
  for (int j = tid; j < C; j += NT) {
    const uint32_t kj = key[j];
    int pos = 0;
    for (int t = 0; t < C; t += 4) {
      const uint4 k4 = *reinterpret_cast<const uint4 *>(key + t);
      pos += k4.x < kj ? 1 : 0;
      pos += k4.y < kj ? 1 : 0;
      pos += k4.z < kj ? 1 : 0;
      pos += k4.w < kj ? 1 : 0;
    }
    cx.s_sorted()[pos] = (uint16_t)j;
  }
  __syncthreads();
  for (int i0 = 0; i0 < C; i0 += NT) {
    const int i = i0 + tid;
    bool start = false;
    int row = kNoRow;
    if (i < C) {
      const uint32_t ki = key[cx.s_sorted()[i]];
      if (ki < 0xffffffffu - (uint32_t)C) {   // a token with a row
        row = (int)(ki >> kOrdBits);
        start = i == 0 || (int)(key[cx.s_sorted()[i - 1]] >> kOrdBits) != row;
      }
    }
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(start);
    int base = 0;
    if (lane == 0 && bal) base = atomicAdd(&cnt[0], __builtin_popcountll(bal));
    base = __shfl(base, 0, kWave);
    if (start) {
      cx.s_seg()[base + __builtin_popcountll(bal & ((1ull << lane) - 1ull))] = (uint16_t)i;
      if (row < m) atomicOr(&cx.s_bitmap()[row >> 5], 1u << (row & 31));
    }
  }
  __syncthreads();
  return cnt[0];
}

// ------------------------------------------------------------------------------------------------
// Step 5: 16 lanes per row, 8 channels per lane.  The row's run of tokens starts at sorted[i0]; a
// run that starts with a creator makes a new row of it.  only_creators: stop after the creator
// (the rows created ahead of the second score pass; their merges follow in the full pass, which
// then starts from the sums written here).
template <int NW>
__device__ __forceinline__ void row_pass(const Ctx<NW> &cx, const Src &src, int64_t tok, int m, int slot_new,
                                         int n_seg, const uint16_t *kbar_blk, bool only_creators, bool skip_creators) {
  constexpr int D = kHeadDim, NG = 4 * NW;
  const Dev &dv = cx.dv;
  const int u = cx.u, b = u / dv.Hkv, h = u % dv.Hkv;
  const int gid = cx.tid >> 4, c16 = cx.tid & 15, ch0 = 8 * c16;
  const int C = dv.C;
  const uint16_t *vsrc = (const uint16_t *)src.v + b * src.v_b + h * src.v_h + tok * src.v_t;
  const float *gsrc = src.g ? src.g + b * src.g_b + h * src.g_h + tok * src.g_t : nullptr;
  float ga[8], be[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ga[e] = dv.gamma ? dv.gamma[h * D + ch0 + e] : 1.f;
    be[e] = dv.beta ? dv.beta[h * D + ch0 + e] : 0.f;
  }
  const uint16_t *sorted = cx.s_sorted();
  const int *pi = cx.s_pi(), *rank = cx.s_rank();
  for (int si = gid; si < n_seg; si += NG) {
    int i = cx.s_seg()[si];
    const int t0 = sorted[i];
    const int row = pi[t0];
    const bool created = rank[t0] >= 0;
    if (only_creators && !created) continue;
    // the run's length (tokens of this row)
    int n_run = 1;
    while (i + n_run < C && pi[sorted[i + n_run]] == row && rank[sorted[i + n_run]] < 0) ++n_run;
    if (only_creators) n_run = 1;
    if (skip_creators && created && n_run == 1) continue;   // made by the earlier pass, nothing merges into it
    const int64_t ro = (int64_t)u * dv.Mcap + row;
    double sk[8];
    float sv[8];
    float rho, w;
    int n;
    // first token's rows are asked for together with the sums
    uint4 kraw = *reinterpret_cast<const uint4 *>(kbar_blk + (int64_t)t0 * D + ch0);
    uint4 vraw = *reinterpret_cast<const uint4 *>(vsrc + (int64_t)t0 * src.v_t + ch0);
    float g0 = gsrc ? gsrc[(int64_t)t0 * src.g_t] : 1.f;
    int first_tok = 0;
    if (created && !skip_creators) {
      float kf[8], vf[8];
      unpack16<bf16_t>(kraw, kf);
      unpack16<bf16_t>(vraw, vf);
      float nn = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sk[e] = (double)kf[e];
        sv[e] = vf[e];
        nn += vf[e] * vf[e];
      }
      rho = sqrtf(group_sum<16>(nn));
      w = 1.f;
      n = 1;
      first_tok = 1;
    } else {
      const double2 *pk = reinterpret_cast<const double2 *>(dv.sK + ro * D + ch0);
      const float4 *pv = reinterpret_cast<const float4 *>(dv.sV + ro * D + ch0);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const double2 x = pk[q];
        sk[2 * q] = x.x;
        sk[2 * q + 1] = x.y;
      }
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const float4 x = pv[q];
        sv[4 * q] = x.x; sv[4 * q + 1] = x.y; sv[4 * q + 2] = x.z; sv[4 * q + 3] = x.w;
      }
      rho = dv.rho[ro];
      w = dv.w[ro];
      n = dv.n[ro];
      first_tok = created ? 1 : 0;   // skip_creators: the creator is already in the sums
    }
    for (int q = first_tok; q < n_run; ++q) {
      if (q > 0) {
        const int t = sorted[i + q];
        kraw = *reinterpret_cast<const uint4 *>(kbar_blk + (int64_t)t * D + ch0);
        vraw = *reinterpret_cast<const uint4 *>(vsrc + (int64_t)t * src.v_t + ch0);
        g0 = gsrc ? gsrc[(int64_t)t * src.g_t] : 1.f;
      }
      float kf[8], vf[8];
      unpack16<bf16_t>(kraw, kf);
      unpack16<bf16_t>(vraw, vf);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sk[e] = fma((double)g0, (double)kf[e], sk[e]);
        sv[e] = fmaf(g0, vf[e], sv[e]);
      }
      w += g0;
      n += 1;
    }
    {
      double2 *pk = reinterpret_cast<double2 *>(dv.sK + ro * D + ch0);
      float4 *pv = reinterpret_cast<float4 *>(dv.sV + ro * D + ch0);
#pragma unroll
      for (int q = 0; q < 4; ++q) pk[q] = make_double2(sk[2 * q], sk[2 * q + 1]);
#pragma unroll
      for (int q = 0; q < 2; ++q) pv[q] = make_float4(sv[4 * q], sv[4 * q + 1], sv[4 * q + 2], sv[4 * q + 3]);
      if (c16 == 0) {
        dv.rho[ro] = rho;
        dv.w[ro] = w;
        dv.n[ro] = n;
      }
    }
    // readout row: LN_s on the key sums (fp64), stored radius on the value sums
    double s = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += sk[e];
    const double mean = group_sum<16>(s) / (double)D;
    double qq = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const double dl = sk[e] - mean;
      qq += dl * dl;
    }
    const double rden = 1.0 / sqrt(group_sum<16>(qq) / (double)D + (double)dv.ln_eps);
    float nn = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) nn += sv[e] * sv[e];
    const float vs = rho / fmaxf(sqrtf(group_sum<16>(nn)), dv.norm_eps);
    uint32_t kw[4], vw[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const double y0 = (sk[e] - mean) * rden * (double)ga[e] + (double)be[e];
      const double y1 = (sk[e + 1] - mean) * rden * (double)ga[e + 1] + (double)be[e + 1];
      kw[e >> 1] = (uint32_t)float_to_bf16_bits((float)y0) | ((uint32_t)float_to_bf16_bits((float)y1) << 16);
      vw[e >> 1] = (uint32_t)float_to_bf16_bits(sv[e] * vs) | ((uint32_t)float_to_bf16_bits(sv[e + 1] * vs) << 16);
    }
    uint16_t *kh = (uint16_t *)dv.khat + slot_new * dv.slot_elems + ro * D + ch0;
    uint16_t *vh = (uint16_t *)dv.vhat + slot_new * dv.slot_elems + ro * D + ch0;
    *reinterpret_cast<uint4 *>(kh) = make_uint4(kw[0], kw[1], kw[2], kw[3]);
    *reinterpret_cast<uint4 *>(vh) = make_uint4(vw[0], vw[1], vw[2], vw[3]);
  }
}

// Rows [0, m) that received no token: their readout moves to the new version unchanged.
template <int NW>
__device__ __forceinline__ void copy_untouched(const Ctx<NW> &cx, int m, int slot_old, int slot_new) {
  constexpr int D = kHeadDim, NG = 4 * NW, UN = 4;
  const Dev &dv = cx.dv;
  const int gid = cx.tid >> 4, c16 = cx.tid & 15;
  const uint32_t *bm = cx.s_bitmap();
  const int64_t ubase = (int64_t)cx.u * dv.Mcap * D;
  const uint16_t *ko = (const uint16_t *)dv.khat + slot_old * dv.slot_elems + ubase;
  const uint16_t *vo = (const uint16_t *)dv.vhat + slot_old * dv.slot_elems + ubase;
  uint16_t *kn = (uint16_t *)dv.khat + slot_new * dv.slot_elems + ubase;
  uint16_t *vn = (uint16_t *)dv.vhat + slot_new * dv.slot_elems + ubase;
  for (int r0 = gid; r0 < m; r0 += NG * UN) {
    uint4 kk[UN], vv[UN];
    bool on[UN];
#pragma unroll
    for (int q = 0; q < UN; ++q) {
      const int r = r0 + q * NG;
      on[q] = r < m && !((bm[r >> 5] >> (r & 31)) & 1u);
      if (on[q]) {
        kk[q] = *reinterpret_cast<const uint4 *>(ko + (int64_t)r * D + 8 * c16);
        vv[q] = *reinterpret_cast<const uint4 *>(vo + (int64_t)r * D + 8 * c16);
      }
    }
#pragma unroll
    for (int q = 0; q < UN; ++q) {
      const int r = r0 + q * NG;
      if (on[q]) {
        *reinterpret_cast<uint4 *>(kn + (int64_t)r * D + 8 * c16) = kk[q];
        *reinterpret_cast<uint4 *>(vn + (int64_t)r * D + 8 * c16) = vv[q];
      }
    }
  }
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void fold_fused_kernel(Dev dv, Src src, FoldRunArgs run) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int NT = 64 * NW, D = kHeadDim;
  const int C = dv.C;
  Ctx<NW> cx{dv, smem, fold_lds(C, dv.Mcap, NW), (int)blockIdx.x, (int)threadIdx.x, (int)(threadIdx.x & 63),
             __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))};
  const int u = cx.u, tid = cx.tid;
  uint16_t *kbar_blk = (uint16_t *)dv.kbar + (int64_t)u * C * D;
  const int n_words = (dv.Mcap + 31) / 32;
  const float qnan = __uint_as_float(0x7fc00000u);

  for (int si = 0; si < run.n; ++si) {
    const FoldStep st = run.s[si];
    const int m = st.m, m_after = st.m_after, n_app = m_after - m;
    for (int i = tid; i < n_words; i += NT) cx.s_bitmap()[i] = 0u;
    int n_seg;
    if (n_app == C) {
      // room for the whole block (state creation included): no scores; the memory keys are
      // still needed, as the new rows' key sums
      const int lane = cx.lane, l32 = lane & 31;
      for (int g0 = cx.wave; g0 < C / 32; g0 += NW) {
        const int j = g0 * 32 + l32;
        const int b = u / dv.Hkv, h = u % dv.Hkv;
        const uint16_t *krow = (const uint16_t *)src.k + b * src.k_b + h * src.k_h + (st.tok + j) * src.k_t;
        bf16x8 kreg[8];
        memory_keys(dv, krow, h, true, kbar_blk + (int64_t)j * D, lane, kreg);
      }
      for (int j = tid; j < C; j += NT) {
        cx.s_rank()[j] = j;
        cx.s_pi()[j] = m + j;
        cx.s_app()[j] = qnan;
        cx.s_best()[j] = qnan;
      }
      __syncthreads();
      n_seg = order_tokens(cx, m, true);
      row_pass(cx, src, st.tok, m, st.sn, n_seg, kbar_blk, false, false);
    } else {
      score_pass(cx, src, st.tok, st.so, 0, m, true, kbar_blk);
      if (n_app > 0) {
        select_tokens(cx, m, n_app);
        // the new rows first, so that the remaining tokens can be scored against them too
        n_seg = order_tokens(cx, m, false);
        row_pass(cx, src, st.tok, m, st.sn, n_seg, kbar_blk, true, false);
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        score_pass(cx, src, st.tok, st.sn, m, m_after, false, kbar_blk);
        for (int i = tid; i < n_words; i += NT) cx.s_bitmap()[i] = 0u;
        __syncthreads();
      }
      n_seg = order_tokens(cx, m, false);
      row_pass(cx, src, st.tok, m, st.sn, n_seg, kbar_blk, false, n_app > 0);
    }
    if (!run.in_place) copy_untouched(cx, m, st.so, st.sn);
    // what the fold decided, for the record and for the entry point's optional outputs
    {
      const int64_t base = (int64_t)u * C;
      for (int j = tid; j < C; j += NT) {
        const int p = cx.s_pi()[j];
        const float2 sc = make_float2(cx.s_app()[j], cx.s_best()[j]);
        dv.pi[base + j] = p;
        dv.score[base + j] = sc;
        if (run.trace_assign && st.trace >= 0) run.trace_assign[st.trace * run.trace_stride + base + j] = p;
        if (run.trace_score && st.trace >= 0)
          reinterpret_cast<float2 *>(run.trace_score)[st.trace * run.trace_stride + base + j] = sc;
      }
    }
    // the next fold of the run reads what this one wrote (this workgroup's own stores)
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
}

}  // namespace

bool fold_fused_fits(const Dev &dv) {
  if (!(dv.io == 1 && dv.d == kHeadDim && dv.C % 64 == 0 && dv.C <= 1024 && dv.Mcap <= (1 << 20))) return false;
  return fold_lds(dv.C, dv.Mcap, 16).total <= 96 * 1024;
}

hipError_t launch_fold_fused(const Dev &dv, const Src &src, const FoldRunArgs &run, int n_waves, hipStream_t st) {
  if (run.n <= 0) return hipSuccess;
  if (n_waves == 16) {
    const size_t lds = fold_lds(dv.C, dv.Mcap, 16).total;
    static bool once = (hipFuncSetAttribute((const void *)fold_fused_kernel<16>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024), true);
    (void)once;
    hipLaunchKernelGGL(fold_fused_kernel<16>, dim3(dv.U), dim3(1024), lds, st, dv, src, run);
  } else {
    const size_t lds = fold_lds(dv.C, dv.Mcap, 8).total;
    static bool once = (hipFuncSetAttribute((const void *)fold_fused_kernel<8>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024), true);
    (void)once;
    hipLaunchKernelGGL(fold_fused_kernel<8>, dim3(dv.U), dim3(512), lds, st, dv, src, run);
  }
  return hipGetLastError();
}

}  // namespace kvm
