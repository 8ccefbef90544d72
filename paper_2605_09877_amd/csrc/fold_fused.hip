// A run of folds in one launch, one workgroup per (sequence, KV head) unit (bf16, head_dim 128).
//
// A fold (sections "Append", "Merge" and the readout equations of the paper's Method section) is a
// chain of small dependent steps: similarity of the block to the normalised state, selection of
// the tokens to append, creation of their rows, similarity of the remaining tokens to the new
// rows, winner-take-all accumulation, readout refresh.  Units are independent of each other, and
// consecutive folds of one unit depend on each other through that unit's state alone, so one
// workgroup walks a unit through all of a run's folds with workgroup barriers between the steps:
// no launch boundaries inside the chain and none between its folds.  Two shapes of workgroup: 16
// waves with up to 160 KiB of LDS when the folds have the chip to themselves (decode, a prefill
// whose folds outweigh its attention); 8 waves at 128 registers and under 96 KiB when they run
// beside a prefill's attention launches, whose workgroups leave room for exactly that on a compute
// unit (a larger workgroup would wait until a unit has drained, which a running attention launch
// never lets happen).  Per fold:
//   1. the block's memory keys k-bar = LN_s(zero_r(k)), computed by a launch of their own ahead of
//      the run (they depend on k alone, so they are not part of the chain), are read as matrix-core
//      operands by the wave that owns the 32 tokens;
//   2. D[row, token] = K-hat_tile . K-bar^T on the matrix cores, state rows streaming HBM/L2 ->
//      LDS in 64-row tiles, two stages of several tiles: append score s_j = max over all rows,
//      merge target = argmax over rows >= S (a lane owns a token and scans rows in ascending
//      order: ties keep the lowest row);
//   3. when the budget has room for some of the block: the n_append smallest (s_j, j) are taken
//      (ranks by counting), their rows are created, and step 2 runs again over the new rows for
//      the tokens that were not taken (a strictly larger score moves a token);
//   4. every merging token pushes itself on its target row's list in LDS (an exchange on the
//      row's head); the token that finds the list empty enters the row in the list of touched rows;
//   5. 16 lanes per touched row (8 channels each): the sums are asked for, the row's list is
//      walked, its tokens are added in ascending position, sums and the readout row (LN_s in
//      fp64 on keys, stored radius on values) are written; rows nothing was added to are copied
//      to the new state version (prefill) or left alone (in place).
// Integer decisions rest on fp64 LN_s and fp64 key sums, as everywhere in this library.
//
// With fewer units than compute units one workgroup per unit leaves most of the chip idle, so a
// unit can be given `split` workgroups (a power of two) that divide its state rows among them in
// 64-row tiles, tile t belonging to workgroup t mod split: a workgroup scores the whole block
// against its own rows, merges the tokens bound for its own rows, creates the new rows that fall
// to it and copies its own untouched rows.  Everything a workgroup reads of the state it wrote
// itself, so the only data that crosses workgroups is each token's partial winner: one exchange
// per scoring pass through a small table in global memory.  An entry is one 64-bit word (score,
// row, a 16-bit tag of the exchange it belongs to) written and read with relaxed device-scope
// atomics: no fences, no flags beside the data; a reader spins on the tag, with a clock limit that
// ends the wait and raises an error word instead of hanging.  The workgroups of a launch must be
// able to be resident together (the host checks the grid against the chip); kernels that run
// beside it on other streams only delay a workgroup's start, they never wait for this kernel.
#include <cstddef>

#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr int kNoRow = 0x7fffffff;
constexpr int kTileBytes = kTileElems * 2;   // 16 KiB
constexpr int kListMax = 16;                 // tokens of a row taken from its list in one go
// NW waves per workgroup; a stage of the K-hat stream is NW / 4 tiles, two stages are in LDS
__host__ __device__ constexpr int stage_tiles(int NW) { return NW / 4; }

// LN_s parameters when the caller gave none (gamma = 1, beta = 0): read like given ones, so that
// the kernels carry no per-element branches.
__device__ const float kOnes[kHeadDim] = {
    1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1,
    1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1,
    1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1,
    1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1};
__device__ const float kZeros[kHeadDim] = {};

__device__ __forceinline__ bool beats(float sa, int ia, float sb, int ib) {
  return sa > sb || (sa == sb && ia < ib);
}

// LDS layout of one workgroup (bytes from the start of dynamic shared memory).
struct FoldLds {
  uint32_t tiles;    // 2 * stage_tiles tiles of K-hat; outside the score passes also scratch for sort keys
  uint32_t app;      // float [C]  append score s_j
  uint32_t best;     // float [C]  winning merge score
  uint32_t pi;       // int   [C]  target row
  uint32_t rank;     // int   [C]  rank among the appended tokens, or -1
  uint32_t next;     // int   [C]  next token on the same row's list, or -1
  uint32_t creator;  // int   [C]  token that creates new row number a
  uint32_t rows;     // int   [C]  rows that receive tokens in this fold
  uint32_t merge;    // float/int [3][NW * 32] partial winners of waves that share tokens
  uint32_t masks;    // u64   [C / 64] taken-token masks
  uint32_t counters; // int   [4]
  uint32_t head;     // int   [Mcap] last token pushed on the row's list, or -1
  uint32_t lall;     // float [C]  this workgroup's own winners of a scoring pass (split > 1)
  uint32_t lbest;    // float [C]
  uint32_t lidx;     // int   [C]
  uint32_t total;
};
__host__ __device__ inline FoldLds fold_lds(int C, int Mcap, int NW, int split = 1) {
  FoldLds l;
  uint32_t o = 0;
  auto take = [&](uint32_t bytes) {
    const uint32_t at = o;
    o += (bytes + 15u) & ~15u;
    return at;
  };
  l.tiles = take(2 * stage_tiles(NW) * kTileBytes);
  l.app = take(4u * C);
  l.best = take(4u * C);
  l.pi = take(4u * C);
  l.rank = take(4u * C);
  l.next = take(4u * C);
  l.creator = take(4u * C);
  l.rows = take(4u * C);
  l.merge = take(3u * 4u * NW * 32);
  l.masks = take(8u * ((C + 63) / 64));
  l.counters = take(16);
  l.head = take(4u * Mcap);
  l.lall = take(split > 1 ? 4u * C : 0u);
  l.lbest = take(split > 1 ? 4u * C : 0u);
  l.lidx = take(split > 1 ? 4u * C : 0u);
  l.total = o;
  return l;
}

struct Ctx {
  unsigned char *smem;
  FoldLds l;
  int u, tid, lane, wave;
  int part, split;   // this workgroup's number among the unit's workgroups, and how many they are
  // the workgroup that owns a state row: 64-row tiles dealt round robin
  __device__ bool owns(int row) const { return ((row >> 6) & (split - 1)) == part; }
  __device__ float *s_lall() const { return (float *)(smem + l.lall); }
  __device__ float *s_lbest() const { return (float *)(smem + l.lbest); }
  __device__ int *s_lidx() const { return (int *)(smem + l.lidx); }
  __device__ float *s_app() const { return (float *)(smem + l.app); }
  __device__ float *s_best() const { return (float *)(smem + l.best); }
  __device__ int *s_pi() const { return (int *)(smem + l.pi); }
  __device__ int *s_rank() const { return (int *)(smem + l.rank); }
  __device__ int *s_next() const { return (int *)(smem + l.next); }
  __device__ int *s_creator() const { return (int *)(smem + l.creator); }
  __device__ int *s_rows() const { return (int *)(smem + l.rows); }
  __device__ int *s_cnt() const { return (int *)(smem + l.counters); }
  __device__ int *s_head() const { return (int *)(smem + l.head); }
  __device__ unsigned long long *s_masks() const { return (unsigned long long *)(smem + l.masks); }
};

// Development aid (compiled in only with -DKVM_FOLD_STAMPS): the first workgroup leaves the clock
// at its phase boundaries in the `creator` scratch, which this path does not use.
#ifdef KVM_FOLD_STAMPS
#define FOLD_STAMP()                                                                        \
  do {                                                                                      \
    if (blockIdx.x == 0 && threadIdx.x == 0 && cx.s_cnt()[3] < 240)                         \
      reinterpret_cast<long long *>(dv.creator)[cx.s_cnt()[3]++] = (long long)wall_clock64(); \
  } while (0)
#else
#define FOLD_STAMP() \
  do {               \
  } while (0)
#endif

// ------------------------------------------------------------------------------------------------
// Step 2: one pass of the block's tokens over state rows [row0, row1) of readout version `slot`.
// first: rows are the state before the append; every token gets s_j and its best row >= S.
// Otherwise rows are the ones created in this fold; a token that was not taken moves to one of
// them when that score is strictly larger than its stored best.
template <int NW>
__device__ __forceinline__ void score_pass(const Dev &dv, const Ctx &cx, int slot, int row0, int row1, bool first,
                                           const uint16_t *kbar_blk) {
  constexpr int D = kHeadDim, ST = stage_tiles(NW);
  const int lane = cx.lane, wave = cx.wave, u = cx.u;
  const int g = lane >> 5, l32 = lane & 31;
  const int C = dv.C, TG = C / 32;
  // Tiles are 64-row blocks of the state counted from row 0; this workgroup takes the ones that
  // fall to it, tile t_first, t_first + split, ...: local tile number lt <-> tile t_first + lt * split.
  const int t_lo = row0 >> 6, t_hi = (row1 + kTileKeys - 1) >> 6;
  const int t_first = t_lo + ((cx.part - t_lo) & (cx.split - 1));
  const int n_tiles = t_first < t_hi ? (t_hi - t_first + cx.split - 1) / cx.split : 0;
  const int n_stages = (n_tiles + ST - 1) / ST;
  const int row_lo = row0 > dv.S ? row0 : dv.S;   // first row that may win a merge
  uint16_t *Ks = (uint16_t *)(cx.smem + cx.l.tiles);
  const uint32_t ks_addr = lds_addr_of(Ks);
  const char *khat = (const char *)dv.khat + (slot * dv.slot_elems + (int64_t)u * dv.Mcap * D) * 2;
  uint32_t koff[8];
  ktile_offsets(lane, koff);
  // a tile is sixteen 1-KiB pieces of four rows; wave w fetches pieces w, w + NW, ... of every
  // tile.  The chunk permutation of a piece depends on (piece % 4) = (w % 4).
  const DmaLane dl = dma_lane(lane);
  const int wq = wave & 3;
  const uint32_t kcol = wq == 0 ? dl.kcol[0] : wq == 1 ? dl.kcol[1] : wq == 2 ? dl.kcol[2] : dl.kcol[3];
  auto issue_stage = [&](int sg) {
#pragma unroll
    for (int i = 0; i < ST; ++i) {
      const int t = ST * sg + i;
      if (t < n_tiles) {
        const int base = (t_first + t * cx.split) * kTileKeys, valid = row1 - base;
#pragma unroll
        for (int n = 0; n < 16 / NW; ++n) {
          const int piece = wave + NW * n;
          int r = 4 * piece + (int)dl.rl;
          r = r < valid ? r : valid - 1;   // rows past the end repeat the last one (masked below)
          dma16(khat + (uint32_t)base * (D * 2), (uint32_t)r * (D * 2) + kcol,
                ks_addr + (uint32_t)(ST * (sg & 1) + i) * kTileBytes + (uint32_t)piece * 1024u);
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
    // The memory keys of this round's token groups, as B operands (lane = 32 g + i holds token i,
    // channels 16 ks + 8 g .. + 7): the block's rows go through LDS as 64-token tiles in the K
    // layout (coalesced 1-KiB pieces) instead of sixteen scattered bytes per lane and step.  When
    // they fit the ring's second half they travel together with the first stage of K-hat.
    const int kb_tiles = (Gp + 1) / 2;
    const bool together = kb_tiles <= ST;
    const int kb_buf0 = together ? ST : 0;
#pragma unroll
    for (int i = 0; i < 2 * ST; ++i)
      if (i < kb_tiles) {
        const char *from = (const char *)(kbar_blk + (int64_t)(g0 / 2 + i) * kTileKeys * D);
#pragma unroll
        for (int n = 0; n < 16 / NW; ++n) {
          const int piece = wave + NW * n;
          dma16(from, (uint32_t)(4 * piece + (int)dl.rl) * (D * 2) + kcol,
                ks_addr + (uint32_t)(kb_buf0 + i) * kTileBytes + (uint32_t)piece * 1024u);
        }
      }
    if (together && n_stages > 0) issue_stage(0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    bf16x8 kreg[8];
    {
      const int gsel = active ? gi : 0;
      const uint16_t *Kb = Ks + (kb_buf0 + gsel / 2) * kTileElems;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) kreg[ks] = ktile_frag(Kb, koff, gsel & 1, ks);
    }
    if (!together) {
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();   // every wave has its operands: the ring is free for K-hat
      if (n_stages > 0) issue_stage(0);
    }
    // The winner is kept as a wave-uniform code (32-row block number * 16 + accumulator element)
    // and turned into a row at the end: selecting a scalar costs no register per candidate.
    float best_all = -INFINITY, best = -INFINITY;
    int best_code = -1;
    for (int sg = 0; sg < n_stages; ++sg) {
      // (together: stage 0 has landed with the memory keys; this wait is for the operand reads,
      // after which the ring's second half may be overwritten by stage 1)
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      if (sg + 1 < n_stages) issue_stage(sg + 1);
      if (active) {
#pragma unroll
        for (int i = 0; i < ST; ++i) {
          const int t = ST * sg + i;
          if (t < n_tiles && (t & (wpg - 1)) == sub) {   // wpg is a power of two: NW and C / 32 are
            const uint16_t *Kt = Ks + (ST * (sg & 1) + i) * kTileElems;
            // the tile's two 32-row blocks, one accumulation chain each (channels in ascending
            // order), interleaved; four K fragments in flight from LDS
            f32x16 acc[2];
            {
              bf16x8 kf[4];
#pragma unroll
              for (int q = 0; q < 4; ++q) kf[q] = ktile_frag(Kt, koff, q & 1, q >> 1);
              const f32x16 zero = {0.f};
#pragma unroll
              for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int rh = 0; rh < 2; ++rh) {
                  const int slot2 = (2 * ks + rh) & 3;
                  acc[rh] = mfma32(kf[slot2], kreg[ks], ks == 0 ? zero : acc[rh]);
                  if (ks + 2 < 8) kf[slot2] = ktile_frag(Kt, koff, rh, ks + 2);
                }
              // pin that order: four LDS reads up front, then one read behind every matrix
              // instruction, so that no matrix instruction waits for the read issued just before it
              __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
              for (int q = 0; q < 12; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
              }
              __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
            }
#pragma unroll
            for (int rh = 0; rh < 2; ++rh) {
              const int blk = 2 * (t_first + t * cx.split) + rh, base = 32 * blk;
              if (base < row1 && base + 32 > row0) {
                const bool edge = base < row_lo || base + 32 > row1;
                if (edge) {
#pragma unroll
                  for (int v = 0; v < 16; ++v) {
                    const int i2 = base + mfma_row(v, g);
                    const float sc = acc[rh][v];
                    if (i2 < row1 && i2 >= row0) {
                      best_all = fmaxf(best_all, sc);
                      if (i2 >= row_lo && sc > best) {
                        best = sc;
                        best_code = 16 * blk + v;
                      }
                    }
                  }
                } else {
#pragma unroll
                  for (int v = 0; v < 16; ++v) {
                    const float sc = acc[rh][v];
                    const bool up = sc > best;
                    best = up ? sc : best;
                    best_code = up ? 16 * blk + v : best_code;
                  }
                }
              }
            }
          }
        }
      }
    }
    int best_i = best_code < 0 ? kNoRow : 32 * (best_code >> 4) + mfma_row(best_code & 15, g);
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
      if (cx.split > 1) {
        // this workgroup's rows only: the unit's winner is settled by the exchange that follows
        cx.s_lall()[j] = best_all;
        cx.s_lbest()[j] = best;
        cx.s_lidx()[j] = best_i;
      } else if (first) {
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
// The exchange after a scoring pass (split > 1): every workgroup of the unit publishes its own
// winners and reads the others'; all of them end up with the same unit-wide result in LDS, as
// score_pass leaves it when a unit has one workgroup.
// Table: [unit][exchange parity][workgroup][2][C] 64-bit words; word 0 of a token = (merge score,
// row in 16 bits, tag), word 1 = (append score, tag).  A workgroup cannot be two exchanges ahead of
// a sibling (it needs the sibling's entries of the exchange in between), so two parities suffice.
// tag: the low 16 bits of the exchange's number, which the host never reuses within a state's life
// before every entry has been rewritten many times; the table starts zeroed and 0 is never a tag.
__device__ __forceinline__ unsigned long long xchg_pack(float score, uint32_t low16, uint32_t tag) {
  return ((unsigned long long)__float_as_uint(score) << 32) | ((unsigned long long)(low16 & 0xffffu) << 16) |
         (unsigned long long)(tag & 0xffffu);
}
// gave_up: a word in LDS, set by the first wait of the workgroup that ran into the limit; from then
// on its waits return at once (a workgroup loses at most one time limit, whatever went wrong),
// with an entry that names no row, so that nothing downstream indexes with it.
__device__ __forceinline__ unsigned long long xchg_wait(const unsigned long long *p, uint32_t tag, int32_t *err,
                                                        volatile int *gave_up) {
  unsigned long long v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if ((uint32_t)(v & 0xffffu) == tag) return v;
  const unsigned long long t0 = wall_clock64();   // 100 MHz
  while (*gave_up == 0) {
    __builtin_amdgcn_s_sleep(4);
    v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((uint32_t)(v & 0xffffu) == tag) return v;
    if (wall_clock64() - t0 > 20000000ull) {   // 200 ms: a sibling that never came
      *gave_up = 1;
      __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
  return xchg_pack(-INFINITY, 0xffffu, tag);
}
template <int NW>
__device__ __forceinline__ void exchange_winners(const Dev &dv, const Ctx &cx, unsigned long long *xtab,
                                                 uint32_t xnum, bool first, int32_t *err) {
  constexpr int NT = 64 * NW;
  const int C = dv.C;
  const uint32_t tag = xnum & 0xffffu;
  volatile int *gave_up = cx.s_cnt() + 2;
  unsigned long long *base = xtab + (((size_t)cx.u * 2 + (xnum & 1u)) * cx.split) * 2 * C;
  for (int j = cx.tid; j < C; j += NT) {
    float best = cx.s_lbest()[j], best_all = cx.s_lall()[j];
    int best_i = cx.s_lidx()[j];
    unsigned long long *mine = base + (size_t)cx.part * 2 * C;
    __hip_atomic_store(mine + j, xchg_pack(best, best_i == kNoRow ? 0xffffu : (uint32_t)best_i, tag), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    if (first)
      __hip_atomic_store(mine + C + j, xchg_pack(best_all, 0, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // the siblings' entries: all of them asked for at once (each read goes to memory, one or two
    // microseconds away), then the stragglers waited for one by one
    unsigned long long w0[kFoldMaxSplit - 1], w1[kFoldMaxSplit - 1];
#pragma unroll
    for (int o = 1; o < kFoldMaxSplit; ++o)
      if (o < cx.split) {
        const unsigned long long *theirs = base + (size_t)((cx.part + o) & (cx.split - 1)) * 2 * C;
        w0[o - 1] = __hip_atomic_load(theirs + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (first) w1[o - 1] = __hip_atomic_load(theirs + C + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
#pragma unroll
    for (int o = 1; o < kFoldMaxSplit; ++o)
      if (o < cx.split) {
        const unsigned long long *theirs = base + (size_t)((cx.part + o) & (cx.split - 1)) * 2 * C;
        if ((uint32_t)(w0[o - 1] & 0xffffu) != tag) w0[o - 1] = xchg_wait(theirs + j, tag, err, gave_up);
        const float ob = __uint_as_float((uint32_t)(w0[o - 1] >> 32));
        const uint32_t oi16 = (uint32_t)(w0[o - 1] >> 16) & 0xffffu;
        const int oi = oi16 == 0xffffu ? kNoRow : (int)oi16;
        if (oi != kNoRow && (best_i == kNoRow || beats(ob, oi, best, best_i))) {
          best = ob;
          best_i = oi;
        }
        if (first) {
          if ((uint32_t)(w1[o - 1] & 0xffffu) != tag) w1[o - 1] = xchg_wait(theirs + C + j, tag, err, gave_up);
          best_all = fmaxf(best_all, __uint_as_float((uint32_t)(w1[o - 1] >> 32)));
        }
      }
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
  __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// Step 3: the n_app tokens with the smallest (s_j, position) are taken; a taken token's rank among
// the taken ones, in position order, is the new row it creates.
template <int NW>
__device__ __forceinline__ void select_tokens(const Dev &dv, const Ctx &cx, int m, int n_app) {
  constexpr int NT = 64 * NW;
  const int C = dv.C, tid = cx.tid, lane = cx.lane;
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
      cx.s_creator()[a] = j;
    } else {
      cx.s_rank()[j] = -1;
    }
  }
  __syncthreads();
}

// 1 / sqrt(x) in fp64 from the hardware estimate and two Newton steps (y <- y (1.5 - 0.5 x y^2)):
// within a few units of the last place, against some 300 instructions for the correctly rounded
// division of the correctly rounded root; the result is rounded to bf16 afterwards.
__device__ __forceinline__ double rsqrt64(double x) {
  double y = __builtin_amdgcn_rsq(x);
  const double hx = 0.5 * x;
  y = y * fma(-hx * y, y, 1.5);
  y = y * fma(-hx * y, y, 1.5);
  return y;
}

// Readout row of sums (sk, sv, rho): LN_s on the key sums in fp64, stored radius on the value sums;
// 16 lanes hold the row, 8 channels each.  Rounding to bf16 is the hardware's (nearest even).
__device__ __forceinline__ void write_readout16(const Dev &dv, int slot, int64_t ro, int ch0, const double (&sk)[8],
                                                const float (&sv)[8], float rho, const float (&ga)[8],
                                                const float (&be)[8]) {
  constexpr int D = kHeadDim;
  double s = 0.0;
#pragma unroll
  for (int e = 0; e < 8; ++e) s += sk[e];
  const double mean = group_sum<16>(s) * (1.0 / (double)D);   // D is a power of two: exact
  double qq = 0.0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const double dl = sk[e] - mean;
    qq += dl * dl;
  }
  const double rden = rsqrt64(group_sum<16>(qq) * (1.0 / (double)D) + (double)dv.ln_eps);
  float nn = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) nn += sv[e] * sv[e];
  // (hardware root and reciprocal, an ulp of fp32 each: far below the bf16 the result is rounded to)
  const float vs = rho * __builtin_amdgcn_rcpf(fmaxf(__builtin_amdgcn_sqrtf(group_sum<16>(nn)), dv.norm_eps));
  uint32_t kw[4], vw[4];
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const double y0 = (sk[e] - mean) * rden * (double)ga[e] + (double)be[e];
    const double y1 = (sk[e + 1] - mean) * rden * (double)ga[e + 1] + (double)be[e + 1];
    kw[e >> 1] = pack_bf16((float)y0, (float)y1);
    vw[e >> 1] = pack_bf16(sv[e] * vs, sv[e + 1] * vs);
  }
  uint16_t *kh = (uint16_t *)dv.khat + slot * dv.slot_elems + ro * D + ch0;
  uint16_t *vh = (uint16_t *)dv.vhat + slot * dv.slot_elems + ro * D + ch0;
  *reinterpret_cast<uint4 *>(kh) = make_uint4(kw[0], kw[1], kw[2], kw[3]);
  *reinterpret_cast<uint4 *>(vh) = make_uint4(vw[0], vw[1], vw[2], vw[3]);
}

struct RowCtx {
  const uint16_t *vsrc, *kbar;
  const float *gsrc;
  int64_t v_t, g_t;
  float ga[8], be[8];
  int gid, c16, ch0;
};
__device__ __forceinline__ RowCtx row_ctx(const Dev &dv, const Ctx &cx, const Src &src, int64_t tok,
                                          const uint16_t *kbar_blk) {
  constexpr int D = kHeadDim;
  RowCtx rc;
  const int u = cx.u, b = u / dv.Hkv, h = u % dv.Hkv;
  rc.gid = cx.tid >> 4;
  rc.c16 = cx.tid & 15;
  rc.ch0 = 8 * rc.c16;
  rc.vsrc = (const uint16_t *)src.v + b * src.v_b + h * src.v_h + tok * src.v_t;
  rc.gsrc = src.g ? src.g + b * src.g_b + h * src.g_h + tok * src.g_t : nullptr;
  rc.kbar = kbar_blk;
  rc.v_t = src.v_t;
  rc.g_t = src.g_t;
  const float *gam = dv.gamma ? dv.gamma + h * D : kOnes, *bet = dv.beta ? dv.beta + h * D : kZeros;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    rc.ga[e] = gam[rc.ch0 + e];
    rc.be[e] = bet[rc.ch0 + e];
  }
  return rc;
}

// New rows m .. m + n_app - 1 from their creator tokens: ungated copy of the memory key and the
// value, radius = the value's norm.
template <int NW>
__device__ __forceinline__ void create_rows(const Dev &dv, const Ctx &cx, const RowCtx &rc, int m, int n_app,
                                            int slot_new) {
  constexpr int D = kHeadDim, NG = 4 * NW;
  for (int a = rc.gid; a < n_app; a += NG) {
    if (!cx.owns(m + a)) continue;
    const int t = cx.s_creator()[a];
    const int64_t ro = (int64_t)cx.u * dv.Mcap + m + a;
    const uint4 kraw = *reinterpret_cast<const uint4 *>(rc.kbar + (int64_t)t * D + rc.ch0);
    const uint4 vraw = *reinterpret_cast<const uint4 *>(rc.vsrc + (int64_t)t * rc.v_t + rc.ch0);
    float kf[8], vf[8];
    unpack16<bf16_t>(kraw, kf);
    unpack16<bf16_t>(vraw, vf);
    double sk[8];
    float nn = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sk[e] = (double)kf[e];
      nn += vf[e] * vf[e];
    }
    const float rho = sqrtf(group_sum<16>(nn));
    double2 *pk = reinterpret_cast<double2 *>(dv.sK + ro * D + rc.ch0);
    float4 *pv = reinterpret_cast<float4 *>(dv.sV + ro * D + rc.ch0);
#pragma unroll
    for (int q = 0; q < 4; ++q) pk[q] = make_double2(sk[2 * q], sk[2 * q + 1]);
    pv[0] = make_float4(vf[0], vf[1], vf[2], vf[3]);
    pv[1] = make_float4(vf[4], vf[5], vf[6], vf[7]);
    if (rc.c16 == 0) {
      dv.rho[ro] = rho;
      dv.w[ro] = 1.f;
      dv.n[ro] = 1;
    }
    write_readout16(dv, slot_new, ro, rc.ch0, sk, vf, rho, rc.ga, rc.be);
  }
}

// Step 4: the lists.  Every token that merges pushes itself on its row's list; the one that finds
// the list empty enters the row in `rows`.  Returns the number of touched rows.
template <int NW>
__device__ __forceinline__ int build_lists(const Dev &dv, const Ctx &cx) {
  constexpr int NT = 64 * NW;
  const int C = dv.C, tid = cx.tid, lane = cx.lane;
  int *cnt = cx.s_cnt();
  if (tid == 0) cnt[0] = 0;
  for (int i = tid; i < dv.Mcap; i += NT) cx.s_head()[i] = -1;
  __syncthreads();
  for (int j0 = 0; j0 < C; j0 += NT) {
    const int j = j0 + tid;
    bool leader = false;
    int row = kNoRow;
    if (j < C && cx.s_rank()[j] < 0) {
      row = cx.s_pi()[j];
      row = row != kNoRow && cx.owns(row) ? row : kNoRow;   // other rows are other workgroups' work
      if (row != kNoRow) {
        const int old = atomicExch(&cx.s_head()[row], j);
        cx.s_next()[j] = old;
        leader = old < 0;
      }
    }
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(leader);
    int base = 0;
    if (lane == 0 && bal) base = atomicAdd(&cnt[0], __builtin_popcountll(bal));
    base = __shfl(base, 0, kWave);
    if (leader) cx.s_rows()[base + __builtin_popcountll(bal & ((1ull << lane) - 1ull))] = row;
  }
  __syncthreads();
  return cnt[0];
}

// Minimum over the 16 lanes of a group, in every lane.
__device__ __forceinline__ int group_min16(int x) {
  auto mn = [](int a, int b) { return a < b ? a : b; };
  x = mn(x, (int)__builtin_amdgcn_mov_dpp((uint32_t)x, 0xB1, 0xF, 0xF, true));
  x = mn(x, (int)__builtin_amdgcn_mov_dpp((uint32_t)x, 0x4E, 0xF, 0xF, true));
  x = mn(x, (int)__builtin_amdgcn_mov_dpp((uint32_t)x, 0x141, 0xF, 0xF, true));
  x = mn(x, (int)__builtin_amdgcn_mov_dpp((uint32_t)x, 0x140, 0xF, 0xF, true));
  return x;
}

// Step 5: the touched rows, 16 lanes each.
struct RowLoad {
  double2 k2[4];
  float4 v4[2];
  uint4 kraw, vraw;
  float rho, w, gt;
  int n, mine, len, t_cur, row;
};

template <int NW>
__device__ __forceinline__ void merge_rows(const Dev &dv, const Ctx &cx, const RowCtx &rc, int slot_new, int n_rows) {
  constexpr int D = kHeadDim, NG = 4 * NW;
  const int C = dv.C;
  const int *next = cx.s_next(), *pi = cx.s_pi(), *rank = cx.s_rank();
  auto fetch = [&](RowLoad &L, int t) {
    L.kraw = *reinterpret_cast<const uint4 *>(rc.kbar + (int64_t)t * D + rc.ch0);
    L.vraw = *reinterpret_cast<const uint4 *>(rc.vsrc + (int64_t)t * rc.v_t + rc.ch0);
    L.gt = rc.gsrc ? rc.gsrc[(int64_t)t * rc.g_t] : 1.f;
  };
  auto start = [&](RowLoad &L, int ri) {
    const int row = cx.s_rows()[ri];
    L.row = row;
    const int64_t ro = (int64_t)cx.u * dv.Mcap + row;
    // the sums are asked for first; the list is walked while they travel
    const double2 *pk = reinterpret_cast<const double2 *>(dv.sK + ro * D + rc.ch0);
    const float4 *pv = reinterpret_cast<const float4 *>(dv.sV + ro * D + rc.ch0);
#pragma unroll
    for (int q = 0; q < 4; ++q) L.k2[q] = pk[q];
    L.v4[0] = pv[0];
    L.v4[1] = pv[1];
    L.rho = dv.rho[ro];
    L.w = dv.w[ro];
    L.n = dv.n[ro];
    // lane i of the group keeps the i-th token of the list (any order); longer lists are scanned
    int mine = kNoRow, len = 0;
    for (int t = cx.s_head()[row]; t >= 0 && len <= kListMax; t = next[t], ++len)
      if (len == rc.c16) mine = t;
    L.mine = mine;
    L.len = len;
    // the first token (the smallest position) is asked for together with the sums
    L.t_cur = len <= kListMax ? group_min16(mine) : kNoRow;
    if (L.t_cur != kNoRow) fetch(L, L.t_cur);
  };
  auto finish = [&](RowLoad &L) {
    const int64_t ro = (int64_t)cx.u * dv.Mcap + L.row;
    double sk[8];
    float sv[8];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      sk[2 * q] = L.k2[q].x;
      sk[2 * q + 1] = L.k2[q].y;
    }
    sv[0] = L.v4[0].x; sv[1] = L.v4[0].y; sv[2] = L.v4[0].z; sv[3] = L.v4[0].w;
    sv[4] = L.v4[1].x; sv[5] = L.v4[1].y; sv[6] = L.v4[1].z; sv[7] = L.v4[1].w;
    float w = L.w;
    int n = L.n;
    auto add_fetched = [&]() {
      float kf[8], vf[8];
      unpack16<bf16_t>(L.kraw, kf);
      unpack16<bf16_t>(L.vraw, vf);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sk[e] = fma((double)L.gt, (double)kf[e], sk[e]);
        sv[e] = fmaf(L.gt, vf[e], sv[e]);
      }
      w += L.gt;
      n += 1;
    };
    if (L.len <= kListMax) {
      // ascending position: the smallest token not yet added, len times
      int t_cur = L.t_cur;
      for (int q = 0; q < L.len; ++q) {
        add_fetched();
        if (q + 1 < L.len) {
          t_cur = group_min16(L.mine > t_cur ? L.mine : kNoRow);
          fetch(L, t_cur);
        }
      }
    } else {
      // a long list (many tokens on one row): scan the block's targets in position order instead
      for (int t = 0; t < C; ++t)
        if (pi[t] == L.row && rank[t] < 0) {
          fetch(L, t);
          add_fetched();
        }
    }
    {
      double2 *qk = reinterpret_cast<double2 *>(dv.sK + ro * D + rc.ch0);
      float4 *qv = reinterpret_cast<float4 *>(dv.sV + ro * D + rc.ch0);
#pragma unroll
      for (int q = 0; q < 4; ++q) qk[q] = make_double2(sk[2 * q], sk[2 * q + 1]);
      qv[0] = make_float4(sv[0], sv[1], sv[2], sv[3]);
      qv[1] = make_float4(sv[4], sv[5], sv[6], sv[7]);
      if (rc.c16 == 0) {
        dv.w[ro] = w;
        dv.n[ro] = n;
      }
    }
    write_readout16(dv, slot_new, ro, rc.ch0, sk, sv, L.rho, rc.ga, rc.be);
  };
  for (int ri = rc.gid; ri < n_rows; ri += NG) {
    RowLoad A;
    start(A, ri);
    finish(A);
  }
}

// Rows [0, m) that received no token: their readout moves to the new version unchanged.
// all: no lists were built in this fold (every token made a row of its own): every row moves.
template <int NW>
__device__ __forceinline__ void copy_untouched(const Dev &dv, const Ctx &cx, int m, int slot_old, int slot_new,
                                               bool all) {
  constexpr int D = kHeadDim, UN = 4, NG = 4 * NW;
  const int gid = cx.tid >> 4, c16 = cx.tid & 15;
  const int *head = cx.s_head();
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
      on[q] = r < m && (all || head[r] < 0) && cx.owns(r);
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

// The kernel's one argument.  The steps of the run are read from the kernel-argument segment by
// index (a scalar load with a computed offset): as a by-value array indexed by the loop variable
// the compiler would either copy them to private memory or hold all of them in scalar registers.
struct FoldKernelArgs {
  Dev dv;
  Src src;
  FoldRunArgs run;
};

template <int NW>
__global__ __launch_bounds__(64 * NW, 4) void fold_fused_kernel(FoldKernelArgs args) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int D = kHeadDim, NT = 64 * NW;
  const Dev &dv = args.dv;
  const Src &src = args.src;
  const int run_n = args.run.n, run_in_place = args.run.in_place;
  int32_t *const trace_assign = args.run.trace_assign;
  float *const trace_score = args.run.trace_score;
  const int64_t trace_stride = args.run.trace_stride;
  const FoldStep *steps = reinterpret_cast<const FoldStep *>(
      (const char *)__builtin_amdgcn_kernarg_segment_ptr() + offsetof(FoldKernelArgs, run) + offsetof(FoldRunArgs, s));
  const int C = dv.C;
  // Workgroup -> (unit, part).  The workgroups of a unit read the same block of tokens: where the
  // number of units allows it they get ids 8 apart, which the hardware hands to one accelerator
  // die, whose L2 then fetches the block once.
  const int split = args.run.split;
  const int bid = (int)blockIdx.x;
  const bool by_die = dv.U % 8 == 0;
  const int u_ = by_die ? (bid / (8 * split)) * 8 + bid % 8 : bid / split;
  const int part_ = by_die ? (bid / 8) % split : bid % split;
  Ctx cx{smem, fold_lds(C, dv.Mcap, NW, split), u_, (int)threadIdx.x, (int)(threadIdx.x & 63),
         __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), part_, split};
  unsigned long long *const xtab = args.run.xtab;
  int32_t *const xerr = args.run.err;
  const int u = cx.u, tid = cx.tid;
  const float qnan = __uint_as_float(0x7fc00000u);
#ifdef KVM_FOLD_STAMPS
  if (threadIdx.x == 0) cx.s_cnt()[3] = 0;
#endif
  if (threadIdx.x == 0) cx.s_cnt()[2] = 0;   // no wait has given up (read after barriers only)

  for (int si = 0; si < run_n; ++si) {
    FOLD_STAMP();
    const FoldStep st = steps[si];
    const int m = st.m, m_after = st.m_after, n_app = m_after - m;
    // the block's memory keys: slab `kbar_block` of the scratch, this unit's C rows
    const uint16_t *kbar_blk = (const uint16_t *)dv.kbar + ((int64_t)st.kbar_block * dv.Ufull + u) * C * D;
    if (n_app == C) {
      // room for the whole block (state creation included): no scores
      for (int j = tid; j < C; j += NT) {
        cx.s_rank()[j] = j;
        cx.s_pi()[j] = m + j;
        cx.s_app()[j] = qnan;
        cx.s_best()[j] = qnan;
        cx.s_creator()[j] = j;
      }
      __syncthreads();
      const RowCtx rc = row_ctx(dv, cx, src, st.tok, kbar_blk);
      create_rows<NW>(dv, cx, rc, m, n_app, st.sn);
      FOLD_STAMP();
      if (!run_in_place) copy_untouched<NW>(dv, cx, m, st.so, st.sn, true);
    } else {
      score_pass<NW>(dv, cx, st.so, 0, m, true, kbar_blk);
      if (split > 1) exchange_winners<NW>(dv, cx, xtab, st.xnum, true, xerr);
      FOLD_STAMP();
      const RowCtx rc = row_ctx(dv, cx, src, st.tok, kbar_blk);
      if (n_app > 0) {
        select_tokens<NW>(dv, cx, m, n_app);
        // the new rows first, so that the remaining tokens can be scored against them too
        create_rows<NW>(dv, cx, rc, m, n_app, st.sn);
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        score_pass<NW>(dv, cx, st.sn, m, m_after, false, kbar_blk);
        if (split > 1) exchange_winners<NW>(dv, cx, xtab, st.xnum + 1u, false, xerr);
      }
      FOLD_STAMP();
      const int n_rows = build_lists<NW>(dv, cx);
      FOLD_STAMP();
      merge_rows<NW>(dv, cx, rc, st.sn, n_rows);
      FOLD_STAMP();
      if (!run_in_place) copy_untouched<NW>(dv, cx, m, st.so, st.sn, false);
    }
    FOLD_STAMP();
    // what the fold decided, for the record and for the entry point's optional outputs
    if (cx.part == 0) {
      const int64_t base = (int64_t)u * C;
      for (int j = tid; j < C; j += NT) {
        const int p = cx.s_pi()[j];
        const float2 sc = make_float2(cx.s_app()[j], cx.s_best()[j]);
        dv.pi[base + j] = p;
        dv.score[base + j] = sc;
        if (trace_assign && st.trace >= 0) trace_assign[st.trace * trace_stride + base + j] = p;
        if (trace_score && st.trace >= 0)
          reinterpret_cast<float2 *>(trace_score)[st.trace * trace_stride + base + j] = sc;
      }
    }
    // the next fold of the run reads what this one wrote (this workgroup's own stores)
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
  }
}

// The readout rows [0, m) of every unit recomputed from the stored sums (after an import), with the
// arithmetic of the folds above, so that a state that was exported and imported continues to the
// bit like one that was not.
__global__ __launch_bounds__(256) void refresh16_kernel(Dev dv, int m, int slot) {
  constexpr int D = kHeadDim;
  const int u = blockIdx.y, h = u % dv.Hkv;
  const int row = blockIdx.x * 16 + (threadIdx.x >> 4), c16 = threadIdx.x & 15, ch0 = 8 * c16;
  if (row >= m) return;
  const int64_t ro = (int64_t)u * dv.Mcap + row;
  const float *gam = dv.gamma ? dv.gamma + h * D : kOnes, *bet = dv.beta ? dv.beta + h * D : kZeros;
  float ga[8], be[8];
  double sk[8];
  float sv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ga[e] = gam[ch0 + e];
    be[e] = bet[ch0 + e];
    sk[e] = dv.sK[ro * D + ch0 + e];
    sv[e] = dv.sV[ro * D + ch0 + e];
  }
  write_readout16(dv, slot, ro, ch0, sk, sv, dv.rho[ro], ga, be);
}

constexpr size_t kLdsWide = 160 * 1024, kLdsNarrow = 96 * 1024;
bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

}  // namespace

// The shapes this path takes: bf16, head_dim 128; blocks of 2^k * 32 tokens up to 1024 (the waves
// that share a token group split a stage's tiles by a power of two); tables that fit LDS.
bool fold_fused_fits(const Dev &dv, int split) {
  if (!(dv.io == 1 && dv.d == kHeadDim && dv.C % 64 == 0 && dv.C <= 1024 && pow2(dv.C / 32))) return false;
  if (!pow2(split) || split > kFoldMaxSplit || dv.Mcap >= 0xffff) return false;   // rows travel in 16 bits
  return fold_lds(dv.C, dv.Mcap, 16, split).total <= kLdsWide && fold_lds(dv.C, dv.Mcap, 8, split).total <= kLdsNarrow;
}

size_t fold_exchange_bytes(const Dev &dv, int split) {
  return split > 1 ? (size_t)dv.Ufull * 2 * split * 2 * dv.C * sizeof(unsigned long long) : 0;
}

hipError_t launch_refresh16(const Dev &dv, int m, int slot, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  hipLaunchKernelGGL(refresh16_kernel, dim3((m + 15) / 16, dv.U), dim3(256), 0, st, dv, m, slot);
  return hipGetLastError();
}

hipError_t launch_fold_fused(const Dev &dv, const Src &src, const FoldRunArgs &run, bool narrow, hipStream_t st) {
  if (run.n <= 0) return hipSuccess;
  static const hipError_t attr16 = hipFuncSetAttribute((const void *)fold_fused_kernel<16>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsWide);
  static const hipError_t attr8 = hipFuncSetAttribute((const void *)fold_fused_kernel<8>,
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsNarrow);
  if (attr16 != hipSuccess) return attr16;
  if (attr8 != hipSuccess) return attr8;
  const int split = run.split;
  if (split < 1 || (split > 1 && (!run.xtab || !run.err))) return hipErrorInvalidValue;
  if (split > 1) {
    // the unit's workgroups wait for each other: all of the grid must fit the chip at once (one
    // workgroup of either shape per compute unit at least)
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if ((int64_t)dv.U * split > cus) return hipErrorInvalidValue;
  }
  FoldKernelArgs args{dv, src, run};
  const unsigned grid = (unsigned)(dv.U * split);
  if (narrow)
    hipLaunchKernelGGL(fold_fused_kernel<8>, dim3(grid), dim3(512), fold_lds(dv.C, dv.Mcap, 8, split).total, st, args);
  else
    hipLaunchKernelGGL(fold_fused_kernel<16>, dim3(grid), dim3(1024), fold_lds(dv.C, dv.Mcap, 16, split).total, st, args);
  return hipGetLastError();
}

}  // namespace kvm
