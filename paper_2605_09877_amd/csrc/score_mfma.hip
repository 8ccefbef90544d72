// Similarity of an overflow block to the normalised state on the gfx950 matrix cores (bf16,
// head_dim 128): s_j = max_i k-bar_j . s-hat^K_i and pi(j) = argmax_{i >= S} ("Append" and
// "Merge" equations of the paper).
//
// D[row, token] = K-hat_tile . K-bar^T: a lane holds one token column, so the running maximum
// and its row index are per-lane scalars scanned in ascending row order (ties keep the lowest
// row); the two lane halves of a token are merged once at the end.  Each wave keeps the memory
// keys of its 32 tokens in registers; state rows stream HBM -> LDS (direct loads, swizzled,
// double buffered) in 64-row tiles.  The rows are split over gridDim.y workgroups so that one
// fold fills the chip; each split leaves a candidate per token and index_kernel merges them.
#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr int kTileTok = 128;  // tokens per workgroup (32 per wave)

__global__ __launch_bounds__(256, 2) void score_mfma_kernel(Dev dv, int slot, int row0, int row1, int first_pass) {
  __shared__ __attribute__((aligned(1024))) uint16_t Ks[2][kTileElems];
  constexpr int D = kHeadDim;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int u = blockIdx.z;
  const int tok0 = blockIdx.x * kTileTok + 32 * wave;
  const bool wave_active = tok0 < dv.C;  // C is a multiple of 32: a wave is all in or all out
  const int j = tok0 + l32;
  const int64_t tj = (int64_t)u * dv.C + (wave_active ? j : 0);

  // this workgroup's share of the row tiles
  const int tiles_all = (row1 - row0 + kTileKeys - 1) / kTileKeys;
  const int per_split = (tiles_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int t_begin = (int)blockIdx.y * per_split;
  const int t_end = min(t_begin + per_split, tiles_all);

  bf16x8 kreg[8];
  if (wave_active) {
    const uint16_t *krow = (const uint16_t *)dv.kbar + tj * D;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      Frag8 f;
      f.q = *reinterpret_cast<const uint4 *>(krow + 16 * ks + 8 * g);
      kreg[ks] = f.v;
    }
  }
  float best_all = -INFINITY, best = -INFINITY;
  int best_i = 0x7fffffff;
  uint32_t koff[8];
  ktile_offsets(lane, koff);

  const char *khat = (const char *)dv.khat + (slot * dv.slot_elems + ((int64_t)u * dv.Mcap + row0) * D) * 2;
  const DmaLane dl = dma_lane(lane);
  const uint32_t ks_addr = lds_addr_of(&Ks[0][0]);
  auto issue_tile = [&](int t) {
    const int base = t * kTileKeys;
    tile_dma<false, 4>(khat + (uint32_t)base * (D * 2), D * 2, row1 - row0 - base,
                       ks_addr + (uint32_t)(t & 1) * (kTileElems * 2), wave, dl);
  };
  if (t_begin < t_end) issue_tile(t_begin);
  for (int t = t_begin; t < t_end; ++t) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (t + 1 < t_end) issue_tile(t + 1);
    if (!wave_active) continue;
    const uint16_t *Kt = Ks[t & 1];
    f32x16 acc[2];
    {
      bf16x8 kf[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) kf[i] = ktile_frag(Kt, koff, i & 1, i >> 1);
      const f32x16 zero = {0.f};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          const int sl = (2 * ks + blk) & 7;
          acc[blk] = mfma32(kf[sl], kreg[ks], ks == 0 ? zero : acc[blk]);
          if (ks + 4 < 8) kf[sl] = ktile_frag(Kt, koff, blk, ks + 4);
        }
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
    // rows this lane sees, ascending: blk, then v
    const int base = row0 + t * kTileKeys;
    const bool edge = base < dv.S || base + kTileKeys > row1;
    if (edge) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = base + 32 * blk + mfma_row(v, g);
          const float sc = acc[blk][v];
          if (i < row1) {
            best_all = fmaxf(best_all, sc);
            if (i >= dv.S && sc > best) {
              best = sc;
              best_i = i;
            }
          }
        }
    } else {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float sc = acc[blk][v];
          if (sc > best) {
            best = sc;
            best_i = base + 32 * blk + mfma_row(v, g);
          }
        }
    }
  }
  if (!wave_active) return;
  best_all = fmaxf(best_all, best);
  {
    const float ob = __shfl_xor(best, 32, kWave);
    const int oi = __shfl_xor(best_i, 32, kWave);
    const float oa = __shfl_xor(best_all, 32, kWave);
    if (ob > best || (ob == best && oi < best_i)) {
      best = ob;
      best_i = oi;
    }
    best_all = fmaxf(best_all, oa);
  }
  if (g == 0) {
    if (first_pass) {
      dv.cand[tj * kScoreSplits + blockIdx.y] = make_float4(best_all, best, __int_as_float(best_i), 0.f);
    } else if (dv.app[tj] < 0 && best_i != 0x7fffffff && best > dv.score[tj].y) {
      dv.score[tj].y = best;
      dv.pi[tj] = best_i;
    }
  }
}

}  // namespace

// first_pass: returns the number of row splits used through *n_splits (candidates are left in
// dv.cand for index_kernel); otherwise one split updates score/pi in place.
hipError_t launch_score_mfma(const Dev &dv, int slot, int row0, int row1, bool first_pass, int *n_splits,
                             hipStream_t st) {
  if (row1 <= row0) return hipSuccess;
  const int tiles = (row1 - row0 + kTileKeys - 1) / kTileKeys;
  int splits = first_pass ? (tiles >= kScoreSplits ? kScoreSplits : 1) : 1;
  if (n_splits) *n_splits = splits;
  dim3 grid((dv.C + kTileTok - 1) / kTileTok, splits, dv.U);
  hipLaunchKernelGGL(score_mfma_kernel, grid, dim3(256), 0, st, dv, slot, row0, row1, first_pass ? 1 : 0);
  return hipGetLastError();
}

}  // namespace kvm
