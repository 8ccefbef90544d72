// Similarity of an overflow block to the normalised state on the gfx950 matrix cores (bf16,
// head_dim 128): s_j = max_i k-bar_j . s-hat^K_i and pi(j) = argmax_{i >= S} ("Append" and
// "Merge" equations of the paper).
//
// D[row, token] = K-hat_tile . K-bar^T: a lane holds one token column, so the running maximum
// and its row index are per-lane scalars scanned in ascending row order (ties keep the lowest
// row); the two lane halves of a token are merged once at the end.  Each wave keeps the memory
// keys of its 32 tokens in registers; state rows stream through LDS in 64-row tiles.
#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr int kTileTok = 128;  // tokens per workgroup (32 per wave)

__global__ __launch_bounds__(256, 2) void score_mfma_kernel(Dev dv, int slot, int row0, int row1, int first_pass) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kTileKeys * kKStride];
  constexpr int D = kHeadDim;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, l32 = lane & 31;
  const int u = blockIdx.y;
  const int tok0 = blockIdx.x * kTileTok + 32 * wave;
  const bool wave_active = tok0 < dv.C;  // C is a multiple of 32: a wave is all in or all out
  const int j = tok0 + l32;
  const int64_t tj = (int64_t)u * dv.C + (wave_active ? j : 0);

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

  const uint16_t *khat = (const uint16_t *)dv.khat + slot * dv.slot_elems + (int64_t)u * dv.Mcap * D;
  const int n_tiles = (row1 - row0 + kTileKeys - 1) / kTileKeys;
  uint4 kr[4];
  tile_rows_load(khat + (int64_t)row0 * D, D, min(kTileKeys, row1 - row0), tid, kr);
  for (int it = 0; it < n_tiles; ++it) {
    __syncthreads();
    tile_rows_to_lds(Ks, tid, kr);
    __syncthreads();
    const int base = row0 + it * kTileKeys;
    if (it + 1 < n_tiles)
      tile_rows_load(khat + (int64_t)(base + kTileKeys) * D, D, min(kTileKeys, row1 - base - kTileKeys),
                     tid, kr);
    if (!wave_active) continue;
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
        acc[blk] = mfma32(tile_rows_frag(Ks, blk, ks, lane), kreg[ks], acc[blk]);
    // rows this lane sees, ascending: blk, then v
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
      dv.score[tj] = make_float2(best_all, best);
      dv.pi[tj] = best_i;
      dv.app[tj] = -1;
    } else if (dv.app[tj] < 0 && best_i != 0x7fffffff && best > dv.score[tj].y) {
      dv.score[tj].y = best;
      dv.pi[tj] = best_i;
    }
  }
}

}  // namespace

hipError_t launch_score_mfma(const Dev &dv, int slot, int row0, int row1, bool first_pass, hipStream_t st) {
  if (row1 <= row0) return hipSuccess;
  dim3 grid((dv.C + kTileTok - 1) / kTileTok, dv.U);
  hipLaunchKernelGGL(score_mfma_kernel, grid, dim3(256), 0, st, dv, slot, row0, row1, first_pass ? 1 : 0);
  return hipGetLastError();
}

}  // namespace kvm
