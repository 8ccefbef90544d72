// Similarity of an overflow block to the normalised state on the gfx950 matrix cores (bf16,
// head_dim 128): s_j = max_i k-bar_j . s-hat^K_i and pi(j) = argmax_{i >= S} ("Append" and
// "Merge" equations of the paper).
//
// D[row, token] = K-hat_tile . K-bar^T: a lane holds one token column, so the running maximum
// and its row index are per-lane scalars scanned in ascending row order (ties keep the lowest
// row).  A workgroup owns 64 tokens and walks all state rows in stages of two 64-row tiles,
// which stream HBM/L2 -> LDS (direct loads, swizzled, one stage ahead).  Its eight waves split
// a stage as (token half) x (row half of a tile) x (which tile of the stage): a wave keeps the
// memory keys of its 32 tokens in registers and multiplies them with 32 rows per stage.  The
// kernel is bound by latencies (a wave's matrix instructions form one dependent chain per
// tile), so the point of the split is to have four waves per SIMD in flight.  The two lane
// halves of a token and then the four waves that share it are merged once at the end.  One fold
// launches (C / 64) x units workgroups: for the 32k-context workload 512, one resident round.
#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr int kTileTok = 64;  // tokens per workgroup (32 per wave)
constexpr int kXcds = 8;

// best eligible candidate a against b: larger score wins, equal scores keep the lower row
__device__ __forceinline__ bool beats(float sa, int ia, float sb, int ib) {
  return sa > sb || (sa == sb && ia < ib);
}

__global__ __launch_bounds__(512, 2) void score_mfma_kernel(Dev dv, int slot, int row0, int row1, int first_pass) {
  __shared__ __attribute__((aligned(1024))) uint16_t Ks[2][2][kTileElems];  // [stage parity][tile of the stage]
  constexpr int D = kHeadDim;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int th = wave & 1, rh = (wave >> 1) & 1, tp = wave >> 2;  // token half, row half, tile of the stage
  const int g = lane >> 5, l32 = lane & 31;
  // Workgroup -> (unit, token tile).  Consecutive workgroup ids go round-robin over the 8 XCDs,
  // each with its own L2: id % 8 picks the XCD and id / 8 walks that XCD's own units, so that
  // all the workgroups that stream one unit's state rows share one L2.
  const int tpu = (dv.C + kTileTok - 1) / kTileTok;
  const int seq = blockIdx.x / kXcds;
  const int u = (seq / tpu) * kXcds + blockIdx.x % kXcds;
  if (u >= dv.U) return;
  const int tok0 = (seq % tpu) * kTileTok + 32 * th;
  const bool wave_active = tok0 < dv.C;  // C is a multiple of 32: a wave is all in or all out
  const int j = tok0 + l32;
  const int64_t tj = (int64_t)u * dv.C + (wave_active ? j : 0);
  const int n_tiles = (row1 - row0 + kTileKeys - 1) / kTileKeys;
  const int n_stages = (n_tiles + 1) / 2;

  float best_all = -INFINITY, best = -INFINITY;
  int best_i = 0x7fffffff;
  uint32_t koff[8];
  ktile_offsets(lane, koff);

  const char *khat = (const char *)dv.khat + (slot * dv.slot_elems + ((int64_t)u * dv.Mcap + row0) * D) * 2;
  const DmaLane dl = dma_lane(lane);
  const uint32_t ks_addr = lds_addr_of(&Ks[0][0][0]);
  auto issue_stage = [&](int sg) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int t = 2 * sg + i;
      if (t < n_tiles) {
        const int base = t * kTileKeys;
        tile_dma<false, 8>(khat + (uint32_t)base * (D * 2), D * 2, row1 - row0 - base,
                           ks_addr + (uint32_t)(2 * (sg & 1) + i) * (kTileElems * 2), wave, dl);
      }
    }
  };
  // the first stage's tiles and the memory keys travel together; the wait at the top of the
  // loop is for everything outstanding
  if (n_stages > 0) issue_stage(0);
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
  for (int sg = 0; sg < n_stages; ++sg) {
    // stage sg has landed for every wave, and every wave is done reading stage sg - 1
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (sg + 1 < n_stages) issue_stage(sg + 1);
    const int t = 2 * sg + tp;
    if (!wave_active || t >= n_tiles) continue;
    const uint16_t *Kt = Ks[sg & 1][tp];
    // one accumulation chain over the channels in ascending order (the order the one-launch fold
    // path uses too, so that both paths produce the same fp32 scores)
    f32x16 acc0;
    {
      bf16x8 kf[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) kf[i] = ktile_frag(Kt, koff, rh, i);
      const f32x16 zero = {0.f};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) acc0 = mfma32(kf[ks], kreg[ks], ks == 0 ? zero : acc0);
    }
    // rows this lane sees, ascending in v
    const int base = row0 + t * kTileKeys + 32 * rh;
    const bool edge = base < dv.S || base + 32 > row1;
    if (edge) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = base + mfma_row(v, g);
        const float sc = acc0[v];
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
      for (int v = 0; v < 16; ++v) {
        const float sc = acc0[v];
        if (sc > best) {
          best = sc;
          best_i = base + mfma_row(v, g);
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
  // and the three other waves with the same tokens, through LDS: the tile buffers are free once
  // every wave has left the loop
  __syncthreads();
  float *x_all = reinterpret_cast<float *>(&Ks[0][0][0]), *x_best = x_all + 256;
  int *x_idx = reinterpret_cast<int *>(x_all + 512);
  const int part = 2 * tp + rh;  // 0..3: which share of the rows this wave looked at
  if (part != 0 && g == 0) {
    const int xi = 64 * part + 32 * th + l32;
    x_all[xi] = best_all;
    x_best[xi] = best;
    x_idx[xi] = best_i;
  }
  __syncthreads();
  if (part == 0 && g == 0 && wave_active) {
#pragma unroll
    for (int o = 1; o < 4; ++o) {
      const int xi = 64 * o + 32 * th + l32;
      best_all = fmaxf(best_all, x_all[xi]);
      if (beats(x_best[xi], x_idx[xi], best, best_i)) {
        best = x_best[xi];
        best_i = x_idx[xi];
      }
    }
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

// first_pass: rows are the pre-append state, every token gets s_j and its best eligible row.
// Otherwise rows are the ones appended in this fold and only tokens that were not appended
// themselves may move to them (strictly larger score only).
hipError_t launch_score_mfma(const Dev &dv, int slot, int row0, int row1, bool first_pass, hipStream_t st) {
  if (row1 <= row0) return hipSuccess;
  dim3 grid((unsigned)((dv.U + kXcds - 1) / kXcds * kXcds * ((dv.C + kTileTok - 1) / kTileTok)));
  hipLaunchKernelGGL(score_mfma_kernel, grid, dim3(512), 0, st, dv, slot, row0, row1, first_pass ? 1 : 0);
  return hipGetLastError();
}

}  // namespace kvm
