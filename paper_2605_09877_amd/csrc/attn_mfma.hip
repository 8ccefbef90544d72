// Fused prefill attention for bf16, head_dim 128 on the gfx950 matrix cores.
//
// One workgroup (4 waves) owns 128 consecutive queries of one chunk for one query head; each
// wave owns 32 of them.  Keys are visited in 64-key tiles through three regions that share one
// online softmax ("Readout" equations of the paper): normalised state rows (scale tau_state,
// all visible), window tokens before the chunk (scale tau_bswa, all visible), and the chunk's
// own tokens (causal).  Per tile and wave:
//   S^T[key, query] = K_tile . Q^T      16 MFMA 32x32x16, K from LDS, Q^T kept in registers
//   online softmax down the key axis: a lane holds one query column, so the running max and
//                                     sum are per-lane scalars plus one exchange with lane^32
//   O^T[d, query]  += V_tile^T . P^T    16 MFMA; V is stored transposed in LDS so that both
//                                     operands are key-contiguous; P^T is S^T's own register
//                                     layout, no shuffle needed
// The mask is never materialised: it is the tile loop bounds plus a compare on diagonal tiles.
#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kTileQ = 128;

__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(Dev dv, AttnArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kTileKeys * kKStride];
  __shared__ __attribute__((aligned(16))) uint16_t Vts[kHeadDim * kVtStride];
  constexpr int D = kHeadDim;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, l32 = lane & 31;
  const int hq = blockIdx.y, b = blockIdx.z;
  const int hkv = hq / (dv.Hq / dv.Hkv);
  const int u = b * dv.Hkv + hkv;
  const int Q0 = blockIdx.x * kTileQ;
  const int wq0 = Q0 + 32 * wave;
  const int myq = wq0 + l32;
  const int nq = a.nq;
  const int m = a.m;

  // Q^T fragments: query myq, channels 16*ks + 8*g .. +7
  bf16x8 qreg[8];
  {
    const int qc = myq < nq ? myq : nq - 1;
    const uint16_t *qrow = (const uint16_t *)a.q + b * a.q_b + (int64_t)qc * a.q_t + hq * a.q_h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      Frag8 f;
      f.q = *reinterpret_cast<const uint4 *>(qrow + 16 * ks + 8 * g);
      qreg[ks] = f.v;
    }
  }
  const float rs = kLog2e * rsqrtf((float)D);
  const float c_state = (dv.tau_state ? dv.tau_state[hq] : 1.f) * rs;
  const float c_bswa = (dv.tau_bswa ? dv.tau_bswa[hq] : 1.f) * rs;

  const int n_st = (m + kTileKeys - 1) / kTileKeys;
  const int qend = (Q0 + kTileQ < nq) ? Q0 + kTileQ : nq;  // one past the last valid query here
  const int n_win = (int)((a.s + qend - a.b + kTileKeys - 1) / kTileKeys);
  const int n_tiles = n_st + n_win;
  const int64_t last_pos = a.s + nq - 1;

  const uint16_t *khat = (const uint16_t *)dv.khat + (int64_t)u * dv.Mcap * D;
  const uint16_t *vhat = (const uint16_t *)dv.vhat + (int64_t)u * dv.Mcap * D;
  const uint16_t *ring_k = (const uint16_t *)dv.winK + (int64_t)u * dv.L * D;
  const uint16_t *ring_v = (const uint16_t *)dv.winV + (int64_t)u * dv.L * D;
  const uint16_t *in_k = (const uint16_t *)a.in.k + b * a.in.k_b + hkv * a.in.k_h;
  const uint16_t *in_v = (const uint16_t *)a.in.v + b * a.in.v_b + hkv * a.in.v_h;

  uint4 kr[4], vr[4];
  auto issue_loads = [&](int it) {
    const uint16_t *kb_, *vb_;
    int64_t kst, vst;
    int valid;
    if (it < n_st) {
      const int row0 = it * kTileKeys;
      kb_ = khat + (int64_t)row0 * D;
      vb_ = vhat + (int64_t)row0 * D;
      kst = vst = D;
      valid = m - row0;
    } else {
      const int64_t p0 = a.b + (int64_t)(it - n_st) * kTileKeys;
      valid = (int)(last_pos - p0 + 1);
      if (p0 >= a.t0) {
        kb_ = in_k + (p0 - a.t0) * a.in.k_t;
        vb_ = in_v + (p0 - a.t0) * a.in.v_t;
        kst = a.in.k_t;
        vst = a.in.v_t;
      } else {
        const int slot = (int)(p0 % dv.L);
        kb_ = ring_k + (int64_t)slot * D;
        vb_ = ring_v + (int64_t)slot * D;
        kst = vst = D;
      }
    }
    valid = valid < kTileKeys ? valid : kTileKeys;
    tile_rows_load(kb_, kst, valid, tid, kr);
    // V: thread takes keys 4*(tid/16) .. +3, channels 8*(tid%16) .. +7
    const int c8 = (tid & 15) * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      int key = 4 * (tid >> 4) + kk;
      key = key < valid ? key : valid - 1;
      vr[kk] = *reinterpret_cast<const uint4 *>(vb_ + (int64_t)key * vst + c8);
    }
  };
  auto store_lds = [&]() {
    tile_rows_to_lds(Ks, tid, kr);
    // transpose the 4 keys x 8 channels block in registers: one 8-byte store per channel
    const uint32_t *w0 = reinterpret_cast<const uint32_t *>(&vr[0]);
    const uint32_t *w1 = reinterpret_cast<const uint32_t *>(&vr[1]);
    const uint32_t *w2 = reinterpret_cast<const uint32_t *>(&vr[2]);
    const uint32_t *w3 = reinterpret_cast<const uint32_t *>(&vr[3]);
    const int d0 = (tid & 15) * 8, key0 = 4 * (tid >> 4);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t lo, hi;
      if (e & 1) {
        lo = (w0[e >> 1] >> 16) | (w1[e >> 1] & 0xffff0000u);
        hi = (w2[e >> 1] >> 16) | (w3[e >> 1] & 0xffff0000u);
      } else {
        lo = (w0[e >> 1] & 0xffffu) | (w1[e >> 1] << 16);
        hi = (w2[e >> 1] & 0xffffu) | (w3[e >> 1] << 16);
      }
      *reinterpret_cast<uint2 *>(Vts + (d0 + e) * kVtStride + key0) = make_uint2(lo, hi);
    }
  };

  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[i][v] = 0.f;
  float m_run = -INFINITY, l_part = 0.f;

  issue_loads(0);
  for (int it = 0; it < n_tiles; ++it) {
    __syncthreads();
    store_lds();
    __syncthreads();
    if (it + 1 < n_tiles) issue_loads(it + 1);

    const bool is_state = it < n_st;
    const int row0 = it * kTileKeys;
    const int64_t p0 = a.b + (int64_t)(it - n_st) * kTileKeys;
    bool need_mask;
    float scale;
    if (is_state) {
      scale = c_state;
      need_mask = m - row0 < kTileKeys;
    } else {
      scale = c_bswa;
      if (p0 > a.s + wq0 + 31) continue;  // every key of the tile lies after this wave's queries
      need_mask = p0 + kTileKeys - 1 > a.s + wq0;
    }

    f32x16 sacc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[i][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
        sacc[blk] = mfma32(tile_rows_frag(Ks, blk, ks, lane), qreg[ks], sacc[blk]);
    }

    float tmax = -INFINITY;
    if (need_mask) {
      // keys up to `lim` (tile-local) are visible to this lane's query
      const int lim = is_state ? (m - row0 - 1) : (int)(a.s + myq - p0);
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = 32 * blk + mfma_row(v, g);
          const float t = key <= lim ? sacc[blk][v] * scale : -INFINITY;
          sacc[blk][v] = t;
          tmax = fmaxf(tmax, t);
        }
    } else {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float t = sacc[blk][v] * scale;
          sacc[blk][v] = t;
          tmax = fmaxf(tmax, t);
        }
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = exp2f(m_run - m_new);
    m_run = m_new;
    l_part *= alpha;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[i][v] *= alpha;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = exp2f(sacc[blk][v] - m_new);
        l_part += p;
        sacc[blk][v] = p;
      }

#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int blk = ks >> 1, v0 = (ks & 1) * 8;
      Frag8 pb;
#pragma unroll
      for (int e = 0; e < 4; ++e) pb.w[e] = pack_bf16(sacc[blk][v0 + 2 * e], sacc[blk][v0 + 2 * e + 1]);
#pragma unroll
      for (int dblk = 0; dblk < 4; ++dblk) {
        const uint16_t *vrow = Vts + (32 * dblk + l32) * kVtStride + 16 * ks + 4 * g;
        Frag8 av;
        av.d[0] = *reinterpret_cast<const uint2 *>(vrow);
        av.d[1] = *reinterpret_cast<const uint2 *>(vrow + 8);
        oacc[dblk] = mfma32(av.v, pb.v, oacc[dblk]);
      }
    }
  }

  const float l = l_part + __shfl_xor(l_part, 32, kWave);
  if (myq < nq) {
    const float inv = 1.f / l;
    uint16_t *orow = (uint16_t *)a.out + b * a.o_b + (int64_t)myq * a.o_t + hq * a.o_h;
#pragma unroll
    for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const uint32_t lo = pack_bf16(oacc[dblk][4 * vq] * inv, oacc[dblk][4 * vq + 1] * inv);
        const uint32_t hi = pack_bf16(oacc[dblk][4 * vq + 2] * inv, oacc[dblk][4 * vq + 3] * inv);
        *reinterpret_cast<uint2 *>(orow + 32 * dblk + 8 * vq + 4 * g) = make_uint2(lo, hi);
      }
    if (a.lse && g == 0)
      a.lse[b * a.lse_b + (int64_t)myq * a.lse_t + hq * a.lse_h] = (m_run + log2f(l)) * kLn2;
  }
}

}  // namespace

hipError_t launch_attn_mfma(const Dev &dv, const AttnArgs &a, hipStream_t st) {
  if (a.nq <= 0) return hipSuccess;
  dim3 grid((a.nq + kTileQ - 1) / kTileQ, dv.Hq, dv.B);
  hipLaunchKernelGGL(attn_mfma_kernel, grid, dim3(256), 0, st, dv, a);
  return hipGetLastError();
}

}  // namespace kvm
