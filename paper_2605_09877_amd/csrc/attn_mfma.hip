// Fused prefill attention for bf16, head_dim 128 on the gfx950 matrix cores.
//
// A workgroup of NW waves owns 32*NW consecutive queries of one chunk for one query head; each
// wave owns 32 of them.  Keys are visited in 64-key tiles through three regions that share one
// online softmax ("Readout" equations of the paper): normalised state rows (scale tau_state,
// all visible), window tokens before the chunk (scale tau_bswa, all visible), and the chunk's
// own tokens (causal).  Per tile and wave:
//   QK : S^T[key, query] = K_tile . Q^T   16 MFMA 32x32x16, K from LDS, Q^T kept in registers
//   SM : online softmax down the key axis; a lane holds one query column, so the running max and
//        sum are per-lane scalars plus one exchange with lane^32
//   PV : O^T[d, query] += V_tile^T . P^T  16 MFMA; V^T fragments come out of the row-major V
//        tile through the transposing LDS read; P^T is S^T's own register layout, no shuffle
// K and V tiles go from HBM/L2 straight into LDS (16 B per lane, swizzled rows) ahead of use,
// one barrier per tile.  The mask is never materialised: it is the tile loop bounds plus a
// compare on diagonal tiles.
//
// The kernel runs NW = 4 (128 queries per workgroup, two workgroups per CU; the four tile buffers,
// two K and two V, fill 64 KiB of LDS).  Eight waves on 256 queries halve the tile bytes per flop
// but measured slower, both with one barrier per tile and with the two halves of the workgroup
// running half a tile apart: the waves of one workgroup then move in step and their matrix and
// softmax phases coincide instead of overlapping.
#include <type_traits>

#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kXcds = 8;  // accelerator dies, each with its own L2

template <int NW>
__device__ __forceinline__ void attn_body(const Dev &dv, const AttnArgs &a, uint16_t *Ks, uint16_t *Vs) {
  constexpr int D = kHeadDim;
  constexpr int kTileQ = 32 * NW;
  constexpr int kVBufs = 2;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
  const int g = lane >> 5, l32 = lane & 31;
  // Workgroup -> work item.  The tpc * Gq workgroups that read the same K and V (query tiles of one
  // chunk x query heads of one KV group) are given to one XCD, whose L2 then serves all but the
  // first read of every tile: consecutive workgroup ids go round-robin over the 8 XCDs, so id % 8
  // picks the XCD and id / 8 walks that XCD's own sequence of (group, member) pairs.
  // The workgroup's 32 * NW query rows: with grouped queries (NW query heads or a multiple per KV
  // head) the waves take the same 32 positions of NW different heads, so that all of them end at
  // the same causal tile (no wave idles at the barriers while another finishes the diagonal, and
  // the workgroup stops loading tiles a position block sooner); otherwise consecutive positions
  // of one head.
  const int Gq = dv.Hq / dv.Hkv;
  const bool by_head = Gq % NW == 0;
  const int span = by_head ? 32 : kTileQ;   // positions a workgroup covers
  const int hpw = by_head ? NW : 1;         // heads a workgroup covers
  const int tpc = (dv.C + span - 1) / span;
  const int per_group = tpc * (Gq / hpw);
  const int n_groups = a.n_chunks * dv.Hkv * dv.B;
  const int xcd = blockIdx.x % kXcds, seq = blockIdx.x / kXcds;
  const int group = (seq / per_group) * kXcds + xcd;
  if (group >= n_groups) return;
  const int member = seq % per_group;
  const int qt = member % tpc, gq = (member / tpc) * hpw + (by_head ? wave : 0);
  const int ci = group % a.n_chunks;
  const int hkv = (group / a.n_chunks) % dv.Hkv;
  const int b = group / (a.n_chunks * dv.Hkv);
  const int hq = __builtin_amdgcn_readfirstlane(hkv * Gq + gq);
  const int u = b * dv.Hkv + hkv;
  const int Q0 = (tpc - 1 - qt) * span;                                  // longest causal part first
  const int nq = ci == a.n_chunks - 1 ? a.nq_total - ci * dv.C : dv.C;  // queries of this chunk
  if (Q0 >= nq) return;
  const int64_t cs = a.s + (int64_t)ci * dv.C;                           // chunk start position
  const int64_t wb = cs + dv.C - dv.L > 0 ? cs + dv.C - dv.L : 0;        // first window position
  const int wq0 = by_head ? Q0 : Q0 + 32 * wave;
  const int myq = wq0 + l32;
  const int m = a.m[ci];

  // Q^T fragments: query myq, channels 16*ks + 8*g .. +7
  bf16x8 qreg[8];
  {
    const int qc = myq < nq ? myq : nq - 1;
    const uint16_t *qrow =
        (const uint16_t *)a.q + b * a.q_b + ((int64_t)ci * dv.C + qc) * a.q_t + hq * a.q_h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      Frag8 f;
      f.q = *reinterpret_cast<const uint4 *>(qrow + 16 * ks + 8 * g);
      qreg[ks] = f.v;
    }
  }
  const float rs = kLog2e * rsqrtf((float)D);
  float c_state = (dv.tau_state ? dv.tau_state[hq] : 1.f) * rs;
  float c_bswa = (dv.tau_bswa ? dv.tau_bswa[hq] : 1.f) * rs;
  // The softmax below takes the row maximum on raw dot products and applies a positive scale
  // afterwards; for a negative temperature the region's dot products are negated, by flipping
  // the sign of Q^T when the tile loop enters the region (exact in bf16, and K . (-Q) = -(K . Q)
  // bit for bit).  Two bits of one wave-uniform scalar, so that the test is a scalar one.
  const int neg_bits = __builtin_amdgcn_readfirstlane((c_state < 0.f ? 1 : 0) | (c_bswa < 0.f ? 2 : 0));
  c_state = fabsf(c_state);
  c_bswa = fabsf(c_bswa);

  const int n_st = __builtin_amdgcn_readfirstlane((m + kTileKeys - 1) / kTileKeys);
  const int qend = (Q0 + span < nq) ? Q0 + span : nq;  // one past the last valid query here
  const int n_win = (int)((cs + qend - wb + kTileKeys - 1) / kTileKeys);
  const int n_tiles = __builtin_amdgcn_readfirstlane(n_st + n_win);

  // Tile sources, all wave-uniform: state rows of this chunk's version; window positions from the
  // call's own k/v (at or after t0) or from the ring (before t0).  Positions are kept relative
  // to the chunk start so that the per-tile arithmetic is 32-bit.
  // All of it is wave-uniform, which the compiler cannot see through the 64-bit divisions above:
  // each value is pinned to scalar registers once, so that the per-tile address arithmetic and
  // the loads' base operands are scalar instructions.
  auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
  auto uni_ptr = [](const char *p_) {
    const uint64_t x = (uint64_t)p_;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(x >> 32));
    return (const char *)(((uint64_t)hi << 32) | (uint64_t)lo);
  };
  const char *khat = uni_ptr((const char *)dv.khat + (a.slot[ci] * dv.slot_elems + (int64_t)u * dv.Mcap * D) * 2);
  const char *vhat = uni_ptr((const char *)dv.vhat + (a.slot[ci] * dv.slot_elems + (int64_t)u * dv.Mcap * D) * 2);
  const char *ring_k = uni_ptr((const char *)dv.winK + (int64_t)u * dv.L * D * 2);
  const char *ring_v = uni_ptr((const char *)dv.winV + (int64_t)u * dv.L * D * 2);
  const uint32_t kst_in = (uint32_t)uni((int)(a.in.k_t * 2)), vst_in = (uint32_t)uni((int)(a.in.v_t * 2));
  const char *in_k = uni_ptr((const char *)a.in.k + (b * a.in.k_b + hkv * a.in.k_h + (cs - a.t0) * a.in.k_t) * 2);
  const char *in_v = uni_ptr((const char *)a.in.v + (b * a.in.v_b + hkv * a.in.v_h + (cs - a.t0) * a.in.v_t) * 2);
  const int wrel = uni((int)(wb - cs));                              // first window position (<= 0)
  const int t0rel = uni(a.t0 - cs < -(1 << 30) ? -(1 << 30) : (int)(a.t0 - cs));
  const int ring_slot0 = uni((int)(wb % dv.L));
  const int last_rel = uni(nq - 1);

  // Per-lane fragment offsets (elements) from the start of the K / V buffers.  K has two buffers
  // and its offsets flip after every tile; V buffers are addressed by tile number.
  uint32_t koff[8], voff[2];
  ktile_offsets(lane, koff);
  vtile_offsets(lane, voff);
  const DmaLane dl = dma_lane(lane);
  const uint32_t ks_addr = lds_addr_of(Ks), vs_addr = lds_addr_of(Vs);

  struct TileSrc {
    const char *k, *v;
    uint32_t kst, vst;
    int valid;
  };
  auto tile_src = [&](int it) {
    TileSrc t;
    if (it < n_st) {
      const int row0 = it * kTileKeys;
      t.k = khat + (uint32_t)row0 * (D * 2);
      t.v = vhat + (uint32_t)row0 * (D * 2);
      t.kst = t.vst = D * 2;
      t.valid = m - row0;
    } else {
      const int w = it - n_st;
      const int prel = wrel + w * kTileKeys;
      t.valid = last_rel - prel + 1;
      if (prel >= t0rel) {
        t.k = in_k + (int64_t)prel * (int64_t)kst_in;
        t.v = in_v + (int64_t)prel * (int64_t)vst_in;
        t.kst = kst_in;
        t.vst = vst_in;
      } else {
        int slot = ring_slot0 + w * kTileKeys;
        slot = slot >= dv.L ? slot - dv.L : slot;   // a window is at most L long: one wrap
        t.k = ring_k + (uint32_t)slot * (D * 2);
        t.v = ring_v + (uint32_t)slot * (D * 2);
        t.kst = t.vst = D * 2;
      }
    }
    return t;
  };
  auto issue_tile = [&](int it) {
    const TileSrc t = tile_src(it);
    tile_dma<false, NW>(t.k, t.kst, t.valid, ks_addr + (uint32_t)(it & 1) * (kTileElems * 2), wave, dl);
    tile_dma<true, NW>(t.v, t.vst, t.valid, vs_addr + (uint32_t)(it % kVBufs) * (kTileElems * 2), wave, dl);
  };

  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[i][v] = 0.f;
  float m_run = -INFINITY, l_part = 0.f;
  Frag8 pb[4];  // P^T of the tile just scored, packed for the second product

  // O^T += V^T . P^T for the tile whose P^T is in pb.  The first eight V^T fragments are asked
  // for ahead of the softmax (pv_fetch), so that their LDS latency is not waited for here.
  bf16x8 vf[8];
  auto pv_fetch = [&](auto parity) {
    const uint16_t *Vt = Vs + decltype(parity)::value * kTileElems;
#pragma unroll
    for (int i = 0; i < 8; ++i) vf[i] = vtile_frag(Vt, voff, i & 3, i >> 2);
  };
  auto do_pv = [&](auto parity) {
    const uint16_t *Vt = Vs + decltype(parity)::value * kTileElems;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int dblk = 0; dblk < 4; ++dblk) {
        const int i = 4 * ks + dblk, slot = i & 7;
        oacc[dblk] = mfma32(vf[slot], pb[ks].v, oacc[dblk]);
        if (i + 8 < 16) vf[slot] = vtile_frag(Vt, voff, dblk, ks + 2);
      }
  };

  // S^T = K . Q^T and the online softmax for the tile in the current K buffer; leaves P^T in pb.
  auto do_qk_softmax = [&](bool is_state, int row0, int64_t p0, auto parity) {
    const uint16_t *Kt = Ks + decltype(parity)::value * kTileElems;
    const float scale = is_state ? c_state : c_bswa;
    const bool need_mask = is_state ? (m - row0 < kTileKeys) : (p0 + kTileKeys - 1 > cs + wq0);
    f32x16 sacc[2];
    // a rolling window of eight K fragments in flight from LDS, so that a matrix instruction does
    // not wait for the read issued just before it
    {
      bf16x8 kf[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) kf[i] = ktile_frag(Kt, koff, i & 1, i >> 1);
      const f32x16 zero = {0.f};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
          const int slot = (2 * ks + blk) & 7;
          sacc[blk] = mfma32(kf[slot], qreg[ks], ks == 0 ? zero : sacc[blk]);
          if (ks + 4 < 8) kf[slot] = ktile_frag(Kt, koff, blk, ks + 4);
        }
      }
      // pin that order: 8 LDS reads up front, then one read behind every matrix instruction
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
    pv_fetch(parity);
    if (need_mask) {
      // keys up to `lim` (tile-local) are visible to this lane's query
      const int lim = is_state ? (m - row0 - 1) : (int)(cs + myq - p0);
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          sacc[blk][v] = (32 * blk + mfma_row(v, g)) <= lim ? sacc[blk][v] : -INFINITY;
    }
    float smax = sacc[0][0];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int v = 0; v < 16; ++v) smax = fmaxf(smax, sacc[blk][v]);
    smax = xhalf_max(smax);  // the other lane half holds the other 32 keys of the same query
    // m_run is the reference point of the exponentials rather than the running maximum itself: it
    // moves, and what is accumulated is rescaled, only when the maximum of some query of the wave
    // has risen more than kSlack (log2 units) above it.  Until then p = 2^(s - m_run) may exceed
    // 1, by at most 2^kSlack: harmless in fp32 and in bf16 (same relative precision at any
    // magnitude), and the division by the sum, taken against the same reference, is unchanged.
    // Some maximum among 32 queries creeps up in most tiles; a jump of this size is rare after
    // the first.
    constexpr float kSlack = 8.f;
    const float m_new = fmaxf(m_run, smax * scale);
    if (__builtin_amdgcn_ballot_w64(m_new > m_run + kSlack) != 0) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_part *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[i][v] *= alpha;
    }
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        sacc[blk][v] = __builtin_amdgcn_exp2f(fmaf(sacc[blk][v], scale, -m_run));
      }
    // The row sum is taken over the probabilities as rounded to bf16 for the second product, two
    // per instruction (v_dot2c_f32_bf16 with a pair of ones): numerator and denominator of the
    // output then see the same rounded values.
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pb[ks].w[e] = pack_bf16(sacc[ks >> 1][(ks & 1) * 8 + 2 * e], sacc[ks >> 1][(ks & 1) * 8 + 2 * e + 1]);
        l_part = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pb[ks].w[e]), ones, l_part, false);
      }
  };

  // One barrier per tile: it publishes tile `it` (every wave has waited for its own share of the
  // loads) and frees the buffers of tile it - 1 for the loads of tile it + 1.  (Measured and
  // dropped: a second barrier per tile that lets K and V loads run a tile and a half ahead, and
  // touching the lines of later tiles to pull them into L2 early; neither beat this loop.)
  bool q_negated = false;
  // Q^T is in registers from here on: said explicitly, or the compiler, which does not count the
  // tile loads, would wait for "its" loads inside the loop and drain the tile loads with them
  __builtin_amdgcn_s_waitcnt(0);
  issue_tile(0);
  // One tile; the buffer pair it lives in (tile number mod 2) is a compile-time constant, so
  // that the buffer's offset folds into the LDS instructions instead of costing address updates.
  auto tile_step = [&](int it, auto parity) {
    const bool is_state = it < n_st;
    if (((neg_bits & (is_state ? 1 : 2)) != 0) != q_negated) {
      asm volatile("" ::: "memory");  // stays a (rarely taken) branch
      q_negated = !q_negated;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        Frag8 f;
        f.v = qreg[ks];
#pragma unroll
        for (int e = 0; e < 4; ++e) f.w[e] ^= 0x80008000u;
        qreg[ks] = f.v;
      }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (it + 1 < n_tiles) issue_tile(it + 1);
    const int64_t p0 = wb + (int64_t)(it - n_st) * kTileKeys;
    // skip tiles whose keys all lie after this wave's queries
    if (is_state || p0 <= cs + wq0 + 31) {
      do_qk_softmax(is_state, it * kTileKeys, p0, parity);
      do_pv(parity);
    }
  };
  for (int it = 0; it < n_tiles; it += 2) {
    tile_step(it, std::integral_constant<int, 0>{});
    if (it + 1 < n_tiles) tile_step(it + 1, std::integral_constant<int, 1>{});
  }
  const float l = xhalf_sum(l_part);
  if (myq < nq) {
    const float inv = 1.f / l;
    uint16_t *orow = (uint16_t *)a.out + b * a.o_b + ((int64_t)ci * dv.C + myq) * a.o_t + hq * a.o_h;
#pragma unroll
    for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const uint32_t lo = pack_bf16(oacc[dblk][4 * vq] * inv, oacc[dblk][4 * vq + 1] * inv);
        const uint32_t hi = pack_bf16(oacc[dblk][4 * vq + 2] * inv, oacc[dblk][4 * vq + 3] * inv);
        *reinterpret_cast<uint2 *>(orow + 32 * dblk + 8 * vq + 4 * g) = make_uint2(lo, hi);
      }
    if (a.lse && g == 0)
      a.lse[b * a.lse_b + ((int64_t)ci * dv.C + myq) * a.lse_t + hq * a.lse_h] = (m_run + log2f(l)) * kLn2;
  }
}

// Static LDS: 2 K + 2 V tile buffers = 64 KiB, two workgroups per CU.
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel_q128(Dev dv, AttnArgs a) {
  __shared__ __attribute__((aligned(32768))) uint16_t Ks[2 * kTileElems];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs[2 * kTileElems];
  attn_body<4>(dv, a, Ks, Vs);
}

}  // namespace

hipError_t launch_attn_mfma(const Dev &dv, const AttnArgs &a, hipStream_t st) {
  if (a.nq_total <= 0) return hipSuccess;
  const int Gq = dv.Hq / dv.Hkv;
  const bool by_head = Gq % 4 == 0;  // as in the kernel: four heads x 32 positions, or 128 positions of one head
  const int span = by_head ? 32 : 128;
  const int per_group = ((dv.C + span - 1) / span) * (by_head ? Gq / 4 : Gq);
  const int n_groups = a.n_chunks * dv.Hkv * dv.B;
  dim3 grid((unsigned)((n_groups + kXcds - 1) / kXcds * kXcds * per_group));
  hipLaunchKernelGGL(attn_mfma_kernel_q128, grid, dim3(256), 0, st, dv, a);
  return hipGetLastError();
}

}  // namespace kvm
