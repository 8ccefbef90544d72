// Attention part of the backward pass for bf16, head_dim 128 on the gfx950 matrix cores.
//
// One kernel body in three roles.  Each wave keeps 32 "stationary" vectors in registers, as B
// operands, and walks 64-row "streamed" tiles that come through LDS:
//   role dQ : stationary = 32 queries (q and dout rows), streamed = keys (state rows of the
//             visited version, then window tokens; K and V rows)           -> dq
//   roles dK, dV: stationary = 32 keys (K and V rows), streamed = the chunk's queries, head
//             after head of the group (q and dout rows)                    -> dk resp. dv (or
//             the adjoint of the state readout).  One kernel for both would hold two sets of
//             result registers and run one wave per SIMD (measured: 550 us per chunk of the bench
//             workload); apart they run two per SIMD, at the price of the logits computed once
//             more.
// Per streamed tile and wave, with X the streamed "key-like" tile (K or q) and Y the streamed
// "value-like" tile (V or dout):
//   S^T  = X . staK^T           16 matrix instructions (32x32x16)    logits, transposed
//   dP^T = Y . staV^T           16
//   P^T  = exp(tau * scale * S^T - lse),  dS^T = P^T * (dP^T - D)   lse and D belong to the query:
//          to the lane's own column in role dQ, to the row in roles dK, dV (then they come from LDS)
//   O1^T += X^T . (tau dS^T)    16      dq^T resp. dk^T          (roles dQ, dK)
//   O2^T += Y^T . P^T           16      dv^T                     (role dV, which skips dP^T and dS^T)
// Both products that need a streamed tile transposed read it through the transposing LDS load
// from the one swizzled image that the first two products read row by row.  Tiles are filled by
// direct global -> LDS loads one tile ahead, one barrier per tile, like the forward kernel.
#include <type_traits>

#include "kvm_device.h"
#include "kvm_internal.h"
#include "kvm_mfma.h"

namespace kvm {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kXcds = 8;
constexpr int kStaPerWg = 128;                                      // stationary vectors per workgroup (4 waves)
constexpr int kBwdTileBytes = 4 * kTileElems * 2 + 2 * 2 * 64 * 4;  // 2 stages x 2 images + row scalars
constexpr int kBwdLdsBytes = kBwdTileBytes + 2 * 4 * kHeadDim * 4;  // + the LN_s parameter sums of the dK role

// Transposed (A-operand) fragment of a K-swizzled row-major tile: lane gets channel
// 32*dblk + lane%32 and rows 16*ks + 4*g + {0..3}, 16*ks + 8 + 4*g + {0..3}.  Lane j of a group
// of 16 addresses row 4*g + j/4 (+ 8 for the second read) and the 8 bytes at channel
// 32*dblk + 16*half + 4*(j%4); chunk q of row r sits in slot q ^ (r & 15).
__device__ __forceinline__ void ttile_offsets(int lane, uint32_t (&off)[4][2]) {
  const int j = lane & 15, t = j >> 2, c = j & 3;
  const int g = lane >> 5, half = (lane >> 4) & 1;
  const int x = 2 * half + (c >> 1);
#pragma unroll
  for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int r = 8 * hi + 4 * g + t;
      const int slot = ((dblk ^ (2 * hi + g)) << 2) | (x ^ t);
      off[dblk][hi] = (uint32_t)(r * kHeadDim + 8 * slot + 4 * (c & 1));
    }
}
__device__ __forceinline__ bf16x8 ttile_frag(const uint16_t *tile, const uint32_t (&off)[4][2], int dblk, int ks) {
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(KVM_LDS_V4(tile + off[dblk][0] + 16 * ks * kHeadDim));
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(KVM_LDS_V4(tile + off[dblk][1] + 16 * ks * kHeadDim));
  Frag8 f;
  f.d[0] = __builtin_bit_cast(uint2, lo);
  f.d[1] = __builtin_bit_cast(uint2, hi);
  return f.v;
}

struct MfmaChunk {
  int64_t cs, wb;   // chunk start, first window position
  int32_t nq, m;    // queries of the chunk, state rows it saw
  int32_t nq_ext;   // queries from the chunk start on that see the chunk's own tokens as window keys
  int32_t folded;   // the chunk's tokens were folded later on: their first gradient share is in the ring
  int32_t ring_row0;  // where in the ring ([U, ring rows, d]) the chunk's tokens have that share
  int32_t section;    // roles dK, dV: kSecBoth, or only the window-key / only the state-row workgroups
};


template <int kRole>
__global__ __launch_bounds__(256, 2) void bwd_mfma_kernel(Bwd a, MfmaChunk c) {
  constexpr bool kKeysSta = kRole != kRoleDQ;
  constexpr bool kWantDS = kRole != kRoleDV;  // dP^T, dS^T and the first result
  extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
  float *rowsc = reinterpret_cast<float *>(lds + 4 * kTileElems);  // [stage][lse * log2e | D][64]
  constexpr int D = kHeadDim;
  const Dev &dv = a.dv;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 5, l32 = lane & 31;
  const int G = dv.Hq / dv.Hkv;
  const int n_keys_win = c.nq;  // roles dK, dV: the window keys of a launch are the chunk's own tokens
  const int n_st_wg = (c.m + kStaPerWg - 1) / kStaPerWg;
  const int tpc = (c.nq + kStaPerWg - 1) / kStaPerWg;
  // Consecutive workgroup ids go round-robin over the 8 XCDs: a unit's workgroups share one L2.
  // Roles dK, dV: the grid has two sections, the window-key workgroups of all units first and the
  // state-row workgroups after them.  The former stream a whole window of queries and the latter
  // one chunk: started first, the long ones are done when the short ones have had two rounds
  // (interleaved unit by unit, the last long ones would start after the first round of short ones).
  const int n_win_wg = (n_keys_win + kStaPerWg - 1) / kStaPerWg;
  const int groups8 = (dv.U + kXcds - 1) / kXcds * kXcds;
  int wg = blockIdx.x, per_group = G * tpc;
  bool section_state = false;
  if constexpr (kKeysSta) {
    section_state = c.section == kSecState || (c.section == kSecBoth && wg >= groups8 * n_win_wg);
    per_group = section_state ? n_st_wg : n_win_wg;
    if (section_state && c.section == kSecBoth) wg -= groups8 * n_win_wg;
  }
  const int xcd = wg % kXcds, seq = wg / kXcds;
  const int u = (seq / per_group) * kXcds + xcd;
  if (u >= dv.U) return;
  const int member = seq % per_group;
  const int b = u / dv.Hkv, h = u % dv.Hkv;
  const float scale = rsqrtf((float)D);

  // ---- stationary vectors
  bool col_ok;
  const uint16_t *sk_row, *sv_row;
  int colq = 0;          // role dQ: the lane's query within the chunk
  int64_t kpos = -1;     // roles dK, dV, window keys: the lane's key position
  int hq_sta = 0, st_row = 0;
  bool sta_state = false;
  int wg_first = 0;      // roles dK, dV, window keys: first key position of the workgroup, relative to cs
  if constexpr (!kKeysSta) {
    const int qt = member % tpc, gq = member / tpc;
    hq_sta = __builtin_amdgcn_readfirstlane(h * G + gq);
    colq = kStaPerWg * qt + 32 * wave + l32;
    col_ok = colq < c.nq;
    const int qc = col_ok ? colq : c.nq - 1;
    const int64_t qrow = ((int64_t)b * a.T + c.cs + qc) * dv.Hq + hq_sta;
    sk_row = (const uint16_t *)a.q + qrow * D;
    sv_row = (const uint16_t *)a.dout + qrow * D;
  } else {
    sta_state = section_state;
    if (sta_state) {
      st_row = kStaPerWg * member + 32 * wave + l32;
      col_ok = st_row < c.m;
      const int64_t ro = ((int64_t)u * dv.Mcap + (col_ok ? st_row : c.m - 1)) * D;
      sk_row = (const uint16_t *)a.khat + ro;
      sv_row = (const uint16_t *)a.vhat + ro;
    } else {
      const int64_t first = c.cs + (int64_t)kStaPerWg * member;
      wg_first = (int)(first - c.cs);
      kpos = first + 32 * wave + l32;
      col_ok = kpos < c.cs + c.nq;
      const int64_t tok = ((int64_t)b * a.T + (col_ok ? kpos : c.cs + c.nq - 1)) * dv.Hkv + h;
      sk_row = (const uint16_t *)a.k + tok * D;
      sv_row = (const uint16_t *)a.v + tok * D;
    }
  }
  bf16x8 sk[8], sv[8];
  float lse2_col = 0.f, d_col = 0.f;

  // ---- streamed tiles
  int n_st = 0, n_tiles, qt0 = 0, per_head = 1;
  int nq_str = c.nq;  // roles dK, dV: queries streamed, from the chunk start on
  if constexpr (!kKeysSta) {
    n_st = (c.m + kTileKeys - 1) / kTileKeys;
    const int qt = member % tpc;
    const int qend = kStaPerWg * (qt + 1) < c.nq ? kStaPerWg * (qt + 1) : c.nq;
    n_tiles = n_st + (int)((c.cs + qend - c.wb + kTileKeys - 1) / kTileKeys);
  } else {
    nq_str = sta_state ? c.nq : c.nq_ext;
    const int n_qt = (nq_str + kTileKeys - 1) / kTileKeys;
    qt0 = (!sta_state && wg_first > 0) ? wg_first / kTileKeys : 0;
    per_head = n_qt - qt0;
    n_tiles = G * per_head;
    // Order of the streamed tiles: the last query tile first, and for each query tile the heads
    // of the group one after the other.  The workgroups of a unit that share a stream differ in
    // where their first visible tile lies, not in where the last one does: walking backwards
    // they all start on the same tile and stay in step, so that one of them brings a tile into
    // the XCD's L2 and the others find it there (ascending, head by head, they ran up to six
    // tiles apart and the stream was fetched more than twice over).
  }
  n_tiles = __builtin_amdgcn_readfirstlane(n_tiles);

  uint32_t koff[8], toff[4][2];
  ktile_offsets(lane, koff);
  ttile_offsets(lane, toff);
  const DmaLane dl = dma_lane(lane);
  const uint32_t lds_addr = lds_addr_of(lds);

  auto issue_tile = [&](int it) {
    const char *xb, *yb;
    uint32_t stride;
    int valid;
    if constexpr (!kKeysSta) {
      if (it < n_st) {
        const int64_t ro = ((int64_t)u * dv.Mcap + (int64_t)it * kTileKeys) * D * 2;
        xb = (const char *)a.khat + ro;
        yb = (const char *)a.vhat + ro;
        stride = D * 2;
        valid = c.m - it * kTileKeys;
      } else {
        const int64_t p0 = c.wb + (int64_t)(it - n_st) * kTileKeys;
        const int64_t tok = ((int64_t)b * a.T + p0) * dv.Hkv + h;
        xb = (const char *)a.k + tok * D * 2;
        yb = (const char *)a.v + tok * D * 2;
        stride = (uint32_t)dv.Hkv * D * 2;
        valid = (int)(c.cs + c.nq - p0);
      }
    } else {
      const int gq = it % G, qtile = qt0 + per_head - 1 - it / G;
      const int64_t qrow = ((int64_t)b * a.T + c.cs + (int64_t)qtile * kTileKeys) * dv.Hq + h * G + gq;
      xb = (const char *)a.q + qrow * D * 2;
      yb = (const char *)a.dout + qrow * D * 2;
      stride = (uint32_t)dv.Hq * D * 2;
      valid = nq_str - qtile * kTileKeys;
    }
    const uint32_t at = lds_addr + (uint32_t)(2 * (it & 1)) * (kTileElems * 2);
    tile_dma<false, 4>(xb, stride, valid, at, wave, dl);
    tile_dma<false, 4>(yb, stride, valid, at + kTileElems * 2, wave, dl);
  };
  // roles dK, dV: lse and D of a tile's 64 query rows, fetched by the first wave a tile ahead and
  // put into LDS just before the barrier that publishes the tile
  float rs_lse = 0.f, rs_d = 0.f;
  auto fetch_rowsc = [&](int it) {
    if constexpr (kKeysSta) {
      if (wave == 0) {
        const int gq = it % G, qtile = qt0 + per_head - 1 - it / G;
        int r = qtile * kTileKeys + lane;
        r = r < nq_str ? r : nq_str - 1;
        const int64_t qrow = ((int64_t)b * a.T + c.cs + r) * dv.Hq + h * G + gq;
        rs_lse = a.lse[qrow] * kLog2e;
        rs_d = a.delta[qrow];
      }
    }
  };
  auto store_rowsc = [&](int it) {
    if constexpr (kKeysSta) {
      if (wave == 0) {
        rowsc[(it & 1) * 128 + lane] = rs_lse;
        rowsc[(it & 1) * 128 + 64 + lane] = rs_d;
      }
    }
  };

  f32x16 o1[4];  // the role's result, transposed: dq^T, dk^T or dv^T
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) o1[i][v] = 0.f;
  float tau_sum_state = 0.f, tau_sum_bswa = 0.f;  // role dQ: sum of dS * S over state / window keys

  auto tile_step = [&](int it, auto parity) {
    store_rowsc(it);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (it + 1 < n_tiles) {
      issue_tile(it + 1);
      fetch_rowsc(it + 1);
    }
    const uint16_t *X = lds + (2 * decltype(parity)::value) * kTileElems;
    const uint16_t *Y = X + kTileElems;
    // what this tile is, and whether any of it is visible to this wave's columns
    bool tile_state;   // logits of this tile use the state temperature
    bool need_mask;    // wave-uniform: whether any pair of the tile is invisible to this wave
    int lim_lane = 0;  // role dQ: tile rows <= lim_lane are visible to the lane's query
    int lo_lane = 0, hi_row = 0;  // roles dK, dV: tile rows lo_lane .. hi_row are visible to the lane's key
    int hq;
    if constexpr (!kKeysSta) {
      hq = hq_sta;
      tile_state = it < n_st;
      const int wave_q0 = kStaPerWg * (member % tpc) + 32 * wave;  // the wave's first query
      if (tile_state) {
        lim_lane = c.m - it * kTileKeys - 1;
        need_mask = lim_lane < kTileKeys - 1;
      } else {
        const int p0rel = (int)(c.wb - c.cs) + (it - n_st) * kTileKeys;
        if (p0rel > wave_q0 + 31) return;  // all keys after the wave's queries
        lim_lane = colq - p0rel;           // visible rows: p0rel + r <= colq
        need_mask = p0rel + kTileKeys - 1 > wave_q0;
      }
    } else {
      const int gq = it % G, qtile = qt0 + per_head - 1 - it / G;
      hq = __builtin_amdgcn_readfirstlane(h * G + gq);
      tile_state = sta_state;
      const int row_pos0 = qtile * kTileKeys;  // the tile's first query, relative to the chunk start
      hi_row = nq_str - 1 - row_pos0;          // rows beyond the last query are padding
      need_mask = hi_row < kTileKeys - 1;
      if (!sta_state) {
        const int wave_k0 = wg_first + 32 * wave;  // the wave's first key, relative to the chunk start
        if (wave_k0 > row_pos0 + kTileKeys - 1) return;  // all queries before the wave's keys
        lo_lane = wave_k0 + l32 - row_pos0;              // visible rows: key position <= query position
        need_mask = need_mask || wave_k0 + 31 > row_pos0;
      }
    }
    const float tau = tile_state ? (dv.tau_state ? dv.tau_state[hq] : 1.f) : (dv.tau_bswa ? dv.tau_bswa[hq] : 1.f);
    const float cexp = tau * scale * kLog2e;

    // Role dK takes the two 32-row halves of the tile one after the other -- logits and
    // dout . v^T of the half, the elementwise step, then the half's share of the result -- so
    // that half the logit registers are live; the other roles take them together.
    f32x16 sacc[2], dacc[2];
    Frag8 pP[4], pS[4];
    float tsum = 0.f;
    auto elementwise = [&](auto masked, auto blk_c) {
      {
        constexpr int blk = decltype(blk_c)::value;
        float lse_r[16], d_r[16];
        if constexpr (kKeysSta) {
          const float *rl = rowsc + decltype(parity)::value * 128 + 32 * blk + 4 * g;
#pragma unroll
          for (int v4 = 0; v4 < 4; ++v4) {
            const float4 x = *reinterpret_cast<const float4 *>(rl + 8 * v4);
            const float4 y = *reinterpret_cast<const float4 *>(rl + 64 + 8 * v4);
            lse_r[4 * v4] = x.x; lse_r[4 * v4 + 1] = x.y; lse_r[4 * v4 + 2] = x.z; lse_r[4 * v4 + 3] = x.w;
            d_r[4 * v4] = y.x; d_r[4 * v4 + 1] = y.y; d_r[4 * v4 + 2] = y.z; d_r[4 * v4 + 3] = y.w;
          }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = 32 * blk + mfma_row(v, g);
          bool vis = true;
          float lse2, dd;
          if constexpr (!kKeysSta) {
            if constexpr (decltype(masked)::value) vis = r <= lim_lane;
            lse2 = lse2_col;
            dd = d_col;
          } else {
            if constexpr (decltype(masked)::value) vis = r >= lo_lane && r <= hi_row;
            lse2 = lse_r[v];
            dd = d_r[v];
          }
          const float s = sacc[blk][v];
          const float p = vis ? __builtin_amdgcn_exp2f(fmaf(s, cexp, -lse2)) : 0.f;
          sacc[blk][v] = p;
          if constexpr (kWantDS) {
            const float ds = p * (dacc[blk][v] - dd);
            tsum = fmaf(ds, s, tsum);
            dacc[blk][v] = ds * tau;
          }
        }
      }
    };
    auto first_products = [&](auto blk_c) {
      constexpr int blk = decltype(blk_c)::value;
      const f32x16 zero = {0.f};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        sacc[blk] = mfma32(ktile_frag(X, koff, blk, ks), sk[ks], ks == 0 ? zero : sacc[blk]);
        if constexpr (kWantDS) dacc[blk] = mfma32(ktile_frag(Y, koff, blk, ks), sv[ks], ks == 0 ? zero : dacc[blk]);
      }
    };
    auto second_product = [&](auto blk_c) {
      constexpr int blk = decltype(blk_c)::value;
#pragma unroll
      for (int ks = 2 * blk; ks < 2 * blk + 2; ++ks) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v0 = (ks & 1) * 8 + 2 * e;
          if constexpr (kWantDS)
            pS[ks].w[e] = pack_bf16(dacc[blk][v0], dacc[blk][v0 + 1]);
          else
            pP[ks].w[e] = pack_bf16(sacc[blk][v0], sacc[blk][v0 + 1]);
        }
#pragma unroll
        for (int dblk = 0; dblk < 4; ++dblk) {
          if constexpr (kWantDS)
            o1[dblk] = mfma32(ttile_frag(X, toff, dblk, ks), pS[ks].v, o1[dblk]);
          else
            o1[dblk] = mfma32(ttile_frag(Y, toff, dblk, ks), pP[ks].v, o1[dblk]);
        }
      }
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    using Masked = std::integral_constant<bool, true>;
    using Plain = std::integral_constant<bool, false>;
    if constexpr (kRole == kRoleDK) {
      first_products(B0{});
      if (need_mask) elementwise(Masked{}, B0{}); else elementwise(Plain{}, B0{});
      second_product(B0{});
      first_products(B1{});
      if (need_mask) elementwise(Masked{}, B1{}); else elementwise(Plain{}, B1{});
      second_product(B1{});
    } else if constexpr (kRole == kRoleDV) {
      first_products(B0{});
      first_products(B1{});
      if (need_mask) {
        elementwise(Masked{}, B0{});
        elementwise(Masked{}, B1{});
      } else {
        elementwise(Plain{}, B0{});
        elementwise(Plain{}, B1{});
      }
      second_product(B0{});
      second_product(B1{});
    } else {
      // role dQ has no registers for two variants of the elementwise step: it always compares
      (void)need_mask;
      first_products(B0{});
      first_products(B1{});
      elementwise(Masked{}, B0{});
      elementwise(Masked{}, B1{});
      second_product(B0{});
      second_product(B1{});
    }
    if constexpr (!kKeysSta) {
      if (tile_state) tau_sum_state += tsum; else tau_sum_bswa += tsum;
    }
  };

  // The first tile is asked for ahead of the stationary vectors, so that the two travel together
  // (short loops -- few streamed tiles per workgroup -- feel every round trip of the prologue).
  if (n_tiles > 0) {
    issue_tile(0);
    fetch_rowsc(0);
  }
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    Frag8 f;
    f.q = *reinterpret_cast<const uint4 *>(sk_row + 16 * ks + 8 * g);
    sk[ks] = f.v;
    if constexpr (kWantDS) {
      f.q = *reinterpret_cast<const uint4 *>(sv_row + 16 * ks + 8 * g);
      sv[ks] = f.v;
    }
  }
  if constexpr (!kKeysSta) {
    const int qc = col_ok ? colq : c.nq - 1;
    const int64_t qrow = ((int64_t)b * a.T + c.cs + qc) * dv.Hq + hq_sta;
    lse2_col = a.lse[qrow] * kLog2e;
    // D = dout . out of the lane's query: the lane has half of the dout row already; the other
    // roles, which run after this one, read D from memory
    const uint16_t *o_row = (const uint16_t *)a.out + qrow * D;
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint4 ov = *reinterpret_cast<const uint4 *>(o_row + 16 * ks + 8 * g);
      Frag8 f;
      f.v = sv[ks];
      float of[8], df[8];
      unpack16<bf16_t>(ov, of);
      unpack16<bf16_t>(f.q, df);
#pragma unroll
      for (int e = 0; e < 8; ++e) part = fmaf(of[e], df[e], part);
    }
    d_col = xhalf_sum(part);
    if (col_ok && g == 0) a.delta[qrow] = d_col;
  }

  // the stationary vectors are in registers from here on (the compiler does not count the tile
  // loads; said explicitly so that it does not wait for "its" loads inside the loop)
  __builtin_amdgcn_s_waitcnt(0);
  for (int it = 0; it < n_tiles; it += 2) {
    tile_step(it, std::integral_constant<int, 0>{});
    if (it + 1 < n_tiles) tile_step(it + 1, std::integral_constant<int, 1>{});
  }

  // ---- results (nothing of what follows is to be prepared, or kept in registers, during the loop)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (!kKeysSta) {
    if (col_ok) {
      const int64_t qrow = ((int64_t)b * a.T + c.cs + colq) * dv.Hq + hq_sta;
      uint16_t *orow = (uint16_t *)a.dq + qrow * D;
#pragma unroll
      for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const uint32_t lo = pack_bf16(o1[dblk][4 * vq] * scale, o1[dblk][4 * vq + 1] * scale);
          const uint32_t hi = pack_bf16(o1[dblk][4 * vq + 2] * scale, o1[dblk][4 * vq + 3] * scale);
          *reinterpret_cast<uint2 *>(orow + 32 * dblk + 8 * vq + 4 * g) = make_uint2(lo, hi);
        }
    }
    const float ts = wave_sum(col_ok ? tau_sum_state : 0.f) * scale;
    const float tb = wave_sum(col_ok ? tau_sum_bswa : 0.f) * scale;
    if (lane == 0) {
      atomicAdd(a.par64 + 2 * dv.Hkv * D + hq_sta, (double)ts);
      atomicAdd(a.par64 + 2 * dv.Hkv * D + dv.Hq + hq_sta, (double)tb);
    }
  } else {
    if (col_ok) {
      // The chunk's own tokens as window keys: this launch has streamed every query that sees
      // them, so dk (which carries the logit scale) resp. dv is complete once the share the
      // token got when its fold was undone (kept in fp32 in a ring of the last window's blocks and one more)
      // is added, and goes out in the I/O dtype.
      if (!sta_state) {
        const float os = kRole == kRoleDK ? scale : 1.f;
        const int64_t tok = ((int64_t)b * a.T + kpos) * dv.Hkv + h;
        uint16_t *orow = (uint16_t *)(kRole == kRoleDK ? a.dk : a.dv_out) + tok * D;
        const float *ring = (kRole == kRoleDK ? a.dk_acc : a.dv_acc) +
                            ((int64_t)u * a.ring_rows + c.ring_row0 + (int)(kpos - c.cs)) * D;
#pragma unroll
        for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const int ch = 32 * dblk + 8 * vq + 4 * g;
            float4 x4 = c.folded ? *reinterpret_cast<const float4 *>(ring + ch) : make_float4(0.f, 0.f, 0.f, 0.f);
            x4.x += o1[dblk][4 * vq] * os;
            x4.y += o1[dblk][4 * vq + 1] * os;
            x4.z += o1[dblk][4 * vq + 2] * os;
            x4.w += o1[dblk][4 * vq + 3] * os;
            *reinterpret_cast<uint2 *>(orow + ch) = make_uint2(pack_bf16(x4.x, x4.y), pack_bf16(x4.z, x4.w));
          }
      }
    }
    // State rows: the readout's adjoint goes straight on into the adjoint of the sums.  A lane
    // holds half of its row's channels (four at a time: 32*dblk + 8*vq + 4*g ..), the lane 32
    // away the other half, so a sum over the row is a sum over the lane's registers plus one
    // exchange between the wave's halves.
    if (sta_state) {
      const int64_t ro = ((int64_t)u * dv.Mcap + (col_ok ? st_row : 0)) * D;
      if constexpr (kRole == kRoleDK) {
        // k-hat = LN_s(sK) * gamma + beta.  The standardised sums x-hat and 1 / sqrt(var + eps) of
        // the visited version are kept beside its readout, so everything the row needs is asked
        // for at once: one memory round trip, not a chain of them.
        const float rden = a.rden[(int64_t)u * dv.Mcap + (col_ok ? st_row : 0)];
        float xh[4][16], pg[4][16], pb[4][16];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const int ch = 32 * dblk + 8 * vq + 4 * g;
            const float4 x4 = *reinterpret_cast<const float4 *>(a.xhat + ro + ch);
            const float4 g4 = dv.gamma ? *reinterpret_cast<const float4 *>(dv.gamma + h * D + ch) : make_float4(1.f, 1.f, 1.f, 1.f);
            const float xs[4] = {x4.x, x4.y, x4.z, x4.w}, gs[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float dkh = o1[dblk][4 * vq + e] * scale;
              xh[dblk][4 * vq + e] = xs[e];
              pb[dblk][4 * vq + e] = dkh * gs[e];  // dk-hat * gamma for now
              pg[dblk][4 * vq + e] = dkh;
              s1 += dkh * gs[e];
              s2 += dkh * gs[e] * xs[e];
            }
          }
        const float m1 = xhalf_sum(s1) / (float)D, m2 = xhalf_sum(s2) / (float)D;
        float *red = reinterpret_cast<float *>(reinterpret_cast<char *>(lds) + kBwdTileBytes);  // [gamma | beta][wave][D]
        // the adjoint of the sums; what the parameter gradients sum over the rows is kept:
        // pg = dk-hat * x-hat (dgamma), pb = dk-hat (dbeta), zero for rows beyond the state
#pragma unroll
        for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const int ch = 32 * dblk + 8 * vq + 4 * g;
            float add[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float dkh = pg[dblk][4 * vq + e], x = xh[dblk][4 * vq + e];
              add[e] = (pb[dblk][4 * vq + e] - m1 - x * m2) * rden;
              pg[dblk][4 * vq + e] = col_ok ? dkh * x : 0.f;
              pb[dblk][4 * vq + e] = col_ok ? dkh : 0.f;
            }
            if (col_ok) {
              float4 x4 = *reinterpret_cast<const float4 *>(a.dsK + ro + ch);
              x4.x += add[0]; x4.y += add[1]; x4.z += add[2]; x4.w += add[3];
              *reinterpret_cast<float4 *>(a.dsK + ro + ch) = x4;
            }
          }
        // Sums over the 32 rows (lanes) of this half of the wave, for 64 channels at once: a
        // butterfly in which every exchange also halves the number of channels a lane carries --
        // the lane whose bit is set keeps the upper half of its channels and hands the lower half
        // to its partner, and the other way round -- so that 62 exchanges do the work of 64 x 5.
        // Register i stands for channel 32*(i/16) + 8*((i%16)/4) + 4*g + i%4; after the five
        // steps a lane holds the sums of registers base, base + 1, base = 32*b0 + 16*b1 + 8*b2 +
        // 4*b3 + 2*b4 (b_k = bit k of its lane number).
        auto rows_sum = [&](float (&v)[4][16], int which) {
          float *f = &v[0][0];
#define KVM_BFLY(N, BIT, XCHG)                                  \
  {                                                             \
    const bool up = (lane & BIT) != 0;                          \
    _Pragma("unroll") for (int i = 0; i < N / 2; ++i) {         \
      const float send = up ? f[i] : f[i + N / 2];              \
      const float keep = up ? f[i + N / 2] : f[i];              \
      f[i] = keep + XCHG(send);                                 \
    }                                                           \
  }
#define KVM_X1(x) dpp_get<0xB1>(x)
#define KVM_X2(x) dpp_get<0x4E>(x)
#define KVM_X4(x) __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(x), 0x101F))
#define KVM_X8(x) __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(x), 0x201F))
#define KVM_X16(x) __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(x), 0x401F))
          KVM_BFLY(64, 1, KVM_X1)
          KVM_BFLY(32, 2, KVM_X2)
          KVM_BFLY(16, 4, KVM_X4)
          KVM_BFLY(8, 8, KVM_X8)
          KVM_BFLY(4, 16, KVM_X16)
#undef KVM_BFLY
#undef KVM_X1
#undef KVM_X2
#undef KVM_X4
#undef KVM_X8
#undef KVM_X16
          const int i0 = 32 * (lane & 1) + 16 * ((lane >> 1) & 1) + 8 * ((lane >> 2) & 1) + 4 * ((lane >> 3) & 1) +
                         2 * ((lane >> 4) & 1);
          const int ch0 = 32 * (i0 >> 4) + 8 * ((i0 & 15) >> 2) + 4 * g + (i0 & 3);
          red[(4 * which + wave) * D + ch0] = f[0];
          red[(4 * which + wave) * D + ch0 + 1] = f[1];
        };
        rows_sum(pg, 0);
        rows_sum(pb, 1);
        __syncthreads();
        {
          const int which = tid / D, ch = tid % D;
          const float sum4 = red[(4 * which) * D + ch] + red[(4 * which + 1) * D + ch] + red[(4 * which + 2) * D + ch] +
                             red[(4 * which + 3) * D + ch];
          if (sum4 != 0.f) atomicAdd(a.par64 + (which * dv.Hkv + h) * D + ch, (double)sum4);
        }
      } else if constexpr (kRole == kRoleDV) {
        // v-hat = rho * sV / max(|sV|, eps)
        float svr[4][16];
        float nn = 0.f, dot = 0.f;
#pragma unroll
        for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const float4 x4 = *reinterpret_cast<const float4 *>(a.wsV + ro + 32 * dblk + 8 * vq + 4 * g);
            const float xs[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              svr[dblk][4 * vq + e] = xs[e];
              nn += xs[e] * xs[e];
              dot += o1[dblk][4 * vq + e] * xs[e];
            }
          }
        const float nrm = sqrtf(xhalf_sum(nn));
        const float den = fmaxf(nrm, dv.norm_eps);
        dot = xhalf_sum(dot) / den;  // dv-hat . unit vector
        const float rho = dv.rho[(int64_t)u * dv.Mcap + (col_ok ? st_row : 0)];
        const float back = nrm > dv.norm_eps ? rho * dot / (den * den) : 0.f;
        if (col_ok) {
#pragma unroll
          for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
              const int ch = 32 * dblk + 8 * vq + 4 * g;
              float4 x4 = *reinterpret_cast<const float4 *>(a.dsV + ro + ch);
              x4.x += rho / den * o1[dblk][4 * vq] - back * svr[dblk][4 * vq];
              x4.y += rho / den * o1[dblk][4 * vq + 1] - back * svr[dblk][4 * vq + 1];
              x4.z += rho / den * o1[dblk][4 * vq + 2] - back * svr[dblk][4 * vq + 2];
              x4.w += rho / den * o1[dblk][4 * vq + 3] - back * svr[dblk][4 * vq + 3];
              *reinterpret_cast<float4 *>(a.dsV + ro + ch) = x4;
            }
          if (g == 0) a.drho[(int64_t)u * dv.Mcap + st_row] += dot;
        }
      }
    }
  }
}

}  // namespace

bool backward_on_mfma(const Dev &dv) { return dv.io == 1 && dv.d == kHeadDim && dv.C % 64 == 0; }

// The three launches of one chunk: dq (and the temperature sums), dk, dv (or the readout's adjoint).
hipError_t launch_backward_mfma(const Bwd &a, int64_t cs, int nq, int m, bool folded, int role, int section,
                                hipStream_t st) {
  const Dev &dv = a.dv;
  static bool allowed = false;  // more than 64 KiB of LDS per workgroup has to be asked for once
  if (!allowed) {
    const void *kernels[3] = {(const void *)bwd_mfma_kernel<kRoleDQ>, (const void *)bwd_mfma_kernel<kRoleDK>,
                              (const void *)bwd_mfma_kernel<kRoleDV>};
    for (const void *k : kernels) {
      const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kBwdLdsBytes);
      if (e != hipSuccess) return e;
    }
    allowed = true;
  }
  MfmaChunk c;
  c.cs = cs;
  c.wb = cs + dv.C - dv.L > 0 ? cs + dv.C - dv.L : 0;
  c.nq = nq;
  c.m = m;
  // the chunk's tokens are window keys for the queries of one window from the chunk start on
  const int64_t ext = a.T - cs < dv.L ? a.T - cs : dv.L;
  c.nq_ext = (int)ext;
  c.folded = folded ? 1 : 0;
  c.ring_row0 = (int)((cs / dv.C) % (a.ring_rows / dv.C)) * dv.C;
  c.section = section;
  const int G = dv.Hq / dv.Hkv;
  const unsigned groups = (unsigned)((dv.U + kXcds - 1) / kXcds * kXcds);
  const int n_win_wg = (nq + kStaPerWg - 1) / kStaPerWg, n_st_wg = (m + kStaPerWg - 1) / kStaPerWg;
  if (role == kRoleDQ) {
    hipLaunchKernelGGL((bwd_mfma_kernel<kRoleDQ>), dim3(groups * G * n_win_wg), dim3(256), kBwdLdsBytes, st, a, c);
    return hipGetLastError();
  }
  const int per_k = section == kSecBoth ? n_st_wg + n_win_wg : section == kSecState ? n_st_wg : n_win_wg;
  if (per_k == 0) return hipSuccess;
  if (role == kRoleDK)
    hipLaunchKernelGGL((bwd_mfma_kernel<kRoleDK>), dim3(groups * per_k), dim3(256), kBwdLdsBytes, st, a, c);
  else
    hipLaunchKernelGGL((bwd_mfma_kernel<kRoleDV>), dim3(groups * per_k), dim3(256), kBwdLdsBytes, st, a, c);
  return hipGetLastError();
}

}  // namespace kvm
