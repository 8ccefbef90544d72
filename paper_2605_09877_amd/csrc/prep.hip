// Attention weight preparation in front of the KVM layer (the paper's appendix "GPTAlpha-2
// Attention weight preparation"; merge gate: Method, "KVM weight preparation"), memory bound:
//   v~ <- (1 - lambda) v~ + lambda v~first          value residual
//   a  =  a~_t + alpha * (a~_{t-1} - a~_t)          token shift of q, k, v (first token unshifted)
//   q, k <- RoPE_r(LN(q)), RoPE_r(LN(k))            LayerNorm with bias per head, rotary on r channels
//   g  =  1 + ELU(x W_g)                            merge gate, one scalar per KV head
// One row (token, head) is handled by d_h / kN adjacent lanes, 16 bytes of channels each, so a
// wave takes several adjacent heads, and walks a run of consecutive tokens of them; statistics
// and the rotation partner come through lane exchanges.
// Arithmetic is fp32; the rotation angles are evaluated in fp64 once per position (a table),
// because position * frequency loses its low bits in fp32 at 32k tokens.
#include "../../include/kvm.h"
#include "kvm_device.h"
#include "kvm_mfma.h"

namespace kvm {
namespace {

__global__ __launch_bounds__(256) void rope_table_kernel(float2 *tab, int64_t n_pos, int64_t pos0, int half,
                                                         double base) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_pos * half) return;
  const int64_t t = i / half;
  const int c = (int)(i % half);
  const double ang = (double)(pos0 + t) * pow(base, -(double)c / (double)half);  // base^(-2c/r)
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}

struct RowArgs {
  const void *in;       // [B, T, H, d] simple q, k or v
  const void *first;    // [B, T, H, d] first-layer value, or null (value residual)
  const void *prev;     // [B, H, d] row of the token before this call, or null
  void *out;            // [B, T, H, d]
  const float *alpha;   // [H, d] or null
  const float *lambda;  // [H, d] or null
  const float *gamma, *beta;  // [H, d] or null
  const float2 *tab;    // [T, r/2] (cos, sin)
  int64_t T;
  int H, r, normalise;
  float eps;
};

// kN fp32 parameters starting at p (16-byte aligned), or the neutral value when p is null.
template <int kN>
__device__ __forceinline__ void load_params(const float *p, float neutral, float (&f)[kN]) {
  if (p) {
#pragma unroll
    for (int i = 0; i < kN; i += 4) {
      const float4 x = *reinterpret_cast<const float4 *>(p + i);
      f[i] = x.x; f[i + 1] = x.y; f[i + 2] = x.z; f[i + 3] = x.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kN; ++i) f[i] = neutral;
  }
}

// kNorm: LayerNorm + rotation (q, k); kResidual: value residual (v).
// A wave takes 64 / (D / kN) adjacent heads (one per lane group: together a contiguous piece of a
// token) and walks kRun consecutive tokens of them, so that the token shift's "previous token" is
// the row the lane group has just had in registers instead of a second read of it (one extra row
// per run), and the per-head parameters are fetched once per run.  Tokens go in blocks of kAhead
// whose loads are all requested before the first of them is worked on.
constexpr int kRun = 16, kAhead = 4;
template <typename T, int D, bool kNorm, bool kResidual>
__global__ __launch_bounds__(256) void prep_rows_kernel(RowArgs a, uint32_t n_hg, uint32_t n_runs, uint32_t n_waves) {
  constexpr int VEC = Vec16<T>::kN;
  constexpr int LPT = D / VEC;   // lanes per row
  constexpr int RPW = 64 / LPT;  // heads per wave
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPT, cl = lane % LPT;
  const uint32_t wg = blockIdx.x * 4u + wave;  // adjacent waves: adjacent head groups of one token run
  if (wg >= n_waves) return;
  const uint32_t hg = wg % n_hg, br = wg / n_hg, run = br % n_runs, b = br / n_runs;
  const uint32_t H = (uint32_t)a.H, T_ = (uint32_t)a.T;
  const uint32_t h_raw = hg * RPW + sub;
  const bool live = h_raw < H;
  const uint32_t h = live ? h_raw : H - 1;  // idle lane groups repeat the last head, store nothing
  const int c0 = cl * VEC;
  const int pc = (int)h * D + c0;  // offset into the per-head parameter arrays
  const uint32_t t_begin = run * kRun, t_end = t_begin + kRun < T_ ? t_begin + kRun : T_;
  const int64_t row_stride = (int64_t)H * D;  // elements between tokens
  const int64_t off0 = (((int64_t)b * T_ + t_begin) * H + h) * D + c0;
  const bool resid = kResidual && a.first && a.lambda;

  float al[VEC], lm[VEC], ga[VEC], be[VEC];
  load_params<VEC>(a.alpha ? a.alpha + pc : nullptr, 0.f, al);
  load_params<VEC>(resid ? a.lambda + pc : nullptr, 0.f, lm);
  if (kNorm) {
    load_params<VEC>(a.gamma ? a.gamma + pc : nullptr, 1.f, ga);
    load_params<VEC>(a.beta ? a.beta + pc : nullptr, 0.f, be);
  }
  // the row before the run (already residual-mixed when it comes from the previous call)
  float prev[VEC];
  bool have_prev = false;
  if (a.alpha) {
    if (t_begin > 0) {
      Vec16<T>::load((const T *)a.in + off0 - row_stride, prev);
      if (resid) {
        float f[VEC];
        Vec16<T>::load((const T *)a.first + off0 - row_stride, f);
#pragma unroll
        for (int i = 0; i < VEC; ++i) prev[i] = (1.f - lm[i]) * prev[i] + lm[i] * f[i];
      }
      have_prev = true;
    } else if (a.prev) {
      Vec16<T>::load((const T *)a.prev + (int64_t)(b * H + h) * D + c0, prev);
      have_prev = true;
    }
  }
  for (uint32_t t0 = t_begin; t0 < t_end; t0 += kAhead) {
    float y[kAhead][VEC], f[kAhead][VEC];
#pragma unroll
    for (int k = 0; k < kAhead; ++k) {
      const uint32_t t = t0 + k < t_end ? t0 + k : t_end - 1;
      const int64_t off = off0 + (int64_t)(t - t_begin) * row_stride;
      Vec16<T>::load((const T *)a.in + off, y[k]);
      if (resid) Vec16<T>::load((const T *)a.first + off, f[k]);
    }
#pragma unroll
    for (int k = 0; k < kAhead; ++k) {
      const uint32_t t = t0 + k;
      if (t >= t_end) break;
      if (resid) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) y[k][i] = (1.f - lm[i]) * y[k][i] + lm[i] * f[k][i];
      }
      float z[VEC];  // the row after the shift; y[k] stays the next token's "previous"
#pragma unroll
      for (int i = 0; i < VEC; ++i) z[i] = have_prev ? y[k][i] + al[i] * (prev[i] - y[k][i]) : y[k][i];
      if (a.alpha) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) prev[i] = y[k][i];
        have_prev = true;
      }
      if (kNorm) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) s += z[i];
        const float mean = group_sum<LPT>(s) * (1.f / (float)D);
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          z[i] -= mean;
          q += z[i] * z[i];
        }
        const float rstd = rsqrtf(group_sum<LPT>(q) * (1.f / (float)D) + a.eps);
#pragma unroll
        for (int i = 0; i < VEC; ++i) z[i] = z[i] * rstd * ga[i] + be[i];
        if (a.r > 0) {
          // channel c < r/2 pairs with c + r/2, which sits r/2/VEC lanes away (a power of two)
          const int half = a.r / 2, hop = half / VEC;
          float o[VEC];
#pragma unroll
          for (int i = 0; i < VEC; ++i) o[i] = __shfl_xor(z[i], hop, kWave);
          if (c0 < a.r) {
            const bool lower = c0 < half;
            float cs[2 * VEC];  // (cos, sin) of this lane's channels
            load_params<2 * VEC>((const float *)(a.tab + (int64_t)t * half + (lower ? c0 : c0 - half)), 0.f, cs);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
              z[i] = lower ? z[i] * cs[2 * i] - o[i] * cs[2 * i + 1] : z[i] * cs[2 * i] + o[i] * cs[2 * i + 1];
          }
        }
      }
      if (live) Vec16<T>::store((T *)a.out + off0 + (int64_t)(t - t_begin) * row_stride, z);
    }
  }
}

// Merge gate: a wave takes kGateTok tokens; lanes stride over the model width, 16 bytes of x each,
// heads in blocks of eight; the per-lane partial dot products are summed across the wave at the
// end.  kFull: the number of KV heads is a multiple of 8, so a row of eight gate weights is two
// aligned 16-byte loads.
constexpr int kGateTok = 8;
template <typename T, bool kFull>
__global__ __launch_bounds__(256) void gate_kernel(const T *x, const float *w, float *gate, int64_t n_tok,
                                                   int dm, int Hkv) {
  constexpr int VEC = Vec16<T>::kN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t tok0 = ((int64_t)blockIdx.x * 4 + wave) * kGateTok;
  if (tok0 >= n_tok) return;
  const T *xr[kGateTok];
#pragma unroll
  for (int k = 0; k < kGateTok; ++k) xr[k] = x + (tok0 + k < n_tok ? tok0 + k : n_tok - 1) * dm;
  for (int h0 = 0; h0 < Hkv; h0 += 8) {
    float acc[kGateTok][8];
#pragma unroll
    for (int k = 0; k < kGateTok; ++k)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[k][j] = 0.f;
    for (int c0 = lane * VEC; c0 < dm; c0 += 64 * VEC) {
      float xv[kGateTok][VEC];
#pragma unroll
      for (int k = 0; k < kGateTok; ++k) Vec16<T>::load(xr[k] + c0, xv[k]);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        float wv[8];
        const float *wrow = w + (int64_t)(c0 + i) * Hkv + h0;
        if (kFull) {
          load_params<8>(wrow, 0.f, wv);
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j) wv[j] = h0 + j < Hkv ? wrow[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int k = 0; k < kGateTok; ++k) acc[k][j] = fmaf(xv[k][i], wv[j], acc[k][j]);
      }
    }
#pragma unroll
    for (int k = 0; k < kGateTok; ++k)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float z = wave_sum(acc[k][j]);
        if (lane == 0 && tok0 + k < n_tok && h0 + j < Hkv)
          gate[(tok0 + k) * Hkv + h0 + j] = 1.f + (z > 0.f ? z : expm1f(z));
      }
  }
}

// The merge gate on the matrix cores (bf16 x, at most 32 KV heads, d_model a multiple of 128).
// W_g is fp32; it is split once per call into two bf16 halves, hi = bf16(w) and lo = bf16(w - hi),
// transposed to [32 heads (zero rows beyond H_kv)][d_model], so that x W_g = x hi + x lo with the
// products exact and the sums in fp32: the same 1e-6-relative arithmetic as the vector version.
constexpr int kGateHeads = 32;
__global__ __launch_bounds__(256) void gate_split_kernel(const float *w, uint16_t *hi, uint16_t *lo, int dm, int Hkv) {
  const int i = blockIdx.x * 256 + threadIdx.x;  // over kGateHeads * dm
  if (i >= kGateHeads * dm) return;
  const int h = i / dm, c = i - h * dm;
  const float x = h < Hkv ? w[(int64_t)c * Hkv + h] : 0.f;
  const uint16_t a = float_to_bf16_bits(x);
  hi[i] = a;
  lo[i] = float_to_bf16_bits(x - bf16_bits_to_float(a));
}

// A wave takes 64 tokens (two blocks of 32 rows of the matrix instruction) and all heads; x goes
// from global memory straight into the A operand (lane = token row, 16 bytes = its 8 channels of
// the step), W's halves into the B operand (lane = head).  Per 128 channels: 16 loads of x in
// flight per lane, 32 matrix instructions.
__global__ __launch_bounds__(256) void gate_mfma_kernel(const uint16_t *x, const uint16_t *hi, const uint16_t *lo,
                                                        float *gate, int64_t n_tok, int dm, int Hkv) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int64_t tok0 = ((int64_t)blockIdx.x * 4 + wave) * 64;
  if (tok0 >= n_tok) return;
  const uint16_t *xr[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int64_t t = tok0 + 32 * tb + l32;
    xr[tb] = x + (t < n_tok ? t : n_tok - 1) * dm + 8 * g;
  }
  const bool head_lane = l32 < ((Hkv + 7) & ~7);  // lanes of the zero rows need not load them
  const uint16_t *hr = hi + (int64_t)l32 * dm + 8 * g, *lr = lo + (int64_t)l32 * dm + 8 * g;
  f32x16 acc[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[tb][v] = 0.f;
  for (int c0 = 0; c0 < dm; c0 += 128) {
    Frag8 xa[2][8], wh[8], wl[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) xa[tb][ks].q = *reinterpret_cast<const uint4 *>(xr[tb] + c0 + 16 * ks);
      wh[ks].q = wl[ks].q = make_uint4(0u, 0u, 0u, 0u);
      if (head_lane) {
        wh[ks].q = *reinterpret_cast<const uint4 *>(hr + c0 + 16 * ks);
        wl[ks].q = *reinterpret_cast<const uint4 *>(lr + c0 + 16 * ks);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        acc[tb] = mfma32(xa[tb][ks].v, wh[ks].v, acc[tb]);
        acc[tb] = mfma32(xa[tb][ks].v, wl[ks].v, acc[tb]);
      }
  }
  if (l32 < Hkv) {
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t t = tok0 + 32 * tb + mfma_row(v, g);
        const float z = acc[tb][v];
        if (t < n_tok) gate[t * Hkv + l32] = 1.f + (z > 0.f ? z : expm1f(z));
      }
  }
}

template <typename T, bool kNorm, bool kResidual>
hipError_t launch_rows(const RowArgs &a, int d, int batch, hipStream_t st) {
  const int heads_per_wave = 64 / (d / Vec16<T>::kN);
  const uint32_t n_hg = (uint32_t)((a.H + heads_per_wave - 1) / heads_per_wave);
  const uint32_t n_runs = (uint32_t)((a.T + kRun - 1) / kRun);
  const int64_t n_waves = (int64_t)batch * n_runs * n_hg;
  if (n_waves >= (1ll << 31)) return hipErrorInvalidValue;
  dim3 grid((unsigned)((n_waves + 3) / 4));
  if (d == 64)
    hipLaunchKernelGGL((prep_rows_kernel<T, 64, kNorm, kResidual>), grid, dim3(256), 0, st, a, n_hg, n_runs,
                       (uint32_t)n_waves);
  else
    hipLaunchKernelGGL((prep_rows_kernel<T, 128, kNorm, kResidual>), grid, dim3(256), 0, st, a, n_hg, n_runs,
                       (uint32_t)n_waves);
  return hipGetLastError();
}

bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// Scratch layout: the rotation table, then (when the matrix-core gate applies) W_g's two bf16 halves.
bool gate_on_mfma(const kvm_prep_params *p) {
  return p->io_dtype == KVM_BF16 && p->d_model > 0 && p->d_model % 128 == 0 && p->n_kv_heads <= kGateHeads;
}
size_t rope_table_bytes(const kvm_prep_params *p, int64_t T) {
  const size_t n = (size_t)T * (size_t)(p->rope_dims / 2) * sizeof(float2);
  return ((n ? n : 16) + 255) & ~(size_t)255;
}
size_t gate_split_bytes(const kvm_prep_params *p) {
  return gate_on_mfma(p) ? 2 * (size_t)kGateHeads * (size_t)p->d_model * 2 : 0;
}

bool valid(const kvm_prep_params *p) {
  if (!p || p->batch <= 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0) return false;
  if (p->head_dim != 64 && p->head_dim != 128) return false;
  if (p->io_dtype != KVM_F32 && p->io_dtype != KVM_BF16) return false;
  const int vec = p->io_dtype == KVM_F32 ? 4 : 8;
  const int r = p->rope_dims;
  if (r < 0 || r > p->head_dim) return false;
  if (r > 0) {
    const int half = r / 2;
    if (r % 2 || half % vec) return false;
    const int hop = half / vec;
    if (hop & (hop - 1)) return false;  // the rotation partner must be a power-of-two lane hop away
  }
  if (p->d_model < 0 || p->d_model % vec) return false;
  return true;
}

}  // namespace
}  // namespace kvm

extern "C" size_t kvm_prepare_scratch_bytes(const kvm_prep_params *p, int64_t T) {
  if (!kvm::valid(p) || T <= 0) return 0;
  return kvm::rope_table_bytes(p, T) + kvm::gate_split_bytes(p);
}

extern "C" int kvm_prepare_qkv(const kvm_prep_params *p, const void *q_raw, const void *k_raw,
                               const void *v_raw, const void *v_first, const void *x, const void *prev_q,
                               const void *prev_k, const void *prev_v, void *q_out, void *k_out,
                               void *v_out, float *gate_out, void *scratch, int64_t T, int64_t pos0,
                               void *stream_) {
  using namespace kvm;
  if (!valid(p) || T <= 0 || pos0 < 0) return KVM_ERR_ARG;
  if (!q_raw || !k_raw || !v_raw || !q_out || !k_out || !v_out || !scratch) return KVM_ERR_ARG;
  if (q_raw == q_out || k_raw == k_out || v_raw == v_out) return KVM_ERR_ARG;  // the shift reads token t - 1
  const void *ptrs[] = {q_raw, k_raw, v_raw, v_first, x, prev_q, prev_k, prev_v, q_out, k_out, v_out, scratch};
  for (const void *q : ptrs)
    if (!al16(q)) return KVM_ERR_ARG;
  const void *prm[] = {p->alpha_q, p->alpha_k, p->alpha_v, p->lambda_v, p->lnq_gamma, p->lnq_beta,
                       p->lnk_gamma, p->lnk_beta, p->w_gate};
  for (const void *q : prm)
    if (!al16(q)) return KVM_ERR_ARG;
  const bool gate = x != nullptr;
  if (gate && (!p->w_gate || !gate_out || p->d_model <= 0)) return KVM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream_;
  const int d = p->head_dim, r = p->rope_dims, half = r / 2;
  const float eps = p->ln_eps > 0.f ? p->ln_eps : 1e-5f;
  float2 *tab = (float2 *)scratch;
  if (half > 0) {
    const int64_t n = T * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, tab, T, pos0, half,
                       p->rope_base > 0.0 ? p->rope_base : 10000.0);
    if (hipGetLastError() != hipSuccess) return KVM_ERR_HIP;
  }
  auto rows = [&](const void *in, const void *first, const void *prev, void *out, const float *alpha,
                  const float *lambda, const float *gamma, const float *beta, int H, int normalise) -> int {
    RowArgs a;
    a.in = in; a.first = first; a.prev = prev; a.out = out;
    a.alpha = alpha; a.lambda = lambda; a.gamma = gamma; a.beta = beta;
    a.tab = tab; a.T = T; a.H = H; a.r = r; a.normalise = normalise; a.eps = eps;
    const int64_t n_rows = (int64_t)p->batch * T * H;
    if (n_rows >= (1ll << 31)) return KVM_ERR_ARG;  // rows are indexed with 32 bits
    hipError_t e;
    if (p->io_dtype == KVM_F32)
      e = normalise ? launch_rows<float, true, false>(a, d, p->batch, st) : launch_rows<float, false, true>(a, d, p->batch, st);
    else
      e = normalise ? launch_rows<bf16_t, true, false>(a, d, p->batch, st)
                    : launch_rows<bf16_t, false, true>(a, d, p->batch, st);
    return e == hipSuccess ? KVM_OK : KVM_ERR_HIP;
  };
  int rc = rows(q_raw, nullptr, prev_q, q_out, p->alpha_q, nullptr, p->lnq_gamma, p->lnq_beta, p->n_q_heads, 1);
  if (rc != KVM_OK) return rc;
  rc = rows(k_raw, nullptr, prev_k, k_out, p->alpha_k, nullptr, p->lnk_gamma, p->lnk_beta, p->n_kv_heads, 1);
  if (rc != KVM_OK) return rc;
  rc = rows(v_raw, v_first, prev_v, v_out, p->alpha_v, p->lambda_v, nullptr, nullptr, p->n_kv_heads, 0);
  if (rc != KVM_OK) return rc;
  if (gate) {
    const int64_t n_tok = (int64_t)p->batch * T;
    dim3 grid((unsigned)((n_tok + 4 * kGateTok - 1) / (4 * kGateTok)));
    const bool full = p->n_kv_heads % 8 == 0;
    const float *wg = p->w_gate;
    const int dm = p->d_model, hk = p->n_kv_heads;
    if (gate_on_mfma(p)) {
      uint16_t *hi = (uint16_t *)((char *)scratch + rope_table_bytes(p, T)), *lo = hi + (size_t)kGateHeads * dm;
      hipLaunchKernelGGL(gate_split_kernel, dim3((unsigned)((kGateHeads * dm + 255) / 256)), dim3(256), 0, st, wg, hi,
                         lo, dm, hk);
      hipLaunchKernelGGL(gate_mfma_kernel, dim3((unsigned)((n_tok + 255) / 256)), dim3(256), 0, st,
                         (const uint16_t *)x, hi, lo, gate_out, n_tok, dm, hk);
    } else if (p->io_dtype == KVM_F32) {
      if (full)
        hipLaunchKernelGGL((gate_kernel<float, true>), grid, dim3(256), 0, st, (const float *)x, wg, gate_out, n_tok, dm, hk);
      else
        hipLaunchKernelGGL((gate_kernel<float, false>), grid, dim3(256), 0, st, (const float *)x, wg, gate_out, n_tok, dm, hk);
    } else {
      if (full)
        hipLaunchKernelGGL((gate_kernel<bf16_t, true>), grid, dim3(256), 0, st, (const bf16_t *)x, wg, gate_out, n_tok, dm, hk);
      else
        hipLaunchKernelGGL((gate_kernel<bf16_t, false>), grid, dim3(256), 0, st, (const bf16_t *)x, wg, gate_out, n_tok, dm, hk);
    }
    if (hipGetLastError() != hipSuccess) return KVM_ERR_HIP;
  }
  return KVM_OK;
}
