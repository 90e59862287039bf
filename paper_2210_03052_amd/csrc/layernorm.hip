// Fused add-bias + residual + LayerNorm (Sec. III-C1): one trip over memory.
// One wavefront owns one token row; the row lives in registers between the
// single 128-bit load and the single 128-bit store.  Mean and variance are fp32,
// two-pass over the registers (no E[x^2]-E[x]^2 cancellation).
#include "common.h"

namespace bt {

// CPL = 16-byte chunks per lane; a row has H/8 chunks, chunk c = lane + 64*i.
// PART: the GEMM output arrives as nsplit fp32 slices xpart[s][T][H] of a split-K product, added here in
// slice order (the reduction of the split costs no kernel of its own); otherwise x is fp16 [T,H].
// STREAM: the tensors exceed the memory-side cache, so rows are loaded and stored with the non-temporal
// hint (measured +9 % on a 1.2 GB pass); at cache-resident sizes the next kernel wants the rows cached.
template <int CPL, bool PART, bool STREAM>
__global__ __launch_bounds__(256) void bias_residual_ln_kernel(
    // what the loads at the top need first: it fits the 14 dwords preloaded into SGPRs at wave launch
    const half_t* x, const half_t* residual, const half_t* __restrict__ bias, int T, int H, int nsplit, float eps,
    const float* __restrict__ xpart, const int32_t* __restrict__ res_rows, const half_t* __restrict__ gamma,
    const half_t* __restrict__ beta, half_t* y, const int32_t* __restrict__ out_idx, int out_rows) {
  // res_rows: the residual of packed row i is row res_rows[i] of `residual` (pack fused into the read).
  // out_idx: y is the padded tensor [out_rows, H]; this wave owns padded row r, which is packed row
  //   `lo` if out_idx[lo] == r (out_idx is increasing: uniform binary search) and a zero row otherwise
  //   (unpack fused into the store, Sec. III-D).
  const int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int chunks = H >> 3;
  size_t obase;
  if (out_idx) {
    const int r = row;
    if (r >= out_rows) return;
    int lo = 0, hi = T;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (out_idx[mid] < r) lo = mid + 1; else hi = mid;
    }
    obase = (size_t)r * H;
    if (!(lo < T && out_idx[lo] == r)) {
      const half8_t z = {(half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f};
      for (int c = lane; c < chunks; c += kWave) *reinterpret_cast<half8_t*>(y + obase + c * 8) = z;
      return;
    }
    row = lo;
  } else {
    if (row >= T) return;
    obase = (size_t)row * H;
  }
  const size_t base = (size_t)row * H;
  const size_t rbase = res_rows ? (size_t)res_rows[row] * H : base;

  float v[CPL][8];
  half8_t gm[CPL], bt[CPL];  // gamma and beta are requested with the row, not after the two reductions
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int c = lane + i * kWave;
    if (c < chunks) {
      gm[i] = *reinterpret_cast<const half8_t*>(gamma + c * 8);
      bt[i] = *reinterpret_cast<const half8_t*>(beta + c * 8);
      const half8_t r = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(residual + rbase + c * 8))
                               : *reinterpret_cast<const half8_t*>(residual + rbase + c * 8);
      if constexpr (PART) {
        float acc8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int sl = 0; sl < nsplit; ++sl) {
          const float* src = xpart + (size_t)sl * T * H + base + c * 8;
          const float4_t lo = *reinterpret_cast<const float4_t*>(src), hi = *reinterpret_cast<const float4_t*>(src + 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) { acc8[e] += lo[e]; acc8[4 + e] += hi[e]; }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[i][e] = acc8[e] + (float)r[e];
      } else {
        const half8_t a = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(x + base + c * 8))
                                 : *reinterpret_cast<const half8_t*>(x + base + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[i][e] = (float)a[e] + (float)r[e];
      }
      if (bias) {
        const half8_t b = *reinterpret_cast<const half8_t*>(bias + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[i][e] += (float)b[e];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += v[i][e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[i][e] = 0.f;
    }
  }
  const float inv_h = 1.0f / (float)H;
  const float mean = wave_sum(sum) * inv_h;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    if (lane + i * kWave < chunks) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = v[i][e] - mean;
        sq += d * d;
      }
    }
  }
  const float rstd = rsqrtf(wave_sum(sq) * inv_h + eps);
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int c = lane + i * kWave;
    if (c < chunks) {
      half8_t o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (half_t)((v[i][e] - mean) * rstd * (float)gm[i][e] + (float)bt[i][e]);
      if (STREAM) __builtin_nontemporal_store(o, reinterpret_cast<half8_t*>(y + obase + c * 8));
      else store_through(y + obase + c * 8, __builtin_bit_cast(uint4_t, o));  // see store_through
    }
  }
}

// Normalisation of a row whose scaled values u = gamma (.) z and partial sums (sum z, sum z^2) were
// produced by a GEMM epilogue (EPI_RESID): y = rstd (u - mu gamma) + beta.  Used once, at the end of a
// stack whose inner LayerNorms are folded into the GEMMs that follow them.  The partial sums are added
// in the order the GEMMs add them (two halves in index order, then the two halves), so the statistics
// are the ones the folded GEMMs used.
__global__ __launch_bounds__(256) void ln_finalize_kernel(const half_t* __restrict__ u, const float2* __restrict__ part,
                                                          int np, const half_t* __restrict__ gamma,
                                                          const half_t* __restrict__ beta, float eps, int T, int H,
                                                          half_t* __restrict__ y, const int32_t* __restrict__ out_idx,
                                                          int out_rows) {
  // out_idx: y is the padded tensor [out_rows, H]; this wave owns padded row r, which is packed row `lo` if
  // out_idx[lo] == r and a zero row otherwise (unpack fused into the store, as in bias_residual_ln_kernel).
  const int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  size_t obase;
  if (out_idx) {
    const int r = row;
    if (r >= out_rows) return;
    int lo = 0, hi = T;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (out_idx[mid] < r) lo = mid + 1; else hi = mid;
    }
    obase = (size_t)r * H;
    if (!(lo < T && out_idx[lo] == r)) {
      const half8_t z = {(half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f};
      for (int c = lane; c < (H >> 3); c += kWave) *reinterpret_cast<half8_t*>(y + obase + c * 8) = z;
      return;
    }
    row = lo;
  } else {
    if (row >= T) return;
    obase = (size_t)row * H;
  }
  const float inv_h = 1.0f / (float)H;
  const int half_np = (np + 1) >> 1;
  float a0 = 0.f, b0 = 0.f, a1 = 0.f, b1 = 0.f;
  for (int q0 = 0; q0 < np; q0 += kWave) {  // lane q holds partial q0+q; added in index order via shuffles
    const float2 v = q0 + lane < np ? part[(size_t)row * np + q0 + lane] : make_float2(0.f, 0.f);
    const int n_here = min(np - q0, kWave);
    for (int q = 0; q < n_here; ++q) {
      const float x = __shfl(v.x, q, kWave), z = __shfl(v.y, q, kWave);
      if (q0 + q < half_np) { a0 += x; b0 += z; } else { a1 += x; b1 += z; }
    }
  }
  const float mu = (a0 + a1) * inv_h;
  const float rstd = rsqrtf(fmaxf((b0 + b1) * inv_h - mu * mu, 0.f) + eps);
  const size_t base = (size_t)row * H;
  for (int c = lane; c < (H >> 3); c += kWave) {
    const half8_t a = *reinterpret_cast<const half8_t*>(u + base + c * 8);
    const half8_t g = *reinterpret_cast<const half8_t*>(gamma + c * 8);
    const half8_t b = *reinterpret_cast<const half8_t*>(beta + c * 8);
    half8_t o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (half_t)(rstd * ((float)a[e] - mu * (float)g[e]) + (float)b[e]);
    *reinterpret_cast<half8_t*>(y + obase + c * 8) = o;
  }
}

// c[n] = sum_k W[n][k] gamma[k],  d[n] = sum_k W[n][k] beta[k] + bias[n]: the two vectors that move a
// LayerNorm (gamma, beta) into the epilogue of the GEMM with weight W.  One wavefront per output n.
__global__ __launch_bounds__(256) void fold_vectors_kernel(const half_t* __restrict__ W,
                                                           const half_t* __restrict__ gamma,
                                                           const half_t* __restrict__ beta,
                                                           const half_t* __restrict__ bias, int N, int K,
                                                           float* __restrict__ c, float* __restrict__ d) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  float sc = 0.f, sd = 0.f;
  for (int k = lane * 8; k < K; k += kWave * 8) {
    const half8_t w = *reinterpret_cast<const half8_t*>(W + (size_t)n * K + k);
    const half8_t g = *reinterpret_cast<const half8_t*>(gamma + k);
    const half8_t b = *reinterpret_cast<const half8_t*>(beta + k);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sc = __builtin_fmaf((float)w[e], (float)g[e], sc);
      sd = __builtin_fmaf((float)w[e], (float)b[e], sd);
    }
  }
  sc = wave_sum(sc);
  sd = wave_sum(sd);
  if (lane == 0) {
    c[n] = sc;
    d[n] = sd + (bias ? (float)bias[n] : 0.f);
  }
}

bt_status ln_finalize_dispatch(const bt_half* u, const float2* part, int np, const bt_half* gamma,
                               const bt_half* beta, float eps, int T, int H, bt_half* y, hipStream_t st,
                               const int32_t* out_idx, int out_rows) {
  ln_finalize_kernel<<<((out_idx ? out_rows : T) + 3) / 4, 256, 0, st>>>(
      reinterpret_cast<const half_t*>(u), part, np, reinterpret_cast<const half_t*>(gamma),
      reinterpret_cast<const half_t*>(beta), eps, T, H, reinterpret_cast<half_t*>(y), out_idx, out_rows);
  return launch_status();
}

bt_status fold_vectors_dispatch(const bt_half* W, const bt_half* gamma, const bt_half* beta, const bt_half* bias,
                                int N, int K, float* c, float* d, hipStream_t st) {
  fold_vectors_kernel<<<(N + 3) / 4, 256, 0, st>>>(reinterpret_cast<const half_t*>(W),
                                                   reinterpret_cast<const half_t*>(gamma),
                                                   reinterpret_cast<const half_t*>(beta),
                                                   reinterpret_cast<const half_t*>(bias), N, K, c, d);
  return launch_status();
}

bt_status layernorm_dispatch(const bt_half* x, const float* xpart, int nsplit, const bt_half* bias,
                             const bt_half* residual, const bt_half* gamma, const bt_half* beta, float eps, int T,
                             int H, bt_half* y, hipStream_t st, const int32_t* res_rows, const int32_t* out_idx,
                             int out_rows) {
  const half_t* px = reinterpret_cast<const half_t*>(x);
  const half_t* pb = reinterpret_cast<const half_t*>(bias);
  const half_t* pr = reinterpret_cast<const half_t*>(residual);
  const half_t* pg = reinterpret_cast<const half_t*>(gamma);
  const half_t* pe = reinterpret_cast<const half_t*>(beta);
  half_t* py = reinterpret_cast<half_t*>(y);
  const int chunks = H / 8;
  dim3 grid(((out_idx ? out_rows : T) + 3) / 4), block(256);
  const bool stream = (size_t)T * H * 6 > ((size_t)256 << 20);  // three tensors larger than the 256 MB Infinity Cache
#define BT_LN(CPL)                                                                                             \
  do {                                                                                                         \
    if (xpart) bias_residual_ln_kernel<CPL, true, false><<<grid, block, 0, st>>>(px, pr, pb, T, H, nsplit, eps, xpart, res_rows, pg, pe, py, out_idx, out_rows); \
    else if (stream) bias_residual_ln_kernel<CPL, false, true><<<grid, block, 0, st>>>(px, pr, pb, T, H, nsplit, eps, xpart, res_rows, pg, pe, py, out_idx, out_rows); \
    else bias_residual_ln_kernel<CPL, false, false><<<grid, block, 0, st>>>(px, pr, pb, T, H, nsplit, eps, xpart, res_rows, pg, pe, py, out_idx, out_rows); \
  } while (0)
  if (chunks <= 64) BT_LN(1);
  else if (chunks <= 128) BT_LN(2);
  else if (chunks <= 256) BT_LN(4);
  else if (chunks <= 512) BT_LN(8);
  else BT_LN(16);
#undef BT_LN
  return launch_status();
}

}  // namespace bt

extern "C" bt_status bt_add_bias_residual_layernorm(const bt_half* d_x, const bt_half* d_bias,
                                                    const bt_half* d_residual, const bt_half* d_gamma,
                                                    const bt_half* d_beta, float eps, int T, int H, bt_half* d_y,
                                                    bt_stream stream) {
  if (T < 0 || H < 8 || (H % 8) != 0 || !(eps >= 0.f)) return BT_ERR_INVALID_ARG;
  if (H > 8192) return BT_ERR_UNSUPPORTED;
  if (T == 0) return BT_OK;
  if (!d_x || !d_residual || !d_gamma || !d_beta || !d_y) return BT_ERR_INVALID_ARG;
  if (!bt::aligned16(d_x) || !bt::aligned16(d_residual) || !bt::aligned16(d_gamma) || !bt::aligned16(d_beta) ||
      !bt::aligned16(d_y) || (d_bias && !bt::aligned16(d_bias)))
    return BT_ERR_INVALID_ARG;
  return bt::layernorm_dispatch(d_x, nullptr, 0, d_bias, d_residual, d_gamma, d_beta, eps, T, H, d_y,
                                static_cast<hipStream_t>(stream), nullptr, nullptr, 0);
}

extern "C" bt_status bt_add_bias_residual_layernorm_kslices(const float* d_slices, int n_slices, const bt_half* d_bias,
                                                            const bt_half* d_residual, const bt_half* d_gamma,
                                                            const bt_half* d_beta, float eps, int T, int H,
                                                            bt_half* d_y, bt_stream stream) {
  if (T < 0 || H < 8 || (H % 8) != 0 || !(eps >= 0.f) || n_slices < 1 || n_slices > 8) return BT_ERR_INVALID_ARG;
  if (H > 8192) return BT_ERR_UNSUPPORTED;
  if (T == 0) return BT_OK;
  if (!d_slices || !d_residual || !d_gamma || !d_beta || !d_y) return BT_ERR_INVALID_ARG;
  if (!bt::aligned16(d_slices) || !bt::aligned16(d_residual) || !bt::aligned16(d_gamma) || !bt::aligned16(d_beta) ||
      !bt::aligned16(d_y) || (d_bias && !bt::aligned16(d_bias)))
    return BT_ERR_INVALID_ARG;
  return bt::layernorm_dispatch(nullptr, d_slices, n_slices, d_bias, d_residual, d_gamma, d_beta, eps, T, H, d_y,
                                static_cast<hipStream_t>(stream), nullptr, nullptr, 0);
}
