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
    // Everything the kernel touches before its first batch of row loads is in flight comes first and fills exactly
    // the 14 dwords that are preloaded into SGPRs at wave launch: the output index (decides the first branch), the
    // four tensors of that batch, the residual's row index and the two sizes.  The rest arrives by scalar loads
    // whose latency then hides behind the row loads (with gamma, beta and the output index behind such loads the
    // kernel began with two exposed round trips to the kernel-argument buffer).
    // xin: x (fp16 [T,H]), or with PART the fp32 K slices [nsplit][T][H] of x.
    const void* __restrict__ xin, const half_t* residual, const half_t* __restrict__ gamma,
    const half_t* __restrict__ beta, const int32_t* __restrict__ out_idx, const int32_t* __restrict__ res_rows, int T,
    int H, const half_t* __restrict__ bias, half_t* y, int nsplit, float eps, int out_rows) {
  const half_t* x = static_cast<const half_t*>(xin);
  const float* xpart = static_cast<const float*>(xin);
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

  // Every load of the row is issued before the first value is used, as straight-line code: chunk indices past the
  // row are clamped (the lane's copy is ignored later) and a missing bias reads gamma with weight 0, so no branch
  // splits the loads into batches that would each wait for the previous one -- the kernel is one memory round trip,
  // not one per chunk and per operand.
  float v[CPL][8];
  half8_t gm[CPL], bt[CPL], rs[CPL], bs[CPL];  // gamma and beta are requested with the row, not after the reductions
  int cc[CPL];
#pragma unroll
  for (int i = 0; i < CPL; ++i) cc[i] = min(lane + i * kWave, chunks - 1) * 8;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    rs[i] = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(residual + rbase + cc[i]))
                   : *reinterpret_cast<const half8_t*>(residual + rbase + cc[i]);
    gm[i] = *reinterpret_cast<const half8_t*>(gamma + cc[i]);
    bt[i] = *reinterpret_cast<const half8_t*>(beta + cc[i]);
  }
  half8_t xs[PART ? 1 : CPL];
  if constexpr (!PART) {
#pragma unroll
    for (int i = 0; i < CPL; ++i)
      xs[i] = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(x + base + cc[i]))
                     : *reinterpret_cast<const half8_t*>(x + base + cc[i]);
  }
  // the bias pointer is not among the preloaded kernel arguments: its loads go last, so that the scalar load of the
  // pointer completes behind the row loads already in flight
  __builtin_amdgcn_sched_barrier(0);
  const half_t* const bsrc = bias ? bias : gamma;
  const float bw = bias ? 1.f : 0.f;
#pragma unroll
  for (int i = 0; i < CPL; ++i) bs[i] = *reinterpret_cast<const half8_t*>(bsrc + cc[i]);
  if constexpr (PART) {
    // K slices of the product, four at a time where the registers allow (slice indices past nsplit are clamped
    // and their values dropped): at the usual widths the up to eight slices cost two round trips, not one each
    constexpr int G = CPL <= 2 ? 4 : (CPL <= 4 ? 2 : 1);
#pragma unroll
    for (int i = 0; i < CPL; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) v[i][e] = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += G) {
      float4_t lo[G][CPL], hi[G][CPL];
#pragma unroll
      for (int k = 0; k < G; ++k)
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
          const float* src = xpart + (size_t)min(s0 + k, nsplit - 1) * T * H + base + cc[i];
          lo[k][i] = *reinterpret_cast<const float4_t*>(src);
          hi[k][i] = *reinterpret_cast<const float4_t*>(src + 4);
        }
#pragma unroll
      for (int k = 0; k < G; ++k) {  // in slice order
        const bool live = s0 + k < nsplit;
#pragma unroll
        for (int i = 0; i < CPL; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[i][e] += live ? lo[k][i][e] : 0.f;
            v[i][4 + e] += live ? hi[k][i][e] : 0.f;
          }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < CPL; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) v[i][e] = (float)xs[i][e];
  }
  // pinned here (after every load of the row has been issued): left alone, the compiler moves the gamma / beta loads down to the stores, a round trip of their own
#pragma unroll
  for (int i = 0; i < CPL; ++i) asm volatile("" : "+v"(gm[i]), "+v"(bt[i]), "+v"(bs[i]));
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const bool mine = lane + i * kWave < chunks;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float t = (v[i][e] + (float)rs[i][e]) + bw * (float)bs[i][e];
      v[i][e] = mine ? t : 0.f;
      sum += v[i][e];
    }
  }
  const float inv_h = 1.0f / (float)H;
  const float mean = wave_sum(sum) * inv_h;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const bool mine = lane + i * kWave < chunks;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float d = mine ? v[i][e] - mean : 0.f;
      sq += d * d;
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
    if (xpart) bias_residual_ln_kernel<CPL, true, false><<<grid, block, 0, st>>>(xpart, pr, pg, pe, out_idx, res_rows, T, H, pb, py, nsplit, eps, out_rows); \
    else if (stream) bias_residual_ln_kernel<CPL, false, true><<<grid, block, 0, st>>>(px, pr, pg, pe, out_idx, res_rows, T, H, pb, py, nsplit, eps, out_rows); \
    else bias_residual_ln_kernel<CPL, false, false><<<grid, block, 0, st>>>(px, pr, pg, pe, out_idx, res_rows, T, H, pb, py, nsplit, eps, out_rows); \
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
