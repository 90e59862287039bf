// Unfused element-wise kernels: the baselines of the kernel-fusion ablations (Sec. IV-A: add-bias + residual
// and LayerNorm as two trips over memory; Sec. IV-B: add-bias + GELU as a kernel of its own behind the GEMM).
// For `bench.py --sweep` only -- built into libbt_peaks.so, never used by the encoder path, whose kernels
// fuse these steps.  Plain, coalesced, 16 bytes per lane; fp32 arithmetic, fp16 in and out.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half_t;
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

// y = x + bias (+ residual): one 16-byte chunk per thread, a row of H halves is H/8 consecutive threads.
__global__ __launch_bounds__(256) void unfused_add_bias_residual_kernel(const half8_t* __restrict__ x,
                                                                        const half8_t* __restrict__ bias,
                                                                        const half8_t* __restrict__ residual,
                                                                        size_t total, int chunks, half8_t* __restrict__ y) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const half8_t a = x[i], b = bias[i % chunks];
  half8_t o;
  if (residual) {
    const half8_t r = residual[i];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (half_t)((float)a[e] + (float)b[e] + (float)r[e]);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (half_t)((float)a[e] + (float)b[e]);
  }
  y[i] = o;
}

// y = GELU(x + bias), exact (erf) form.
__global__ __launch_bounds__(256) void unfused_bias_gelu_kernel(const half8_t* __restrict__ x,
                                                                const half8_t* __restrict__ bias, size_t total,
                                                                int chunks, half8_t* __restrict__ y) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const half8_t a = x[i], b = bias[i % chunks];
  half8_t o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float v = (float)a[e] + (float)b[e];
    o[e] = (half_t)(0.5f * v * (1.0f + erff(v * 0.70710678118654752f)));
  }
  y[i] = o;
}

// Plain LayerNorm of rows of H <= 8192 halves: one wavefront per row, two passes over registers.
__global__ __launch_bounds__(256) void unfused_layernorm_kernel(const half_t* __restrict__ x,
                                                                const half_t* __restrict__ gamma,
                                                                const half_t* __restrict__ beta, float eps, int T, int H,
                                                                half_t* __restrict__ y) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  const int chunks = H >> 3;
  const size_t base = (size_t)row * H;
  float v[16][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = lane + i * 64;
    if (c < chunks) {
      const half8_t a = *reinterpret_cast<const half8_t*>(x + base + c * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) { v[i][e] = (float)a[e]; sum += v[i][e]; }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
  const float mean = sum / (float)H;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
    if (lane + i * 64 < chunks) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; sq += d * d; }
    }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
  const float rstd = rsqrtf(sq / (float)H + eps);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = lane + i * 64;
    if (c < chunks) {
      const half8_t g = *reinterpret_cast<const half8_t*>(gamma + c * 8), b = *reinterpret_cast<const half8_t*>(beta + c * 8);
      half8_t o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (half_t)((v[i][e] - mean) * rstd * (float)g[e] + (float)b[e]);
      *reinterpret_cast<half8_t*>(y + base + c * 8) = o;
    }
  }
}

static inline bool ok16(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// All return 0 on success, 1 on a bad argument, 4 on a HIP error (the status codes of bt.h).  T rows of H
// halves, H % 8 == 0; device pointers, 16-byte aligned; d_residual may be NULL (bias only).
extern "C" int bt_unfused_add_bias_residual(const void* d_x, const void* d_bias, const void* d_residual, int T, int H,
                                            void* d_y, void* stream) {
  if (T < 1 || H < 8 || (H % 8) || !ok16(d_x) || !ok16(d_bias) || !ok16(d_y) || (d_residual && !ok16(d_residual))) return 1;
  const size_t total = (size_t)T * (H / 8);
  unfused_add_bias_residual_kernel<<<(unsigned)((total + 255) / 256), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const half8_t*>(d_x), static_cast<const half8_t*>(d_bias), static_cast<const half8_t*>(d_residual),
      total, H / 8, static_cast<half8_t*>(d_y));
  return hipGetLastError() == hipSuccess ? 0 : 4;
}

extern "C" int bt_unfused_bias_gelu(const void* d_x, const void* d_bias, int T, int H, void* d_y, void* stream) {
  if (T < 1 || H < 8 || (H % 8) || !ok16(d_x) || !ok16(d_bias) || !ok16(d_y)) return 1;
  const size_t total = (size_t)T * (H / 8);
  unfused_bias_gelu_kernel<<<(unsigned)((total + 255) / 256), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const half8_t*>(d_x), static_cast<const half8_t*>(d_bias), total, H / 8, static_cast<half8_t*>(d_y));
  return hipGetLastError() == hipSuccess ? 0 : 4;
}

extern "C" int bt_unfused_layernorm(const void* d_x, const void* d_gamma, const void* d_beta, float eps, int T, int H,
                                    void* d_y, void* stream) {
  if (T < 1 || H < 8 || (H % 8) || H > 8192 || !ok16(d_x) || !ok16(d_gamma) || !ok16(d_beta) || !ok16(d_y)) return 1;
  unfused_layernorm_kernel<<<(unsigned)((T + 3) / 4), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const half_t*>(d_x), static_cast<const half_t*>(d_gamma), static_cast<const half_t*>(d_beta), eps, T, H,
      static_cast<half_t*>(d_y));
  return hipGetLastError() == hipSuccess ? 0 : 4;
}
