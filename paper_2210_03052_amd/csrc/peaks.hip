// Measurement kernels for `bench.py --peaks`: what this very GPU sustains on the two resources the
// rooflines are priced against, so that a report can carry the measured denominators next to the
// published ones.  Built into libbt_peaks.so, a library of its own: nothing on the encoder path uses it.
//   bt_peak_mfma_f16     a loop of independent 32x32x16 fp16 MFMAs on register operands (no memory traffic)
//   bt_peak_stream_read  a read-only stream over a buffer much larger than the caches
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

// Each wavefront keeps 4 independent accumulators busy; operands are either constants (pattern 0: the
// clock stays high) or pseudo-random fp16 values in [-1, 1) (pattern 1: the switching activity of real
// data, under which the clock settles lower).  The accumulators are written out so nothing is elided.
__global__ __launch_bounds__(256) void peak_mfma_kernel(int iters, int pattern, float* __restrict__ sink) {
  const uint32_t t = blockIdx.x * 256u + threadIdx.x;
  half8_t a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t h = (t * 2654435761u) ^ ((uint32_t)(i * 8 + e) * 40503u);
      h ^= h >> 13; h *= 2246822519u; h ^= h >> 16;
      const float r = (float)(int)(h & 0xffffu) * (1.0f / 32768.0f) - 1.0f;
      a[i][e] = (_Float16)(pattern ? r : 0.5f);
      b[i][e] = (_Float16)(pattern ? -r * 0.5f : 0.25f);
    }
  float16_t acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[i], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[t] = s;
}

// 16 bytes per lane per step, grid-stride, every loaded word folded into one value per thread.
__global__ __launch_bounds__(256) void peak_read_kernel(const uint4_t* __restrict__ src, size_t n_vec,
                                                        uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint32_t x = 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride) {
    const uint4_t v = __builtin_nontemporal_load(src + i);
    x ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = x;
}

// Both return 0 on success, 1 on a bad argument, 4 on a HIP error (the status codes of bt.h).
// d_sink: blocks * 256 floats.  FLOPs of one launch: blocks * 4 waves * iters * 4 * 2*32*32*16.
extern "C" int bt_peak_mfma_f16(int iters, int blocks, int pattern, float* d_sink, void* stream) {
  if (iters < 1 || blocks < 1 || !d_sink || (pattern != 0 && pattern != 1)) return 1;
  peak_mfma_kernel<<<(unsigned)blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(iters, pattern, d_sink);
  return hipGetLastError() == hipSuccess ? 0 : 4;
}

// d_src: bytes (a multiple of 16, 16-byte aligned); d_sink: blocks * 256 words.
extern "C" int bt_peak_stream_read(const void* d_src, size_t bytes, int blocks, uint32_t* d_sink, void* stream) {
  if (!d_src || !d_sink || blocks < 1 || bytes < 16 || (bytes & 15u) || (reinterpret_cast<uintptr_t>(d_src) & 15u))
    return 1;
  peak_read_kernel<<<(unsigned)blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const uint4_t*>(d_src), bytes / 16, d_sink);
  return hipGetLastError() == hipSuccess ? 0 : 4;
}
