// Internal helpers shared by the HIP translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bt.h"

namespace bt {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline bt_status launch_status() {
  return hipGetLastError() == hipSuccess ? BT_OK : BT_ERR_HIP;
}

// Blocks are dealt round-robin to the 8 XCDs (block i runs on XCD i % 8), each
// with a private L2.  Remap a linear block id so that every XCD works on one
// contiguous range of the logical tile order and neighbouring tiles share L2.
__device__ __forceinline__ int xcd_remap(int id, int n) {
  constexpr int kXcd = 8;
  const int x = id % kXcd, local = id / kXcd;
  const int base = n / kXcd, rem = n % kXcd;
  return x * base + (x < rem ? x : rem) + local;
}

// Butterfly reductions over the 64 lanes of a wavefront.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

}  // namespace bt
