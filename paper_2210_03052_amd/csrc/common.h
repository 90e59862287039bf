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

// Epilogue forms of the packed GEMM (see store_tile in gemm.hip) and their operands.
// Row statistics of a LayerNorm travel as partial sums: part[m][p] = (sum z, sum z^2) of row m over the
// columns of column tile p of the producing GEMM, p < np.  They are written once each and added up
// in a fixed order by whoever needs the mean and variance: no atomics, bit-reproducible.
enum { EPI_PLAIN = 0, EPI_FOLD = 1, EPI_RESID = 2, EPI_PARTIAL = 3 };
struct GemmEpi {
  const int32_t* a_rows = nullptr;  // any form: row m of the product reads row a_rows[m] of A (pack fused into the load)
  const half_t* bias = nullptr;     // PLAIN / RESID: [N] or null
  // FOLD: the A operand is u = gamma (.) z of a LayerNorm whose row sums are ln_part
  const float2* ln_part = nullptr;  // [M][ln_np]
  int ln_np = 0;
  const float* fold_c = nullptr;    // [N]  W gamma
  const float* fold_d = nullptr;    // [N]  W beta + bias
  float inv_h = 0.f, eps = 0.f;     // 1/width and epsilon of that LayerNorm (also used by RESID)
  // RESID: v = acc + bias + residual; C = out_gamma (.) v; part_out[m][p] = (sum v, sum v^2) over column tile p
  const half_t* resid = nullptr;        // [M][N]: plain residual, or u_r if resid_part is set
  const int32_t* resid_rows = nullptr;  // plain residual only: row m of the residual is row resid_rows[m] of `resid`
                                        // (the padded input tensor: pack fused into the read)
  const float2* resid_part = nullptr;   // [M][resid_np] or null
  int resid_np = 0;
  const half_t* resid_gamma = nullptr;  // [N] (with resid_part): residual = rstd (u_r - mu gamma) + beta
  const half_t* resid_beta = nullptr;
  const half_t* out_gamma = nullptr;    // [N]
  float2* part_out = nullptr;           // [M][part_np]
  int part_np = 0;                      // set by the launcher: number of column tiles
  // PARTIAL (split-K): workgroup (tile, s) multiplies K range [s K/ksplit, (s+1) K/ksplit) and stores its
  // fp32 accumulators to partial[s][M][N]; whoever consumes the product adds the ksplit slices in order.
  float* partial = nullptr;
  int ksplit = 1;
};

// Stores with device scope: written through the XCD's L2 instead of staying dirty in it until the
// write-back that ends every kernel (during which no CU computes).  As assembly because the scope is
// not expressible on a plain store; the s_nop covers the hazard of a wide store whose data registers are
// overwritten by the next instruction.  16 and 8 bytes per lane.
__device__ __forceinline__ void store_through(half_t* gptr, const uint4_t& v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1"
               ::"v"((half_t __attribute__((address_space(1)))*)gptr), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(half_t* gptr, const uint2_t& v) {
  asm volatile("global_store_dwordx2 %0, %1, off sc1\n\ts_nop 0"
               ::"v"((half_t __attribute__((address_space(1)))*)gptr), "v"(v) : "memory");
}

__device__ __forceinline__ void store_through(float* gptr, const float4_t& v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1"
               ::"v"((float __attribute__((address_space(1)))*)gptr), "v"(v) : "memory");
}

// Cross-lane moves inside a row of 16 lanes through the data-parallel-primitive operand path (no LDS trip,
// unlike ds_bpermute, which is what __shfl compiles to).  CTRL: 0xB1 = lane ^ 1, 0x4E = lane ^ 2 (quad
// permutations), 0x141 = 7 - lane within 8 (half mirror), 0x140 = 15 - lane within 16 (mirror).
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) {
  return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, dpp_move<CTRL>(__builtin_bit_cast(int, v)));
}

// Sum / maximum over the 64 lanes of a wavefront, the same value in every lane: four steps inside each row
// of 16 lanes (after the two quad steps every lane of a quad holds the quad's value, so the mirrors combine
// whole quads), then the four row results are read as scalars and combined in a fixed order.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ int wave_max(int v) {
  v = max(v, dpp_move<0xB1>(v));
  v = max(v, dpp_move<0x4E>(v));
  v = max(v, dpp_move<0x141>(v));
  v = max(v, dpp_move<0x140>(v));
  return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
             max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

}  // namespace bt
