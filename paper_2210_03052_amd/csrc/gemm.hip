// Packed-token GEMM with fused epilogue (Sec. III-C2):  C = act(A W^T + bias).
// A [M,K] and W [N,K] are both K-contiguous, which is exactly the operand order
// the gfx950 MFMA wants: every lane feeds 8 consecutive K values of one row.
//
// Tiling: 256 threads = 4 wavefronts in a 2x2 grid; block tile BM x BN x 64,
// wave tile (BM/2) x (BN/2) made of 32x32x16 fp16 MFMA blocks with fp32
// accumulators.  Operand tiles are staged in LDS (double-buffered, rows padded
// by 16 bytes so that 128-bit reads of 16 consecutive rows hit 64 distinct
// banks); the next K-slab is fetched from global memory into registers while the
// current one is multiplied.  The product is computed transposed (W is the MFMA
// A operand), so each lane ends up with 4 consecutive output columns of one row
// and stores them with one 8-byte write after bias/activation in fp32.
#include "common.h"

namespace bt {

constexpr int kGemmThreads = 256;
constexpr int kBK = 64;            // K-slab per stage (halves)
constexpr int kLdsStride = kBK + 8;  // halves; 144-byte rows

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_tanh(float x) {
  const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  return 0.5f * x * (1.0f + tanhf(u));
}

template <int BM, int BN, int ACT>
__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(const half_t* __restrict__ A,
                                                            const half_t* __restrict__ W,
                                                            const half_t* __restrict__ bias, half_t* __restrict__ C,
                                                            int M, int N, int K, int tiles_n, int n_tiles) {
  constexpr int WM = BM / 2, WN = BN / 2;      // wave tile
  constexpr int MI = WM / 32, NI = WN / 32;    // 32x32 blocks per wave
  constexpr int A_CH = BM * (kBK / 8) / kGemmThreads;  // 16-byte chunks per thread
  constexpr int B_CH = BN * (kBK / 8) / kGemmThreads;
  static_assert(A_CH >= 1 && B_CH >= 1, "tile too small for 256 threads");

  __shared__ __attribute__((aligned(16))) half_t sA[2][BM * kLdsStride];
  __shared__ __attribute__((aligned(16))) half_t sB[2][BN * kLdsStride];

  const int tile = xcd_remap(blockIdx.x, n_tiles);
  const int tm = tile / tiles_n, tn = tile - tm * tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, hf = lane >> 5;

  // global -> register staging: chunk c = tid + 256*i covers row c/8, halves (c%8)*8..+7
  const half_t* a_ptr[A_CH];
  const half_t* b_ptr[B_CH];
  int a_lds[A_CH], b_lds[B_CH];
  const int kc = (tid & 7) * 8;
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int row = (tid >> 3) + i * (kGemmThreads / 8);
    const int gr = min(m0 + row, M - 1);  // rows past M are read clamped, never stored
    a_ptr[i] = A + (size_t)gr * K + kc;
    a_lds[i] = row * kLdsStride + kc;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int row = (tid >> 3) + i * (kGemmThreads / 8);
    const int gr = min(n0 + row, N - 1);
    b_ptr[i] = W + (size_t)gr * K + kc;
    b_lds[i] = row * kLdsStride + kc;
  }

  uint4_t ra[A_CH], rb[B_CH];
  const uint4_t zero4 = {0u, 0u, 0u, 0u};
  auto fetch = [&](int k0) {
    const bool in = (k0 + kc) < K;  // K % 8 == 0: a chunk is entirely inside or outside
#pragma unroll
    for (int i = 0; i < A_CH; ++i) ra[i] = in ? *reinterpret_cast<const uint4_t*>(a_ptr[i] + k0) : zero4;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[i] = in ? *reinterpret_cast<const uint4_t*>(b_ptr[i] + k0) : zero4;
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<uint4_t*>(&sA[buf][a_lds[i]]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<uint4_t*>(&sB[buf][b_lds[i]]) = rb[i];
  };

  float16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (K + kBK - 1) / kBK;
  fetch(0);
  stage(0);
  __syncthreads();

  const int a_rd = (wm * WM + l32) * kLdsStride + hf * 8;
  const int b_rd = (wn * WN + l32) * kLdsStride + hf * 8;

  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) fetch((kt + 1) * kBK);
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      half8_t fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        fa[i] = *reinterpret_cast<const half8_t*>(&sA[buf][a_rd + i * 32 * kLdsStride + ks * 16]);
#pragma unroll
      for (int j = 0; j < NI; ++j)
        fb[j] = *reinterpret_cast<const half8_t*>(&sB[buf][b_rd + j * 32 * kLdsStride + ks * 16]);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          // transposed product: D[n][m] += W[n][k] * A[m][k]
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) stage(buf ^ 1);
    __syncthreads();
  }

  // Epilogue.  acc[i][j][4g+t] = C[m][n] with m = m0 + wm*WM + i*32 + l32,
  // n = n0 + wn*WN + j*32 + 8g + 4hf + t.
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int m = m0 + wm * WM + i * 32 + l32;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * WN + j * 32 + 8 * g + 4 * hf;
        if (n >= N) continue;  // N % 8 == 0: the 4 columns are all in or all out
        float v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = acc[i][j][4 * g + t];
        if (bias) {
          const half4_t bv = *reinterpret_cast<const half4_t*>(bias + n);
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] += (float)bv[t];
        }
        if (ACT == BT_ACT_GELU_ERF) {
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = gelu_erf(v[t]);
        } else if (ACT == BT_ACT_GELU_TANH) {
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = gelu_tanh(v[t]);
        }
        half4_t o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = (half_t)v[t];
        *reinterpret_cast<half4_t*>(C + (size_t)m * N + n) = o;
      }
    }
  }
}

template <int BM, int BN>
static bt_status launch_gemm(const half_t* A, const half_t* W, const half_t* bias, half_t* C, int M, int N, int K,
                             bt_act act, hipStream_t st) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const long long n_tiles = (long long)tiles_m * tiles_n;
  if (n_tiles > 0x7fffffffLL) return BT_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_tiles), block(kGemmThreads);
  switch (act) {
    case BT_ACT_NONE:
      gemm_kernel<BM, BN, BT_ACT_NONE><<<grid, block, 0, st>>>(A, W, bias, C, M, N, K, tiles_n, (int)n_tiles);
      break;
    case BT_ACT_GELU_ERF:
      gemm_kernel<BM, BN, BT_ACT_GELU_ERF><<<grid, block, 0, st>>>(A, W, bias, C, M, N, K, tiles_n, (int)n_tiles);
      break;
    case BT_ACT_GELU_TANH:
      gemm_kernel<BM, BN, BT_ACT_GELU_TANH><<<grid, block, 0, st>>>(A, W, bias, C, M, N, K, tiles_n, (int)n_tiles);
      break;
    default:
      return BT_ERR_INVALID_ARG;
  }
  return launch_status();
}

// Tile choice: the packed token count is small next to 256 compute units, so
// prefer the largest tile that still yields at least ~2 workgroups per CU.
bt_status gemm_dispatch(const bt_half* A, const bt_half* W, const bt_half* bias, int M, int N, int K, bt_act act,
                        bt_half* C, hipStream_t st) {
  const half_t* a = reinterpret_cast<const half_t*>(A);
  const half_t* w = reinterpret_cast<const half_t*>(W);
  const half_t* b = reinterpret_cast<const half_t*>(bias);
  half_t* c = reinterpret_cast<half_t*>(C);
  auto tiles = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
  constexpr long long kTarget = 512;
  if (tiles(128, 128) >= kTarget) return launch_gemm<128, 128>(a, w, b, c, M, N, K, act, st);
  if (tiles(128, 64) >= kTarget) return launch_gemm<128, 64>(a, w, b, c, M, N, K, act, st);
  return launch_gemm<64, 64>(a, w, b, c, M, N, K, act, st);
}

}  // namespace bt

extern "C" bt_status bt_gemm_bias_act(const bt_half* d_A, const bt_half* d_W, const bt_half* d_bias, int M, int N,
                                      int K, bt_act act, bt_half* d_C, bt_stream stream) {
  if (M < 0 || N < 8 || K < 8 || (N % 8) != 0 || (K % 8) != 0) return BT_ERR_INVALID_ARG;
  if (act != BT_ACT_NONE && act != BT_ACT_GELU_ERF && act != BT_ACT_GELU_TANH) return BT_ERR_INVALID_ARG;
  if (M == 0) return BT_OK;
  if (!d_A || !d_W || !d_C || !bt::aligned16(d_A) || !bt::aligned16(d_W) || !bt::aligned16(d_C))
    return BT_ERR_INVALID_ARG;
  if (d_bias && (reinterpret_cast<uintptr_t>(d_bias) & 7u)) return BT_ERR_INVALID_ARG;
  return bt::gemm_dispatch(d_A, d_W, d_bias, M, N, K, act, d_C, static_cast<hipStream_t>(stream));
}
