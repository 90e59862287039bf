// Packed-token GEMM with fused epilogue (Sec. III-C2):  C = act(A W^T + bias).
// A [M,K] and W [N,K] are both K-contiguous, which is exactly the operand order
// the gfx950 MFMA wants: every lane feeds 8 consecutive K values of one row.
//
// Main kernel (K % 64 == 0): WGM x WGN wavefronts, block tile BM x BN x 64, wave tile
// (BM/WGM) x (BN/WGN) of 32x32x16 fp16 MFMA blocks with fp32 accumulators.
// Operand slabs travel global memory -> LDS directly (global_load_lds_dwordx4: no
// register staging), NS stages deep, so that NS-1 slabs are in flight while one is
// multiplied; each wave waits only for its own oldest slab (s_waitcnt vmcnt) and one
// s_barrier per slab publishes it.  LDS rows are unpadded (a DMA instruction fills
// 1 KB contiguously) and XOR-swizzled at 16-byte granularity on the *global* side,
// so the 128-bit operand reads of 16 consecutive rows still hit 64 distinct banks.
// The product is computed transposed (W is the MFMA A operand): each lane ends up
// with 4 consecutive output columns of one row; bias/activation run in fp32 and the
// fp16 tile leaves through LDS with 16-byte stores.
//
// Fallback kernel (any K % 8 == 0): register-staged, zero-fills the K tail.
#include <type_traits>

#include "common.h"

namespace bt {

constexpr int kGemmThreads = 256;  // fallback kernel

#define BT_AS1 __attribute__((address_space(1)))
#define BT_AS3 __attribute__((address_space(3)))

// Exact-form GELU, x * Phi(x).  With h(a) = Phi(-a) = 0.5 erfc(a / sqrt 2), a = |x|:
//   Phi(x) = x >= 0 ? 1 - h : h,  so  x Phi(x) = max(x, 0) - a h(a)  in both cases.
// log2 h(a) is smooth (-1 at a = 0, ~ -a^2/2 log2 e further out), so h = exp2(P(a)) with P a degree-7
// polynomial fitted (weighted least squares iterated to minimax) to log2 h on [0, 6]: |P - log2 h| <=
// 4.8e-6 there, i.e. h to 3.3e-6 RELATIVE, and the small negative outputs keep their fp16 digits
// too.  In fp32 arithmetic the result is within 6e-7 of x Phi(x) everywhere and rounds to the same
// fp16 value as the fp64 definition for 99.9 % of inputs (1 ulp otherwise).  The leading
// coefficient is negative and P decreases monotonically, so beyond the fitted range exp2(P)
// underflows to 0 (a h(a) < 3e-9 there anyway).  Nine VALU instructions, one transcendental; the
// epilogue runs once per output element and is not overlapped with MFMA work.
__device__ __forceinline__ float gelu_erf(float x) {
  const float a = fabsf(x);
  float p = __builtin_fmaf(a, -1.83486475e-06f, 6.15994941e-05f);
  p = __builtin_fmaf(a, p, -0.000930535374f);
  p = __builtin_fmaf(a, p, 0.00850793719f);
  p = __builtin_fmaf(a, p, -0.0539601706f);
  p = __builtin_fmaf(a, p, -0.458464265f);
  p = __builtin_fmaf(a, p, -1.15125108f);
  p = __builtin_fmaf(a, p, -0.999995291f);
  return __builtin_fmaf(-a, __builtin_amdgcn_exp2f(p), fmaxf(x, 0.f));
}
// tanh form: 0.5 x (1 + tanh u) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3).
__device__ __forceinline__ float gelu_tanh(float x) {
  constexpr float k1 = -2.0f * 1.4426950408889634f * 0.7978845608028654f, k3 = k1 * 0.044715f;
  const float e = __builtin_amdgcn_exp2f(x * __builtin_fmaf(x * x, k3, k1));
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

// One 16-byte-per-lane DMA from global memory straight into LDS: lane i's 16 bytes land at
// lds_base + 16*i (lds_base is wave-uniform and travels in M0).  Issued through inline assembly so
// that the compiler does not serialise later LDS reads behind every outstanding DMA; completion is
// tracked by hand with s_waitcnt vmcnt + s_barrier.  The s_nop covers the M0-write -> LDS-DMA hazard.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr)
               : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(BT_AS3 const void*)p;
}

// s_waitcnt vmcnt(n), other counters untouched (gfx9 encoding: vmcnt = [15:14|3:0]).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Calls f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// Shared epilogue.  acc[i][j][4g+t] = C[m][n] with m = m_base + i*32 + l32, n = n_base + j*32 + 8g + 4hf + t.
// Three forms, all on the fp32 accumulators, one rounding to fp16:
//   EPI_PLAIN  C = act(acc + bias)                                         (Sec. III-C2)
//   EPI_FOLD   C = act(rstd_m (acc - mu_m c_n) + d_n): the A operand was u = gamma (.) z, the scaled
//              but NOT yet normalised input of a LayerNorm; since LN(z) W^T = rstd (u W^T - mu c) + d
//              with c = W gamma, d = W beta + bias, the normalisation moves into this epilogue and the
//              LayerNorm kernel in front of the GEMM disappears.  mu, rstd come from per-row sums.
//   EPI_RESID  v = acc + bias + residual, C = u = gamma_out (.) v, and this wave's partial row sums of
//              v and v^2 are stored for the LayerNorm that follows (add-bias + residual of
//              Sec. III-C1 fused here; the normalisation itself is folded into the next GEMM).  The
//              residual is either a plain tensor or itself a folded LayerNorm output
//              rstd (u_r - mu gamma_r) + beta_r.
// mu, rstd (FOLD: of the A operand's rows; RESID: of the residual's rows) and the residual tile are
// fetched by the caller before the K loop so that their latency is not exposed here.
// The fp16 tile of this wave is then transposed through a private LDS region (rows padded to WN+8
// halves) so that global memory is written with 16-byte-per-lane stores, 8 lanes covering 128
// contiguous bytes of an output row.
// Per-column epilogue operands of one lane (its 4*NI groups of 4 columns).  They do not depend on the
// product, so the kernels request them before the K loop: the L2 is cold at kernel start and a fetch
// issued in the epilogue would sit fully exposed at the end of every tile.  Unused members are dead code.
template <int NI>
struct EpiVecs {
  half4_t bias[NI][4];             // PLAIN / RESID (accumulator layout: this lane's 4*NI groups of 4 columns)
  float4_t fc[NI][4], fd[NI][4];   // FOLD: W gamma, W beta + bias
  // RESID, in the layout of the row-contiguous store pass (this lane's 8 consecutive columns):
  half8_t og8, rg8, rb8;           // output gamma; gamma / beta of a folded residual
};

template <int NI, int EPI>
__device__ __forceinline__ void load_epi_vecs(const GemmEpi& ep, const half_t* bias /* = ep.bias */, int N,
                                              int n_base, int lane, EpiVecs<NI>& v) {
  const int hf = lane >> 5;
  const half4_t zero = {(half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f};
#pragma unroll
  for (int j = 0; j < NI; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int nc = min(n_base + j * 32 + 8 * g + 4 * hf, N - 4);  // columns past N: clamped, never stored
      if constexpr (EPI == EPI_FOLD) {
        v.fc[j][g] = *reinterpret_cast<const float4_t*>(ep.fold_c + nc);
        v.fd[j][g] = *reinterpret_cast<const float4_t*>(ep.fold_d + nc);
      } else {
        v.bias[j][g] = bias ? *reinterpret_cast<const half4_t*>(bias + nc) : zero;
      }
    }
  if constexpr (EPI == EPI_RESID) {
    constexpr int LPR = NI * 4;  // lanes per row of the store pass
    const int nc = min(n_base + (lane % LPR) * 8, N - 8);
    v.og8 = *reinterpret_cast<const half8_t*>(ep.out_gamma + nc);
    if (ep.resid_part) {
      v.rg8 = *reinterpret_cast<const half8_t*>(ep.resid_gamma + nc);
      v.rb8 = *reinterpret_cast<const half8_t*>(ep.resid_beta + nc);
    }
  }
}

// Number of row-contiguous store passes over a wave tile of MI x NI blocks, and the residual tile of EPI_RESID in
// that layout: pass p, lane (rr, cc) holds the 8 residual values of row p*RPP + rr, columns cc .. cc+7.
template <int MI, int NI>
struct ResidTile {
  static constexpr int LPR = NI * 4, RPP = 64 / LPR, P = MI * 32 / RPP;
  uint4_t r[P];
};

template <int MI, int NI, int WGN, int ACT, int EPI>
__device__ __forceinline__ void store_tile(const float16_t (&acc)[MI][NI], const GemmEpi& ep, const EpiVecs<NI>& vec,
                                           const float (&mu)[MI], const float (&rstd)[MI],
                                           const ResidTile<MI, NI>& rres, int tile_n,
                                           int wn, int row_in_tile, float2* red /* LDS [WGN][rows of the tile] */,
                                           int tile_rows, half_t* __restrict__ C, int M, int N, int m_base,
                                           int n_base, int lane,
                                           half_t* stage /* this wave's LDS region: MI*32 x (NI*32+8) halves */) {
  constexpr int WN = NI * 32, LD = WN + 8;
  const int l32 = lane & 31, hf = lane >> 5;
  const bool folded_resid = EPI == EPI_RESID && ep.resid_part != nullptr;
  // rows of this wave's tile in the store pass: WN/8 lanes per row
  constexpr int LPR = WN / 8, RPP = 64 / LPR;  // lanes per row, rows per pass
  const int rr = lane / LPR, cc = (lane % LPR) * 8;
  // One 32-row block at a time: arithmetic on the accumulators, fp16 block to LDS, then the row-contiguous
  // pass straight to memory -- the stores of block i drain while the arithmetic of block i+1 runs.
  // EPI_RESID: the accumulator pass only adds the bias; the residual, the row sums and the output scale live
  // in the row pass, where the residual arrives as whole 16-byte pieces of a row (requested like that, 8 lanes
  // per 128-byte line, instead of 8-byte pieces gathered in accumulator layout) and a row's partial sums are
  // an exchange among the LPR neighbouring lanes that share the row.
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int j = 0; j < NI; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int nl = j * 32 + 8 * g + 4 * hf;
        float v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = acc[i][j][4 * g + t];
        if constexpr (EPI == EPI_FOLD) {
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = __builtin_fmaf(rstd[i], v[t] - mu[i] * vec.fc[j][g][t], vec.fd[j][g][t]);
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] += (float)vec.bias[j][g][t];
        }
        if constexpr (EPI != EPI_RESID) {
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            if (ACT == BT_ACT_GELU_ERF) v[t] = gelu_erf(v[t]);
            else if (ACT == BT_ACT_GELU_TANH) v[t] = gelu_tanh(v[t]);
          }
        }
        half4_t o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = (half_t)v[t];
        *reinterpret_cast<half4_t*>(stage + (i * 32 + l32) * LD + nl) = o;
      }
    }
#pragma unroll
    for (int r0 = i * 32; r0 < (i + 1) * 32; r0 += RPP) {
      const int mr = m_base + r0 + rr, n = n_base + cc;
      uint4_t out4 = *reinterpret_cast<const uint4_t*>(stage + (r0 + rr) * LD + cc);
      const bool ok = mr < M && n < N;
      if constexpr (EPI == EPI_RESID) {
        const half8_t h8 = __builtin_bit_cast(half8_t, out4);
        const half8_t r8 = __builtin_bit_cast(half8_t, rres.r[r0 / RPP]);
        // mean and 1/sigma of the residual's row: lane (r0+rr) % 32 holds them in accumulator layout
        const float mu_r = __shfl(mu[i], (r0 + rr) & 31, kWave), rstd_r = __shfl(rstd[i], (r0 + rr) & 31, kWave);
        float s0 = 0.f, s1 = 0.f;
        half8_t u8;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float r = folded_resid
                              ? __builtin_fmaf(rstd_r, (float)r8[e] - mu_r * (float)vec.rg8[e], (float)vec.rb8[e])
                              : (float)r8[e];
          const float v = ok ? (float)h8[e] + r : 0.f;
          s0 += v;
          s1 = __builtin_fmaf(v, v, s1);
          u8[e] = (half_t)(v * (float)vec.og8[e]);
        }
        out4 = __builtin_bit_cast(uint4_t, u8);
        // the LPR (4, 8 or 16) lanes of a row are neighbours inside one row of 16 lanes
        s0 += dpp_move<0xB1>(s0);
        s1 += dpp_move<0xB1>(s1);
        s0 += dpp_move<0x4E>(s0);
        s1 += dpp_move<0x4E>(s1);
        if constexpr (LPR >= 8) {
          s0 += dpp_move<0x141>(s0);
          s1 += dpp_move<0x141>(s1);
        }
        if constexpr (LPR >= 16) {
          s0 += dpp_move<0x140>(s0);
          s1 += dpp_move<0x140>(s1);
        }
        if ((lane % LPR) == 0) red[wn * tile_rows + row_in_tile + r0 + rr] = make_float2(s0, s1);
      }
      // Device-scope (write-through) stores: the tile leaves the L2 as it is produced.  Plain stores leave
      // 1-2 MB of dirty lines in every XCD's L2 and the kernel then ends with their write-back, ~3 us for
      // a 14 MB product with every CU idle; written through, that overlaps the tail of the computation
      // (3 % off a 12-layer forward).  Non-temporal stores save the same but the next kernel reads slower.
      if (ok) store_through(C + ((size_t)mr * N + n), out4);
    }
  }
  if constexpr (EPI == EPI_RESID) {
    // Row sums of this wave's columns are in LDS; after the barrier the wavefronts of tile column 0 add the
    // WGN contributions in order and store ONE partial per row and column tile.
    __syncthreads();
    if (wn == 0 && hf == 0) {
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int r = row_in_tile + i * 32 + l32, m = m_base + i * 32 + l32;
        float2 t = red[r];
#pragma unroll
        for (int w = 1; w < WGN; ++w) {
          const float2 u = red[w * tile_rows + r];
          t.x += u.x;
          t.y += u.y;
        }
        if (m < M) ep.part_out[(size_t)m * ep.part_np + tile_n] = t;
      }
    }
  }
}

// Split-K epilogue: the fp32 accumulators of this wave's tile, one 32-row block at a time through a private
// LDS region (rows padded by 4 floats) so that they leave as whole row segments, 16 bytes per lane, WN/4
// lanes per row, instead of 16-byte pieces scattered over 32 rows.
template <int MI, int NI>
__device__ __forceinline__ void store_partial(const float16_t (&acc)[MI][NI], float* __restrict__ P, int M, int N,
                                              int m_base, int n_base, int lane,
                                              float* stage /* this wave's LDS region: 32 x (NI*32+4) floats */) {
  constexpr int WN = NI * 32, LD = WN + 4;
  constexpr int LPR = WN / 4, RPP = 64 / LPR;  // lanes per row, rows per pass
  const int l32 = lane & 31, hf = lane >> 5;
  const int rr = lane / LPR, cc = (lane % LPR) * 4;
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4_t v;
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = acc[i][j][4 * g + t];
        *reinterpret_cast<float4_t*>(stage + l32 * LD + j * 32 + 8 * g + 4 * hf) = v;
      }
    // same wavefront reads what it wrote: LDS operations of a wave complete in order
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += RPP) {
      const int mr = m_base + i * 32 + r0 + rr, n = n_base + cc;
      const float4_t v = *reinterpret_cast<const float4_t*>(stage + (r0 + rr) * LD + cc);
      if (mr < M && n < N) store_through(P + ((size_t)mr * N + n), v);  // N % 8 == 0: 4 columns all in or all out
    }
  }
}

// Mean and 1/sigma of the rows m_base + i*32 + l32 from their partial sums, in two steps so that the
// loads can be issued ahead of the operand slabs and collected after them:
//   request_row_sums: the two 32-lane halves each request one half of a row's partials (up to
//     kMaxHalfParts each, clamped indices, no branches).  Issued through inline assembly so that the
//     compiler does not put a wait for ALL outstanding memory operations in front of their first use;
//   finish_row_sums: after the caller has waited (s_waitcnt vmcnt), add them in index order,
//     exchange the halves, derive mu and rstd.
constexpr int kMaxHalfParts = 4;  // np <= 8: H <= 1024 at 128-wide column tiles; more falls back to a loop

template <int MI>
__device__ __forceinline__ void request_row_sums(const float2* __restrict__ part, int np, int M, int m_base, int l32,
                                                 int hf, float2 (&v)[MI][kMaxHalfParts]) {
  const int half_np = (np + 1) >> 1, p0 = hf * half_np, p1 = min(np, p0 + half_np);
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const float2* row = part + (size_t)min(m_base + i * 32 + l32, M - 1) * np;
#pragma unroll
    for (int q = 0; q < kMaxHalfParts; ++q) {
      const float2* src = row + min(p0 + q, max(p1 - 1, 0));
      asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(v[i][q]) : "v"(src) : "memory");
    }
  }
}

template <int MI>
__device__ __forceinline__ void finish_row_sums(const float2* __restrict__ part, int np, int M, int m_base, int l32,
                                                int hf, float inv_h, float eps, float2 (&v)[MI][kMaxHalfParts],
                                                float (&mu)[MI], float (&rstd)[MI]) {
  const int half_np = (np + 1) >> 1, p0 = hf * half_np, p1 = min(np, p0 + half_np);
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int q = 0; q < kMaxHalfParts; ++q) {
      asm volatile("" : "+v"(v[i][q]));  // ordered after the caller's wait
      if (p0 + q < p1) {
        a += v[i][q].x;
        b += v[i][q].y;
      }
    }
    if (half_np > kMaxHalfParts) {  // wide rows: the rest with ordinary loads
      const float2* row = part + (size_t)min(m_base + i * 32 + l32, M - 1) * np;
      for (int p = p0 + kMaxHalfParts; p < p1; ++p) {
        const float2 u = row[p];
        a += u.x;
        b += u.y;
      }
    }
    a += __shfl_xor(a, 32, kWave);
    b += __shfl_xor(b, 32, kWave);
    mu[i] = a * inv_h;
    rstd[i] = rsqrtf(fmaxf(b * inv_h - mu[i] * mu[i], 0.f) + eps);
  }
}

// The residual tile requested through inline assembly, exactly ResidTile::P load instructions whatever M and N
// (addresses clamped into the matrix; positions outside it are ignored by the epilogue): the K loop counts
// outstanding memory instructions by hand and must know this number.  rrow[p]: the residual row of store pass p
// of this lane (clamped, and already translated through resid_rows where the residual is the padded input).
template <int MI, int NI>
__device__ __forceinline__ void request_resid(const half_t* __restrict__ resid, const int (&rrow)[ResidTile<MI, NI>::P],
                                              int N, int n_base, int lane, ResidTile<MI, NI>& rres) {
  const int n = min(n_base + (lane % ResidTile<MI, NI>::LPR) * 8, N - 8);
#pragma unroll
  for (int p = 0; p < ResidTile<MI, NI>::P; ++p) {
    const half_t* src = resid + (size_t)rrow[p] * N + n;
    uint4_t t;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(t) : "v"(src) : "memory");
    rres.r[p] = t;
  }
}

// The same tile with ordinary loads (fallback kernel).
template <int MI, int NI>
__device__ __forceinline__ void load_resid(const half_t* __restrict__ resid, const int32_t* __restrict__ rows, int M,
                                           int N, int m_base, int n_base, int lane, ResidTile<MI, NI>& rres) {
  constexpr int LPR = ResidTile<MI, NI>::LPR, RPP = ResidTile<MI, NI>::RPP;
  const int n = min(n_base + (lane % LPR) * 8, N - 8);
#pragma unroll
  for (int p = 0; p < ResidTile<MI, NI>::P; ++p) {
    const int m = min(m_base + p * RPP + lane / LPR, M - 1);
    rres.r[p] = *reinterpret_cast<const uint4_t*>(resid + (size_t)(rows ? rows[m] : m) * N + n);
  }
}

// ---------------------------------------------------------------------------
// Pipelined kernel: direct-to-LDS slabs, NS stages, WGM x WGN wavefronts.
// ---------------------------------------------------------------------------
// SHAPE (0 = fan-out, N >= 2K; 1 = neither; 2 = deep reduction, K >= 2N) changes nothing in the code: it is
// part of the kernel's name, so that a kernel trace tells the four products of an encoder layer apart
// (QKV and FFN-up are fan-out, the output projection is square, FFN-down is deep) when they share a tile shape.
template <int BM, int BN, int WGM, int WGN, int NS, int ACT, int EPI, int SHAPE>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_pipe_kernel(
    // Argument order: what the prologue and the K loop need comes first and fits the 14 dwords that are
    // preloaded into SGPRs at wave launch (-amdgpu-kernarg-preload-count), so the first DMA does not
    // wait for a scalar load of the kernel arguments; the epilogue descriptor is fetched behind it.
    const half_t* __restrict__ A, const half_t* __restrict__ W, const int32_t* __restrict__ a_rows /* = ep.a_rows */,
    const half_t* __restrict__ bias /* = ep.bias */, int M, int N, int K, int tiles_n, int tiles_m, int group_m,
    half_t* __restrict__ C, const GemmEpi ep) {
  constexpr int BK = 64, KS = BK / 16;
  constexpr int NWAVES = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;   // wave tile
  constexpr int MI = WM / 32, NI = WN / 32;     // 32x32 MFMA blocks per wave tile
  constexpr int CPR = BK / 8;                   // 16-byte chunks per LDS row
  constexpr int RPI = 64 / CPR;                 // rows one DMA instruction (64 lanes x 16 B) fills
  constexpr int LA = BM / RPI / NWAVES, LB = BN / RPI / NWAVES;  // DMA instructions per wave per slab
  constexpr int TOT = LA + LB;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
  static_assert(LA * RPI * NWAVES == BM && LB * RPI * NWAVES == BN, "tile rows must split evenly over the waves");
  static_assert(NS >= 2 && (NS - 1) * TOT < 64, "vmcnt range");

  // per-wave epilogue staging: the fp16 wave tile, or (split-K) one 32-row block of fp32 accumulators
  constexpr int STAGE_HALVES = EPI == EPI_PARTIAL ? 2 * 32 * (WN + 4) : WM * (WN + 8);
  constexpr int PIPE_HALVES = NS * (BM + BN) * BK;
  constexpr int LDS_HALVES = PIPE_HALVES > NWAVES * STAGE_HALVES ? PIPE_HALVES : NWAVES * STAGE_HALVES;
  __shared__ __attribute__((aligned(1024))) half_t smem[LDS_HALVES];
  half_t* const sA = smem;                 // [NS][BM*BK]
  half_t* const sB = smem + NS * BM * BK;  // [NS][BN*BK]

  // Tile order.  Block ids are dealt round-robin to the 8 XCDs; xcd_remap gives every XCD one
  // contiguous run of the logical order, and the logical order walks strips of `group_m` tile rows
  // column by column, so the tiles an XCD works on together form a near-square patch of C whose A
  // and W panels fit its private L2 instead of streaming all of W through every L2.
  // split-K (EPI_PARTIAL): the grid holds ksplit copies of the tile grid, copy s works on K slice s
  const int n_tiles = tiles_m * tiles_n;
  const int split = EPI == EPI_PARTIAL ? (int)blockIdx.x / n_tiles : 0;
  const int k_len = EPI == EPI_PARTIAL ? K / ep.ksplit : K, k_off = split * k_len;
  const int lin = xcd_remap((int)blockIdx.x - split * n_tiles, n_tiles);
  const int per_group = group_m * tiles_n;
  const int first_m = (lin / per_group) * group_m;
  const int rows_here = min(tiles_m - first_m, group_m);
  const int in_group = lin - (lin / per_group) * per_group;
  const int tm = first_m + in_group % rows_here, tn = in_group / rows_here;
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: LDS DMA bases live in M0
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, hf = lane >> 5;

  // The bias of the plain epilogue is requested right behind the first operand slabs (a cheap broadcast
  // load whose latency then hides behind the K loop).  The folded forms hold more per-column operands than
  // there are registers to park them across the K loop; they load them right before the epilogue.  Their
  // residual tile and partial row sums are requested in the last steady round (see below).
  ResidTile<MI, NI> rres;  // dead (and removed by the compiler) in the other epilogue forms
  EpiVecs<NI> vec;
  __shared__ float2 red[EPI == EPI_RESID ? WGN * BM : 1];
  float2 psum[MI][kMaxHalfParts];
  constexpr bool kStats = EPI == EPI_FOLD || EPI == EPI_RESID;
  // without statistics (a plain residual) the requests still issue, at a harmless valid address, so that
  // the number of memory instructions in flight is a compile-time constant
  const float2* const stat_src = EPI == EPI_FOLD ? ep.ln_part : (EPI == EPI_RESID ? ep.resid_part : nullptr);
  const float2* const stat_part = stat_src ? stat_src : reinterpret_cast<const float2*>(W);
  const int stat_np = stat_src ? (EPI == EPI_FOLD ? ep.ln_np : ep.resid_np) : 0;
  constexpr int kLateLoads = (EPI == EPI_RESID ? ResidTile<MI, NI>::P : 0) + (kStats ? MI * kMaxHalfParts : 0);
  static_assert((NS - 2) * TOT + kLateLoads < 64, "vmcnt range");

  // DMA source pointers.  Instruction q of this wave fills LDS rows [r0, r0+8) of the slab; lane i
  // lands at row r0 + i/8, physical chunk i%8, and therefore fetches logical chunk
  // (i%8) ^ ((row>>1)&7) of that row from global memory.
  const half_t* ga[LA];
  const half_t* gb[LB];
#pragma unroll
  for (int q = 0; q < LA; ++q) {
    const int r = (wave * LA + q) * RPI + lane / CPR;
    const int c = (lane % CPR) ^ ((r >> 1) & (CPR - 1));
    const int ar = min(m0 + r, M - 1);  // rows past M: clamped reads, never stored
    ga[q] = A + (size_t)(a_rows ? a_rows[ar] : ar) * K + k_off + c * 8;
  }
#pragma unroll
  for (int q = 0; q < LB; ++q) {
    const int r = (wave * LB + q) * RPI + lane / CPR;
    const int c = (lane % CPR) ^ ((r >> 1) & (CPR - 1));
    gb[q] = W + (size_t)min(n0 + r, N - 1) * K + k_off + c * 8;
  }
  // Residual rows of this lane's store passes (EPI_RESID): resolved here, with the operand row indices and
  // before the first DMA, so that the late residual requests need no dependent index load.
  int rrow[ResidTile<MI, NI>::P];
#pragma unroll
  for (int p = 0; p < ResidTile<MI, NI>::P; ++p) {
    const int m = min(m0 + wm * WM + p * ResidTile<MI, NI>::RPP + lane / ResidTile<MI, NI>::LPR, M - 1);
    rrow[p] = (EPI == EPI_RESID && ep.resid_rows) ? ep.resid_rows[m] : m;
    // collected here: the wait for this load must not end up in the K loop, where the compiler cannot see
    // the DMA instructions in flight and would wait for all of them
    if constexpr (EPI == EPI_RESID) asm volatile("" : "+v"(rrow[p]));
  }
  const uint32_t lds_a = lds_addr(sA) + wave * LA * RPI * BK * 2;  // bytes
  const uint32_t lds_b = lds_addr(sB) + wave * LB * RPI * BK * 2;
  // DMA instruction q (0 <= q < TOT) of this wave for slab `slab` into stage `stage`: A rows, then W rows.
  auto issue_one = [&](int q, int slab, int stage) {
    if (q < LA) dma16(ga[q < LA ? q : 0] + slab * BK, lds_a + stage * (BM * BK * 2) + q * (RPI * BK * 2));
    else dma16(gb[q >= LA ? q - LA : 0] + slab * BK, lds_b + stage * (BN * BK * 2) + (q - LA) * (RPI * BK * 2));
  };

  float16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Slab schedule.  Slab kt lives in stage (kt - pre) mod NS, with pre = (nk - (NS-1)) mod NS, so that
  // the nk slabs split into `pre` leading slabs (stage known at run time only), a steady state of
  // whole rounds of NS slabs whose stages are compile-time constants, and the last NS-1 slabs, which
  // fetch nothing.  In the steady state and the tail every LDS offset is an immediate, every DMA
  // target a constant and every wait count exact: no branches, no address arithmetic in the loop.
  const int nk = k_len / BK;  // >= NS - 1 (checked by the launcher)
  const int pre = (nk - (NS - 1)) % NS;
  const int rounds = (nk - (NS - 1) - pre) / NS;
  {
    int st = pre == 0 ? 0 : NS - pre;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) {
#pragma unroll
      for (int q = 0; q < TOT; ++q) issue_one(q, s, st);
      st = st + 1 == NS ? 0 : st + 1;
    }
  }
  // These loads sit between the DMA of the first NS-1 slabs and of the later ones in the in-order queue the
  // hand-written waits count: a wait for slab k then also waits for as many of the younger entries as there
  // are loads here -- more than needed, never less, and only for the first slabs.
  if constexpr (EPI == EPI_PLAIN) load_epi_vecs<NI, EPI>(ep, bias, N, n0 + wn * WN, lane, vec);

  // operand read offsets (halves): row*BK + ((2ks+hf) ^ swz(row))*8 ; swz depends on l32 only
  const int swz = (l32 >> 1) & (CPR - 1);
  const half_t* const pa0 = sA + (wm * WM + l32) * BK;
  const half_t* const pb0 = sB + (wn * WN + l32) * BK;
  int co[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) co[ks] = ((2 * ks + hf) ^ swz) * 8;
  half8_t fa[2][MI], fb[2][NI];
  auto read_frags = [&](auto stage, int ks, int slot) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
      fa[slot][i] = *reinterpret_cast<const half8_t*>(pa0 + co[ks] + stage * (BM * BK) + i * 32 * BK);
#pragma unroll
    for (int j = 0; j < NI; ++j)
      fb[slot][j] = *reinterpret_cast<const half8_t*>(pb0 + co[ks] + stage * (BN * BK) + j * 32 * BK);
  };
  auto mfmas = [&](int slot) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
        // transposed product: D[n][m] += W[n][k] * A[m][k]
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0);
  };
  // One slab.  The fragments of k-step ks+1 are read from LDS while the MFMAs of k-step ks run; the
  // DMA instructions for slab kt+NS-1 (FETCH) are spread over the first KS-1 k-steps into the stage
  // that the previous hand-over freed.  The hand-over to the next slab sits in front of the last
  // k-step's MFMAs: every fragment of this slab is in registers (lgkmcnt 0), this wave's share of
  // the next slab has landed (at most IN_FLIGHT younger memory instructions stay in flight), and
  // the barrier publishes both facts, so the next slab may be read and this stage refilled.
  auto slab = [&](int kt, auto stage, auto fetch_c, auto last_c, auto in_flight_c) {
    constexpr bool FETCH = decltype(fetch_c)::value, LAST = decltype(last_c)::value;
    constexpr int IN_FLIGHT = decltype(in_flight_c)::value;  // memory instructions issued after slab kt+1
    const auto fstage = (stage + (NS - 1)) % NS, nstage = (stage + 1) % NS;
#pragma unroll
    for (int ks = 0; ks < KS - 1; ++ks) {
      read_frags(stage, ks + 1, (ks + 1) & 1);
      if (FETCH) {
#pragma unroll
        for (int q = ks * TOT / (KS - 1); q < (ks + 1) * TOT / (KS - 1); ++q) issue_one(q, kt + NS - 1, fstage);
      }
      mfmas(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!LAST) {
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0), other counters untouched
      wait_vmcnt<IN_FLIGHT>();
      __builtin_amdgcn_s_barrier();
      read_frags(nstage, 0, 0);
    }
    mfmas((KS - 1) & 1);
    __builtin_amdgcn_sched_barrier(0);
  };
  using std::integral_constant;
  using yes = std::true_type;
  using no = std::false_type;

  wait_vmcnt<(NS - 2) * TOT>();  // slab 0 has landed
  __builtin_amdgcn_s_barrier();
  int kt = 0;
  {
    int st = pre == 0 ? 0 : NS - pre;
    read_frags(st, 0, 0);
    for (; kt < pre; ++kt) {  // leading slabs: run-time stage
      slab(kt, st, yes{}, no{}, integral_constant<int, (NS - 2) * TOT>{});
      st = st + 1 == NS ? 0 : st + 1;
    }
  }
  // The epilogue operands that are expensive to fetch (residual tile: one cache line per lane; partial
  // row sums; kLateLoads instructions in all) are requested at the start of the LAST steady round, about
  // 2 NS slabs before they are needed: early enough to arrive in time, late enough not to sit in front of
  // the first operand slabs in the in-order memory pipeline (issued at kernel start they delayed the whole
  // K loop by more than a microsecond).  The waits that follow count them: they are younger than the
  // NS-2 slabs in flight at that moment and older than every slab requested afterwards.
  // They are requested through inline assembly and collected by hand, so from request to collection the
  // code is straight-line (no loop, no join): the compiler must not get a chance to copy a destination
  // register before its data has arrived.
  float mu[MI], rstd[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i) { mu[i] = 0.f; rstd[i] = 1.f; }
  auto late_requests = [&]() {
    if constexpr (EPI == EPI_RESID) request_resid<MI, NI>(ep.resid, rrow, N, n0 + wn * WN, lane, rres);
    if constexpr (kStats) request_row_sums<MI>(stat_part, stat_np, M, m0 + wm * WM, l32, hf, psum);
  };
  auto late_collect = [&]() {
    if constexpr (kLateLoads > 0) {
      wait_vmcnt<0>();
      if constexpr (EPI == EPI_RESID) {
#pragma unroll
        for (int p = 0; p < ResidTile<MI, NI>::P; ++p) asm volatile("" : "+v"(rres.r[p]));  // ordered after the wait
      }
      finish_row_sums<MI>(stat_part, stat_np, M, m0 + wm * WM, l32, hf, ep.inv_h, ep.eps, psum, mu, rstd);
    }
  };
  for (int r = 0; r + 1 < rounds; ++r) {  // steady state: compile-time stages
    static_for<NS>([&](auto s) { slab(kt + decltype(s)::value, s, yes{}, no{}, integral_constant<int, (NS - 2) * TOT>{}); });
    kt += NS;
  }
  if (rounds > 0) {  // last steady round + the last NS-1 slabs (which fetch nothing)
    late_requests();
    static_for<NS>([&](auto s) {
      constexpr int S = decltype(s)::value;
      slab(kt + S, s, yes{}, no{}, integral_constant<int, (NS - 2) * TOT + (S <= NS - 3 ? kLateLoads : 0)>{});
    });
    static_for<NS - 1>([&](auto j) {
      constexpr int J = decltype(j)::value;
      slab(kt + NS + J, j, no{}, integral_constant<bool, J == NS - 2>{},
           integral_constant<int, (NS - 3 - J > 0 ? NS - 3 - J : 0) * TOT>{});
    });
    late_collect();
  } else {  // short K: the late requests go behind all operand slabs and the remaining waits allow for them
    late_requests();
    static_for<NS - 1>([&](auto j) {
      constexpr int J = decltype(j)::value;
      slab(kt + J, j, no{}, integral_constant<bool, J == NS - 2>{},
           integral_constant<int, (NS - 3 - J > 0 ? NS - 3 - J : 0) * TOT + kLateLoads>{});
    });
    late_collect();
  }
  if (!stat_src) {  // a plain residual: no LayerNorm to rebuild
#pragma unroll
    for (int i = 0; i < MI; ++i) { mu[i] = 0.f; rstd[i] = 1.f; }
  }
  if constexpr (EPI == EPI_FOLD || EPI == EPI_RESID) load_epi_vecs<NI, EPI>(ep, bias, N, n0 + wn * WN, lane, vec);
  if constexpr (EPI == EPI_PARTIAL) {
    __builtin_amdgcn_s_barrier();  // every wave is done reading the last slab: LDS becomes staging space
    store_partial<MI, NI>(acc, ep.partial + (size_t)split * M * N, M, N, m0 + wm * WM, n0 + wn * WN, lane,
                          reinterpret_cast<float*>(smem + wave * STAGE_HALVES));
  } else {
    __builtin_amdgcn_s_barrier();  // every wave is done reading the last slab: LDS becomes staging space
    store_tile<MI, NI, WGN, ACT, EPI>(acc, ep, vec, mu, rstd, rres, tn, wn, wm * WM, red, BM, C, M, N, m0 + wm * WM,
                                      n0 + wn * WN, lane, smem + wave * STAGE_HALVES);
  }
}

// ---------------------------------------------------------------------------
// Fallback kernel: register-staged, 64x64x64 tile, padded LDS rows, K tail zero-filled.
// ---------------------------------------------------------------------------
template <int ACT, int EPI>
__global__ __launch_bounds__(kGemmThreads) void gemm_simple_kernel(const half_t* __restrict__ A,
                                                                   const half_t* __restrict__ W, const GemmEpi ep,
                                                                   half_t* __restrict__ C, int M, int N, int K,
                                                                   int tiles_n) {
  constexpr int BM = 64, BN = 64, BK = 64, LDS = BK + 8, CH = BM * (BK / 8) / kGemmThreads;
  __shared__ __attribute__((aligned(16))) half_t sA[BM * LDS];
  __shared__ __attribute__((aligned(16))) half_t sB[BN * LDS];
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x - tm * tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, hf = lane >> 5;
  const int kc = (tid & 7) * 8;
  float16_t acc[1][1];
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[0][0][r] = 0.f;
  const uint4_t zero4 = {0u, 0u, 0u, 0u};
  for (int k0 = 0; k0 < K; k0 += BK) {
    const bool in = (k0 + kc) < K;  // K % 8 == 0: a chunk is entirely inside or outside
    uint4_t ra[CH], rb[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int row = (tid >> 3) + i * (kGemmThreads / 8);
      const int ar = min(m0 + row, M - 1);
      ra[i] = in ? *reinterpret_cast<const uint4_t*>(A + (size_t)(ep.a_rows ? ep.a_rows[ar] : ar) * K + k0 + kc) : zero4;
      rb[i] = in ? *reinterpret_cast<const uint4_t*>(W + (size_t)min(n0 + row, N - 1) * K + k0 + kc) : zero4;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int row = (tid >> 3) + i * (kGemmThreads / 8);
      *reinterpret_cast<uint4_t*>(&sA[row * LDS + kc]) = ra[i];
      *reinterpret_cast<uint4_t*>(&sB[row * LDS + kc]) = rb[i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const half8_t fa = *reinterpret_cast<const half8_t*>(&sA[(wm * 32 + l32) * LDS + ks * 16 + hf * 8]);
      const half8_t fb = *reinterpret_cast<const half8_t*>(&sB[(wn * 32 + l32) * LDS + ks * 16 + hf * 8]);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb, fa, acc[0][0], 0, 0, 0);
    }
  }
  __syncthreads();  // operand tiles are dead: reuse them as per-wave staging space (32 x 40 halves each)
  float mu[1] = {0.f}, rstd[1] = {1.f};
  ResidTile<1, 1> rres;
  __shared__ float2 red[EPI == EPI_RESID ? 2 * BM : 1];
  const float2* const stat_part = EPI == EPI_FOLD ? ep.ln_part : (EPI == EPI_RESID ? ep.resid_part : nullptr);
  const int stat_np = EPI == EPI_FOLD ? ep.ln_np : ep.resid_np;
  if (EPI != EPI_PLAIN && stat_part) {
    float2 psum[1][kMaxHalfParts];
    request_row_sums<1>(stat_part, stat_np, M, m0 + wm * 32, l32, hf, psum);
    wait_vmcnt<0>();
    finish_row_sums<1>(stat_part, stat_np, M, m0 + wm * 32, l32, hf, ep.inv_h, ep.eps, psum, mu, rstd);
  }
  if constexpr (EPI == EPI_RESID) load_resid<1, 1>(ep.resid, ep.resid_rows, M, N, m0 + wm * 32, n0 + wn * 32, lane, rres);
  EpiVecs<1> vec;
  load_epi_vecs<1, EPI>(ep, ep.bias, N, n0 + wn * 32, lane, vec);
  store_tile<1, 1, 2, ACT, EPI>(acc, ep, vec, mu, rstd, rres, tn, wn, wm * 32, red, BM, C, M, N, m0 + wm * 32, n0 + wn * 32,
                                lane, (wave < 2 ? sA : sB) + (wave & 1) * 32 * 40);
}

// act x epilogue combinations that exist: PLAIN and FOLD with any activation, RESID without one.
static bt_status launch_simple(const half_t* A, const half_t* W, half_t* C, int M, int N, int K, bt_act act, int epi,
                               GemmEpi ep, hipStream_t st, int* np_out);

template <int BM, int BN, int WGM, int WGN, int NS>
static bt_status launch_pipe(const half_t* A, const half_t* W, half_t* C, int M, int N, int K, bt_act act, int epi,
                             GemmEpi ep, hipStream_t st, int* np_out) {
  if (K / 64 < NS - 1) return launch_simple(A, W, C, M, N, K, act, epi, ep, st, np_out);  // pipeline deeper than K
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  ep.part_np = tiles_n;
  if (np_out) *np_out = ep.part_np;
  const long long n_tiles = (long long)tiles_m * tiles_n;
  if (n_tiles > 0x7fffffffLL) return BT_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_tiles), block(WGM * WGN * 64);
  // strip height: the per-XCD share of tiles (n_tiles/8) should cover a patch with gm*BM ~ gn*BN
  int group_m = (int)(sqrt((double)n_tiles / 8.0 * BN / BM) + 0.5);
  group_m = group_m < 1 ? 1 : (group_m > tiles_m ? tiles_m : group_m);
#define BT_LAUNCH_S(ACT, EPI, SHAPE) \
  gemm_pipe_kernel<BM, BN, WGM, WGN, NS, ACT, EPI, SHAPE><<<grid, block, 0, st>>>(A, W, ep.a_rows, ep.bias, M, N, K, tiles_n, tiles_m, group_m, C, ep)
  // the shape class is spelled out only where two products of a layer can meet in one instantiation
  // (no activation); the FFN-up product is told apart by its activation already
#define BT_LAUNCH(ACT, EPI)                                                     \
  do {                                                                          \
    if constexpr ((ACT) == BT_ACT_NONE && (EPI) == EPI_PLAIN) {                 \
      if (N >= 2 * K) BT_LAUNCH_S(ACT, EPI, 0);                                 \
      else if (K >= 2 * N) BT_LAUNCH_S(ACT, EPI, 2);                            \
      else BT_LAUNCH_S(ACT, EPI, 1);                                            \
    } else if constexpr ((ACT) == BT_ACT_NONE && (EPI) == EPI_FOLD) {           \
      if (N >= 2 * K) BT_LAUNCH_S(ACT, EPI, 0);                                 \
      else BT_LAUNCH_S(ACT, EPI, 1);                                            \
    } else if constexpr ((EPI) == EPI_RESID) {                                  \
      if (K >= 2 * N) BT_LAUNCH_S(ACT, EPI, 2);                                 \
      else BT_LAUNCH_S(ACT, EPI, 1);                                            \
    } else {                                                                    \
      BT_LAUNCH_S(ACT, EPI, 1);                                                 \
    }                                                                           \
  } while (0)
  if (epi == EPI_RESID) {
    // only for shapes with one 32x32 block per wavefront: the residual tile and the partial row sums wait in
    // registers across the last slabs, and the two largest shapes have none to spare (they would spill, which
    // the hand-collected loads do not survive).  128x128 fits (192 registers) but gains nothing where it could
    // be chosen: folded and plain layers are level from 2 700 to 5 400 tokens of width 768 with it.
    if constexpr ((BM / WGM) * (BN / WGN) == 32 * 32) BT_LAUNCH(BT_ACT_NONE, EPI_RESID);
    else return BT_ERR_UNSUPPORTED;
  } else if (epi == EPI_FOLD) {
    if (act == BT_ACT_NONE) BT_LAUNCH(BT_ACT_NONE, EPI_FOLD);
    else if (act == BT_ACT_GELU_ERF) BT_LAUNCH(BT_ACT_GELU_ERF, EPI_FOLD);
    else BT_LAUNCH(BT_ACT_GELU_TANH, EPI_FOLD);
  } else {
    if (act == BT_ACT_NONE) BT_LAUNCH(BT_ACT_NONE, EPI_PLAIN);
    else if (act == BT_ACT_GELU_ERF) BT_LAUNCH(BT_ACT_GELU_ERF, EPI_PLAIN);
    else BT_LAUNCH(BT_ACT_GELU_TANH, EPI_PLAIN);
  }
#undef BT_LAUNCH
#undef BT_LAUNCH_S
  return launch_status();
}

static bt_status launch_simple(const half_t* A, const half_t* W, half_t* C, int M, int N, int K, bt_act act, int epi,
                               GemmEpi ep, hipStream_t st, int* np_out) {
  const int tiles_n = (N + 63) / 64;
  ep.part_np = tiles_n;
  if (np_out) *np_out = ep.part_np;
  const long long n_tiles = (long long)((M + 63) / 64) * tiles_n;
  if (n_tiles > 0x7fffffffLL) return BT_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_tiles), block(kGemmThreads);
#define BT_LAUNCH(ACT, EPI) gemm_simple_kernel<ACT, EPI><<<grid, block, 0, st>>>(A, W, ep, C, M, N, K, tiles_n)
  if (epi == EPI_RESID) {
    BT_LAUNCH(BT_ACT_NONE, EPI_RESID);
  } else if (epi == EPI_FOLD) {
    if (act == BT_ACT_NONE) BT_LAUNCH(BT_ACT_NONE, EPI_FOLD);
    else if (act == BT_ACT_GELU_ERF) BT_LAUNCH(BT_ACT_GELU_ERF, EPI_FOLD);
    else BT_LAUNCH(BT_ACT_GELU_TANH, EPI_FOLD);
  } else {
    if (act == BT_ACT_NONE) BT_LAUNCH(BT_ACT_NONE, EPI_PLAIN);
    else if (act == BT_ACT_GELU_ERF) BT_LAUNCH(BT_ACT_GELU_ERF, EPI_PLAIN);
    else BT_LAUNCH(BT_ACT_GELU_TANH, EPI_PLAIN);
  }
#undef BT_LAUNCH
  return launch_status();
}

// Tile choice by a small cost model.  Every tile shape is bound by how fast a compute unit ingests
// operand slabs (~85 GB/s here whatever the shape), so one 64-deep slab costs a time proportional to
// BM+BN, and the grid runs in ceil(tiles / 256) rounds of one tile per compute unit.  slab_us and
// epi_us (epilogue + pipeline fill) were measured per shape on MI355X; GELU adds to the epilogue.
// Returns the index into kGemmTiles.  K % 64 == 0.
struct GemmTile { int bm, bn; float slab_us, epi_us; bool resid_form; };
static const GemmTile kGemmTiles[6] = {{256, 128, 0.607f, 2.2f, false}, {192, 128, 0.482f, 1.5f, false},
                                       {128, 128, 0.384f, 1.5f, false}, {128, 64, 0.298f, 0.78f, true},
                                       {64, 128, 0.287f, 0.84f, true},  {64, 64, 0.183f, 0.4f, true}};
// Time of one round (one tile per compute unit) of shape t, by the model above.
static float gemm_round_us(const GemmTile& t, int K, bt_act act) {
  const float act_us = act != BT_ACT_NONE ? 9e-5f * t.bm * t.bn : 0.f;
  return (float)(K / 64) * t.slab_us + t.epi_us + act_us;
}

static int gemm_tile_choice(int M, int N, int K, bt_act act, int epi, float* us_out = nullptr) {
  int best = -1;
  float best_us = 0.f;
  for (int c = 0; c < 6; ++c) {
    const GemmTile& t = kGemmTiles[c];
    if (epi == EPI_RESID && !t.resid_form) continue;  // see launch_pipe
    const long long tiles = (long long)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
    const long long rounds = (tiles + 255) / 256;
    const float us = (float)rounds * gemm_round_us(t, K, act);
    if (best < 0 || us < best_us) { best = c; best_us = us; }
  }
  if (us_out) *us_out = best_us;
  return best;
}

// The staircase of the round model: a tile grid that needs a little more than a whole number of rounds pays a
// whole round for its few last tiles (608 tiles of 256 x 128 for the FFN-up product of 4 648 tokens at width
// 1024: the third round runs 96 tiles on 256 compute units).  Rows are independent, so such a product can run as
// two launches: the rows that fill whole rounds of one shape, then the remaining rows with whatever shape suits
// them (measured for that product: 49 us against 58.5 us; bit-identical rows where both parts use the shape of the
// single launch).  Returns the number of leading rows for the first launch and its shape, or 0: one launch.
// The second launch costs a launch gap, and the model's constants are from single-round runs: a split must
// promise 5 %.
constexpr float kLaunchUs = 2.5f;
static int gemm_msplit_choice(int M, int N, int K, bt_act act, int* main_tile) {
  float single_us = 0.f;
  (void)gemm_tile_choice(M, N, K, act, EPI_PLAIN, &single_us);
  int best_rows = 0;
  float best_us = 0.95f * single_us;
  for (int c = 0; c < 6; ++c) {
    const GemmTile& t = kGemmTiles[c];
    const long long tn = (N + t.bn - 1) / t.bn, tm = (M + t.bm - 1) / t.bm, tiles = tm * tn;
    const long long full = tiles / 256;
    if (full < 1 || tiles % 256 == 0 || tn > 256) continue;
    const long long rows_main = (full * 256 / tn) * t.bm;  // whole tile rows that fit `full` rounds
    if (rows_main <= 0 || rows_main >= M) continue;
    const long long rounds_main = ((rows_main / t.bm) * tn + 255) / 256;
    float rest_us = 0.f;
    (void)gemm_tile_choice((int)(M - rows_main), N, K, act, EPI_PLAIN, &rest_us);
    const float us = (float)rounds_main * gemm_round_us(t, K, act) + rest_us + kLaunchUs;
    if (us < best_us) { best_us = us; best_rows = (int)rows_main; *main_tile = c; }
  }
  return best_rows;
}

static bt_status gemm_launch_tile(int tile, const half_t* a, const half_t* w, half_t* c, int M, int N, int K,
                                  bt_act act, int epi, const GemmEpi& ep, hipStream_t st, int* np_out) {
#define BT_PIPE(BM, BN, WGM, WGN, NS) launch_pipe<BM, BN, WGM, WGN, NS>(a, w, c, M, N, K, act, epi, ep, st, np_out)
  switch (tile) {
    case 0: return BT_PIPE(256, 128, 4, 2, 3);
    case 1: return BT_PIPE(192, 128, 2, 4, 3);
    case 2: return BT_PIPE(128, 128, 2, 4, 4);
    case 3: return BT_PIPE(128, 64, 4, 2, 4);
    case 4: return BT_PIPE(64, 128, 2, 4, 4);
    default: return BT_PIPE(64, 64, 2, 2, 4);
  }
#undef BT_PIPE
}

bt_status gemm_dispatch(const bt_half* A, const bt_half* W, int M, int N, int K, bt_act act, int epi,
                        const GemmEpi& ep, bt_half* C, hipStream_t st, int* np_out) {
  const half_t* a = reinterpret_cast<const half_t*>(A);
  const half_t* w = reinterpret_cast<const half_t*>(W);
  half_t* c = reinterpret_cast<half_t*>(C);
  if (epi == EPI_RESID && act != BT_ACT_NONE) return BT_ERR_INVALID_ARG;
  if ((K % 64) != 0) return launch_simple(a, w, c, M, N, K, act, epi, ep, st, np_out);
  if (epi == EPI_PLAIN) {  // nothing of the plain epilogue is indexed by row: the row ranges are independent products
    int main_tile = 0;
    const int m1 = gemm_msplit_choice(M, N, K, act, &main_tile);
    if (m1 > 0) {
      const bt_status s = gemm_launch_tile(main_tile, a, w, c, m1, N, K, act, epi, ep, st, np_out);
      if (s != BT_OK) return s;
      GemmEpi rest = ep;
      if (rest.a_rows) rest.a_rows += m1;  // gathered rows: the index moves, the matrix stays
      return gemm_dispatch(reinterpret_cast<const bt_half*>(rest.a_rows ? a : a + (size_t)m1 * K), W, M - m1, N, K, act,
                           epi, rest, reinterpret_cast<bt_half*>(c + (size_t)m1 * N), st, np_out);
    }
  }
  return gemm_launch_tile(gemm_tile_choice(M, N, K, act, epi), a, w, c, M, N, K, act, epi, ep, st, np_out);
}

// Split-K for token counts so small that the tile grid leaves most compute units idle and every tile
// walks the whole K alone (Sec. IV-E, small batches): workgroup (tile, s) multiplies K slice s and stores
// fp32 partial sums; the add-bias + residual + LayerNorm kernel that consumes the product adds the slices.
// gemm_splitk_choice: how many K slices to use for an M x N x K product (1 = do not split).  Slices times
// tiles stays within one round of the chip; a slice keeps at least the three slabs the pipeline needs; the
// slices divide K/64 evenly.  slices * M * N <= kSplitKFloats (256 tiles of 64 x 64).
// Larger tiles over K slices for the deep FFN-down product at a few thousand tokens (fewer operand bytes per
// compute unit) were measured and are not used: at 2 308 x 768 x 3072, 128 x 128 tiles x 2 slices run 18.4 us
// against 16.0 us unsplit -- the K loop halves but 14 MB of fp32 slices leave through the write path
// (and the LayerNorm kernel reads them back), which costs more than the shorter loop saves.
int gemm_splitk_choice(int M, int N, int K) {
  if ((K % 64) != 0 || M < 1) return 1;
  const long long t64 = (long long)((M + 63) / 64) * ((N + 63) / 64);
  if (t64 > 128) return 1;
  const int nk = K / 64;
  int best = 1;
  for (int s = 2; s <= 8; ++s)
    if (nk % s == 0 && nk / s >= 3 && t64 * s <= 256) best = s;
  return best;
}

bt_status gemm_splitk_dispatch(const bt_half* A, const bt_half* W, int M, int N, int K, int ksplit, float* partial,
                               hipStream_t st) {
  constexpr int BM = 64, BN = 64, NS = 4;
  if (ksplit < 2 || (K % (64 * ksplit)) != 0 || K / ksplit / 64 < NS - 1 || !partial) return BT_ERR_INVALID_ARG;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int n_tiles = tiles_m * tiles_n;
  GemmEpi ep;
  ep.partial = partial;
  ep.ksplit = ksplit;
  int group_m = (int)(sqrt((double)n_tiles / 8.0) + 0.5);
  group_m = group_m < 1 ? 1 : (group_m > tiles_m ? tiles_m : group_m);
  const dim3 grid((unsigned)(n_tiles * ksplit)), block(256);
  const half_t* a = reinterpret_cast<const half_t*>(A);
  const half_t* w = reinterpret_cast<const half_t*>(W);
  // shape class as in launch_pipe: a trace tells the split FFN-down product (deep) from the split projection
  if (K >= 2 * N)
    gemm_pipe_kernel<BM, BN, 2, 2, NS, BT_ACT_NONE, EPI_PARTIAL, 2><<<grid, block, 0, st>>>(a, w, nullptr, nullptr, M, N, K, tiles_n, tiles_m, group_m, nullptr, ep);
  else
    gemm_pipe_kernel<BM, BN, 2, 2, NS, BT_ACT_NONE, EPI_PARTIAL, 1><<<grid, block, 0, st>>>(a, w, nullptr, nullptr, M, N, K, tiles_n, tiles_m, group_m, nullptr, ep);
  return launch_status();
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
  bt::GemmEpi ep;
  ep.bias = reinterpret_cast<const bt::half_t*>(d_bias);
  return bt::gemm_dispatch(d_A, d_W, M, N, K, act, bt::EPI_PLAIN, ep, d_C, static_cast<hipStream_t>(stream), nullptr);
}

extern "C" size_t bt_gemm_kslices_bytes(int M, int N, int K) {
  if (M < 1 || N < 8 || K < 8) return 0;
  const int sl = bt::gemm_splitk_choice(M, N, K);
  return sl > 1 ? (size_t)sl * (size_t)M * (size_t)N * sizeof(float) : 0;
}

extern "C" bt_status bt_gemm_kslices(const bt_half* d_A, const bt_half* d_W, int M, int N, int K, bt_half* d_C,
                                     float* d_slices, size_t slices_bytes, int* n_slices, bt_stream stream) {
  if (M < 0 || N < 8 || K < 8 || (N % 8) != 0 || (K % 8) != 0 || !n_slices) return BT_ERR_INVALID_ARG;
  *n_slices = 0;
  if (M == 0) return BT_OK;
  if (!d_A || !d_W || !bt::aligned16(d_A) || !bt::aligned16(d_W)) return BT_ERR_INVALID_ARG;
  const int sl = bt::gemm_splitk_choice(M, N, K);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (sl > 1) {
    if (!d_slices || (reinterpret_cast<uintptr_t>(d_slices) & 15u)) return BT_ERR_WORKSPACE;
    if (slices_bytes < (size_t)sl * (size_t)M * (size_t)N * sizeof(float)) return BT_ERR_WORKSPACE;
    const bt_status r = bt::gemm_splitk_dispatch(d_A, d_W, M, N, K, sl, d_slices, st);
    if (r == BT_OK) *n_slices = sl;
    return r;
  }
  if (!d_C || !bt::aligned16(d_C)) return BT_ERR_INVALID_ARG;
  bt::GemmEpi ep;
  return bt::gemm_dispatch(d_A, d_W, M, N, K, BT_ACT_NONE, bt::EPI_PLAIN, ep, d_C, st, nullptr);
}

extern "C" bt_status bt_gemm_row_split(int M, int N, int K, bt_act act, int* rows_first) {
  if (M < 0 || N < 1 || K < 1 || (N % 8) != 0 || (K % 8) != 0 || !rows_first) return BT_ERR_INVALID_ARG;
  if (act != BT_ACT_NONE && act != BT_ACT_GELU_ERF && act != BT_ACT_GELU_TANH) return BT_ERR_INVALID_ARG;
  int tile = 0;
  *rows_first = (K % 64) != 0 || M < 1 ? 0 : bt::gemm_msplit_choice(M, N, K, act, &tile);
  return BT_OK;
}

extern "C" bt_status bt_gemm_tile_shape(int M, int N, int K, bt_act act, int* bm, int* bn) {
  if (M < 0 || N < 1 || K < 1 || (N % 8) != 0 || (K % 8) != 0 || !bm || !bn) return BT_ERR_INVALID_ARG;
  if (act != BT_ACT_NONE && act != BT_ACT_GELU_ERF && act != BT_ACT_GELU_TANH) return BT_ERR_INVALID_ARG;
  *bm = *bn = 64;  // the register-staged fallback kernel: K not a multiple of 64, or shorter than the pipeline
  if ((K % 64) != 0) return BT_OK;
  const int c = bt::gemm_tile_choice(M, N, K, act, bt::EPI_PLAIN);
  const bt::GemmTile& t = bt::kGemmTiles[c];
  if (K / 64 < (c < 2 ? 3 : 4) - 1) return BT_OK;  // stages of that shape: 3 for the two widest, else 4
  *bm = t.bm;
  *bn = t.bn;
  return BT_OK;
}
