// Fused variable-length multi-head attention (eq. (1), Sec. III-E).
//
// One kernel for every sequence length: a workgroup owns one (sequence, head,
// tile of BQ = 32*NW query rows); it walks the sequence's own keys in tiles of
// 64 and keeps the running row maximum / row sum (online softmax), so the
// L x L logit matrix never exists in memory and no padded row or column is
// touched -- the valid range comes from cu_seqlens, the prefix sum of Sec. III-D.
//
// MFMA mapping (32x32x16 fp16, fp32 accumulate), chosen so that softmax needs no
// cross-lane traffic beyond one exchange between the two 32-lane halves:
//   S^T[key][q] = K[key][:] . Q[q][:]      A operand = K tile (LDS), B = Q (registers)
//   O^T[d][q]  += V^T[d][key] * P^T[key][q] A operand = V^T tile (LDS), B = P
// In both accumulators a lane owns ONE query column (q = lane % 32), so the row
// maximum, the rescale factor and the row sum are per-lane scalars, and the
// fp32 S^T accumulator registers of a lane are -- after exp and conversion to
// fp16 -- directly the B operand of the second product (the key order inside a
// 16-key step is permuted identically on the V^T side, which a sum allows).
// K tiles are staged row-major in LDS, V tiles transposed; the next tile is
// prefetched from global memory into registers while the current one is used.
#include "common.h"

namespace bt {

constexpr int kD = BT_HEAD_DIM;   // 64
constexpr int kKT = 64;           // keys per tile
constexpr int kKStride = kD + 8;  // halves per LDS row of the K tile   (144 B)
constexpr int kVStride = kKT + 4; // halves per LDS row of the V^T tile (136 B)

__device__ __forceinline__ half8_t add_bias8(half8_t x, const float* b) {
  half8_t r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (half_t)((float)x[e] + b[e]);
  return r;
}

template <int NW>
__global__ __launch_bounds__(NW * 64) void varlen_mha_kernel(
    const half_t* __restrict__ Q, const half_t* __restrict__ K, const half_t* __restrict__ V, int64_t row_stride,
    const half_t* __restrict__ bq, const half_t* __restrict__ bk, const half_t* __restrict__ bv,
    const int32_t* __restrict__ cu, int B, int heads, float scale_log2e, half_t* __restrict__ out) {
  constexpr int NT = NW * 64;
  constexpr int BQ = NW * 32;
  constexpr int KC = (kKT * 8) / NT;      // 16-byte K chunks per thread per tile
  constexpr int VC = (kKT / 2 * 8) / NT;  // (key pair, chunk) items per thread per tile

  __shared__ __attribute__((aligned(16))) half_t sK[2][kKT * kKStride];
  __shared__ __attribute__((aligned(16))) half_t sV[2][kD * kVStride];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int head = blockIdx.x % heads;
  const int qtile = blockIdx.x / heads;

  // Locate (sequence, q-tile): prefix sum of per-sequence tile counts, 64 at a time.
  int seq = -1, qt = 0;
  {
    int running = 0;
    for (int b0 = 0; b0 < B; b0 += kWave) {
      const int b = b0 + lane;
      const int len = b < B ? cu[b + 1] - cu[b] : 0;
      const int nt = (len + BQ - 1) / BQ;
      int incl = nt;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const int u = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += u;
      }
      const int excl = running + incl - nt;
      const unsigned long long hit = __ballot(qtile >= excl && qtile < excl + nt);
      if (hit) {
        const int src = __ffsll((long long)hit) - 1;
        seq = b0 + src;
        qt = qtile - __shfl(excl, src, kWave);
        break;
      }
      running += __shfl(incl, kWave - 1, kWave);
    }
  }
  if (seq < 0) return;  // same decision in every wave: no barrier is left waiting

  const int tok0 = cu[seq];
  const int L = cu[seq + 1] - tok0;
  const int q0 = qt * BQ;
  const int hofs = head * kD;
  const bool wave_active = q0 + wave * 32 < L;

  // ---- Q fragments (B operand of S^T): rows q0 + wave*32 + l32, halves ks*16 + hf*8 ..+7
  const int q_row = q0 + wave * 32 + l32;
  half8_t qf[4];
  {
    const half_t* qp = Q + (size_t)(tok0 + min(q_row, L - 1)) * row_stride + hofs + hf * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qf[ks] = *reinterpret_cast<const half8_t*>(qp + ks * 16);
      if (bq) {
        float b[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) b[e] = (float)bq[hofs + ks * 16 + hf * 8 + e];
        qf[ks] = add_bias8(qf[ks], b);
      }
    }
  }

  // ---- global -> register staging of one K/V tile
  const int dc = tid & 7;  // 16-byte chunk inside a 64-half row (NT is a multiple of 8)
  float kbias[8], vbias[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    kbias[e] = bk ? (float)bk[hofs + dc * 8 + e] : 0.f;
    vbias[e] = bv ? (float)bv[hofs + dc * 8 + e] : 0.f;
  }
  half8_t rk[KC], rv[VC][2];
  const half_t* kbase = K + (size_t)tok0 * row_stride + hofs + dc * 8;
  const half_t* vbase = V + (size_t)tok0 * row_stride + hofs + dc * 8;
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < KC; ++i) {
      const int key = min(k0 + (tid >> 3) + i * (NT / 8), L - 1);  // rows past L: clamped, masked later
      rk[i] = *reinterpret_cast<const half8_t*>(kbase + (size_t)key * row_stride);
    }
#pragma unroll
    for (int i = 0; i < VC; ++i) {
      const int kp = (tid >> 3) + i * (NT / 8);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int key = min(k0 + 2 * kp + u, L - 1);
        rv[i][u] = *reinterpret_cast<const half8_t*>(vbase + (size_t)key * row_stride);
      }
    }
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < KC; ++i) {
      const int key = (tid >> 3) + i * (NT / 8);
      half8_t x = rk[i];
      if (bk) x = add_bias8(x, kbias);
      *reinterpret_cast<half8_t*>(&sK[buf][key * kKStride + dc * 8]) = x;
    }
#pragma unroll
    for (int i = 0; i < VC; ++i) {
      const int kp = (tid >> 3) + i * (NT / 8);
      half8_t x0 = rv[i][0], x1 = rv[i][1];
      if (bv) {
        x0 = add_bias8(x0, vbias);
        x1 = add_bias8(x1, vbias);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {  // transpose: V^T[d][key], two neighbouring keys per 32-bit write
        half2_t pr;
        pr[0] = x0[e];
        pr[1] = x1[e];
        *reinterpret_cast<half2_t*>(&sV[buf][(dc * 8 + e) * kVStride + 2 * kp]) = pr;
      }
    }
  };

  float16_t o_acc[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;  // per query column; l_run is this half's partial sum

  const int ntiles = (L + kKT - 1) / kKT;
  fetch(0);
  stage(0);
  __syncthreads();

  for (int kt = 0; kt < ntiles; ++kt) {
    const int buf = kt & 1;
    const int k0 = kt * kKT;
    if (kt + 1 < ntiles) fetch(k0 + kKT);

    if (wave_active) {
      // S^T = K Q^T for the two 32-key blocks of the tile
      float16_t s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const half8_t a =
              *reinterpret_cast<const half8_t*>(&sK[buf][(kb * 32 + l32) * kKStride + ks * 16 + hf * 8]);
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qf[ks], s[kb], 0, 0, 0);
        }
      }
      // scale into the log2 domain; mask the keys past the end of the sequence
      const bool ragged = k0 + kKT > L;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float x = s[kb][r] * scale_log2e;
          if (ragged) {
            const int key = k0 + kb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
            if (key >= L) x = -INFINITY;
          }
          s[kb][r] = x;
        }
      float mx = s[0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      const float m_new = fmaxf(m_run, mx);  // finite: every tile holds at least one valid key
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      float psum = 0.f;
      half8_t pf[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(s[kb][r] - m_new);
          psum += p;
          pf[kb][r >> 3][r & 7] = (half_t)p;
        }
      l_run = l_run * alpha + psum;
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
      // O^T += V^T P^T ; 16-key step ks covers S^T registers 8*(ks%2)..+7 of block ks/2,
      // i.e. keys 16ks + {0..3, 8..11} + 4hf, the same order the V^T fragment is read in.
#pragma unroll
      for (int db = 0; db < 2; ++db) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const half_t* vp = &sV[buf][(db * 32 + l32) * kVStride + ks * 16 + 4 * hf];
          const half4_t lo = *reinterpret_cast<const half4_t*>(vp);
          const half4_t hi = *reinterpret_cast<const half4_t*>(vp + 8);
          half8_t a;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a[e] = lo[e];
            a[4 + e] = hi[e];
          }
          o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pf[ks >> 1][ks & 1], o_acc[db], 0, 0, 0);
        }
      }
    }

    if (kt + 1 < ntiles) stage(buf ^ 1);
    __syncthreads();
  }

  if (wave_active && q_row < L) {
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    const float inv = 1.0f / l_tot;
    half_t* op = out + (size_t)(tok0 + q_row) * (heads * kD) + hofs + 4 * hf;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        half4_t o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = (half_t)(o_acc[db][4 * g + t] * inv);
        *reinterpret_cast<half4_t*>(op + db * 32 + 8 * g) = o;
      }
  }
}

template <int NW>
static bt_status launch_mha(const half_t* q, const half_t* k, const half_t* v, int64_t row_stride, const half_t* bq,
                            const half_t* bk, const half_t* bv, const int32_t* cu, int B, int T, int max_len,
                            int heads, float scale, half_t* out, hipStream_t st) {
  constexpr int BQ = NW * 32;
  // number of q-tiles: sum ceil(L_b/BQ) <= min(B*ceil(max_len/BQ), floor(T/BQ) + B)
  const long long by_len = (long long)B * ((max_len + BQ - 1) / BQ);
  const long long by_tok = (long long)T / BQ + B;
  const long long tiles = by_len < by_tok ? by_len : by_tok;
  const long long blocks = tiles * heads;
  if (blocks > 0x7fffffffLL) return BT_ERR_UNSUPPORTED;
  varlen_mha_kernel<NW><<<(unsigned)blocks, NW * 64, 0, st>>>(q, k, v, row_stride, bq, bk, bv, cu, B, heads,
                                                            scale * 1.4426950408889634f, out);
  return launch_status();
}

bt_status mha_dispatch(const bt_half* q, const bt_half* k, const bt_half* v, int64_t row_stride, const bt_half* bq,
                       const bt_half* bk, const bt_half* bv, const int32_t* cu, int B, int T, int max_len, int heads,
                       float scale, bt_half* out, hipStream_t st) {
  auto h = [](const bt_half* p) { return reinterpret_cast<const half_t*>(p); };
  half_t* o = reinterpret_cast<half_t*>(out);
  // Query-tile height: tall tiles re-read K/V less often, short tiles give more
  // workgroups; pick the tallest that still offers ~2 workgroups per compute unit.
  auto blocks = [&](int bqt) { return ((long long)T / bqt + B) * heads; };
  if (max_len > 128 && blocks(128) >= 512)
    return launch_mha<4>(h(q), h(k), h(v), row_stride, h(bq), h(bk), h(bv), cu, B, T, max_len, heads, scale, o, st);
  if (max_len > 32 && blocks(64) >= 512)
    return launch_mha<2>(h(q), h(k), h(v), row_stride, h(bq), h(bk), h(bv), cu, B, T, max_len, heads, scale, o, st);
  return launch_mha<1>(h(q), h(k), h(v), row_stride, h(bq), h(bk), h(bv), cu, B, T, max_len, heads, scale, o, st);
}

}  // namespace bt

extern "C" bt_status bt_varlen_mha(const bt_half* d_q, const bt_half* d_k, const bt_half* d_v, int64_t row_stride,
                                   const bt_half* d_bq, const bt_half* d_bk, const bt_half* d_bv,
                                   const int32_t* d_cu_seqlens, int B, int T, int max_len, int heads, int head_dim,
                                   float scale, bt_half* d_out, void* d_ws, size_t ws_bytes, bt_stream stream) {
  (void)d_ws;
  (void)ws_bytes;
  if (B < 0 || T < 0 || max_len < 0 || heads < 1 || head_dim < 1) return BT_ERR_INVALID_ARG;
  if (head_dim != BT_HEAD_DIM) return BT_ERR_UNSUPPORTED;
  if (row_stride < (int64_t)heads * head_dim || (row_stride % 8) != 0) return BT_ERR_INVALID_ARG;
  if (!(scale > 0.f) || !(scale < INFINITY)) return BT_ERR_INVALID_ARG;
  if (B == 0 || T == 0) return BT_OK;
  if (max_len < 1 || (int64_t)T > (int64_t)B * max_len) return BT_ERR_INVALID_ARG;
  if (!d_q || !d_k || !d_v || !d_cu_seqlens || !d_out) return BT_ERR_INVALID_ARG;
  if (!bt::aligned16(d_q) || !bt::aligned16(d_k) || !bt::aligned16(d_v) || !bt::aligned16(d_out))
    return BT_ERR_INVALID_ARG;
  return bt::mha_dispatch(d_q, d_k, d_v, row_stride, d_bq, d_bk, d_bv, d_cu_seqlens, B, T, max_len, heads, scale,
                          d_out, static_cast<hipStream_t>(stream));
}
