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
//   O^T[d][q]  += V^T[d][key] * P^T[key][q] A operand = V^T fragment, B = P
// In both accumulators a lane owns ONE query column (q = lane % 32), so the row
// maximum, the rescale factor and the row sum are per-lane scalars, and the
// fp32 S^T accumulator registers of a lane are -- after exp and conversion to
// fp16 -- directly the B operand of the second product (the key order inside a
// 16-key step is permuted identically on the V side, which a sum allows).
//
// K and V tiles travel global memory -> LDS by DMA (global_load_lds_dwordx4), NS
// tiles deep, both row-major with the 16-byte chunks XOR-swizzled on the global
// side.  K fragments are plain 128-bit LDS reads; V^T fragments come from the
// transposing LDS read of gfx950 (ds_read_b64_tr_b16), so V is never transposed
// in memory.  Biases: b_q is added to the Q registers; b_k shifts every logit of
// a row by the same amount and cancels in the softmax; b_v is added to the
// output (the probabilities of a row sum to one).
#include "common.h"

namespace bt {

constexpr int kD = BT_HEAD_DIM;  // 64
constexpr int kKT = 64;          // keys per tile

#define BT_AS3 __attribute__((address_space(3)))
typedef __fp16 fp16x4_t __attribute__((__vector_size__(4 * sizeof(__fp16))));  // operand type of the tr16 builtin

__device__ __forceinline__ void mha_dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr)
               : "memory", "m0");
}
// The same DMA with the address split into a wave-uniform base (SGPR pair) and a per-lane 32-bit byte offset:
// walking the key tiles of a sequence then only moves the scalar base, no vector arithmetic per tile.
__device__ __forceinline__ void mha_dma16_sv(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase)
               : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void mha_wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Per-lane constants of the LDS fragment reads.
struct FragAddr {
  int k_rd, swz_k;        // K: row l32, 16-byte chunk (2ks+hf) ^ swz_k
  int v_row, v_c, v_in;   // V: transposing read, see process_tile
  int hf;
};
__device__ __forceinline__ FragAddr make_frag_addr(int lane) {
  FragAddr f;
  const int l32 = lane & 31;
  f.hf = lane >> 5;
  f.k_rd = l32 * kD;
  f.swz_k = (l32 >> 1) & 7;
  // 16-lane group g = lane>>4 covers d = 16*(g&1)..+15 and keys 4*hf..+3 of an 8-key half step;
  // lane j of the group points at key row j>>2, d offset 4*(j&3).
  const int vj = lane & 15, vg = (lane >> 4) & 1;
  f.v_row = 4 * f.hf + (vj >> 2);
  f.v_c = vg * 2 + ((vj & 3) >> 1);
  f.v_in = 4 * (vj & 1);
  return f;
}

// One 64-key tile for the 32 query rows of a wavefront, step by step:  S^T = K Q^T (qk_tile);  mask of a
// ragged last tile;  running maximum and rescale (softmax_max);  P = exp2(S - m), row sums, fp16 P
// (softmax_exp);  O^T += V^T P^T (pv_tile).
__device__ __forceinline__ void qk_tile(const half_t* sk, const half8_t (&qf)[4], const FragAddr& fa,
                                        float16_t (&s)[2]) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const half8_t a =
          *reinterpret_cast<const half8_t*>(sk + fa.k_rd + kb * 32 * kD + (((2 * ks + fa.hf) ^ fa.swz_k) * 8));
      s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qf[ks], s[kb], 0, 0, 0);
    }
  }
}

// Keys past the end of the sequence drop out (only the last tile of a sequence can hold any).
__device__ __forceinline__ void mask_ragged(float16_t (&s)[2], int k0, int L, int hf) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = k0 + kb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      if (key >= L) s[kb][r] = -INFINITY;
    }
}

// x of lane l and of lane l ^ 32 as (value of the lower half, value of the upper half), the same pair in both
// lanes: the cross-half lane swap of gfx950, a VALU operation (no trip through the LDS queue).
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);  // {lo,lo} and {hi,hi} of the halves
  lo = __builtin_bit_cast(float, (unsigned)sw[0]);
  hi = __builtin_bit_cast(float, (unsigned)sw[1]);
}

// m_run is kept in the scaled log2 domain and is only raised when the tile maximum exceeds it by
// more than 8 (a factor 256: probabilities stay <= 256, exact in fp16/fp32 terms), so the rescale
// of the accumulators is skipped for most tiles; any reference maximum gives the same softmax.
__device__ __forceinline__ void softmax_max(const float16_t (&s)[2], float scale_log2e, float& m_run, float& l_run,
                                            float16_t (&o_acc)[2]) {
  // four independent chains, then the exchange between the two 32-lane halves by the lane-swap
  // instruction of gfx950 (a VALU operation: no trip through the LDS queue behind the fragment reads)
  float c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float16_t& t = s[j >> 1];
    const int o = 8 * (j & 1);
    float m = fmaxf(fmaxf(t[o], t[o + 1]), t[o + 2]);  // three-operand maxima
    m = fmaxf(fmaxf(m, t[o + 3]), t[o + 4]);
    m = fmaxf(fmaxf(m, t[o + 5]), t[o + 6]);
    c[j] = fmaxf(m, t[o + 7]);
  }
  float mx = fmaxf(fmaxf(fmaxf(c[0], c[1]), c[2]), c[3]);
  {
    float lo, hi;
    both_halves(mx, lo, hi);
    mx = fmaxf(lo, hi);
  }
  const float mx_s = mx * scale_log2e;            // finite: every tile holds at least one valid key
  const bool raise = mx_s > m_run + 8.0f;         // same in both halves of a query column
  if (__builtin_amdgcn_ballot_w64(raise)) {
    const float m_new = raise ? mx_s : m_run;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
  }
}

__device__ __forceinline__ void softmax_exp(const float16_t (&s)[2], float scale_log2e, float m_run, float& l_run,
                                            half8_t (&pf)[2][2]) {
  // The row sum is taken over the fp16 probabilities, the values the second product multiplies, two per
  // instruction (dot product with (1, 1), fp32 accumulate) instead of one fp32 add per probability.
  typedef __fp16 fp16x2_t __attribute__((ext_vector_type(2)));
  const fp16x2_t ones = {(__fp16)1.0f, (__fp16)1.0f};
  float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r], scale_log2e, -m_run));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r + 1], scale_log2e, -m_run));
      const half2_t h = {(half_t)p0, (half_t)p1};
      pf[kb][r >> 3][r & 7] = h[0];
      pf[kb][r >> 3][(r & 7) + 1] = h[1];
      if (kb == 0) psum0 = __builtin_amdgcn_fdot2(__builtin_bit_cast(fp16x2_t, h), ones, psum0, false);
      else psum1 = __builtin_amdgcn_fdot2(__builtin_bit_cast(fp16x2_t, h), ones, psum1, false);
    }
  l_run += psum0 + psum1;
}

// O^T += V^T P^T ; 16-key step ks covers S^T registers 8*(ks%2)..+7 of block ks/2, i.e. keys
// 16ks + {0..3, 8..11} + 4hf, the order the two transposing reads deliver.
__device__ __forceinline__ void pv_tile(const half_t* sv, const FragAddr& fa, const half8_t (&pf)[2][2],
                                        float16_t (&o_acc)[2]) {
#pragma unroll
  for (int db = 0; db < 2; ++db) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      half8_t a;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int row = 16 * ks + 8 * t + fa.v_row;
        const int chunk = (4 * db + fa.v_c) ^ (((row >> 1) & 1) << 2);
        const half4_t x = __builtin_bit_cast(
            half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4f16((BT_AS3 fp16x4_t*)(sv + row * kD + chunk * 8 + fa.v_in)));
#pragma unroll
        for (int e = 0; e < 4; ++e) a[4 * t + e] = x[e];
      }
      o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pf[ks >> 1][ks & 1], o_acc[db], 0, 0, 0);
    }
  }
}

__device__ __forceinline__ void process_tile(const half_t* sk, const half_t* sv, const half8_t (&qf)[4], int k0, int L,
                                             float scale_log2e, const FragAddr& fa, float& m_run, float& l_run,
                                             float16_t (&o_acc)[2]) {
  float16_t s[2];
  qk_tile(sk, qf, fa, s);
  if (k0 + kKT > L) mask_ragged(s, k0, L, fa.hf);  // wave-uniform
  softmax_max(s, scale_log2e, m_run, l_run, o_acc);
  half8_t pf[2][2];
  softmax_exp(s, scale_log2e, m_run, l_run, pf);
  pv_tile(sv, fa, pf, o_acc);
}

// Locate the (sequence, q-tile) a workgroup owns.  Results are wave-uniform (readfirstlane).
// Up to 64 sequences: workgroups are ordered longest sequence first (by q-tile count, ties by index),
// so the workgroups that walk the most key tiles start first and short ones fill the tail -- the
// work list is never materialised, every wave derives its entry from cu_seqlens with ballots.
// More than 64 sequences: plain sequence order, prefix sum of per-sequence tile counts, 64 at a time.
// Tile counts come from cu_seqlens alone (never from the caller's max_len), so every row of every
// sequence has an owner as long as the grid holds sum ceil(L_b / BQ) <= T / BQ + B workgroups per head.
__device__ __forceinline__ bool locate_tile(const int32_t* __restrict__ cu, int B, int BQ, int qtile, int lane,
                                            int& tok0, int& L, int& qt) {
  if (B <= kWave) {
    const int start = lane < B ? cu[lane] : 0;
    const int len = lane < B ? cu[lane + 1] - start : 0;
    const int nt = (len + BQ - 1) / BQ;
    const int vmax = wave_max(nt);  // largest tile count present: where the walk over the groups starts
    const unsigned long long below = (1ull << lane) - 1ull;
    int running = 0;
    for (int v = vmax; v >= 1; --v) {
      const unsigned long long grp = __ballot(nt == v);  // sequences with exactly v q-tiles
      const int c = __popcll(grp);
      if (qtile < running + c * v) {
        const int idx = qtile - running;
        const int j = idx / v;  // j-th sequence of the group, its q-tile idx % v
        const unsigned long long me = __ballot(nt == v && __popcll(grp & below) == j);
        const int src = __ffsll((long long)me) - 1;  // wave-uniform
        tok0 = __builtin_amdgcn_readlane(start, src);
        L = __builtin_amdgcn_readlane(len, src);
        qt = idx - j * v;
        return true;
      }
      running += c * v;
    }
    return false;
  }
  int running = 0;
  for (int b0 = 0; b0 < B; b0 += kWave) {
    const int b = b0 + lane;
    const int start = b < B ? cu[b] : 0;
    const int len = b < B ? cu[b + 1] - start : 0;
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
      const int src = __ffsll((long long)hit) - 1;  // wave-uniform
      tok0 = __builtin_amdgcn_readlane(start, src);
      L = __builtin_amdgcn_readlane(len, src);
      qt = qtile - __builtin_amdgcn_readlane(excl, src);
      return true;
    }
    running += __builtin_amdgcn_readlane(incl, kWave - 1);
  }
  return false;
}

template <int NW, int NS>
__global__ __launch_bounds__(NW * 64) void varlen_mha_kernel(
    // in the order of first use: the first 14 dwords are preloaded into SGPRs at wave launch
    const int32_t* __restrict__ cu, int B, int heads, float scale_log2e, const half_t* __restrict__ Q,
    const half_t* __restrict__ K, const half_t* __restrict__ V, int64_t row_stride, half_t* __restrict__ out,
    const half_t* __restrict__ bq, const half_t* __restrict__ bv) {
  constexpr int BQ = NW * 32;
  constexpr int TILE = kKT * kD;            // halves per K (or V) tile
  constexpr int PER = 8 / NW;               // DMA instructions per wave per operand tile (8 rows each)
  constexpr int TOT = 2 * PER;              // ... per stage
  static_assert(NW == 1 || NW == 2 || NW == 4, "NW");

  __shared__ __attribute__((aligned(1024))) half_t sK[NS * TILE];
  __shared__ __attribute__((aligned(1024))) half_t sV[NS * TILE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int head = blockIdx.x % heads;
  const int qtile = blockIdx.x / heads;

  int tok0 = 0, L = 0, qt = -1;
  if (!locate_tile(cu, B, BQ, qtile, lane, tok0, L, qt)) return;  // same decision in every wave

  const int q0 = qt * BQ;
  const int hofs = head * kD;
  const bool wave_active = q0 + wave * 32 < L;
  const int ntiles = (L + kKT - 1) / kKT;

  // ---- Q fragments (B operand of S^T): rows q0 + wave*32 + l32, halves ks*16 + hf*8 ..+7
  const int q_row = q0 + wave * 32 + l32;
  half8_t qf[4];
  {
    const half_t* qp = Q + (size_t)(tok0 + min(q_row, L - 1)) * row_stride + hofs + hf * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[ks] = *reinterpret_cast<const half8_t*>(qp + ks * 16);
  }

  // ---- DMA of K/V tiles.  Instruction p of this wave fills LDS rows [8*(wave*PER+p), +8) of the
  // tile; lane i lands at row r = 8*(..) + i/8, physical chunk i%8, and fetches the logical chunk
  //   K: (i%8) ^ ((r>>1)&7)      (128-bit reads of 16 consecutive rows stay conflict-free)
  //   V: (i%8) ^ (4*((r>>1)&1))  (the 4-row x 64-byte windows of the transposing read do)
  const half_t* kbase = K + (size_t)tok0 * row_stride + hofs;
  const half_t* vbase = V + (size_t)tok0 * row_stride + hofs;
  int k_chunk[PER], v_chunk[PER], t_row[PER];
  uint32_t k_off[PER], v_off[PER];  // byte offsets of this lane's 16 bytes inside a tile that lies fully inside the sequence
#pragma unroll
  for (int p = 0; p < PER; ++p) {
    const int r = (wave * PER + p) * 8 + (lane >> 3);
    t_row[p] = r;
    k_chunk[p] = ((lane & 7) ^ ((r >> 1) & 7)) * 8;
    v_chunk[p] = ((lane & 7) ^ (((r >> 1) & 1) << 2)) * 8;
    k_off[p] = (uint32_t)(((int64_t)r * row_stride + k_chunk[p]) * 2);  // < 64 rows x row pitch: fits 32 bits (checked by the host)
    v_off[p] = (uint32_t)(((int64_t)r * row_stride + v_chunk[p]) * 2);
  }
  const uint32_t lds_k = (uint32_t)(uintptr_t)(BT_AS3 const void*)sK + wave * PER * 1024;
  const uint32_t lds_v = (uint32_t)(uintptr_t)(BT_AS3 const void*)sV + wave * PER * 1024;
  const int64_t tile_pitch = (int64_t)kKT * row_stride;  // elements between consecutive key tiles
  auto issue_tile = [&](int kt, int stage) {
    if ((kt + 1) * kKT <= L) {  // wave-uniform: the whole tile lies inside the sequence -> scalar base, fixed lane offsets
      const half_t* kb_ = kbase + kt * tile_pitch;
      const half_t* vb_ = vbase + kt * tile_pitch;
#pragma unroll
      for (int p = 0; p < PER; ++p) {
        mha_dma16_sv(kb_, k_off[p], lds_k + stage * (TILE * 2) + p * 1024);
        mha_dma16_sv(vb_, v_off[p], lds_v + stage * (TILE * 2) + p * 1024);
      }
    } else {
#pragma unroll
      for (int p = 0; p < PER; ++p) {
        const size_t row = (size_t)min(kt * kKT + t_row[p], L - 1) * row_stride;  // rows past L: clamped, masked later
        mha_dma16(kbase + row + k_chunk[p], lds_k + stage * (TILE * 2) + p * 1024);
        mha_dma16(vbase + row + v_chunk[p], lds_v + stage * (TILE * 2) + p * 1024);
      }
    }
  };
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < ntiles) issue_tile(s, s);

  if (bq) {
    half8_t b8[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) b8[ks] = *reinterpret_cast<const half8_t*>(bq + hofs + ks * 16 + hf * 8);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[ks][e] = (half_t)((float)qf[ks][e] + (float)b8[ks][e]);
  }
  // The Q loads must be complete BEFORE the tile loop.  Left to the compiler, their s_waitcnt vmcnt(3..0)
  // land at the first use inside the loop body and are executed by every iteration, where the only
  // loads in flight are the K/V DMA of the next tile just issued: each iteration would wait for its own
  // prefetch.  A use of the registers here moves the wait out of the loop.
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(qf[ks]));

  float16_t o_acc[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;  // per query column; l_run is this half's partial sum

  const FragAddr fa = make_frag_addr(lane);

  int stage = 0;
  for (int kt = 0; kt < ntiles; ++kt) {
    {  // tile kt landed (at most min(ntiles-1-kt, NS-2) younger tiles in flight) and is published
      const int younger = min(ntiles - 1 - kt, NS - 2);
      if (NS >= 4 && younger >= 2) mha_wait_vmcnt<(NS >= 4 ? 2 : 0) * TOT>();
      else if (NS >= 3 && younger == 1) mha_wait_vmcnt<(NS >= 3 ? 1 : 0) * TOT>();
      else mha_wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
    }
    if (kt + NS - 1 < ntiles) issue_tile(kt + NS - 1, stage == 0 ? NS - 1 : stage - 1);
    const int k0 = kt * kKT;

    if (wave_active)
      process_tile(sK + stage * TILE, sV + stage * TILE, qf, k0, L, scale_log2e, fa, m_run, l_run, o_acc);
    stage = stage + 1 == NS ? 0 : stage + 1;
  }

  // Output.  A lane holds 4 consecutive values of one row per register group, so stored directly a
  // row leaves in 8-byte pieces (16 per 128-byte head slice); instead the 32 x 64 block of a wavefront
  // is transposed through LDS (the K/V stages are free once every wave has left the loop) and leaves
  // as whole 128-byte rows, 16 bytes per lane, written through the L2 like the GEMM tiles.
  constexpr int OLD = kD + 8;  // row pitch of the staged block, halves
  __builtin_amdgcn_s_barrier();
  half_t* ostage = ((wave & 2) ? sV : sK) + (wave & 1) * (32 * OLD);
  static_assert(2 * 32 * OLD <= NS * TILE, "two staged blocks fit one operand ring");
  if (wave_active) {
    float l_lo, l_hi;
    both_halves(l_run, l_lo, l_hi);
    const float inv = 1.0f / (l_lo + l_hi);
    // the value bias, all eight pieces requested together (one round trip, and only when there is a bias)
    half4_t bias4[2][4];
    if (bv) {
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) bias4[db][g] = *reinterpret_cast<const half4_t*>(bv + hofs + db * 32 + 8 * g + 4 * hf);
    } else {
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) bias4[db][g] = half4_t{(half_t)0.f, (half_t)0.f, (half_t)0.f, (half_t)0.f};
    }
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        half4_t o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = (half_t)(o_acc[db][4 * g + t] * inv + (float)bias4[db][g][t]);
        *reinterpret_cast<half4_t*>(ostage + l32 * OLD + db * 32 + 8 * g + 4 * hf) = o;
      }
    // same wavefront reads what it wrote: LDS operations of a wave complete in order
    const int rr = lane >> 3, cc = (lane & 7) * 8;
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += 8) {
      const int q = q0 + wave * 32 + r0 + rr;
      const uint4_t v = *reinterpret_cast<const uint4_t*>(ostage + (r0 + rr) * OLD + cc);
      if (q < L) store_through(out + (size_t)(tok0 + q) * (heads * kD) + hofs + cc, v);
    }
  }
}

// ---------------------------------------------------------------------------
// Split-key variant for short sequences / small batches.  The q-parallel kernel
// above gives one wavefront 32 query rows and ALL keys of the sequence, so with
// few, short sequences there are about as many wavefronts as SIMDs and each one
// walks its tiles serially.  Here a workgroup owns 32 query rows and its NK
// wavefronts split the key tiles (wave w takes tiles w, w+NK, ...), each with a
// private LDS ring and no barrier in the loop; the NK partial results
// (running max, sum, unnormalised O) are merged through LDS at the end, which is
// the same rescaling the online softmax applies between tiles.
// ---------------------------------------------------------------------------
template <int NK, int NS>
__global__ __launch_bounds__(NK * 64) void varlen_mha_splitkey_kernel(
    // in the order of first use: the first 14 dwords are preloaded into SGPRs at wave launch
    const int32_t* __restrict__ cu, int B, int heads, float scale_log2e, const half_t* __restrict__ Q,
    const half_t* __restrict__ K, const half_t* __restrict__ V, int64_t row_stride, half_t* __restrict__ out,
    const half_t* __restrict__ bq, const half_t* __restrict__ bv) {
  constexpr int BQ = 32;
  constexpr int TILE = kKT * kD;       // halves per K (or V) tile
  constexpr int WAVE_LDS = NS * 2 * TILE;  // halves per wave: NS x (K tile + V tile), >= 8 KB + 256 B for the merge
  constexpr int TOT = 16;              // DMA instructions per tile pair
  static_assert((NS - 1) * TOT < 64, "vmcnt range");

  __shared__ __attribute__((aligned(1024))) half_t smem[NK * WAVE_LDS];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int head = blockIdx.x % heads;
  const int qtile = blockIdx.x / heads;

  int tok0 = 0, L = 0, qt = -1;
  if (!locate_tile(cu, B, BQ, qtile, lane, tok0, L, qt)) return;  // same decision in every wave

  const int q0 = qt * BQ;
  const int hofs = head * kD;
  const int ntiles = (L + kKT - 1) / kKT;
  const int my_tiles = wave < ntiles ? (ntiles - wave + NK - 1) / NK : 0;  // tiles wave, wave+NK, ...

  const int q_row = q0 + l32;
  half8_t qf[4];
  {
    const half_t* qp = Q + (size_t)(tok0 + min(q_row, L - 1)) * row_stride + hofs + hf * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[ks] = *reinterpret_cast<const half8_t*>(qp + ks * 16);
  }

  const half_t* kbase = K + (size_t)tok0 * row_stride + hofs;
  const half_t* vbase = V + (size_t)tok0 * row_stride + hofs;
  half_t* my_lds = smem + wave * WAVE_LDS;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(BT_AS3 const void*)my_lds;
  auto issue_tile = [&](int kt, int stage) {  // this wave alone fetches all 64 rows of both tiles
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int r = p * 8 + (lane >> 3);
      const size_t row = (size_t)min(kt * kKT + r, L - 1) * row_stride;
      const int kc = ((lane & 7) ^ ((r >> 1) & 7)) * 8;
      const int vc = ((lane & 7) ^ (((r >> 1) & 1) << 2)) * 8;
      mha_dma16(kbase + row + kc, lds_base + stage * (2 * TILE * 2) + p * 1024);
      mha_dma16(vbase + row + vc, lds_base + stage * (2 * TILE * 2) + TILE * 2 + p * 1024);
    }
  };
#pragma unroll
  for (int s = 0; s < (NS > 1 ? NS - 1 : 1); ++s)
    if (s < my_tiles) issue_tile(wave + s * NK, s);

  if (bq) {
    half8_t b8[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) b8[ks] = *reinterpret_cast<const half8_t*>(bq + hofs + ks * 16 + hf * 8);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[ks][e] = (half_t)((float)qf[ks][e] + (float)b8[ks][e]);
  }
  // The Q loads must be complete BEFORE the tile loop.  Left to the compiler, their s_waitcnt vmcnt(3..0)
  // land at the first use inside the loop body and are executed by every iteration, where the only
  // loads in flight are the K/V DMA of the next tile just issued: each iteration would wait for its own
  // prefetch.  A use of the registers here moves the wait out of the loop.
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) asm volatile("" : "+v"(qf[ks]));

  float16_t o_acc[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const FragAddr fa = make_frag_addr(lane);

  int stage = 0;
  for (int it = 0; it < my_tiles; ++it) {
    const int kt = wave + it * NK;
    if (NS == 1) {
      if (it > 0) issue_tile(kt, 0);  // single buffer: fetch, then wait (tile 0 was issued above)
      mha_wait_vmcnt<0>();
    } else {
      const int younger = min(my_tiles - 1 - it, NS - 2);
      if (NS >= 4 && younger >= 2) mha_wait_vmcnt<(NS >= 4 ? 2 : 0) * TOT>();
      else if (NS >= 3 && younger == 1) mha_wait_vmcnt<(NS >= 3 ? 1 : 0) * TOT>();
      else mha_wait_vmcnt<0>();
      // the stage refilled now was read in iteration it-1; those reads completed before its MFMAs issued
      if (it + NS - 1 < my_tiles) issue_tile(kt + (NS - 1) * NK, stage == 0 ? NS - 1 : stage - 1);
    }
    const int k0 = kt * kKT;
    process_tile(my_lds + stage * (2 * TILE), my_lds + stage * (2 * TILE) + TILE, qf, k0, L, scale_log2e, fa, m_run,
                 l_run, o_acc);
    if (NS > 1) stage = stage + 1 == NS ? 0 : stage + 1;
  }

  // ---- merge the NK partial results.  Each wave parks (O^T fp32 [64 d][32 q], m[32], l[32]) in its
  // own LDS ring (all of its tile reads are complete), one barrier, then wave w finishes d-slice w.
  float* po = reinterpret_cast<float*>(my_lds);   // 8 KB
  float* pm = po + kD * 32;                       // 128 B
  float* pl = pm + 32;                            // 128 B
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) po[(db * 32 + 8 * (r >> 2) + 4 * hf + (r & 3)) * 32 + l32] = o_acc[db][r];
  float l_lo, l_hi;
  both_halves(l_run, l_lo, l_hi);
  const float l_tot = l_lo + l_hi;
  if (hf == 0) {
    pm[l32] = m_run;
    pl[l32] = l_tot;
  }
  __syncthreads();
  constexpr int DW = kD / NK;   // d values finished by one wave (16 or 32)
  constexpr int DL = DW / 2;    // ... by one lane (8 or 16), contiguous
  float mw[NK], lw[NK], M = -INFINITY;
#pragma unroll
  for (int w = 0; w < NK; ++w) {
    const float* base = reinterpret_cast<const float*>(smem + w * WAVE_LDS);
    mw[w] = base[kD * 32 + l32];
    lw[w] = base[kD * 32 + 32 + l32];
    M = fmaxf(M, mw[w]);
  }
  float denom = 0.f, sc[NK];
#pragma unroll
  for (int w = 0; w < NK; ++w) {
    sc[w] = __builtin_amdgcn_exp2f(mw[w] - M);  // a wave without tiles has m = -inf: weight 0
    denom += sc[w] * lw[w];
  }
  const float inv = 1.0f / denom;
  const int d0 = wave * DW + hf * DL;
  float o[DL];
#pragma unroll
  for (int i = 0; i < DL; ++i) o[i] = 0.f;
#pragma unroll
  for (int w = 0; w < NK; ++w) {
    const float* base = reinterpret_cast<const float*>(smem + w * WAVE_LDS);
#pragma unroll
    for (int i = 0; i < DL; ++i) o[i] += sc[w] * base[(d0 + i) * 32 + l32];
  }
  if (q_row < L) {
    half_t* op = out + (size_t)(tok0 + q_row) * (heads * kD) + hofs + d0;
    half8_t b8[DL / 8];  // the value bias, requested in one go
#pragma unroll
    for (int c = 0; c < DL / 8; ++c) {
      if (bv) b8[c] = *reinterpret_cast<const half8_t*>(bv + hofs + d0 + c * 8);
      else
#pragma unroll
        for (int e = 0; e < 8; ++e) b8[c][e] = (half_t)0.f;
    }
#pragma unroll
    for (int c = 0; c < DL / 8; ++c) {
      half8_t h8;
#pragma unroll
      for (int e = 0; e < 8; ++e) h8[e] = (half_t)(o[c * 8 + e] * inv + (float)b8[c][e]);
      *reinterpret_cast<half8_t*>(op + c * 8) = h8;
    }
  }
}

template <int NK, int NS>
static bt_status launch_mha_splitkey(const half_t* q, const half_t* k, const half_t* v, int64_t row_stride,
                                     const half_t* bq, const half_t* bv, const int32_t* cu, int B, int T, int max_len,
                                     int heads, float scale, half_t* out, hipStream_t st) {
  constexpr int BQ = 32;
  // q-tiles: sum ceil(L_b/BQ) <= floor(T/BQ) + B, a bound that holds whatever the lengths are (the caller's
  // max_len is only a hint for the choice of kernel: a sequence longer than it is still computed in full)
  const long long blocks = ((long long)T / BQ + B) * heads;
  if (blocks > 0x7fffffffLL) return BT_ERR_UNSUPPORTED;
  varlen_mha_splitkey_kernel<NK, NS><<<(unsigned)blocks, NK * 64, 0, st>>>(
      cu, B, heads, scale * 1.4426950408889634f, q, k, v, row_stride, out, bq, bv);
  return launch_status();
}

template <int NW, int NS>
static bt_status launch_mha(const half_t* q, const half_t* k, const half_t* v, int64_t row_stride, const half_t* bq,
                            const half_t* bv, const int32_t* cu, int B, int T, int max_len, int heads, float scale,
                            half_t* out, hipStream_t st) {
  constexpr int BQ = NW * 32;
  const long long blocks = ((long long)T / BQ + B) * heads;  // see launch_mha_splitkey
  if (blocks > 0x7fffffffLL) return BT_ERR_UNSUPPORTED;
  varlen_mha_kernel<NW, NS><<<(unsigned)blocks, NW * 64, 0, st>>>(
      cu, B, heads, scale * 1.4426950408889634f, q, k, v, row_stride, out, bq, bv);
  return launch_status();
}

bt_status mha_dispatch(const bt_half* q, const bt_half* k, const bt_half* v, int64_t row_stride, const bt_half* bq,
                       const bt_half* bk, const bt_half* bv, const int32_t* cu, int B, int T, int max_len, int heads,
                       float scale, bt_half* out, hipStream_t st) {
  (void)bk;  // adds the same constant to every logit of a row: cancels in the softmax
  auto h = [](const bt_half* p) { return reinterpret_cast<const half_t*>(p); };
  half_t* o = reinterpret_cast<half_t*>(out);
#define BT_MHA_ARGS h(q), h(k), h(v), row_stride, h(bq), h(bv), cu, B, T, max_len, heads, scale, o, st
  // Kernel choice.  Tall query tiles (4 waves x 32 rows) re-read K/V least and start the fewest workgroups
  // (every workgroup pays the search of its work item, the Q load and the first K/V round trip before its
  // first MFMA); they win as soon as there is about one such workgroup per compute unit (measured: 7.7 us
  // against 8.5 us with 2-wave tiles at 16 sequences of up to 256 tokens, 408 workgroups; 39 against 55 us
  // at 16 x up to 1024).  2-wave tiles give more workgroups below that; with too few of those to occupy the
  // SIMDs, the split-key kernel puts two waves on every 32 query rows.  Two K/V stages (32 KB of LDS per
  // workgroup) rather than three: the 120 VGPRs of the kernel allow four waves per SIMD and the third
  // stage would cap residency at three; measured 2-8 % faster from 256 to 1024 keys, never slower.
  auto blocks = [&](int bqt) { return ((long long)T / bqt + B) * heads; };
  if (max_len > 128 && blocks(128) >= 256) return launch_mha<4, 2>(BT_MHA_ARGS);
  if (blocks(64) >= 512) return launch_mha<2, 2>(BT_MHA_ARGS);
  return launch_mha_splitkey<2, 1>(BT_MHA_ARGS);
#undef BT_MHA_ARGS
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
  if (row_stride > (int64_t)1 << 24) return BT_ERR_UNSUPPORTED;  // a 64-row tile is addressed with 32-bit byte offsets
  if (!(scale > 0.f) || !(scale < INFINITY)) return BT_ERR_INVALID_ARG;
  if (B == 0 || T == 0) return BT_OK;
  if (max_len < 1 || (int64_t)T > (int64_t)B * max_len) return BT_ERR_INVALID_ARG;
  if (max_len > BT_MAX_SEQ) return BT_ERR_UNSUPPORTED;
  if (!d_q || !d_k || !d_v || !d_cu_seqlens || !d_out) return BT_ERR_INVALID_ARG;
  if (!bt::aligned16(d_q) || !bt::aligned16(d_k) || !bt::aligned16(d_v) || !bt::aligned16(d_out))
    return BT_ERR_INVALID_ARG;
  if ((d_bq && !bt::aligned16(d_bq)) || (d_bv && !bt::aligned16(d_bv))) return BT_ERR_INVALID_ARG;  // vector loads
  return bt::mha_dispatch(d_q, d_k, d_v, row_stride, d_bq, d_bk, d_bv, d_cu_seqlens, B, T, max_len, heads, scale,
                          d_out, static_cast<hipStream_t>(stream));
}
