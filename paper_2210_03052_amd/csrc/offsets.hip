// Zero-padding algorithm (Sec. III-D, Fig. 4): prefix sum of the mask matrix,
// position array, pack and unpack.  Integer / byte work: bit-exact.
#include <chrono>

#include "common.h"

namespace bt {

constexpr int kOffsetsThreads = 1024;  // 16 wavefronts, one per sentence at a time

// One workgroup.  Wave w owns sentences w, w+16, ...  (the paper assigns one
// warp per sentence inside one threadblock; same decomposition, 64-wide).
//   phase 1: per-sentence valid count (ballot + popcount) -> cu[b+1]
//   phase 2: wave 0 turns the counts into an inclusive scan, cu[0] = 0
//   phase 3: per sentence, ballot/mbcnt ranks every valid token and writes
//            token_idx[cu[b] + rank] = b*S + t
// A length outside [0,S] or a mask entry outside {0,1} sets cu[B] = -1.
// host_total (optional): device-visible host memory that receives the total (or -1) as soon as it
// is known, before the position array is written, so that the host can go on without a stream sync.
// max_out (optional): device word that receives the largest per-sentence valid count; with host_total
// it is also stored to host_total[1], before the total, so that a host that sees the total sees it too.
__global__ __launch_bounds__(kOffsetsThreads) void offsets_kernel(const int32_t* __restrict__ mask,
                                                                 const int32_t* __restrict__ lengths, int B, int S,
                                                                 int32_t* __restrict__ cu,
                                                                 int32_t* __restrict__ token_idx,
                                                                 int32_t* host_total, int32_t* max_out) {
  __shared__ int s_bad, s_max;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwave = kOffsetsThreads / kWave;
  if (threadIdx.x == 0) { s_bad = 0; s_max = 0; }
  __syncthreads();

  for (int b = wave; b < B; b += nwave) {
    int count = 0, bad = 0;
    if (mask) {
      for (int t0 = 0; t0 < S; t0 += kWave) {
        const int t = t0 + lane;
        const int m = t < S ? mask[(size_t)b * S + t] : 0;
        bad |= (m != 0 && m != 1);
        count += __popcll(__ballot(m != 0));
      }
      bad = __any(bad);
    } else {
      count = lengths[b];
      bad = count < 0 || count > S;
      if (bad) count = 0;
    }
    if (lane == 0) {
      cu[b + 1] = count;
      if (bad) s_bad = 1;
      atomicMax(&s_max, count);
    }
  }
  __syncthreads();

  if (wave == 0) {
    int running = 0;
    for (int b0 = 0; b0 < B; b0 += kWave) {
      const int b = b0 + lane;
      int v = b < B ? cu[b + 1] : 0;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const int u = __shfl_up(v, o, kWave);
        if (lane >= o) v += u;
      }
      if (b < B) cu[b + 1] = running + v;
      running += __shfl(v, kWave - 1, kWave);
    }
    if (lane == 0) cu[0] = 0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (max_out) *max_out = s_max;
    if (host_total) {
      if (max_out) __hip_atomic_store(host_total + 1, s_max, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(host_total, s_bad ? -1 : cu[B], __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }

  for (int b = wave; b < B; b += nwave) {
    const int base = cu[b];
    const int len = mask ? 0 : (cu[b + 1] - base);
    int running = 0;
    for (int t0 = 0; t0 < S; t0 += kWave) {
      const int t = t0 + lane;
      const bool valid = t < S && (mask ? mask[(size_t)b * S + t] != 0 : t < len);
      const unsigned long long bal = __ballot(valid);
      const int rank = __popcll(bal & ((1ull << lane) - 1ull));
      if (valid) token_idx[base + running + rank] = b * S + t;
      running += __popcll(bal);
      if (!mask && t0 + kWave >= len) break;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && s_bad) cu[B] = -1;
}

// One 16-byte chunk per thread; a row of H halves is H/8 consecutive threads.
__global__ __launch_bounds__(256) void pack_kernel(const uint4_t* __restrict__ padded,
                                                   const int32_t* __restrict__ token_idx, size_t total, int chunks,
                                                   uint4_t* __restrict__ packed) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const size_t tok = i / chunks;
  const int c = (int)(i - tok * chunks);
  packed[i] = padded[(size_t)token_idx[tok] * chunks + c];
}

// One wavefront per padded row.  The row is valid iff it occurs in the strictly
// increasing token_idx; a uniform binary search finds its packed position.
__global__ __launch_bounds__(256) void unpack_kernel(const uint4_t* __restrict__ packed,
                                                     const int32_t* __restrict__ token_idx, int T, int rows,
                                                     int chunks, uint4_t* __restrict__ padded) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  int lo = 0, hi = T;  // first position with token_idx[pos] >= r
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (token_idx[mid] < r) lo = mid + 1; else hi = mid;
  }
  const bool valid = lo < T && token_idx[lo] == r;
  const uint4_t zero = {0u, 0u, 0u, 0u};
  for (int c = lane; c < chunks; c += kWave)
    padded[(size_t)r * chunks + c] = valid ? packed[(size_t)lo * chunks + c] : zero;
}

}  // namespace bt

using namespace bt;

// Shared body of bt_build_offsets / bt_build_offsets_stats.  h_out[0] receives the total; with `stats`
// h_out[1] receives the largest per-sentence count and d_cu_seqlens has B+2 entries (the last one is
// the device copy of that maximum).
static bt_status build_offsets_impl(const int32_t* d_mask, const int32_t* d_lengths, int B, int S,
                                    int32_t* d_cu_seqlens, int32_t* d_token_idx, int32_t* h_out, bool stats,
                                    bt_stream stream) {
  if ((d_mask == nullptr) == (d_lengths == nullptr)) return BT_ERR_INVALID_ARG;
  if (!d_cu_seqlens || !d_token_idx || !h_out || B < 0 || S < 1) return BT_ERR_INVALID_ARG;
  if (S > BT_MAX_SEQ || (int64_t)B * S >= (int64_t)INT32_MAX) return BT_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // The call waits for a result on the host: it cannot be recorded into a HIP graph.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cap) != hipSuccess) {
    (void)hipGetLastError();
    return BT_ERR_HIP;
  }
  if (cap != hipStreamCaptureStatusNone) return BT_ERR_UNSUPPORTED;
  // Fast path: h_out lies in pinned host memory that the device can write (hipHostMalloc).  The
  // kernel stores the total there the moment it is known and the host polls for it: no copy, no
  // stream synchronisation, and later launches on the stream are ordered after the kernel anyway.
  hipPointerAttribute_t attr;
  int32_t* h_dev = nullptr;
  if (hipPointerGetAttributes(&attr, h_out) == hipSuccess && attr.type == hipMemoryTypeHost && attr.devicePointer)
    h_dev = static_cast<int32_t*>(attr.devicePointer);
  else
    (void)hipGetLastError();  // ordinary host memory: not an error
  constexpr int32_t kPending = INT32_MIN;
  volatile int32_t* slot = h_out;
  if (h_dev) *slot = kPending;
  // B == 0 runs the same kernel: it writes cu[0] = 0 and a total of 0 (no memset, no special case)
  offsets_kernel<<<1, kOffsetsThreads, 0, st>>>(d_mask, d_lengths, B, S, d_cu_seqlens, d_token_idx, h_dev,
                                                stats ? d_cu_seqlens + B + 1 : nullptr);
  if (hipGetLastError() != hipSuccess) return BT_ERR_HIP;
  int32_t res[2] = {kPending, 0};
  if (h_dev) {
    const auto t0 = std::chrono::steady_clock::now();
    for (long spin = 0; (res[0] = slot[0]) == kPending; ++spin) {
      if ((spin & 1023) == 1023 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(200)) break;
      __builtin_ia32_pause();
    }
    if (res[0] != kPending && stats) {
      __atomic_thread_fence(__ATOMIC_ACQUIRE);  // the maximum was stored before the total
      res[1] = slot[1];
    }
  }
  if (res[0] == kPending) {  // pageable h_out, or the store has not shown up: copy and synchronise
    if (hipMemcpyAsync(res, d_cu_seqlens + B, (stats ? 2 : 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st) !=
        hipSuccess)
      return BT_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return BT_ERR_HIP;
  }
  h_out[0] = res[0] < 0 ? 0 : res[0];
  if (stats) h_out[1] = res[0] < 0 ? 0 : res[1];
  return res[0] < 0 ? BT_ERR_INVALID_ARG : BT_OK;
}

extern "C" bt_status bt_build_offsets(const int32_t* d_mask, const int32_t* d_lengths, int B, int S,
                                      int32_t* d_cu_seqlens, int32_t* d_token_idx, int32_t* h_total,
                                      bt_stream stream) {
  return build_offsets_impl(d_mask, d_lengths, B, S, d_cu_seqlens, d_token_idx, h_total, false, stream);
}

extern "C" bt_status bt_build_offsets_stats(const int32_t* d_mask, const int32_t* d_lengths, int B, int S,
                                            int32_t* d_cu_seqlens, int32_t* d_token_idx, int32_t* h_total_max,
                                            bt_stream stream) {
  return build_offsets_impl(d_mask, d_lengths, B, S, d_cu_seqlens, d_token_idx, h_total_max, true, stream);
}

extern "C" bt_status bt_pack(const bt_half* d_padded, const int32_t* d_token_idx, int T, int H,
                             bt_half* d_packed, bt_stream stream) {
  if (T < 0 || H < 8 || (H % 8) != 0) return BT_ERR_INVALID_ARG;
  if (T == 0) return BT_OK;
  if (!d_padded || !d_token_idx || !d_packed || !aligned16(d_padded) || !aligned16(d_packed))
    return BT_ERR_INVALID_ARG;
  const int chunks = H / 8;
  const size_t total = (size_t)T * chunks;
  const size_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffull) return BT_ERR_UNSUPPORTED;
  pack_kernel<<<(unsigned)blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(
      reinterpret_cast<const uint4_t*>(d_padded), d_token_idx, total, chunks, reinterpret_cast<uint4_t*>(d_packed));
  return launch_status();
}

extern "C" bt_status bt_unpack(const bt_half* d_packed, const int32_t* d_token_idx, int T, int B, int S, int H,
                               bt_half* d_padded, bt_stream stream) {
  if (T < 0 || B < 0 || S < 1 || H < 8 || (H % 8) != 0) return BT_ERR_INVALID_ARG;
  if ((int64_t)B * S >= (int64_t)INT32_MAX) return BT_ERR_UNSUPPORTED;
  if ((int64_t)T > (int64_t)B * S) return BT_ERR_INVALID_ARG;
  if (B == 0) return BT_OK;
  if (!d_padded || !aligned16(d_padded)) return BT_ERR_INVALID_ARG;
  if (T > 0 && (!d_packed || !d_token_idx || !aligned16(d_packed))) return BT_ERR_INVALID_ARG;
  const int rows = B * S;
  unpack_kernel<<<(rows + 3) / 4, 256, 0, static_cast<hipStream_t>(stream)>>>(
      reinterpret_cast<const uint4_t*>(d_packed), d_token_idx, T, rows, H / 8, reinterpret_cast<uint4_t*>(d_padded));
  return launch_status();
}
