// Padding-free encoder layer (Fig. 2(c)) and the stack of layers (Sec. IV-E):
// a host-side sequence of launches on the caller's stream, no synchronisation.
//
// Plain pipeline (7 launches per layer):
//   GEMM0 (+bias) -> varlen MHA -> GEMM1 -> bias+residual+LN
//   -> GEMM2 (+bias, GELU in the epilogue) -> GEMM3 -> bias+residual+LN
//
// Folded pipeline (bt_encoder_fwd with fold vectors, 5 launches per layer): the add-bias + residual
// of Sec. III-C1 moves into the epilogue of GEMM1 / GEMM3, which also stores partial row sums of
// the LayerNorm input and writes u = gamma (.) z; the normalisation itself moves into the epilogue
// of the GEMM that consumes the LayerNorm output (GEMM2, next layer's GEMM0) through
//   LN(z) W^T + b = rstd (u W^T - mu c) + d,   c = W gamma,  d = W beta + b,
// and the residual branches rebuild LN(z) = rstd (u - mu gamma) + beta on the fly.  One explicit
// normalisation remains, at the end of the stack.
#include <atomic>

#include "common.h"

namespace bt {
bt_status gemm_dispatch(const bt_half* A, const bt_half* W, int M, int N, int K, bt_act act, int epi,
                        const GemmEpi& ep, bt_half* C, hipStream_t st, int* np_out);
bt_status layernorm_dispatch(const bt_half* x, const float* xpart, int nsplit, const bt_half* bias,
                             const bt_half* residual, const bt_half* gamma, const bt_half* beta, float eps, int T,
                             int H, bt_half* y, hipStream_t st, const int32_t* res_rows, const int32_t* out_idx,
                             int out_rows);
int gemm_splitk_choice(int M, int N, int K);
bt_status gemm_splitk_dispatch(const bt_half* A, const bt_half* W, int M, int N, int K, int ksplit, float* partial,
                               hipStream_t st);
// slices * M * N of any split gemm_splitk_choice allows: at most 256 tiles of 64 x 64 outputs
constexpr size_t kSplitKFloats = (size_t)256 * 64 * 64;
bt_status ln_finalize_dispatch(const bt_half* u, const float2* part, int np, const bt_half* gamma,
                               const bt_half* beta, float eps, int T, int H, bt_half* y, hipStream_t st,
                               const int32_t* out_idx, int out_rows);
bt_status fold_vectors_dispatch(const bt_half* W, const bt_half* gamma, const bt_half* beta, const bt_half* bias,
                                int N, int K, float* c, float* d, hipStream_t st);
bt_status mha_dispatch(const bt_half* q, const bt_half* k, const bt_half* v, int64_t row_stride, const bt_half* bq,
                       const bt_half* bk, const bt_half* bv, const int32_t* cu, int B, int T, int max_len, int heads,
                       float scale, bt_half* out, hipStream_t st);

static inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
static inline const half_t* hp(const bt_half* p) { return reinterpret_cast<const half_t*>(p); }

// Workspace layout for T tokens (every region 256-byte aligned):
//   qkv [T,3H] | attn [T,H] | proj [T,H] (GEMM1 and GEMM3 output) | y1 [T,H] | g [T,F] | ping [T,H] |
//   pong [T,H] | part1 [T, H/64] float2 | part2 [T, H/64] float2   (partial row sums of the two LayerNorms;
//   a column tile of the producing GEMM is at least 64 wide, so H/64 slots per row always suffice)
//   | splitk fp32 [kSplitKFloats]   (K slices of GEMM1 / GEMM3 when the token count is small)
struct Workspace {
  bt_half *qkv, *attn, *proj, *y1, *g, *ping, *pong;
  float2 *part1, *part2;
  float* splitk;
  size_t bytes;
};
static inline size_t part_slots(int H) { return (size_t)(H + 63) / 64; }

static Workspace carve(void* ws, int T, int H, int F) {
  Workspace w;
  uintptr_t base = reinterpret_cast<uintptr_t>(ws);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* r = reinterpret_cast<void*>(base + off);
    off += align256(bytes);
    return r;
  };
  const size_t t = (size_t)T;
  w.qkv = static_cast<bt_half*>(take(t * 3 * H * 2));
  w.attn = static_cast<bt_half*>(take(t * H * 2));
  w.proj = static_cast<bt_half*>(take(t * H * 2));
  w.y1 = static_cast<bt_half*>(take(t * H * 2));
  w.g = static_cast<bt_half*>(take(t * F * 2));
  w.ping = static_cast<bt_half*>(take(t * H * 2));
  w.pong = static_cast<bt_half*>(take(t * H * 2));
  w.part1 = static_cast<float2*>(take(t * part_slots(H) * sizeof(float2)));
  w.part2 = static_cast<float2*>(take(t * part_slots(H) * sizeof(float2)));
  w.splitk = static_cast<float*>(take(kSplitKFloats * sizeof(float)));
  w.bytes = off;
  return w;
}

// Fold vectors of one layer: [c_qkv (3H) | d_qkv (3H) | c_1 (F) | d_1 (F)] fp32.
static inline size_t fold_floats(int H, int F) { return (size_t)6 * H + (size_t)2 * F; }

static bt_status check_layer(const bt_layer* l) {
  if (!l) return BT_ERR_INVALID_ARG;
  if (l->H < 8 || l->heads < 1 || l->head_dim < 1 || l->F < 8 || !(l->ln_eps >= 0.f)) return BT_ERR_INVALID_ARG;
  if (l->gelu_kind != 0 && l->gelu_kind != 1) return BT_ERR_INVALID_ARG;
  if (l->head_dim != BT_HEAD_DIM || l->H != l->heads * l->head_dim || (l->F % 8) != 0 || l->H > 8192)
    return BT_ERR_UNSUPPORTED;
  const void* ptrs[] = {l->w_qkv, l->b_qkv, l->w_o, l->b_o, l->ln0_g, l->ln0_b,
                        l->w_1,   l->b_1,   l->w_2, l->b_2, l->ln1_g, l->ln1_b};
  for (const void* p : ptrs)
    if (!p || !aligned16(p)) return BT_ERR_INVALID_ARG;
  return BT_OK;
}

static bt_status check_stack(const bt_layer* layers, int n_layers) {
  if (!layers || n_layers < 1) return BT_ERR_INVALID_ARG;
  for (int i = 0; i < n_layers; ++i) {
    bt_status s = check_layer(&layers[i]);
    if (s != BT_OK) return s;
    if (layers[i].H != layers[0].H || layers[i].F != layers[0].F || layers[i].heads != layers[0].heads ||
        layers[i].ln_eps != layers[0].ln_eps)
      return BT_ERR_INVALID_ARG;
  }
  return BT_OK;
}

// Where a layer's input rows come from and where its output rows go.  Defaults: packed in, packed out.
struct LayerIo {
  const int32_t* in_rows = nullptr;   // x is the PADDED tensor; packed row i is its row in_rows[i] (first layer)
  const int32_t* out_idx = nullptr;   // y is the PADDED tensor [out_rows, H]; packed row i goes to row out_idx[i],
  int out_rows = 0;                   // every other row is zero-filled (last layer)
};

static bt_status layer_fwd(const bt_layer* l, const bt_half* x, const int32_t* cu, int B, int T, int max_len,
                           bt_half* y, const Workspace& w, hipStream_t st, const LayerIo& io = LayerIo()) {
  const int H = l->H, F = l->F;
  bt_status s;
  GemmEpi ep;
  ep.a_rows = io.in_rows;
  ep.bias = hp(l->b_qkv);
  if ((s = gemm_dispatch(x, l->w_qkv, T, 3 * H, H, BT_ACT_NONE, EPI_PLAIN, ep, w.qkv, st, nullptr)) != BT_OK) return s;
  const float scale = 1.0f / sqrtf((float)l->head_dim);
  if ((s = mha_dispatch(w.qkv, w.qkv + H, w.qkv + 2 * H, 3 * (int64_t)H, nullptr, nullptr, nullptr, cu, B, T,
                        max_len, l->heads, scale, w.attn, st)) != BT_OK)
    return s;
  ep.a_rows = nullptr;
  ep.bias = nullptr;
  // Output projection and FFN-down: with few tokens the K loop is split over otherwise idle compute
  // units and the LayerNorm kernel adds the fp32 slices (no reduction kernel, no fp16 rounding in between).
  const int split1 = gemm_splitk_choice(T, H, H), split3 = gemm_splitk_choice(T, H, F);
  if (split1 > 1) {
    if ((s = gemm_splitk_dispatch(w.attn, l->w_o, T, H, H, split1, w.splitk, st)) != BT_OK) return s;
    if ((s = layernorm_dispatch(nullptr, w.splitk, split1, l->b_o, x, l->ln0_g, l->ln0_b, l->ln_eps, T, H, w.y1, st,
                                io.in_rows, nullptr, 0)) != BT_OK)
      return s;
  } else {
    if ((s = gemm_dispatch(w.attn, l->w_o, T, H, H, BT_ACT_NONE, EPI_PLAIN, ep, w.proj, st, nullptr)) != BT_OK) return s;
    if ((s = layernorm_dispatch(w.proj, nullptr, 0, l->b_o, x, l->ln0_g, l->ln0_b, l->ln_eps, T, H, w.y1, st,
                                io.in_rows, nullptr, 0)) != BT_OK)
      return s;
  }
  const bt_act act = l->gelu_kind == 0 ? BT_ACT_GELU_ERF : BT_ACT_GELU_TANH;
  ep.bias = hp(l->b_1);
  if ((s = gemm_dispatch(w.y1, l->w_1, T, F, H, act, EPI_PLAIN, ep, w.g, st, nullptr)) != BT_OK) return s;
  ep.bias = nullptr;
  if (split3 > 1) {
    if ((s = gemm_splitk_dispatch(w.g, l->w_2, T, H, F, split3, w.splitk, st)) != BT_OK) return s;
    return layernorm_dispatch(nullptr, w.splitk, split3, l->b_2, w.y1, l->ln1_g, l->ln1_b, l->ln_eps, T, H, y, st, nullptr,
                              io.out_idx, io.out_rows);
  }
  if ((s = gemm_dispatch(w.g, l->w_2, T, H, F, BT_ACT_NONE, EPI_PLAIN, ep, w.proj, st, nullptr)) != BT_OK) return s;
  return layernorm_dispatch(w.proj, nullptr, 0, l->b_2, w.y1, l->ln1_g, l->ln1_b, l->ln_eps, T, H, y, st, nullptr,
                            io.out_idx, io.out_rows);
}

// Folded stack.  Between layers the activation lives as (u2 = gamma1 (.) z2, part2); inside a layer
// as (u1 = gamma0 (.) z1, part1).  Each part buffer is rewritten in full by the GEMM that produces it
// (one slot per row and producing wavefront), after its last reader has run: nothing to clear.
// io: with in_rows, x is the padded tensor and packed row i is its row in_rows[i] (gathered by the first GEMM's
// operand load and by the first residual read); with out_idx, y is the padded tensor and the final
// normalisation scatters its rows there and zero-fills the rest.
static bt_status stack_fwd_folded(const bt_layer* layers, int n_layers, const float* fold, const bt_half* x,
                                  const int32_t* cu, int B, int T, int max_len, bt_half* y, const Workspace& w,
                                  hipStream_t st, const LayerIo& io = LayerIo()) {
  const int H = layers[0].H, F = layers[0].F;
  const float inv_h = 1.0f / (float)H, eps = layers[0].ln_eps;
  const float scale = 1.0f / sqrtf((float)layers[0].head_dim);
  const size_t per_layer = fold_floats(H, F);
  bt_status s;
  const bt_half* in = x;  // layer input: plain x for layer 0, u2 of the previous layer afterwards
  int np1 = 0, np2 = 0;   // partial sums per row in part1 (LN0 of this layer) / part2 (LN1 of the previous layer)
  for (int i = 0; i < n_layers; ++i) {
    const bt_layer* l = &layers[i];
    const bt_layer* prev = i > 0 ? &layers[i - 1] : nullptr;
    const float* fv = fold + (size_t)i * per_layer;
    bt_half* u2 = (i & 1) ? w.pong : w.ping;
    {  // GEMM0: QKV projection of LN1_{i-1}(z2) (folded) or of the plain input
      GemmEpi ep;
      if (prev) {
        ep.ln_part = w.part2; ep.ln_np = np2; ep.fold_c = fv; ep.fold_d = fv + 3 * H; ep.inv_h = inv_h; ep.eps = eps;
      } else {
        ep.bias = hp(l->b_qkv);
        ep.a_rows = io.in_rows;
      }
      if ((s = gemm_dispatch(in, l->w_qkv, T, 3 * H, H, BT_ACT_NONE, prev ? EPI_FOLD : EPI_PLAIN, ep, w.qkv, st,
                             nullptr)) != BT_OK)
        return s;
    }
    if ((s = mha_dispatch(w.qkv, w.qkv + H, w.qkv + 2 * H, 3 * (int64_t)H, nullptr, nullptr, nullptr, cu, B, T,
                          max_len, l->heads, scale, w.attn, st)) != BT_OK)
      return s;
    {  // GEMM1: z1 = attn W_o^T + b_o + layer input;  u1 = gamma0 (.) z1, part1 = partial row sums of z1
      GemmEpi ep;
      ep.bias = hp(l->b_o); ep.inv_h = inv_h; ep.eps = eps;
      ep.resid = hp(in);
      if (prev) {
        ep.resid_part = w.part2; ep.resid_np = np2; ep.resid_gamma = hp(prev->ln1_g); ep.resid_beta = hp(prev->ln1_b);
      } else {
        ep.resid_rows = io.in_rows;
      }
      ep.out_gamma = hp(l->ln0_g); ep.part_out = w.part1;
      if ((s = gemm_dispatch(w.attn, l->w_o, T, H, H, BT_ACT_NONE, EPI_RESID, ep, w.y1, st, &np1)) != BT_OK) return s;
    }
    {  // GEMM2: GELU(LN0(z1) W_1^T + b_1), LayerNorm folded
      GemmEpi ep;
      ep.ln_part = w.part1; ep.ln_np = np1; ep.fold_c = fv + 6 * H; ep.fold_d = fv + 6 * H + F;
      ep.inv_h = inv_h; ep.eps = eps;
      const bt_act act = l->gelu_kind == 0 ? BT_ACT_GELU_ERF : BT_ACT_GELU_TANH;
      if ((s = gemm_dispatch(w.y1, l->w_1, T, F, H, act, EPI_FOLD, ep, w.g, st, nullptr)) != BT_OK) return s;
    }
    {  // GEMM3: z2 = g W_2^T + b_2 + LN0(z1);  u2 = gamma1 (.) z2, part2 = partial row sums of z2
      GemmEpi ep;
      ep.bias = hp(l->b_2); ep.inv_h = inv_h; ep.eps = eps;
      ep.resid = hp(w.y1); ep.resid_part = w.part1; ep.resid_np = np1;
      ep.resid_gamma = hp(l->ln0_g); ep.resid_beta = hp(l->ln0_b);
      ep.out_gamma = hp(l->ln1_g); ep.part_out = w.part2;
      if ((s = gemm_dispatch(w.g, l->w_2, T, H, F, BT_ACT_NONE, EPI_RESID, ep, u2, st, &np2)) != BT_OK) return s;
    }
    in = u2;
  }
  const bt_layer* last = &layers[n_layers - 1];
  return ln_finalize_dispatch(in, w.part2, np2, last->ln1_g, last->ln1_b, eps, T, H, y, st, io.out_idx, io.out_rows);
}

// Whether the folded pipeline is the faster one for T tokens (hidden width H, FFN width F).  Its residual
// epilogue exists for the small tile shapes only (64 x 128 for the H-wide products); as long as those tiles fit
// one round of the 256 compute units the two launches saved per layer win, beyond that the small tiles run in
// several rounds and the plain 7-launch layer with its larger tiles is faster (measured: -4 % from 1 280 to
// 2 560 tokens of width 768, -3 % at 2 048 tokens of width 1024; +7 ... +18 % beyond 5 400 tokens).  With so few tokens that the plain layer splits K of its
// H-wide products, the plain layer wins again (the folded epilogue has no split-K form: +1.5 % at 186 tokens).
static bool folded_pays(int T, int H, int F) {
  if ((long long)((T + 63) / 64) * ((H + 127) / 128) > 256) return false;
  return gemm_splitk_choice(T, H, F) == 1 && gemm_splitk_choice(T, H, H) == 1;
}

static bt_status check_io(const bt_half* x, const int32_t* cu, int B, int T, int max_len, bt_half* y, void* ws) {
  if (B < 0 || T < 0 || max_len < 0) return BT_ERR_INVALID_ARG;
  if (B == 0 || T == 0) return BT_OK;
  if (max_len < 1 || (int64_t)T > (int64_t)B * max_len) return BT_ERR_INVALID_ARG;
  if (!x || !cu || !y || x == y || !aligned16(x) || !aligned16(y)) return BT_ERR_INVALID_ARG;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return BT_ERR_WORKSPACE;
  return BT_OK;
}

}  // namespace bt

// Workspace of bt_encoder_layer_fwd_static: one array per GPU, created when the code object is loaded on
// that GPU and held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress -- it is NOT a device address and is never passed to a kernel or a memory call.
static __device__ __align__(256) unsigned char scratch[BT_STATIC_SCRATCH_BYTES];

namespace bt {
// Device address of `scratch` on each GPU, resolved once per device on the first call made with that
// device current (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static bt_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return BT_ERR_HIP;
  }
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return BT_ERR_HIP;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // racing first calls resolve the same address
  }
  *out = p;
  return BT_OK;
}
}  // namespace bt

using namespace bt;

extern "C" const char* bt_status_string(bt_status s) {
  switch (s) {
    case BT_OK: return "ok";
    case BT_ERR_INVALID_ARG: return "invalid argument";
    case BT_ERR_UNSUPPORTED: return "unsupported shape";
    case BT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case BT_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

extern "C" size_t bt_layer_workspace_bytes(const bt_layer* layer, int T, int B, int max_len) {
  (void)B;
  (void)max_len;
  if (!layer || T <= 0 || layer->H < 1 || layer->F < 1) return 0;
  return carve(nullptr, T, layer->H, layer->F).bytes;
}

extern "C" bt_status bt_encoder_layer_fwd(const bt_layer* layer, const bt_half* d_x, const int32_t* d_cu_seqlens,
                                          int B, int T, int max_len, bt_half* d_y, void* d_ws, size_t ws_bytes,
                                          bt_stream stream) {
  bt_status s = check_layer(layer);
  if (s != BT_OK) return s;
  if ((s = check_io(d_x, d_cu_seqlens, B, T, max_len, d_y, d_ws)) != BT_OK) return s;
  if (B == 0 || T == 0) return BT_OK;
  const Workspace w = carve(d_ws, T, layer->H, layer->F);
  if (ws_bytes < w.bytes) return BT_ERR_WORKSPACE;
  return layer_fwd(layer, d_x, d_cu_seqlens, B, T, max_len, d_y, w, static_cast<hipStream_t>(stream));
}

extern "C" bt_status bt_encoder_layer_fwd_static(const bt_layer* layer, const bt_half* d_x,
                                                 const int32_t* d_cu_seqlens, int B, int T, int max_len,
                                                 bt_half* d_y, bt_stream stream) {
  bt_status s = check_layer(layer);
  if (s != BT_OK) return s;
  // any non-null 256-byte aligned value passes the workspace checks; the real address is resolved below
  if ((s = check_io(d_x, d_cu_seqlens, B, T, max_len, d_y, reinterpret_cast<void*>(uintptr_t(256)))) != BT_OK) return s;
  if (B == 0 || T == 0) return BT_OK;
  if (carve(nullptr, T, layer->H, layer->F).bytes > (size_t)BT_STATIC_SCRATCH_BYTES) return BT_ERR_WORKSPACE;
  void* ws = nullptr;
  if ((s = static_scratch(&ws)) != BT_OK) return s;
  const Workspace w = carve(ws, T, layer->H, layer->F);
  return layer_fwd(layer, d_x, d_cu_seqlens, B, T, max_len, d_y, w, static_cast<hipStream_t>(stream));
}

extern "C" size_t bt_encoder_fold_bytes(const bt_layer* layers, int n_layers) {
  if (!layers || n_layers < 1 || layers[0].H < 1 || layers[0].F < 1) return 0;
  return (size_t)n_layers * fold_floats(layers[0].H, layers[0].F) * sizeof(float);
}

extern "C" bt_status bt_encoder_prepare(const bt_layer* layers, int n_layers, float* d_fold, size_t fold_bytes,
                                        bt_stream stream) {
  bt_status s = check_stack(layers, n_layers);
  if (s != BT_OK) return s;
  if (!d_fold || (reinterpret_cast<uintptr_t>(d_fold) & 15u)) return BT_ERR_INVALID_ARG;
  if (fold_bytes < bt_encoder_fold_bytes(layers, n_layers)) return BT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int H = layers[0].H, F = layers[0].F;
  const size_t per_layer = fold_floats(H, F);
  for (int i = 0; i < n_layers; ++i) {
    float* fv = d_fold + (size_t)i * per_layer;
    const bt_layer* l = &layers[i];
    if (i > 0) {  // layer 0 reads a plain input: its c_qkv / d_qkv stay unused
      const bt_layer* p = &layers[i - 1];
      if ((s = fold_vectors_dispatch(l->w_qkv, p->ln1_g, p->ln1_b, l->b_qkv, 3 * H, H, fv, fv + 3 * H, st)) != BT_OK)
        return s;
    }
    if ((s = fold_vectors_dispatch(l->w_1, l->ln0_g, l->ln0_b, l->b_1, F, H, fv + 6 * H, fv + 6 * H + F, st)) != BT_OK)
      return s;
  }
  return BT_OK;
}

extern "C" bt_status bt_encoder_fwd(const bt_layer* layers, int n_layers, const float* d_fold, const bt_half* d_x,
                                    const int32_t* d_cu_seqlens, int B, int T, int max_len, bt_half* d_y, void* d_ws,
                                    size_t ws_bytes, bt_stream stream) {
  bt_status s = check_stack(layers, n_layers);
  if (s != BT_OK) return s;
  if ((s = check_io(d_x, d_cu_seqlens, B, T, max_len, d_y, d_ws)) != BT_OK) return s;
  if (d_fold && (reinterpret_cast<uintptr_t>(d_fold) & 15u)) return BT_ERR_INVALID_ARG;
  if (B == 0 || T == 0) return BT_OK;
  const Workspace w = carve(d_ws, T, layers[0].H, layers[0].F);
  if (ws_bytes < w.bytes) return BT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (d_fold && folded_pays(T, layers[0].H, layers[0].F))
    return stack_fwd_folded(layers, n_layers, d_fold, d_x, d_cu_seqlens, B, T, max_len, d_y, w, st);
  const bt_half* in = d_x;
  for (int i = 0; i < n_layers; ++i) {
    bt_half* outp = (i == n_layers - 1) ? d_y : ((i & 1) ? w.pong : w.ping);
    if ((s = layer_fwd(&layers[i], in, d_cu_seqlens, B, T, max_len, outp, w, st)) != BT_OK) return s;
    in = outp;
  }
  return BT_OK;
}

extern "C" bt_status bt_encoder_fwd_padded(const bt_layer* layers, int n_layers, const float* d_fold,
                                           const bt_half* d_x_padded, const int32_t* d_token_idx,
                                           const int32_t* d_cu_seqlens, int B, int T, int S, bt_half* d_y_padded,
                                           void* d_ws, size_t ws_bytes, bt_stream stream) {
  bt_status s = check_stack(layers, n_layers);
  if (s != BT_OK) return s;
  if (B < 0 || T < 0 || S < 0) return BT_ERR_INVALID_ARG;
  if (d_fold && (reinterpret_cast<uintptr_t>(d_fold) & 15u)) return BT_ERR_INVALID_ARG;
  if (B == 0 || S == 0) return BT_OK;
  if ((int64_t)T > (int64_t)B * S || (int64_t)B * S >= (int64_t)INT32_MAX) return BT_ERR_INVALID_ARG;
  if (!d_x_padded || !d_y_padded || d_x_padded == d_y_padded || !aligned16(d_x_padded) || !aligned16(d_y_padded))
    return BT_ERR_INVALID_ARG;
  if (T > 0 && (!d_token_idx || !d_cu_seqlens)) return BT_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int H = layers[0].H;
  if (T == 0)  // nothing valid: the output is all padding (the unpack kernel zero-fills; no memset node for graphs)
    return bt_unpack(d_x_padded, d_token_idx, 0, B, S, H, d_y_padded, stream);
  if (!d_ws || (reinterpret_cast<uintptr_t>(d_ws) & 255u)) return BT_ERR_WORKSPACE;
  const Workspace w = carve(d_ws, T, H, layers[0].F);
  if (ws_bytes < w.bytes) return BT_ERR_WORKSPACE;
  if (d_fold && folded_pays(T, H, layers[0].F)) {
    LayerIo io;
    io.in_rows = d_token_idx;
    io.out_idx = d_token_idx;
    io.out_rows = B * S;
    return stack_fwd_folded(layers, n_layers, d_fold, d_x_padded, d_cu_seqlens, B, T, S, d_y_padded, w, st, io);
  }
  const bt_half* in = d_x_padded;
  for (int i = 0; i < n_layers; ++i) {
    const bool last = i == n_layers - 1;
    LayerIo io;
    if (i == 0) io.in_rows = d_token_idx;
    if (last) { io.out_idx = d_token_idx; io.out_rows = B * S; }
    bt_half* outp = last ? d_y_padded : ((i & 1) ? w.pong : w.ping);
    if ((s = layer_fwd(&layers[i], in, d_cu_seqlens, B, T, S, outp, w, st, io)) != BT_OK) return s;
    in = outp;
  }
  return BT_OK;
}

// bt_build_offsets followed by bt_encoder_fwd_padded in one call: the token count the first call waits for
// goes straight into the launches of the second, with no host code of the caller in between (while the host
// holds the count and has not launched yet, the device is idle).
extern "C" bt_status bt_encoder_fwd_masked(const bt_layer* layers, int n_layers, const float* d_fold,
                                           const bt_half* d_x_padded, const int32_t* d_mask,
                                           const int32_t* d_lengths, int B, int S, int32_t* d_cu_seqlens,
                                           int32_t* d_token_idx, int32_t* h_total, bt_half* d_y_padded, void* d_ws,
                                           size_t ws_bytes, bt_stream stream) {
  // everything that can be refused is refused before the prefix-sum kernel runs
  bt_status s = check_stack(layers, n_layers);
  if (s != BT_OK) return s;
  if (d_fold && (reinterpret_cast<uintptr_t>(d_fold) & 15u)) return BT_ERR_INVALID_ARG;
  if (B > 0 && S > 0) {
    if (!d_x_padded || !d_y_padded || d_x_padded == d_y_padded || !aligned16(d_x_padded) || !aligned16(d_y_padded))
      return BT_ERR_INVALID_ARG;
    if ((int64_t)B * S >= (int64_t)INT32_MAX) return BT_ERR_UNSUPPORTED;
    if (!d_ws || (reinterpret_cast<uintptr_t>(d_ws) & 255u)) return BT_ERR_WORKSPACE;
    if (ws_bytes < carve(d_ws, B * S, layers[0].H, layers[0].F).bytes) return BT_ERR_WORKSPACE;  // any count fits
  }
  if ((s = bt_build_offsets(d_mask, d_lengths, B, S, d_cu_seqlens, d_token_idx, h_total, stream)) != BT_OK) return s;
  return bt_encoder_fwd_padded(layers, n_layers, d_fold, d_x_padded, d_token_idx, d_cu_seqlens, B, h_total[0], S,
                               d_y_padded, d_ws, ws_bytes, stream);
}

