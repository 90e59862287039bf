// Padding-free encoder layer (Fig. 2(c)) and the stack of layers (Sec. IV-E):
// a host-side sequence of launches on the caller's stream, no synchronisation.
//   GEMM0 (+bias) -> varlen MHA -> GEMM1 -> bias+residual+LN
//   -> GEMM2 (+bias, GELU in the epilogue) -> GEMM3 -> bias+residual+LN
#include "common.h"

namespace bt {
bt_status gemm_dispatch(const bt_half* A, const bt_half* W, const bt_half* bias, int M, int N, int K, bt_act act,
                        bt_half* C, hipStream_t st);
bt_status layernorm_dispatch(const bt_half* x, const bt_half* bias, const bt_half* residual, const bt_half* gamma,
                             const bt_half* beta, float eps, int T, int H, bt_half* y, hipStream_t st);
bt_status mha_dispatch(const bt_half* q, const bt_half* k, const bt_half* v, int64_t row_stride, const bt_half* bq,
                       const bt_half* bk, const bt_half* bv, const int32_t* cu, int B, int T, int max_len, int heads,
                       float scale, bt_half* out, hipStream_t st);

static inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// Workspace layout for T tokens (every region 256-byte aligned):
//   qkv [T,3H] | attn [T,H] | proj [T,H] (GEMM1 and GEMM3 output) | y1 [T,H] | g [T,F] | ping [T,H] | pong [T,H]
struct Workspace {
  bt_half *qkv, *attn, *proj, *y1, *g, *ping, *pong;
  size_t bytes;
};

static Workspace carve(void* ws, int T, int H, int F) {
  Workspace w;
  char* p = static_cast<char*>(ws);
  size_t off = 0;
  auto take = [&](size_t halves) {
    bt_half* r = reinterpret_cast<bt_half*>(p + off);
    off += align256(halves * sizeof(bt_half));
    return r;
  };
  const size_t t = (size_t)T;
  w.qkv = take(t * 3 * H);
  w.attn = take(t * H);
  w.proj = take(t * H);
  w.y1 = take(t * H);
  w.g = take(t * F);
  w.ping = take(t * H);
  w.pong = take(t * H);
  w.bytes = off;
  return w;
}

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

static bt_status layer_fwd(const bt_layer* l, const bt_half* x, const int32_t* cu, int B, int T, int max_len,
                           bt_half* y, const Workspace& w, hipStream_t st) {
  const int H = l->H, F = l->F;
  bt_status s;
  if ((s = gemm_dispatch(x, l->w_qkv, l->b_qkv, T, 3 * H, H, BT_ACT_NONE, w.qkv, st)) != BT_OK) return s;
  const float scale = 1.0f / sqrtf((float)l->head_dim);
  if ((s = mha_dispatch(w.qkv, w.qkv + H, w.qkv + 2 * H, 3 * (int64_t)H, nullptr, nullptr, nullptr, cu, B, T,
                        max_len, l->heads, scale, w.attn, st)) != BT_OK)
    return s;
  if ((s = gemm_dispatch(w.attn, l->w_o, nullptr, T, H, H, BT_ACT_NONE, w.proj, st)) != BT_OK) return s;
  if ((s = layernorm_dispatch(w.proj, l->b_o, x, l->ln0_g, l->ln0_b, l->ln_eps, T, H, w.y1, st)) != BT_OK) return s;
  const bt_act act = l->gelu_kind == 0 ? BT_ACT_GELU_ERF : BT_ACT_GELU_TANH;
  if ((s = gemm_dispatch(w.y1, l->w_1, l->b_1, T, F, H, act, w.g, st)) != BT_OK) return s;
  if ((s = gemm_dispatch(w.g, l->w_2, nullptr, T, H, F, BT_ACT_NONE, w.proj, st)) != BT_OK) return s;
  return layernorm_dispatch(w.proj, l->b_2, w.y1, l->ln1_g, l->ln1_b, l->ln_eps, T, H, y, st);
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

extern "C" bt_status bt_encoder_fwd(const bt_layer* layers, int n_layers, const bt_half* d_x,
                                    const int32_t* d_cu_seqlens, int B, int T, int max_len, bt_half* d_y, void* d_ws,
                                    size_t ws_bytes, bt_stream stream) {
  if (!layers || n_layers < 1) return BT_ERR_INVALID_ARG;
  bt_status s;
  for (int i = 0; i < n_layers; ++i) {
    if ((s = check_layer(&layers[i])) != BT_OK) return s;
    if (layers[i].H != layers[0].H || layers[i].F != layers[0].F || layers[i].heads != layers[0].heads)
      return BT_ERR_INVALID_ARG;
  }
  if ((s = check_io(d_x, d_cu_seqlens, B, T, max_len, d_y, d_ws)) != BT_OK) return s;
  if (B == 0 || T == 0) return BT_OK;
  const Workspace w = carve(d_ws, T, layers[0].H, layers[0].F);
  if (ws_bytes < w.bytes) return BT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bt_half* in = d_x;
  for (int i = 0; i < n_layers; ++i) {
    bt_half* outp = (i == n_layers - 1) ? d_y : ((i & 1) ? w.pong : w.ping);
    if ((s = layer_fwd(&layers[i], in, d_cu_seqlens, B, T, max_len, outp, w, st)) != BT_OK) return s;
    in = outp;
  }
  return BT_OK;
}
