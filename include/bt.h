/*
 * bt.h -- C ABI of the padding-free BERT encoder forward for variable-length
 * batches on AMD MI355X (gfx950).
 *
 * Conventions shared by every entry point
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller
 *     owns all memory; the library never allocates, frees or keeps a pointer.
 *   - fp16 tensors are passed as `const bt_half*` (IEEE binary16 bit patterns),
 *     row-major, innermost dimension contiguous, base address 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it and nothing synchronises, with the one exception
 *     stated at bt_build_offsets.
 *   - Errors are return codes only.  Argument checks happen on the host before
 *     any launch: a call that returns BT_ERR_INVALID_ARG / BT_ERR_UNSUPPORTED /
 *     BT_ERR_WORKSPACE has enqueued nothing -- with one exception, bt_build_offsets
 *     (and its _stats form), which also reports what only the device can see (a bad
 *     length or mask entry) after its kernel has run.  A failed launch gives BT_ERR_HIP.
 *   - T == 0 or B == 0 is a valid no-op (BT_OK, no launch).  A sequence of
 *     length 0 is allowed and contributes nothing.
 *   - Weight matrices are [out_features, in_features] row-major (the reduction
 *     dimension is contiguous), so y = x W^T + b.
 *   - The calls are re-entrant: no global state (one exception, stated at
 *     bt_encoder_layer_fwd_static).
 */
#ifndef BT_H_
#define BT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t bt_half;   /* IEEE binary16 bit pattern */
typedef void*    bt_stream; /* hipStream_t */

typedef enum {
  BT_OK = 0,
  BT_ERR_INVALID_ARG = 1, /* null / misaligned pointer, negative size, bad length */
  BT_ERR_UNSUPPORTED = 2, /* shape outside what the kernels are built for */
  BT_ERR_WORKSPACE = 3,   /* workspace missing or too small */
  BT_ERR_HIP = 4          /* a HIP runtime call or kernel launch failed */
} bt_status;

/* Static, never-NULL description of a status code. */
const char* bt_status_string(bt_status s);

/* Limits the kernels are built for. */
#define BT_MAX_SEQ 4096  /* largest S accepted by bt_build_offsets */
#define BT_HEAD_DIM 64   /* the only head size (standard BERT, Sec. III-B) */

/*
 * Zero-padding algorithm, Sec. III-D / Fig. 4: prefix sum of the mask matrix and
 * the position array that maps packed tokens to the padded tensor.
 *
 * Exactly one of d_mask (int32 [B,S], entries 0 or 1, 1 = valid token) and
 * d_lengths (int32 [B], sequence b has tokens 0..L_b-1 valid) is non-NULL.
 * Outputs:
 *   d_cu_seqlens int32 [B+1]  exclusive prefix sum of the per-sequence valid counts
 *   d_token_idx  int32 [B*S]  capacity; the first T entries are written:
 *                             token_idx[i] = b*S + t of the i-th valid token in
 *                             row-major order
 *   h_total      host int32   T = number of valid tokens
 * This is the one call that blocks the host: *h_total is valid on return.
 *   - h_total in ordinary host memory: the total is copied back and `stream` is
 *     synchronised once.
 *   - h_total in pinned, device-visible host memory (hipHostMalloc): the kernel stores
 *     the total there as soon as it is known and the host polls for it; the stream is
 *     NOT synchronised (d_cu_seqlens / d_token_idx are ready for later work on the same
 *     stream, as for any other call).  About 20 us less host latency per batch.  Each
 *     thread that calls concurrently needs its own h_total.
 * A length outside [0,S] or a mask entry outside {0,1} is detected on the device and
 * reported as BT_ERR_INVALID_ARG after the kernel has run (*h_total = 0, the other
 * outputs are then unspecified).  Requires 1 <= S <= BT_MAX_SEQ, B*S < 2^31.
 * Because the call waits for a device result it cannot be recorded into a HIP graph:
 * on a stream that is being captured it returns BT_ERR_UNSUPPORTED and enqueues nothing
 * (build the offsets before the capture; every other call of this library captures as it is).
 */
bt_status bt_build_offsets(const int32_t* d_mask, const int32_t* d_lengths, int B, int S,
                           int32_t* d_cu_seqlens, int32_t* d_token_idx, int32_t* h_total,
                           bt_stream stream);

/*
 * The same call (Sec. III-D), which also hands back the longest sequence of the batch, so that the
 * caller can pass an exact max_len to the attention and encoder calls:
 *   h_total_max   host int32 [2]   [0] = T, [1] = max_b L_b (per-sentence valid count)
 *   d_cu_seqlens  int32 [B+2]      entries 0..B as above; entry B+1 = the same maximum, on the device
 * Pinned / ordinary host memory, errors and stream capture exactly as for bt_build_offsets
 * (on an error both host words are 0).
 */
bt_status bt_build_offsets_stats(const int32_t* d_mask, const int32_t* d_lengths, int B, int S,
                                 int32_t* d_cu_seqlens, int32_t* d_token_idx, int32_t* h_total_max,
                                 bt_stream stream);

/*
 * Pack (remove padding), Sec. III-D: d_packed[i,:] = d_padded[token_idx[i],:]
 * for i < T.  d_padded is fp16 [B*S,H], d_packed fp16 [T,H]; H % 8 == 0.
 * Bit-exact copy.  The two buffers must not overlap.
 */
bt_status bt_pack(const bt_half* d_padded, const int32_t* d_token_idx, int T, int H,
                  bt_half* d_packed, bt_stream stream);

/*
 * Unpack (rebuild padding), Sec. III-D: d_padded[token_idx[i],:] = d_packed[i,:],
 * every other row of d_padded [B*S,H] is written as zero.  token_idx must be
 * strictly increasing (as bt_build_offsets writes it).  T <= B*S, H % 8 == 0.
 */
bt_status bt_unpack(const bt_half* d_packed, const int32_t* d_token_idx, int T, int B, int S, int H,
                    bt_half* d_padded, bt_stream stream);

/*
 * Fused variable-length multi-head attention, eq. (1) and Sec. III-E: for every
 * sequence b and head j,  O = softmax((Q+bq)(K+bk)^T * scale) (V+bv)  over the
 * L_b = cu_seqlens[b+1]-cu_seqlens[b] tokens of that sequence only -- no padded
 * row or column is ever read or computed.
 *
 * d_q, d_k, d_v point at token 0, head 0 of each operand; token i's head j starts
 * at ptr + i*row_stride + j*head_dim (elements).  row_stride = 3*heads*head_dim
 * with d_k = d_q + heads*head_dim, d_v = d_q + 2*heads*head_dim reads the fused
 * [T, q|k|v] buffer GEMM #0 writes; row_stride = heads*head_dim reads three
 * separate tensors.  row_stride % 8 == 0.
 * d_bq/d_bk/d_bv: optional fp16 [heads*head_dim] biases (NULL = none; 16-byte aligned).  Alg. 1 adds them while
 * the operands are loaded; here b_q is added to the Q registers (fp32 add, fp16 result), b_k is
 * ignored because (q+b_q).b_k is constant along a softmax row and cancels exactly, and b_v is added
 * to the output because the probabilities of a row sum to one -- the same function, fewer roundings.
 * d_out: fp16 [T, heads*head_dim], heads concatenated inside a row.
 * T must equal cu_seqlens[B].  max_len: an upper bound on every L_b, 1 <= max_len <= BT_MAX_SEQ
 * and T <= B*max_len (checked); it only steers the choice among the kernel variants -- the work
 * list is derived from d_cu_seqlens on the device, so a sequence longer than max_len is still
 * computed in full (bt_build_offsets_stats returns the exact value).
 * head_dim must be BT_HEAD_DIM.  d_ws/ws_bytes: reserved, may be NULL/0.
 * Logits, softmax statistics and accumulators are fp32; the probabilities enter
 * the second contraction as fp16.
 */
bt_status bt_varlen_mha(const bt_half* d_q, const bt_half* d_k, const bt_half* d_v, int64_t row_stride,
                        const bt_half* d_bq, const bt_half* d_bk, const bt_half* d_bv,
                        const int32_t* d_cu_seqlens, int B, int T, int max_len, int heads, int head_dim,
                        float scale, bt_half* d_out, void* d_ws, size_t ws_bytes, bt_stream stream);

/*
 * Packed GEMM with fused epilogue, Sec. III-C2: C = act(A W^T + bias).
 * A fp16 [M,K], W fp16 [N,K], bias fp16 [N] or NULL, C fp16 [M,N]; fp32
 * accumulation; the bias and the activation are applied to the fp32 accumulators
 * before the single rounding to fp16.  K % 8 == 0, N % 8 == 0.
 */
typedef enum { BT_ACT_NONE = 0, BT_ACT_GELU_ERF = 1, BT_ACT_GELU_TANH = 2 } bt_act;
bt_status bt_gemm_bias_act(const bt_half* d_A, const bt_half* d_W, const bt_half* d_bias, int M, int N, int K,
                           bt_act act, bt_half* d_C, bt_stream stream);

/*
 * Which block tile bt_gemm_bias_act uses for an M x N x K product (host only, nothing is launched): the
 * library picks among 256x128 ... 64x64 by a cost model of rounds of tiles over the 256 compute units.
 * For reports: with it a caller can state the tile-quantisation ceiling of a measured product,
 * M*N / (tiles * bm * bn) * tiles / (ceil(tiles/256) * 256).  Same argument checks as bt_gemm_bias_act.
 */
bt_status bt_gemm_tile_shape(int M, int N, int K, bt_act act, int* bm, int* bn);

/*
 * Whether bt_gemm_bias_act runs an M x N x K product as two launches over row ranges (host only, nothing is
 * launched).  A tile grid that needs slightly more than a whole number of rounds of the 256 compute units pays a
 * whole round for its last few tiles; rows are independent, so the library then runs the rows that fill whole
 * rounds first and the remaining rows with the tile shape that suits them (Sec. III-C2 product, same function;
 * a row's value can differ in the last fp16 digit from the single launch where the two launches use different
 * tile shapes).  *rows_first = number of leading rows of the first launch, 0 = a single launch.  For reports.
 */
bt_status bt_gemm_row_split(int M, int N, int K, bt_act act, int* rows_first);

/*
 * Fused add-bias + residual + LayerNorm, Sec. III-C1:
 *   y[i,:] = LN(x[i,:] + bias + residual[i,:]) * gamma + beta,   one pass over memory.
 * x, residual, y fp16 [T,H]; bias, gamma, beta fp16 [H]; bias may be NULL.
 * Statistics in fp32, biased variance, eps inside the square root.
 * H % 8 == 0, H <= 8192.  y may alias x or residual.
 */
bt_status bt_add_bias_residual_layernorm(const bt_half* d_x, const bt_half* d_bias, const bt_half* d_residual,
                                         const bt_half* d_gamma, const bt_half* d_beta, float eps, int T, int H,
                                         bt_half* d_y, bt_stream stream);

/*
 * The output projection and the FFN-down product as the encoder layer runs them (Table II, GEMM #1 and #3;
 * Sec. III-C1 for what follows them): a product whose consumer is the add-bias + residual + LayerNorm
 * kernel may leave its reduction over K unfinished.  bt_gemm_kslices decides from the shape alone
 * whether to split K (it does when the tokens are so few that whole tiles would leave most of the chip idle):
 *   *n_slices == 0  the product was written to d_C, fp16 [M,N], as bt_gemm_bias_act without bias writes it;
 *   *n_slices == s  (2..8) d_slices holds s fp32 slices [s][M][N] whose sum is the product (d_C untouched);
 *                   slice i covers K range [i K/s, (i+1) K/s).
 * d_slices: device, 16-byte aligned, at least bt_gemm_kslices_bytes(M, N, K) bytes (0 when the shape is not
 * split; then d_slices may be NULL); BT_ERR_WORKSPACE if it is missing or too small.  n_slices: host.
 * bt_add_bias_residual_layernorm_kslices is bt_add_bias_residual_layernorm with x given as such slices,
 * added in slice order in fp32 (no rounding of the product to fp16 in between); 1 <= n_slices <= 8.
 */
size_t bt_gemm_kslices_bytes(int M, int N, int K);
bt_status bt_gemm_kslices(const bt_half* d_A, const bt_half* d_W, int M, int N, int K, bt_half* d_C,
                          float* d_slices, size_t slices_bytes, int* n_slices, bt_stream stream);
bt_status bt_add_bias_residual_layernorm_kslices(const float* d_slices, int n_slices, const bt_half* d_bias,
                                                 const bt_half* d_residual, const bt_half* d_gamma,
                                                 const bt_half* d_beta, float eps, int T, int H, bt_half* d_y,
                                                 bt_stream stream);

/*
 * One encoder layer's parameters (device pointers, fp16).  Shapes:
 *   w_qkv [3H,H]  rows 0..H-1 produce Q, H..2H-1 K, 2H..3H-1 V;   b_qkv [3H]
 *   w_o [H,H], b_o [H];  ln0_g, ln0_b [H]
 *   w_1 [F,H], b_1 [F];  w_2 [H,F], b_2 [H];  ln1_g, ln1_b [H]
 * gelu_kind: 0 = exact (erf), 1 = tanh approximation.
 */
typedef struct {
  int H, heads, head_dim, F;
  float ln_eps;
  int gelu_kind;
  const bt_half *w_qkv, *b_qkv, *w_o, *b_o, *ln0_g, *ln0_b, *w_1, *b_1, *w_2, *b_2, *ln1_g, *ln1_b;
} bt_layer;

/* Bytes of workspace bt_encoder_layer_fwd / bt_encoder_fwd need for T tokens. */
size_t bt_layer_workspace_bytes(const bt_layer* layer, int T, int B, int max_len);

/*
 * One padding-free post-LN BERT encoder layer on packed tokens, Fig. 2(c):
 *   QKV = x W_qkv^T + b_qkv;  A = varlen MHA(QKV);  y1 = LN(A W_o^T + b_o + x);
 *   y  = LN(GELU(y1 W_1^T + b_1) W_2^T + b_2 + y1).
 * d_x, d_y fp16 [T,H] (must not alias); d_ws 256-byte aligned, at least
 * bt_layer_workspace_bytes() bytes.  H == heads*head_dim, head_dim == BT_HEAD_DIM.
 */
bt_status bt_encoder_layer_fwd(const bt_layer* layer, const bt_half* d_x, const int32_t* d_cu_seqlens,
                               int B, int T, int max_len, bt_half* d_y, void* d_ws, size_t ws_bytes,
                               bt_stream stream);

/*
 * bt_encoder_layer_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same layer, same kernels, same
 * bits; the workspace is a fixed array of BT_STATIC_SCRATCH_BYTES inside the library's code object (one
 * per GPU, held until the process ends) instead of an argument.  The call allocates and frees nothing.
 *   - Limit: bt_layer_workspace_bytes(layer, T, B, max_len) <= BT_STATIC_SCRATCH_BYTES, i.e. about 3 300
 *     tokens for H = 768, F = 3072 and about 2 500 for H = 1024, F = 4096; beyond it the call returns
 *     BT_ERR_WORKSPACE and enqueues nothing.
 *   - The device that owns `stream` must be current.  The first call on a device looks the array's address
 *     up once (hipGetSymbolAddress); make that call outside a stream capture.
 *   - All calls on one GPU share the array: calls that overlap in time on the same GPU (two streams,
 *     two threads) race and give wrong results; calls on one stream are ordered and safe.  Nothing has
 *     to start at zero: every region is written in full by the kernel that produces it before any
 *     kernel reads it, so the previous call's contents never matter.
 * Everything else (argument checks, T == 0, errors) as for bt_encoder_layer_fwd.
 */
#define BT_STATIC_SCRATCH_BYTES (64u << 20)
bt_status bt_encoder_layer_fwd_static(const bt_layer* layer, const bt_half* d_x, const int32_t* d_cu_seqlens,
                                      int B, int T, int max_len, bt_half* d_y, bt_stream stream);

/*
 * LayerNorm folding (optional, for bt_encoder_fwd).  A LayerNorm followed by a linear layer satisfies
 *   LN(z) W^T + b = rstd (u W^T - mu c) + d,   u = gamma (.) z,  c = W gamma,  d = W beta + b,
 * so the add-bias + residual + LayerNorm of Sec. III-C1 can live entirely in GEMM epilogues: the GEMM
 * in front of the LayerNorm adds bias and residual, writes u and accumulates the row sums of z and
 * z^2; the GEMM behind it applies mu, rstd, c and d.  The vectors c, d depend on the weights only;
 * bt_encoder_prepare computes them once (fp32, on the device):
 *   per layer  [ c_qkv (3H) | d_qkv (3H) | c_1 (F) | d_1 (F) ]
 * where c_qkv/d_qkv of layer i use the second LayerNorm of layer i-1 (unused for layer 0).
 * d_fold: device buffer of bt_encoder_fold_bytes() bytes, 16-byte aligned, owned by the caller; it must
 * be recomputed when any weight, bias or LayerNorm parameter of the stack changes.
 */
size_t bt_encoder_fold_bytes(const bt_layer* layers, int n_layers);
bt_status bt_encoder_prepare(const bt_layer* layers, int n_layers, float* d_fold, size_t fold_bytes,
                             bt_stream stream);

/*
 * A stack of n_layers encoder layers (Sec. IV-E): layer i+1 reads layer i's
 * output.  `layers` is a HOST array of n_layers descriptors with identical
 * H / heads / F / ln_eps.  The workspace (sized by bt_layer_workspace_bytes) also
 * holds the ping-pong buffer between layers; d_x is not modified; d_y receives
 * the last layer's output.
 * d_fold == NULL: each layer runs as bt_encoder_layer_fwd does (7 launches per layer).
 * d_fold from bt_encoder_prepare: the library MAY fold the LayerNorms into the GEMM epilogues
 * (5 launches per layer plus one normalisation at the end) and does so where that is the faster
 * pipeline: while ceil(T/64) * ceil(H/128) <= 256 (up to about 2 700 tokens at H = 768) and there are
 * enough tokens that the unfolded layer would not split K (more than about 600 at H = 768); outside that
 * range it runs the unfolded layers.  Same function either way.  The folded results differ from the
 * unfolded ones in two ways: u = gamma (.) z is stored in fp16 instead of LN(z), so every stored value carries
 * a rounding error of 2^-11 |u| that the normalisation then divides by the row's standard deviation; and the
 * variance is formed from the row sums of z and z^2 in fp32 (E[z^2] - mean^2, clamped at 0).  Both are
 * harmless while a row's |mean| stays within about 10 standard deviations -- post-LN BERT rows have
 * |mean| << sigma (a residual of LayerNorm outputs) -- and lose accuracy beyond; for such data leave d_fold
 * NULL.  Row statistics travel as
 * per-tile partial sums that are added in a fixed order: bit-reproducible, like the unfolded path.
 */
bt_status bt_encoder_fwd(const bt_layer* layers, int n_layers, const float* d_fold, const bt_half* d_x,
                         const int32_t* d_cu_seqlens, int B, int T, int max_len, bt_half* d_y,
                         void* d_ws, size_t ws_bytes, bt_stream stream);

/*
 * The same stack on PADDED tensors, with the zero-padding algorithm of Sec. III-D fused into the
 * neighbouring kernels instead of running as kernels of its own: the first GEMM and the first
 * residual read gather their rows of d_x_padded [B*S,H] through d_token_idx (pack), the last
 * LayerNorm scatters its rows into d_y_padded [B*S,H] and zero-fills every padding row (unpack).
 * d_token_idx / d_cu_seqlens / T come from bt_build_offsets for the same B and S.  d_fold: NULL, or the
 * fold vectors of bt_encoder_prepare (same meaning and the same choice of pipeline by token count as for
 * bt_encoder_fwd).  Results are bit-identical to bt_pack + bt_encoder_fwd (same d_fold) + bt_unpack; two
 * launches fewer.  d_x_padded is not modified and must not alias d_y_padded.  T == 0 zero-fills d_y_padded.
 * Workspace as for bt_encoder_fwd (bt_layer_workspace_bytes with this T).
 */
bt_status bt_encoder_fwd_padded(const bt_layer* layers, int n_layers, const float* d_fold,
                                const bt_half* d_x_padded, const int32_t* d_token_idx,
                                const int32_t* d_cu_seqlens, int B, int T, int S, bt_half* d_y_padded, void* d_ws,
                                size_t ws_bytes, bt_stream stream);

/*
 * bt_build_offsets followed by bt_encoder_fwd_padded in one call (Sec. III-D, Fig. 2 (c): the prefix sum of the mask
 * and the packed layers it feeds).  Same kernels, same results, same arguments with the same meaning as in the two
 * calls: d_mask / d_lengths (exactly one non-NULL), d_cu_seqlens [B+1] and d_token_idx [B*S] are written as by
 * bt_build_offsets, *h_total receives the token count (host memory; pinned and device-mapped memory avoids a stream
 * synchronisation), d_y_padded as by bt_encoder_fwd_padded.  What the single call saves is host time: the count that
 * the host waits for goes into the launches of the layers without returning to the caller first, and while the
 * host holds that count without having launched, the device has nothing to do (about 10 us per batch through a
 * scripting-language binding).  The workspace must be large enough for every count: at least
 * bt_layer_workspace_bytes(layers, B*S, B, S).  Errors the host can see are reported before anything runs; a
 * length outside [0, S] is found by the prefix-sum kernel and reported as by bt_build_offsets, and then no layer
 * is launched.  Like
 * bt_build_offsets this call waits on the host and is refused (BT_ERR_UNSUPPORTED) on a capturing stream.
 */
bt_status bt_encoder_fwd_masked(const bt_layer* layers, int n_layers, const float* d_fold,
                                const bt_half* d_x_padded, const int32_t* d_mask, const int32_t* d_lengths, int B,
                                int S, int32_t* d_cu_seqlens, int32_t* d_token_idx, int32_t* h_total,
                                bt_half* d_y_padded, void* d_ws, size_t ws_bytes, bt_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* BT_H_ */
