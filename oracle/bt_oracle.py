"""fp64 numpy oracle of the padded-semantics BERT encoder layer.

TEST INFRASTRUCTURE ONLY.  This module is the yardstick the HIP path is
compared with; it shares no code with it and is never called by it.

Everything here works on *padded* tensors ``[B, S, ...]`` plus a 0/1 validity
mask, i.e. it is the conventional (padded) BERT layer the paper says the
padding-free pipeline must reproduce on the valid tokens ("semantic
preservation", Sec. III-D).  No blocking, no fusion, no reordering: each
function is the textbook definition written out with numpy fp64 primitives
(matmul, exp, cumsum, scipy's erf).

Readings of the paper taken here (each is listed with its reason in the
design notes of the repository):
  * softmax scale is 1/sqrt(d_k) as in eq. (1), d_k = head size;
  * masked keys are excluded from the softmax (logit = -inf);
  * post-LayerNorm: LN(x + sublayer(x)), biased variance, eps a parameter;
  * GELU is the exact erf form  x/2 (1 + erf(x/sqrt 2)); the tanh form of the same
    citation is available as ``gelu_tanh`` / ``gelu_kind="tanh"`` (never the default);
  * outputs at padded positions are zero;
  * a stack of layers feeds the unrounded fp64 output to the next layer.

Pins (see tests/test_oracle_*.py): the worked packing example of Fig. 4,
brute-force scalar masked attention, closed forms and invariants, the dense
special case against torch's float64 CPU library ops, Table II's closed-form
FLOP counts.  Parity with the numeric outputs of the paper's own
implementation is unpinned: the paper prints none.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------
# Zero-padding algorithm (Sec. III-D, Fig. 4): mask -> prefix sum -> offsets
# --------------------------------------------------------------------------
def lengths_to_mask(lengths, S):
    """Right-padded mask [B,S] (int32) with 1 for t < L_b (Sec. III-D)."""
    lengths = np.asarray(lengths, dtype=np.int64)
    if np.any(lengths < 0) or np.any(lengths > S):
        raise ValueError("length outside [0, S]")
    return (np.arange(S)[None, :] < lengths[:, None]).astype(np.int32)


def build_offsets(mask):
    """Prefix sum of the mask matrix and the position array (Sec. III-D).

    mask: [B,S] of 0/1.  Returns (cu_seqlens int32[B+1], token_idx int32[T], T):
    cu_seqlens is the exclusive prefix sum of the per-sentence valid counts,
    token_idx[i] is the flat padded row b*S+t of the i-th valid token taken in
    row-major order -- the map between packed and original tensor.
    """
    mask = np.asarray(mask)
    if mask.ndim != 2 or not np.all((mask == 0) | (mask == 1)):
        raise ValueError("mask must be a [B,S] 0/1 matrix")
    B, S = mask.shape
    flat = mask.reshape(-1).astype(np.int64)
    incl = np.cumsum(flat)                      # inclusive prefix sum
    excl = incl - flat                          # packed position of each valid token
    T = int(incl[-1]) if flat.size else 0
    token_idx = np.empty(T, dtype=np.int32)
    for r in range(flat.size):                  # plain loop: the definition
        if flat[r]:
            token_idx[excl[r]] = r
    per_seq = mask.astype(np.int64).sum(axis=1)
    cu = np.zeros(B + 1, dtype=np.int64)
    for b in range(B):
        cu[b + 1] = cu[b] + per_seq[b]
    return cu.astype(np.int32), token_idx, T


def pack(x_padded, token_idx):
    """Gather the valid rows of [B,S,H] (or [B*S,H]) into [T,H] (Sec. III-D)."""
    H = x_padded.shape[-1]
    flat = x_padded.reshape(-1, H)
    return flat[np.asarray(token_idx, dtype=np.int64)].copy()


def unpack(x_packed, token_idx, B, S):
    """Scatter [T,H] back to [B,S,H]; padded rows are zero (Sec. III-D)."""
    H = x_packed.shape[-1]
    out = np.zeros((B * S, H), dtype=x_packed.dtype)
    out[np.asarray(token_idx, dtype=np.int64)] = x_packed
    return out.reshape(B, S, H)


# --------------------------------------------------------------------------
# Element-wise pieces
# --------------------------------------------------------------------------
def gelu(x):
    """Exact GELU, x * Phi(x) (activation of Sec. III-C2)."""
    x = np.asarray(x, dtype=F64)
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_tanh(x):
    """The tanh form of GELU given beside the exact one in the work Sec. III-C2 cites for the
    activation:  x/2 (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))).  Selected by ``gelu_kind = "tanh"``."""
    x = np.asarray(x, dtype=F64)
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def layer_norm(x, gamma, beta, eps):
    """LayerNorm over the last axis, biased variance (Sec. II-A, III-C1)."""
    x = np.asarray(x, dtype=F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def softmax_rows(logits):
    """Row softmax: subtract row max, exponentiate, divide by row sum."""
    m = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(axis=-1, keepdims=True)


# --------------------------------------------------------------------------
# Multi-head attention, eq. (1), padded with masking
# --------------------------------------------------------------------------
def attention_padded(q, k, v, mask, heads, scale=None):
    """softmax(Q K^T / sqrt(d_k)) V per sentence and head (eq. (1)).

    q, k, v: [B,S,heads*d] (biases already added), mask: [B,S] 0/1.
    Keys with mask 0 get logit -inf; rows with mask 0 are returned as zeros.
    A sentence with no valid key returns zeros.
    """
    q = np.asarray(q, F64); k = np.asarray(k, F64); v = np.asarray(v, F64)
    B, S, HD = q.shape
    d = HD // heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.zeros((B, S, HD), dtype=F64)
    for b in range(B):
        valid = np.asarray(mask[b]) != 0
        if not valid.any():
            continue
        for j in range(heads):
            sl = slice(j * d, (j + 1) * d)
            logits = (q[b, :, sl] @ k[b, :, sl].T) * scale          # [S,S]
            logits[:, ~valid] = -np.inf
            p = softmax_rows(logits)
            out[b, :, sl] = p @ v[b, :, sl]
        out[b, ~valid, :] = 0.0
    return out


def varlen_mha_packed(qkv_packed, cu_seqlens, heads, head_dim, scale=None,
                      bq=None, bk=None, bv=None):
    """Attention on the packed [T, 3*heads*d] QKV buffer (config "MHA alone").

    Rebuilds the padded tensors, calls the padded definition above and gathers
    the valid rows again, so the result is by construction what the padded
    layer gives on the valid tokens.  Row layout: [q | k | v], each heads*d.
    """
    qkv = np.asarray(qkv_packed, F64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    B = cu.size - 1
    HD = heads * head_dim
    lengths = cu[1:] - cu[:-1]
    S = int(max(1, lengths.max())) if B else 1
    mask = lengths_to_mask(lengths, S)
    _, token_idx, T = build_offsets(mask)
    assert T == qkv.shape[0]
    padded = unpack(qkv, token_idx, B, S)
    q = padded[..., 0:HD].copy(); k = padded[..., HD:2 * HD].copy(); v = padded[..., 2 * HD:3 * HD].copy()
    if bq is not None: q += np.asarray(bq, F64)
    if bk is not None: k += np.asarray(bk, F64)
    if bv is not None: v += np.asarray(bv, F64)
    o = attention_padded(q, k, v, mask, heads, scale)
    return pack(o, token_idx)


# --------------------------------------------------------------------------
# Encoder layer, Fig. 2(a) pipeline on padded tensors
# --------------------------------------------------------------------------
class LayerWeights:
    """fp64 copies of one layer's parameters.  Weights are [out, in]."""

    FIELDS = ("w_qkv", "b_qkv", "w_o", "b_o", "ln0_g", "ln0_b",
              "w_1", "b_1", "w_2", "b_2", "ln1_g", "ln1_b")

    def __init__(self, **kw):
        for f in self.FIELDS:
            setattr(self, f, np.asarray(kw[f], dtype=F64))
        self.heads = int(kw["heads"])
        self.eps = float(kw.get("eps", 1e-12))
        self.gelu_kind = str(kw.get("gelu_kind", "erf"))           # "erf" (exact, default) | "tanh"
        if self.gelu_kind not in ("erf", "tanh"):
            raise ValueError("gelu_kind must be 'erf' or 'tanh'")


def encoder_layer(x_padded, mask, w: LayerWeights):
    """One post-LN BERT encoder layer on padded [B,S,H] input (Sec. III-A).

    GEMM0 (+bias) -> masked multi-head attention -> GEMM1 (+bias) -> +residual
    -> LN -> GEMM2 (+bias) -> GELU -> GEMM3 (+bias) -> +residual -> LN.
    Padded rows take part in the GEMMs like any other row (padded semantics)
    and are zeroed in the returned tensor.
    """
    x = np.asarray(x_padded, F64)
    B, S, H = x.shape
    qkv = x @ w.w_qkv.T + w.b_qkv                                   # [B,S,3H]
    q, k, v = qkv[..., :H], qkv[..., H:2 * H], qkv[..., 2 * H:]
    attn = attention_padded(q, k, v, mask, w.heads)
    proj = attn @ w.w_o.T + w.b_o
    y1 = layer_norm(x + proj, w.ln0_g, w.ln0_b, w.eps)
    act = gelu if w.gelu_kind == "erf" else gelu_tanh
    g = act(y1 @ w.w_1.T + w.b_1)
    ffn = g @ w.w_2.T + w.b_2
    y2 = layer_norm(y1 + ffn, w.ln1_g, w.ln1_b, w.eps)
    y2 = y2 * (np.asarray(mask) != 0)[..., None]
    return y2


def encoder_stack(x_padded, mask, layers):
    """N stacked layers; layer i+1 consumes layer i's fp64 output (Sec. IV-E)."""
    y = np.asarray(x_padded, F64)
    for w in layers:
        y = encoder_layer(y, mask, w)
    return y


# --------------------------------------------------------------------------
# Table II: floating-point operation counts of one layer
# --------------------------------------------------------------------------
def table2_flops(batch, max_seq, hidden, alpha, variant):
    """Closed forms of Table II with m = batch*max_seq, k = hidden.

    variant: "baseline" | "zero_padding" | "zero_padding_fmha".
    Returns dict(GEMM0, MHA, GEMM1, GEMM2, GEMM3).
    """
    m = batch * max_seq
    k = hidden
    a = 1.0 if variant == "baseline" else alpha
    a_mha = alpha if variant == "zero_padding_fmha" else 1.0
    return {
        "GEMM0": 6 * a * m * k * k,
        "MHA": 4 * (a_mha * m) ** 2 / batch * k,
        "GEMM1": 2 * a * m * k * k,
        "GEMM2": 8 * a * m * k * k,
        "GEMM3": 8 * a * m * k * k,
    }
