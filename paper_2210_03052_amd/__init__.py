"""Thin ctypes binding of libbt.so, the C-ABI HIP library (see include/bt.h).

Argument marshalling only: every function checks dtypes / devices, allocates
the output tensors with torch (device memory and streams are torch's), and
passes raw device pointers plus the current HIP stream to the entry point of
the same name.  No step of the path is computed here, and there is no
fallback: if the library is not built, ``load_library`` raises.
"""
from __future__ import annotations

import ctypes
import os
import threading as _threading
import weakref as _weakref

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libbt.so")

BT_OK = 0
ACT_NONE, ACT_GELU_ERF, ACT_GELU_TANH = 0, 1, 2
_c = ctypes
_lib = None


class BtError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        msg = _lib.bt_status_string(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} (status {int(code)})")


class bt_layer(_c.Structure):
    _fields_ = [("H", _c.c_int), ("heads", _c.c_int), ("head_dim", _c.c_int), ("F", _c.c_int),
                ("ln_eps", _c.c_float), ("gelu_kind", _c.c_int)] + [
        (n, _c.c_void_p) for n in ("w_qkv", "b_qkv", "w_o", "b_o", "ln0_g", "ln0_b",
                                   "w_1", "b_1", "w_2", "b_2", "ln1_g", "ln1_b")]


PARAM_NAMES = ("w_qkv", "b_qkv", "w_o", "b_o", "ln0_g", "ln0_b", "w_1", "b_1", "w_2", "b_2", "ln1_g", "ln1_b")

_SIGNATURES = {
    "bt_status_string": (_c.c_char_p, [_c.c_int]),
    "bt_build_offsets": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p,
                                    _c.POINTER(_c.c_int32), _c.c_void_p]),
    "bt_build_offsets_stats": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p,
                                          _c.POINTER(_c.c_int32), _c.c_void_p]),
    "bt_pack": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "bt_unpack": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p,
                             _c.c_void_p]),
    "bt_varlen_mha": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p, _c.c_void_p,
                                 _c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                 _c.c_float, _c.c_void_p, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "bt_gemm_bias_act": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                    _c.c_void_p, _c.c_void_p]),
    "bt_add_bias_residual_layernorm": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                                  _c.c_float, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "bt_gemm_kslices_bytes": (_c.c_size_t, [_c.c_int, _c.c_int, _c.c_int]),
    "bt_gemm_kslices": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p,
                                   _c.c_size_t, _c.POINTER(_c.c_int), _c.c_void_p]),
    "bt_add_bias_residual_layernorm_kslices": (_c.c_int, [_c.c_void_p, _c.c_int, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                                          _c.c_void_p, _c.c_float, _c.c_int, _c.c_int, _c.c_void_p,
                                                          _c.c_void_p]),
    "bt_layer_workspace_bytes": (_c.c_size_t, [_c.POINTER(bt_layer), _c.c_int, _c.c_int, _c.c_int]),
    "bt_encoder_layer_fwd": (_c.c_int, [_c.POINTER(bt_layer), _c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int,
                                        _c.c_int, _c.c_void_p, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "bt_encoder_layer_fwd_static": (_c.c_int, [_c.POINTER(bt_layer), _c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int,
                                               _c.c_int, _c.c_void_p, _c.c_void_p]),
    "bt_encoder_fold_bytes": (_c.c_size_t, [_c.POINTER(bt_layer), _c.c_int]),
    "bt_encoder_prepare": (_c.c_int, [_c.POINTER(bt_layer), _c.c_int, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "bt_encoder_fwd": (_c.c_int, [_c.POINTER(bt_layer), _c.c_int, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_int,
                                  _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "bt_gemm_tile_shape": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.POINTER(_c.c_int), _c.POINTER(_c.c_int)]),
    "bt_gemm_row_split": (_c.c_int, [_c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.POINTER(_c.c_int)]),
    "bt_encoder_fwd_padded": (_c.c_int, [_c.POINTER(bt_layer), _c.c_int, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                         _c.c_void_p, _c.c_int, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p,
                                         _c.c_size_t, _c.c_void_p]),
    "bt_encoder_fwd_masked": (_c.c_int, [_c.POINTER(bt_layer), _c.c_int, _c.c_void_p, _c.c_void_p, _c.c_void_p,
                                         _c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p,
                                         _c.POINTER(_c.c_int32), _c.c_void_p, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
}
EXPORTED = tuple(_SIGNATURES)


def load_library(path: str | None = None):
    """dlopen libbt.so and declare the prototypes.  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built: run `python -m paper_2210_03052_amd.build` "
                           "(there is no CPU fallback)")
    lib = _c.CDLL(path)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


# ------------------------------------------------------------------ helpers
def _torch():
    import torch
    return torch


def _stream():
    return _c.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _ptr(t):
    return _c.c_void_p(t.data_ptr()) if t is not None else _c.c_void_p(0)


def _chk(t, dtype, name, ndim=None):
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of dtype {dtype}")
    if ndim is not None and t.dim() != ndim:
        raise TypeError(f"{name}: expected {ndim} dimensions, got {t.dim()}")


def _call(name, *args):
    lib = load_library()
    st = getattr(lib, name)(*args)
    if st != BT_OK:
        raise BtError(st, name)


# ------------------------------------------------------------------ entry points
_tls = _threading.local()


def _pinned_total():
    """Two pinned int32 per host thread: the device writes the token count (and, for the _stats call, the
    longest sequence) there and the host polls it."""
    t = getattr(_tls, "total", None)
    if t is None:
        t = _torch().empty(2, dtype=_torch().int32, pin_memory=True)
        # (tensor, its address as the C pointer, a numpy view for cheap reads): the reads sit between the device
        # writing the count and the first launch that needs it, where every host microsecond is device idle time
        t = _tls.total = (t, _c.cast(t.data_ptr(), _c.POINTER(_c.c_int32)), t.numpy())
    return t


def build_offsets(mask=None, lengths=None, S=None, pinned=True, with_max=False):
    """bt_build_offsets.  Returns (cu_seqlens int32[B+1], token_idx int32[T], T).
    pinned=True hands the library a pinned host word for T (no stream synchronisation);
    pinned=False passes ordinary host memory (copy + one synchronisation).
    with_max=True calls bt_build_offsets_stats and returns (cu_seqlens, token_idx, T, max_len)."""
    torch = _torch()
    if (mask is None) == (lengths is None):
        raise ValueError("give exactly one of mask / lengths")
    if mask is not None:
        _chk(mask, torch.int32, "mask", 2)
        B, S = mask.shape
        dev = mask.device
    else:
        _chk(lengths, torch.int32, "lengths", 1)
        if S is None:
            raise ValueError("S is required with lengths")
        B, dev = lengths.shape[0], lengths.device
    cu = torch.empty(B + 2, dtype=torch.int32, device=dev)
    tok = torch.empty(max(1, B * S), dtype=torch.int32, device=dev)
    cu_view = cu[: B + 1]  # made before the call: it does not depend on the count the host waits for
    name = "bt_build_offsets_stats" if with_max else "bt_build_offsets"
    if pinned:
        _, slot_ptr, slot_np = _pinned_total()
        _call(name, _ptr(mask), _ptr(lengths), B, int(S), _ptr(cu), _ptr(tok), slot_ptr, _stream())
        T, mx = int(slot_np[0]), int(slot_np[1])
    else:
        res = (_c.c_int32 * 2)(-1, -1)
        _call(name, _ptr(mask), _ptr(lengths), B, int(S), _ptr(cu), _ptr(tok),
              _c.cast(res, _c.POINTER(_c.c_int32)), _stream())
        T, mx = int(res[0]), int(res[1])
    if with_max:
        return cu_view, tok[:T], T, mx
    return cu_view, tok[:T], T


def pack(padded, token_idx, out=None):
    """bt_pack: padded fp16 [B,S,H] or [B*S,H] -> packed fp16 [T,H]."""
    torch = _torch()
    _chk(padded, torch.float16, "padded")
    _chk(token_idx, torch.int32, "token_idx", 1)
    H, T = padded.shape[-1], token_idx.shape[0]
    if out is None:
        out = torch.empty((T, H), dtype=torch.float16, device=padded.device)
    _call("bt_pack", _ptr(padded), _ptr(token_idx), T, H, _ptr(out), _stream())
    return out


def unpack(packed, token_idx, B, S, out=None):
    """bt_unpack: packed fp16 [T,H] -> padded fp16 [B,S,H], pads zero."""
    torch = _torch()
    _chk(packed, torch.float16, "packed", 2)
    _chk(token_idx, torch.int32, "token_idx", 1)
    T, H = packed.shape
    if out is None:
        out = torch.empty((B, S, H), dtype=torch.float16, device=packed.device)
    _call("bt_unpack", _ptr(packed), _ptr(token_idx), T, B, S, H, _ptr(out), _stream())
    return out


def varlen_mha(qkv, cu_seqlens, max_len, heads, head_dim=64, scale=None, bq=None, bk=None, bv=None, out=None):
    """bt_varlen_mha on the fused packed buffer qkv fp16 [T, 3*heads*head_dim]."""
    torch = _torch()
    _chk(qkv, torch.float16, "qkv", 2)
    _chk(cu_seqlens, torch.int32, "cu_seqlens", 1)
    HD = heads * head_dim
    T, B = qkv.shape[0], cu_seqlens.shape[0] - 1
    if qkv.shape[1] != 3 * HD:
        raise ValueError("qkv must be [T, 3*heads*head_dim]")
    for b_, n in ((bq, "bq"), (bk, "bk"), (bv, "bv")):
        if b_ is not None:
            _chk(b_, torch.float16, n, 1)
    if scale is None:
        scale = head_dim ** -0.5
    if out is None:
        out = torch.empty((T, HD), dtype=torch.float16, device=qkv.device)
    base, es = qkv.data_ptr(), qkv.element_size()
    _call("bt_varlen_mha", _c.c_void_p(base), _c.c_void_p(base + HD * es), _c.c_void_p(base + 2 * HD * es),
          3 * HD, _ptr(bq), _ptr(bk), _ptr(bv), _ptr(cu_seqlens), B, T, int(max_len), heads, head_dim,
          float(scale), _ptr(out), _c.c_void_p(0), 0, _stream())
    return out


def varlen_mha_separate(q, k, v, cu_seqlens, max_len, heads, head_dim=64, scale=None, out=None):
    """bt_varlen_mha on three separate packed tensors fp16 [T, heads*head_dim]."""
    torch = _torch()
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _chk(t, torch.float16, n, 2)
    _chk(cu_seqlens, torch.int32, "cu_seqlens", 1)
    HD = heads * head_dim
    T, B = q.shape[0], cu_seqlens.shape[0] - 1
    if scale is None:
        scale = head_dim ** -0.5
    if out is None:
        out = torch.empty((T, HD), dtype=torch.float16, device=q.device)
    _call("bt_varlen_mha", _ptr(q), _ptr(k), _ptr(v), HD, None, None, None, _ptr(cu_seqlens), B, T, int(max_len),
          heads, head_dim, float(scale), _ptr(out), _c.c_void_p(0), 0, _stream())
    return out


def gemm_bias_act(a, w, bias=None, act=ACT_NONE, out=None):
    """bt_gemm_bias_act: act(a [M,K] @ w[N,K]^T + bias) -> fp16 [M,N]."""
    torch = _torch()
    _chk(a, torch.float16, "a", 2)
    _chk(w, torch.float16, "w", 2)
    if bias is not None:
        _chk(bias, torch.float16, "bias", 1)
    M, K = a.shape
    N = w.shape[0]
    if w.shape[1] != K:
        raise ValueError("w must be [N,K]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=a.device)
    _call("bt_gemm_bias_act", _ptr(a), _ptr(w), _ptr(bias), M, N, K, int(act), _ptr(out), _stream())
    return out


def gemm_row_split(M, N, K, act=ACT_NONE):
    """bt_gemm_row_split: number of leading rows bt_gemm_bias_act gives a launch of their own (0 = one launch)."""
    rows = _c.c_int(0)
    _call("bt_gemm_row_split", int(M), int(N), int(K), int(act), _c.byref(rows))
    return rows.value


def gemm_tile_shape(M, N, K, act=ACT_NONE):
    """bt_gemm_tile_shape: the (BM, BN) block tile bt_gemm_bias_act uses for this product."""
    bm, bn = _c.c_int(0), _c.c_int(0)
    _call("bt_gemm_tile_shape", int(M), int(N), int(K), int(act), _c.byref(bm), _c.byref(bn))
    return bm.value, bn.value


def add_bias_residual_layernorm(x, bias, residual, gamma, beta, eps, out=None):
    """bt_add_bias_residual_layernorm on fp16 [T,H]."""
    torch = _torch()
    _chk(x, torch.float16, "x", 2)
    _chk(residual, torch.float16, "residual", 2)
    T, H = x.shape
    if out is None:
        out = torch.empty_like(x)
    _call("bt_add_bias_residual_layernorm", _ptr(x), _ptr(bias), _ptr(residual), _ptr(gamma), _ptr(beta),
          float(eps), T, H, _ptr(out), _stream())
    return out


def gemm_kslices(a, w, out=None, slices=None):
    """bt_gemm_kslices: a [M,K] @ w[N,K]^T with the reduction over K possibly left to the consumer.
    Returns (c fp16 [M,N] or None, slices fp32 [s,M,N] or None): exactly one of the two is not None."""
    torch = _torch()
    _chk(a, torch.float16, "a", 2)
    _chk(w, torch.float16, "w", 2)
    M, K = a.shape
    N = w.shape[0]
    nbytes = int(load_library().bt_gemm_kslices_bytes(M, N, K))
    if slices is None and nbytes:
        slices = torch.empty(nbytes // 4, dtype=torch.float32, device=a.device)
    if out is None and not nbytes:
        out = torch.empty((M, N), dtype=torch.float16, device=a.device)
    n = _c.c_int(-1)
    _call("bt_gemm_kslices", _ptr(a), _ptr(w), M, N, K, _ptr(out), _ptr(slices),
          slices.numel() * 4 if slices is not None else 0, _c.byref(n), _stream())
    if n.value == 0:
        return out, None
    return None, slices[: n.value * M * N].view(n.value, M, N)


def add_bias_residual_layernorm_kslices(slices, bias, residual, gamma, beta, eps, out=None):
    """bt_add_bias_residual_layernorm_kslices: x given as fp32 K slices [s,T,H]."""
    torch = _torch()
    _chk(slices, torch.float32, "slices", 3)
    _chk(residual, torch.float16, "residual", 2)
    n, T, H = slices.shape
    if out is None:
        out = torch.empty_like(residual)
    _call("bt_add_bias_residual_layernorm_kslices", _ptr(slices), n, _ptr(bias), _ptr(residual), _ptr(gamma),
          _ptr(beta), float(eps), T, H, _ptr(out), _stream())
    return out


class Layer:
    """Device copies of one layer's parameters plus the C descriptor."""

    def __init__(self, params: dict, device="cuda:0", gelu_kind=0):
        torch = _torch()
        self.tensors = {}
        for n in PARAM_NAMES:
            t = params[n]
            if not isinstance(t, torch.Tensor):
                t = torch.from_numpy(t)
            self.tensors[n] = t.to(device=device, dtype=torch.float16).contiguous()
        self.H = int(self.tensors["w_o"].shape[0])
        self.F = int(self.tensors["w_1"].shape[0])
        self.heads = int(params["heads"])
        self.head_dim = int(params.get("head_dim", self.H // self.heads))
        self.eps = float(params.get("eps", 1e-12))
        self.desc = bt_layer(self.H, self.heads, self.head_dim, self.F, self.eps, int(gelu_kind),
                             *[self.tensors[n].data_ptr() for n in PARAM_NAMES])


def layer_workspace_bytes(layer: Layer, T, B, max_len):
    return int(load_library().bt_layer_workspace_bytes(_c.byref(layer.desc), T, B, max_len))


def _workspace(layer, T, B, max_len, device):
    torch = _torch()
    n = layer_workspace_bytes(layer, T, B, max_len)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device), n


def encoder_layer_fwd(layer: Layer, x, cu_seqlens, max_len, out=None, ws=None):
    """bt_encoder_layer_fwd: packed fp16 [T,H] -> packed fp16 [T,H]."""
    torch = _torch()
    _chk(x, torch.float16, "x", 2)
    _chk(cu_seqlens, torch.int32, "cu_seqlens", 1)
    T, B = x.shape[0], cu_seqlens.shape[0] - 1
    if out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws, _ = _workspace(layer, T, B, max_len, x.device)
    _call("bt_encoder_layer_fwd", _c.byref(layer.desc), _ptr(x), _ptr(cu_seqlens), B, T, int(max_len), _ptr(out),
          _ptr(ws), ws.numel(), _stream())
    return out


def encoder_layer_fwd_static(layer: Layer, x, cu_seqlens, max_len, out):
    """bt_encoder_layer_fwd_static: the same layer with the library's fixed workspace; `out` is required
    (this call is for callers that must not allocate)."""
    torch = _torch()
    _chk(x, torch.float16, "x", 2)
    _chk(out, torch.float16, "out", 2)
    _chk(cu_seqlens, torch.int32, "cu_seqlens", 1)
    T, B = x.shape[0], cu_seqlens.shape[0] - 1
    _call("bt_encoder_layer_fwd_static", _c.byref(layer.desc), _ptr(x), _ptr(cu_seqlens), B, T, int(max_len),
          _ptr(out), _stream())
    return out


_layer_arrays = {}


def _layer_array(layers):
    """The C array of layer descriptors for a list of Layer objects, built once per distinct list.  The key is the
    identity of the Layer objects (immutable once built); weak references tell a recycled id from the original
    and keep the cache from holding device memory alive."""
    key = tuple(map(id, layers))
    hit = _layer_arrays.get(key)
    if hit is None or any(r() is not l for r, l in zip(hit[1], layers)):
        if len(_layer_arrays) > 64:
            _layer_arrays.clear()
        hit = _layer_arrays[key] = ((bt_layer * len(layers))(*[l.desc for l in layers]),
                                    tuple(_weakref.ref(l) for l in layers))
    return hit[0]


def encoder_prepare(layers):
    """bt_encoder_prepare: the fold vectors (fp32, device) that move every LayerNorm of the stack
    into GEMM epilogues.  Depends on the parameters only: compute once, pass to encoder_fwd."""
    torch = _torch()
    lib = load_library()
    arr = _layer_array(layers)
    n = int(lib.bt_encoder_fold_bytes(arr, len(layers)))
    fold = torch.empty(n // 4, dtype=torch.float32, device=layers[0].tensors["w_o"].device)
    _call("bt_encoder_prepare", arr, len(layers), _ptr(fold), n, _stream())
    return fold


def encoder_fwd(layers, x, cu_seqlens, max_len, out=None, ws=None, fold=None):
    """bt_encoder_fwd: the stack of layers on packed fp16 [T,H]; `fold` from encoder_prepare
    selects the LayerNorm-folded pipeline."""
    torch = _torch()
    _chk(x, torch.float16, "x", 2)
    _chk(cu_seqlens, torch.int32, "cu_seqlens", 1)
    if fold is not None:
        _chk(fold, torch.float32, "fold", 1)
    T, B = x.shape[0], cu_seqlens.shape[0] - 1
    if out is None:
        out = torch.empty_like(x)
    if ws is None:
        ws, _ = _workspace(layers[0], T, B, max_len, x.device)
    arr = _layer_array(layers)
    _call("bt_encoder_fwd", arr, len(layers), _ptr(fold), _ptr(x), _ptr(cu_seqlens), B, T, int(max_len), _ptr(out),
          _ptr(ws), ws.numel(), _stream())
    return out


def encoder_fwd_padded(layers, x_padded, token_idx, cu_seqlens, out=None, ws=None, fold=None):
    """bt_encoder_fwd_padded: padded fp16 [B,S,H] in, padded fp16 [B,S,H] out (pads zero); pack and
    unpack run inside the first and last kernels of the stack.  `fold` from encoder_prepare as for encoder_fwd."""
    torch = _torch()
    _chk(x_padded, torch.float16, "x_padded", 3)
    _chk(token_idx, torch.int32, "token_idx", 1)
    _chk(cu_seqlens, torch.int32, "cu_seqlens", 1)
    B, S, _ = x_padded.shape
    T = token_idx.shape[0]
    if out is None:
        out = torch.empty_like(x_padded)
    if ws is None:
        ws, _ = _workspace(layers[0], max(T, 1), B, S, x_padded.device)
    arr = _layer_array(layers)
    if fold is not None:
        _chk(fold, torch.float32, "fold", 1)
    _call("bt_encoder_fwd_padded", arr, len(layers), _ptr(fold), _ptr(x_padded), _ptr(token_idx), _ptr(cu_seqlens),
          B, T, S, _ptr(out), _ptr(ws), ws.numel(), _stream())
    return out


def encoder_fwd_masked(layers, x_padded, mask=None, lengths=None, out=None, ws=None, fold=None):
    """bt_encoder_fwd_masked: build_offsets + encoder_fwd_padded in one call of the library -- the token count goes
    from the prefix-sum kernel into the launches of the layers without passing through Python.
    x_padded fp16 [B,S,H]; exactly one of mask int32 [B,S] / lengths int32 [B].  `ws` must hold B*S tokens
    (layer_workspace_bytes(layers[0], B*S, B, S)).  Returns (out [B,S,H], cu_seqlens [B+1], token_idx [T], T)."""
    torch = _torch()
    _chk(x_padded, torch.float16, "x_padded", 3)
    if (mask is None) == (lengths is None):
        raise ValueError("give exactly one of mask / lengths")
    B, S, _ = x_padded.shape
    if mask is not None:
        _chk(mask, torch.int32, "mask", 2)
        if tuple(mask.shape) != (B, S):
            raise ValueError("mask must be [B,S]")
    else:
        _chk(lengths, torch.int32, "lengths", 1)
        if lengths.shape[0] != B:
            raise ValueError("lengths must be [B]")
    if fold is not None:
        _chk(fold, torch.float32, "fold", 1)
    dev = x_padded.device
    if out is None:
        out = torch.empty_like(x_padded)
    if ws is None:
        ws, _ = _workspace(layers[0], max(B * S, 1), B, S, dev)
    cu = torch.empty(B + 2, dtype=torch.int32, device=dev)
    tok = torch.empty(max(1, B * S), dtype=torch.int32, device=dev)
    cu_view = cu[: B + 1]
    _, slot_ptr, slot_np = _pinned_total()
    _call("bt_encoder_fwd_masked", _layer_array(layers), len(layers), _ptr(fold), _ptr(x_padded), _ptr(mask),
          _ptr(lengths), B, S, _ptr(cu), _ptr(tok), slot_ptr, _ptr(out), _ptr(ws), ws.numel(), _stream())
    T = int(slot_np[0])
    return out, cu_view, tok[:T], T

