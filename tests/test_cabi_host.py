"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2210_03052_amd as bt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(bt.LIB_PATH):
        from paper_2210_03052_amd.build import build_library
        build_library(verbose=False)
    return bt.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bt_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = _declared_symbols()
    assert "bt_varlen_mha" in names and "bt_encoder_layer_fwd" in names and len(names) >= 10
    for n in names:
        assert hasattr(lib, n), f"{n} declared in bt.h but not exported"
    assert set(names) == set(bt.EXPORTED)


def test_status_strings(lib):
    seen = {lib.bt_status_string(i) for i in range(5)}
    assert len(seen) == 5 and all(s for s in seen)
    assert lib.bt_status_string(99)


def test_argument_errors_before_launch(lib):
    one = ctypes.c_void_p(16)      # non-null, aligned, never dereferenced: calls fail before any launch
    odd = ctypes.c_void_p(24)
    tot = ctypes.c_int32(0)
    # build_offsets: both or neither of mask/lengths, bad sizes
    assert lib.bt_build_offsets(None, None, 2, 8, one, one, ctypes.byref(tot), None) == 1
    assert lib.bt_build_offsets(one, one, 2, 8, one, one, ctypes.byref(tot), None) == 1
    assert lib.bt_build_offsets(one, None, 2, 0, one, one, ctypes.byref(tot), None) == 1
    assert lib.bt_build_offsets(one, None, 2, 1 << 20, one, one, ctypes.byref(tot), None) == 2
    two = (ctypes.c_int32 * 2)()
    assert lib.bt_build_offsets_stats(None, None, 2, 8, one, one, two, None) == 1
    assert lib.bt_build_offsets_stats(one, None, 2, 8, one, one, None, None) == 1
    assert lib.bt_build_offsets_stats(one, None, 2, 1 << 20, one, one, two, None) == 2
    # pack / unpack
    assert lib.bt_pack(one, one, 4, 7, one, None) == 1
    assert lib.bt_pack(one, one, -1, 8, one, None) == 1
    assert lib.bt_pack(one, one, 0, 8, one, None) == 0          # T == 0: no-op
    assert lib.bt_pack(odd, one, 4, 8, one, None) == 1          # misaligned
    assert lib.bt_unpack(one, one, 100, 2, 8, 8, one, None) == 1  # T > B*S
    assert lib.bt_unpack(one, one, 0, 0, 8, 8, one, None) == 0
    # mha
    f = ctypes.c_float(0.125)
    assert lib.bt_varlen_mha(one, one, one, 2304, None, None, None, one, 2, 10, 8, 12, 32, f, one, None, 0, None) == 2
    assert lib.bt_varlen_mha(one, one, one, 100, None, None, None, one, 2, 10, 8, 12, 64, f, one, None, 0, None) == 1
    assert lib.bt_varlen_mha(one, one, one, 2304, None, None, None, one, 2, 100, 8, 12, 64, f, one, None, 0, None) == 1
    assert lib.bt_varlen_mha(one, one, one, 2304, None, None, None, one, 0, 0, 8, 12, 64, f, one, None, 0, None) == 0
    assert lib.bt_varlen_mha(one, one, one, 2304, None, None, None, one, 2, 10, 4097, 12, 64, f, one, None, 0,
                             None) == 2                          # max_len beyond BT_MAX_SEQ
    assert lib.bt_varlen_mha(one, one, one, 2304, None, None, None, one, 2, 10, 8, 12, 64, ctypes.c_float(-1.0),
                             one, None, 0, None) == 1
    assert lib.bt_varlen_mha(one, one, one, 2304, None, None, odd, one, 2, 10, 8, 12, 64, f, one, None, 0,
                             None) == 1                          # misaligned value bias
    assert lib.bt_varlen_mha(one, one, one, 2304, odd, None, None, one, 2, 10, 8, 12, 64, f, one, None, 0,
                             None) == 1                          # misaligned query bias
    # gemm / layernorm
    assert lib.bt_gemm_bias_act(one, one, None, 4, 12, 64, 0, one, None) == 1   # N % 8
    assert lib.bt_gemm_bias_act(one, one, None, 4, 16, 60, 0, one, None) == 1   # K % 8
    assert lib.bt_gemm_bias_act(one, one, None, 4, 16, 64, 7, one, None) == 1   # bad activation
    assert lib.bt_gemm_bias_act(one, one, None, 0, 16, 64, 0, one, None) == 0
    assert lib.bt_add_bias_residual_layernorm(one, None, one, one, one, ctypes.c_float(1e-12), 4, 12, one, None) == 1
    assert lib.bt_add_bias_residual_layernorm(one, None, one, one, one, ctypes.c_float(1e-12), 4, 16384, one,
                                              None) == 2
    # K slices: which shapes are split is a host decision; too small a slice buffer is refused before any launch
    n = ctypes.c_int(-1)
    assert lib.bt_gemm_kslices_bytes(186, 768, 3072) % (186 * 768 * 4) == 0
    assert lib.bt_gemm_kslices_bytes(186, 768, 3072) >= 2 * 186 * 768 * 4
    assert lib.bt_gemm_kslices_bytes(2308, 768, 3072) == 0            # enough tiles to fill the chip: not split
    assert lib.bt_gemm_kslices(one, one, 186, 768, 3072, one, one, 16, ctypes.byref(n), None) == 3
    assert lib.bt_gemm_kslices(one, one, 186, 768, 3072, one, None, 0, ctypes.byref(n), None) == 3
    assert lib.bt_gemm_kslices(one, one, 0, 768, 3072, one, None, 0, ctypes.byref(n), None) == 0 and n.value == 0
    assert lib.bt_gemm_kslices(one, one, 186, 768, 3072, one, one, 1 << 30, None, None) == 1
    assert lib.bt_add_bias_residual_layernorm_kslices(one, 9, None, one, one, one, ctypes.c_float(1e-12), 4, 16,
                                                      one, None) == 1
    assert lib.bt_add_bias_residual_layernorm_kslices(None, 2, None, one, one, one, ctypes.c_float(1e-12), 4, 16,
                                                      one, None) == 1


def test_layer_checks(lib):
    one = 256
    good = bt.bt_layer(768, 12, 64, 3072, 1e-12, 0, *[one] * 12)
    n = lib.bt_layer_workspace_bytes(ctypes.byref(good), 100, 4, 64)
    # qkv + attn + proj + y1 + g + ping + pong + two per-row statistics buffers, each 256-byte aligned
    assert n >= 2 * 100 * (3 * 768 + 5 * 768 + 3072) + 2 * 100 * 8 and n % 256 == 0
    assert lib.bt_layer_workspace_bytes(ctypes.byref(good), 0, 4, 64) == 0
    x, y, cu, ws = ctypes.c_void_p(256), ctypes.c_void_p(512), ctypes.c_void_p(768), ctypes.c_void_p(1024)
    call = lambda L, T=100, ws_=ws, nbytes=n, y_=y: lib.bt_encoder_layer_fwd(
        ctypes.byref(L), x, cu, 4, T, 64, y_, ws_, nbytes, None)
    assert call(good, nbytes=n - 1) == 3                       # workspace too small
    assert call(good, ws_=None) == 3
    assert call(good, y_=x) == 1                               # in-place not allowed
    assert call(good, T=0) == 0
    assert call(good, T=4 * 64 + 1) == 1                       # more tokens than B*max_len
    assert call(bt.bt_layer(768, 12, 32, 3072, 1e-12, 0, *[one] * 12)) == 2      # head_dim
    assert call(bt.bt_layer(768, 10, 64, 3072, 1e-12, 0, *[one] * 12)) == 2      # H != heads*d
    assert call(bt.bt_layer(768, 12, 64, 3072, 1e-12, 5, *[one] * 12)) == 1      # gelu kind
    assert call(bt.bt_layer(768, 12, 64, 3072, 1e-12, 0, *([one] * 11 + [0]))) == 1  # null parameter
    arr = (bt.bt_layer * 2)(good, bt.bt_layer(1024, 16, 64, 4096, 1e-12, 0, *[one] * 12))
    assert lib.bt_encoder_fwd(arr, 2, None, x, cu, 4, 100, 64, y, ws, n, None) == 1  # mixed shapes
    assert lib.bt_encoder_fwd(arr, 0, None, x, cu, 4, 100, 64, y, ws, n, None) == 1
    pad = lambda T=100, x_=x, y_=y, ws_=ws, nb=n: lib.bt_encoder_fwd_padded(
        (bt.bt_layer * 1)(good), 1, None, x_, cu, cu, 4, T, 64, y_, ws_, nb, None)
    assert pad(T=4 * 64 + 1) == 1                              # more tokens than B*S
    assert pad(y_=x) == 1                                      # in-place not allowed
    assert pad(x_=None) == 1
    assert pad(ws_=None) == 3 and pad(nb=n - 1) == 3
    assert lib.bt_encoder_fwd_padded((bt.bt_layer * 1)(good), 1, ctypes.c_void_p(4), x, cu, cu, 4, 100, 64, y, ws, n,
                                     None) == 1                 # misaligned fold vectors
    # build_offsets + padded forward in one call: every refusal comes before the prefix-sum kernel would run
    n_all = lib.bt_layer_workspace_bytes(ctypes.byref(good), 4 * 64, 4, 64)
    tot = (ctypes.c_int32 * 2)()
    masked = lambda x_=x, y_=y, ws_=ws, nb=n_all, L=good, fold=None: lib.bt_encoder_fwd_masked(
        (bt.bt_layer * 1)(L), 1, fold, x_, None, cu, 4, 64, cu, cu, tot, y_, ws_, nb, None)
    assert masked(nb=n) == 3                                   # workspace for 100 tokens, but B*S = 256 may come
    assert masked(ws_=None) == 3
    assert masked(x_=None) == 1 and masked(y_=x) == 1
    assert masked(fold=ctypes.c_void_p(4)) == 1                # misaligned fold vectors
    assert masked(L=bt.bt_layer(768, 12, 32, 3072, 1e-12, 0, *[one] * 12)) == 2  # head_dim
    same = (bt.bt_layer * 2)(good, good)
    fb = lib.bt_encoder_fold_bytes(same, 2)
    assert fb == 2 * (6 * 768 + 2 * 3072) * 4
    assert lib.bt_encoder_prepare(same, 2, None, fb, None) == 1            # null fold buffer
    assert lib.bt_encoder_prepare(same, 2, ctypes.c_void_p(256), fb - 4, None) == 3   # too small
    assert lib.bt_encoder_prepare(arr, 2, ctypes.c_void_p(256), fb, None) == 1        # mixed shapes
    assert lib.bt_encoder_fwd(same, 2, ctypes.c_void_p(4), x, cu, 4, 100, 64, y, ws, n, None) == 1  # misaligned fold


def test_no_fallback_when_library_missing(tmp_path):
    import importlib
    mod = importlib.reload(bt)
    try:
        with pytest.raises(RuntimeError, match="not built"):
            mod.load_library(str(tmp_path / "missing.so"))
    finally:
        importlib.reload(bt)


def test_gemm_kernels_use_no_scratch():
    """The GEMM kernels request some operands through inline assembly and collect them by hand; a register
    spill of such a destination before its data has arrived would store garbage.  Every GEMM kernel must
    therefore compile without scratch memory (checked in the compiler's own metadata)."""
    import shutil
    import subprocess
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    src = os.path.join(ROOT, "paper_2210_03052_amd", "csrc", "gemm.hip")
    from paper_2210_03052_amd.build import EXTRA_FLAGS, FLAGS            # the flags libbt.so is built with
    flags = [f for f in FLAGS if f != "-fPIC"] + EXTRA_FLAGS.get("gemm.hip", [])
    out = subprocess.run([hipcc, *flags, "-w", "-S", "--cuda-device-only", "-o", "-", src],
                         capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stderr[-2000:]
    sizes = re.findall(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)", out.stdout)
    assert len(sizes) >= 20
    spilled = [n for n, b in sizes if int(b) != 0]
    assert not spilled, spilled


def test_gelu_polynomial_in_the_kernel_source():
    """The GELU epilogue approximates Phi(-a) by exp2 of a polynomial whose coefficients are literals in
    gemm.hip.  Read them from the source and evaluate the same float32 Horner scheme here: within 1e-6 of
    x Phi(x) (erf from scipy) on a dense grid, and so negative beyond the fitted range that exp2 underflows
    -- so a mistyped coefficient fails without a GPU."""
    import numpy as np
    from scipy.special import erf
    src = open(os.path.join(ROOT, "paper_2210_03052_amd", "csrc", "gemm.hip")).read()
    body = src[src.index("float gelu_erf(float x)"):src.index("float gelu_tanh(float x)")]
    first = re.search(r"fmaf\(a, (-?[0-9.e+-]+)f, (-?[0-9.e+-]+)f\)", body)
    rest = re.findall(r"fmaf\(a, p, (-?[0-9.e+-]+)f\)", body)
    coef = [np.float32(first.group(1)), np.float32(first.group(2))] + [np.float32(c) for c in rest]
    assert len(coef) == 8
    x = np.concatenate([np.linspace(-12, 12, 400001), [-1e4, 1e4, -65504.0, 65504.0]]).astype(np.float32)
    a = np.abs(x)
    p = np.zeros_like(a)
    with np.errstate(over="ignore"):
        for c in coef:
            p = (p * a + c).astype(np.float32)
    got = np.maximum(x, 0) - a * np.exp2(p).astype(np.float32)
    ref = x.astype(np.float64) * 0.5 * (1.0 + erf(x.astype(np.float64) / np.sqrt(2.0)))
    assert np.abs(got - ref).max() <= 1e-6
    assert p[a >= 9].max() < -60 and (np.diff(p[:400001][x[:400001] >= 0]) <= 0).all()


def test_gemm_tile_shape_query_is_host_only():
    """bt_gemm_tile_shape answers on the host (no GPU needed): the shapes the cost model picks for the four
    products of the headline layer, the 128x128 tile just past one round of the 64x128 tiles, the fallback
    for a K that is not a multiple of 64, and the argument checks."""
    assert bt.gemm_tile_shape(2308, 2304, 768) == (192, 128)
    assert bt.gemm_tile_shape(2308, 768, 768) == (64, 128)
    assert bt.gemm_tile_shape(2308, 3072, 768, bt.ACT_GELU_ERF) == (256, 128)
    assert bt.gemm_tile_shape(2308, 768, 3072) == (64, 128)
    assert bt.gemm_tile_shape(2699, 768, 3072) == (128, 128)
    assert bt.gemm_tile_shape(100, 768, 72) == (64, 64)
    for bad in ((10, 7, 64), (10, 8, 60), (-1, 8, 64)):
        with pytest.raises(bt.BtError):
            bt.gemm_tile_shape(*bad)


def test_gemm_row_split_query_is_host_only():
    """bt_gemm_row_split: products whose tile grid fills its rounds run as one launch (the four products of the
    headline layer, the long and the large workload's FFN-down); a grid a little past a whole number of rounds
    gives its leading rows -- whole tile rows, whole rounds -- a launch of their own."""
    for shape in ((2308, 2304, 768), (2308, 768, 768), (2308, 768, 3072), (9894, 768, 3072), (4648, 1024, 4096)):
        assert bt.gemm_row_split(*shape) == 0
    assert bt.gemm_row_split(2308, 3072, 768, bt.ACT_GELU_ERF) == 0
    r = bt.gemm_row_split(2752, 3072, 768, bt.ACT_GELU_ERF)        # 11 x 24 tiles of 256 x 128: 8 past one round
    assert r == 2560                                                # 10 tile rows x 24 = 240 tiles, one round
    r = bt.gemm_row_split(6400, 4096, 1024, bt.ACT_GELU_ERF)
    assert 0 < r < 6400 and r % 64 == 0
    assert bt.gemm_row_split(100, 768, 72) == 0                     # fallback kernel: never split
    with pytest.raises(bt.BtError):
        bt.gemm_row_split(10, 7, 64)
