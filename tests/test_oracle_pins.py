"""Pins for the CPU oracle (no GPU): the oracle is checked against things other
than itself -- the paper's worked packing example, brute-force scalar loops,
closed forms, invariants and the dense special case computed with torch's
float64 CPU library routines."""
import math
import os

import numpy as np
import pytest

from oracle import bt_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- offsets
def _read_golden(path):
    d = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            d[key] = [int(v) for v in vals]
    return d


def test_fig4_worked_example():
    """Sec. III-D, Fig. 4: lengths (5,2,4), max length 5."""
    g = _read_golden(os.path.join(GOLDEN, "fig4_offsets.txt"))
    S = g["S"][0]
    mask = np.array(g["mask"], dtype=np.int32).reshape(-1, S)
    assert np.array_equal(O.lengths_to_mask(g["lengths"], S), mask)
    cu, tok, T = O.build_offsets(mask)
    assert T == g["T"][0]
    assert cu.tolist() == g["cu_seqlens"]
    assert tok.tolist() == g["token_idx"]
    # hidden size 3 as in the figure: packing keeps exactly the valid columns
    x = np.arange(3 * S * 3, dtype=np.float64).reshape(3, S, 3)
    p = O.pack(x, tok)
    assert p.shape == (11, 3)
    assert np.array_equal(p[5], x[1, 0]) and np.array_equal(p[7], x[2, 0])


@pytest.mark.parametrize("seed", range(6))
def test_offsets_bruteforce_any_mask(seed):
    rng = np.random.default_rng(seed)
    B, S = int(rng.integers(1, 7)), int(rng.integers(1, 40))
    mask = (rng.random((B, S)) < 0.6).astype(np.int32)       # holes allowed
    cu, tok, T = O.build_offsets(mask)
    assert np.array_equal(tok, np.flatnonzero(mask.reshape(-1)))
    assert T == int(mask.sum()) == cu[-1]
    assert np.array_equal(np.diff(cu), mask.sum(axis=1))
    x = rng.normal(size=(B, S, 5))
    assert np.array_equal(O.unpack(O.pack(x, tok), tok, B, S), x * mask[..., None])


def test_offsets_degenerate():
    cu, tok, T = O.build_offsets(np.zeros((3, 4), np.int32))
    assert T == 0 and tok.size == 0 and cu.tolist() == [0, 0, 0, 0]
    cu, tok, T = O.build_offsets(np.ones((2, 3), np.int32))
    assert T == 6 and tok.tolist() == list(range(6)) and cu.tolist() == [0, 3, 6]
    with pytest.raises(ValueError):
        O.lengths_to_mask([5], 4)


# ---------------------------------------------------------------- attention
def _brute_attention(q, k, v, mask, heads):
    """Scalar loops, python floats: eq. (1) with masked keys skipped."""
    B, S, HD = q.shape
    d = HD // heads
    out = [[[0.0] * HD for _ in range(S)] for _ in range(B)]
    for b in range(B):
        for j in range(heads):
            for t in range(S):
                if not mask[b][t]:
                    continue
                logit = {}
                for u in range(S):
                    if not mask[b][u]:
                        continue
                    acc = 0.0
                    for c in range(d):
                        acc += float(q[b, t, j * d + c]) * float(k[b, u, j * d + c])
                    logit[u] = acc / math.sqrt(d)
                mx = max(logit.values())
                den = sum(math.exp(x - mx) for x in logit.values())
                for c in range(d):
                    acc = 0.0
                    for u, x in logit.items():
                        acc += math.exp(x - mx) / den * float(v[b, u, j * d + c])
                    out[b][t][j * d + c] = acc
    return np.array(out)


@pytest.mark.parametrize("seed", range(5))
def test_attention_vs_bruteforce(seed):
    rng = np.random.default_rng(100 + seed)
    B, S, heads, d = int(rng.integers(1, 4)), int(rng.integers(2, 9)), int(rng.integers(1, 4)), int(rng.integers(1, 9))
    q, k, v = (rng.normal(size=(B, S, heads * d)) for _ in range(3))
    if seed % 2:
        mask = (rng.random((B, S)) < 0.7).astype(np.int32)
        mask[:, 0] = 1
    else:
        mask = O.lengths_to_mask(rng.integers(1, S + 1, B), S)
    got = O.attention_padded(q, k, v, mask, heads)
    ref = _brute_attention(q, k, v, mask.tolist(), heads)
    assert np.abs(got - ref).max() < 1e-12


def test_softmax_rows_sum_to_one():
    rng = np.random.default_rng(7)
    x = rng.normal(size=(9, 13)) * 30
    x[:, 5:] = -np.inf
    p = O.softmax_rows(x)
    assert np.abs(p.sum(axis=1) - 1).max() < 1e-12
    assert np.all(p[:, 5:] == 0)


def test_attention_closed_forms():
    rng = np.random.default_rng(8)
    heads, d, S = 2, 4, 6
    q, k, v = (rng.normal(size=(2, S, heads * d)) for _ in range(3))
    # a sentence of one token attends to itself only: output row == V row
    mask = O.lengths_to_mask([1, S], S)
    out = O.attention_padded(q, k, v, mask, heads)
    assert np.allclose(out[0, 0], v[0, 0], atol=1e-15)
    assert np.all(out[0, 1:] == 0)
    # identical keys => uniform weights => mean of the valid V rows
    k2 = np.broadcast_to(k[:, :1], k.shape).copy()
    L = 4
    mask = O.lengths_to_mask([L, L], S)
    out = O.attention_padded(q, k2, v, mask, heads)
    assert np.abs(out[:, :L] - v[:, :L].mean(axis=1, keepdims=True)).max() < 1e-13
    # scale: doubling it equals doubling q
    a = O.attention_padded(q, k, v, mask, heads, scale=2.0 / math.sqrt(d))
    b = O.attention_padded(2 * q, k, v, mask, heads)
    assert np.abs(a - b).max() < 1e-12


def test_attention_invariances():
    rng = np.random.default_rng(9)
    B, S, heads, d = 3, 7, 2, 3
    lengths = np.array([4, 7, 2])
    mask = O.lengths_to_mask(lengths, S)
    q, k, v = (rng.normal(size=(B, S, heads * d)) for _ in range(3))
    ref = O.attention_padded(q, k, v, mask, heads)
    # pads never influence valid tokens (finite garbage in every padded slot)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for a in (q2, k2, v2):
        a[mask == 0] = 1e4
    got = O.attention_padded(q2, k2, v2, mask, heads)
    assert np.array_equal(got[mask == 1], ref[mask == 1])
    # sentences are independent
    q3 = q.copy(); q3[1] += 1.0
    got = O.attention_padded(q3, k, v, mask, heads)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[2], ref[2])
    assert not np.allclose(got[1], ref[1])
    # permuting a sentence's tokens permutes its outputs
    perm = np.array([2, 0, 3, 1])
    qp, kp, vp = q.copy(), k.copy(), v.copy()
    for a, src in ((qp, q), (kp, k), (vp, v)):
        a[0, :4] = src[0, perm]
    got = O.attention_padded(qp, kp, vp, mask, heads)
    assert np.abs(got[0, :4] - ref[0, perm]).max() < 1e-13


def test_varlen_packed_matches_padded():
    rng = np.random.default_rng(10)
    heads, d = 2, 4
    lengths = np.array([3, 1, 5])
    cu = np.concatenate([[0], np.cumsum(lengths)])
    T = cu[-1]
    qkv = rng.normal(size=(T, 3 * heads * d))
    bq, bk, bv = (rng.normal(size=heads * d) for _ in range(3))
    got = O.varlen_mha_packed(qkv, cu, heads, d, bq=bq, bk=bk, bv=bv)
    # sentence by sentence, unpadded, with the brute-force loops
    for b in range(3):
        rows = slice(cu[b], cu[b + 1])
        q = (qkv[rows, :8] + bq)[None]; k = (qkv[rows, 8:16] + bk)[None]; v = (qkv[rows, 16:] + bv)[None]
        ref = _brute_attention(q, k, v, [[1] * lengths[b]], heads)[0]
        assert np.abs(got[rows] - ref).max() < 1e-12


# ---------------------------------------------------------------- LN / GELU
def test_layernorm_moments_and_affine():
    rng = np.random.default_rng(11)
    x = rng.normal(size=(5, 64)) * 3 + 2
    y = O.layer_norm(x, np.ones(64), np.zeros(64), 1e-12)
    assert np.abs(y.mean(axis=1)).max() < 1e-12
    assert np.abs(y.var(axis=1) - 1).max() < 1e-9
    g, b = rng.normal(size=64), rng.normal(size=64)
    assert np.allclose(O.layer_norm(x, g, b, 1e-12), y * g + b, atol=1e-14)
    # eps matters as sigma^2/(sigma^2+eps)
    y2 = O.layer_norm(x, np.ones(64), np.zeros(64), 1.0)
    assert np.allclose(y2.var(axis=1), x.var(axis=1) / (x.var(axis=1) + 1.0), atol=1e-12)
    # scalar re-computation of one row
    r = x[0]; mu = sum(r) / 64; var = sum((t - mu) ** 2 for t in r) / 64
    assert np.allclose(y[0], [(t - mu) / math.sqrt(var + 1e-12) for t in r], atol=1e-13)


def test_gelu_closed_forms():
    assert O.gelu(0.0) == 0.0
    assert abs(O.gelu(10.0) - 10.0) < 1e-12 and abs(O.gelu(-10.0)) < 1e-12
    x = np.linspace(-4, 4, 33)
    assert np.abs(O.gelu(x) - O.gelu(-x) - x).max() < 1e-14
    assert abs(O.gelu(1.0) - 0.5 * (1 + math.erf(1 / math.sqrt(2)))) < 1e-15
    assert abs(O.gelu(1.0) - 0.8413447460685429) < 1e-12      # Phi(1)


def test_gelu_tanh_form_pins():
    """The tanh form: closed forms, the odd-part identity (tanh is odd), torch's float64 CPU routine as an
    independent library implementation, and the known distance to the exact form (largest near |x| = 2.7,
    4.7e-4; identical at 0 and in both tails)."""
    import torch
    assert O.gelu_tanh(0.0) == 0.0
    assert abs(O.gelu_tanh(10.0) - 10.0) < 1e-12 and abs(O.gelu_tanh(-10.0)) < 1e-12
    x = np.linspace(-6, 6, 2401)
    assert np.abs(O.gelu_tanh(x) - O.gelu_tanh(-x) - x).max() < 1e-14
    ref = torch.nn.functional.gelu(torch.tensor(x, dtype=torch.float64), approximate="tanh").numpy()
    assert np.abs(O.gelu_tanh(x) - ref).max() < 1e-14
    # scalar re-computation at one point
    u = math.sqrt(2 / math.pi) * (1.5 + 0.044715 * 1.5 ** 3)
    assert abs(O.gelu_tanh(1.5) - 0.75 * (1 + math.tanh(u))) < 1e-15
    gap = np.abs(O.gelu_tanh(x) - O.gelu(x))
    assert 4.5e-4 < gap.max() < 5e-4 and 2.5 < abs(x[gap.argmax()]) < 2.9
    assert gap[np.abs(x) > 5.5].max() < 1e-7


def test_layer_gelu_kind_selects_the_activation():
    """gelu_kind reaches the FFN and nothing else: the two layers differ by exactly the FFN-down image of the
    activation difference, pushed through the last LayerNorm (checked by recomputing that path by hand)."""
    rng = np.random.default_rng(21)
    H, heads, F, S = 8, 2, 16, 4
    p = _tiny_layer(rng, H, heads, F)
    x = rng.normal(size=(1, S, H)) * 2
    mask = np.ones((1, S), np.int32)
    a = O.encoder_layer(x, mask, O.LayerWeights(**p))
    b = O.encoder_layer(x, mask, O.LayerWeights(**p, gelu_kind="tanh"))
    assert 0 < np.abs(a - b).max() < 5e-2
    w = O.LayerWeights(**p)
    qkv = x @ w.w_qkv.T + w.b_qkv
    attn = O.attention_padded(qkv[..., :H], qkv[..., H:2 * H], qkv[..., 2 * H:], mask, heads)
    y1 = O.layer_norm(x + attn @ w.w_o.T + w.b_o, w.ln0_g, w.ln0_b, w.eps)
    h = y1 @ w.w_1.T + w.b_1
    want = O.layer_norm(y1 + O.gelu_tanh(h) @ w.w_2.T + w.b_2, w.ln1_g, w.ln1_b, w.eps)
    assert np.abs(b - want).max() < 1e-13
    with pytest.raises(ValueError):
        O.LayerWeights(**p, gelu_kind="relu")


# ---------------------------------------------------------------- whole layer
def _tiny_layer(rng, H, heads, F, stress=True):
    p = dict(
        w_qkv=rng.normal(0, 0.3, (3 * H, H)), b_qkv=rng.normal(0, 0.3, 3 * H),
        w_o=rng.normal(0, 0.3, (H, H)), b_o=rng.normal(0, 0.3, H),
        ln0_g=rng.normal(1, 0.2, H), ln0_b=rng.normal(0, 0.2, H),
        w_1=rng.normal(0, 0.3, (F, H)), b_1=rng.normal(0, 0.3, F),
        w_2=rng.normal(0, 0.3, (H, F)), b_2=rng.normal(0, 0.3, H),
        ln1_g=rng.normal(1, 0.2, H), ln1_b=rng.normal(0, 0.2, H),
        heads=heads, eps=1e-5)
    return p


def _scalar_layer_one_sentence(x, p):
    """One unpadded sentence through the layer, python scalar loops only."""
    L, H = len(x), len(x[0])
    heads = p["heads"]; d = H // heads

    def linear(rows, w, b):
        return [[sum(r[i] * w[o][i] for i in range(len(r))) + b[o] for o in range(len(w))] for r in rows]

    def ln(rows, g, b, eps):
        out = []
        for r in rows:
            mu = sum(r) / len(r)
            var = sum((t - mu) ** 2 for t in r) / len(r)
            out.append([(t - mu) / math.sqrt(var + eps) * g[i] + b[i] for i, t in enumerate(r)])
        return out

    qkv = linear(x, p["w_qkv"], p["b_qkv"])
    attn = [[0.0] * H for _ in range(L)]
    for j in range(heads):
        for t in range(L):
            lg = [sum(qkv[t][j * d + c] * qkv[u][H + j * d + c] for c in range(d)) / math.sqrt(d) for u in range(L)]
            mx = max(lg); e = [math.exp(a - mx) for a in lg]; s = sum(e)
            for c in range(d):
                attn[t][j * d + c] = sum(e[u] / s * qkv[u][2 * H + j * d + c] for u in range(L))
    proj = linear(attn, p["w_o"], p["b_o"])
    y1 = ln([[x[t][i] + proj[t][i] for i in range(H)] for t in range(L)], p["ln0_g"], p["ln0_b"], p["eps"])
    h = linear(y1, p["w_1"], p["b_1"])
    g = [[0.5 * a * (1 + math.erf(a / math.sqrt(2))) for a in r] for r in h]
    f = linear(g, p["w_2"], p["b_2"])
    return ln([[y1[t][i] + f[t][i] for i in range(H)] for t in range(L)], p["ln1_g"], p["ln1_b"], p["eps"])


def test_layer_vs_scalar_loops():
    rng = np.random.default_rng(12)
    H, heads, F, S = 8, 2, 16, 5
    p = _tiny_layer(rng, H, heads, F)
    lengths = [3, 5, 1]
    mask = O.lengths_to_mask(lengths, S)
    x = rng.normal(size=(3, S, H))
    x[mask == 0] = 123.0                               # garbage in the pads
    got = O.encoder_layer(x, mask, O.LayerWeights(**p))
    plist = {k: (v.tolist() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    for b, L in enumerate(lengths):
        ref = np.array(_scalar_layer_one_sentence(x[b, :L].tolist(), plist))
        assert np.abs(got[b, :L] - ref).max() < 1e-11
        assert np.all(got[b, L:] == 0)


def test_dense_layer_vs_torch_float64():
    """All lengths == S: the layer is the textbook dense layer; torch CPU
    float64 library ops serve as an independent routine."""
    import torch
    import torch.nn.functional as Fn
    rng = np.random.default_rng(13)
    B, S, H, heads, F = 2, 6, 16, 4, 32
    p = _tiny_layer(rng, H, heads, F)
    x = rng.normal(size=(B, S, H))
    got = O.encoder_layer(x, np.ones((B, S), np.int32), O.LayerWeights(**p))
    t = {k: torch.tensor(v, dtype=torch.float64) for k, v in p.items() if isinstance(v, np.ndarray)}
    X = torch.tensor(x, dtype=torch.float64)
    qkv = Fn.linear(X, t["w_qkv"], t["b_qkv"])
    q, k, v = (a.reshape(B, S, heads, H // heads).transpose(1, 2) for a in qkv.split(H, dim=-1))
    a = Fn.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(B, S, H)
    y1 = Fn.layer_norm(X + Fn.linear(a, t["w_o"], t["b_o"]), (H,), t["ln0_g"], t["ln0_b"], p["eps"])
    f = Fn.linear(Fn.gelu(Fn.linear(y1, t["w_1"], t["b_1"])), t["w_2"], t["b_2"])
    y2 = Fn.layer_norm(y1 + f, (H,), t["ln1_g"], t["ln1_b"], p["eps"])
    assert np.abs(got - y2.numpy()).max() < 1e-12


def test_stack_feeds_output_forward():
    rng = np.random.default_rng(14)
    H, heads, F, S = 8, 2, 16, 4
    layers = [O.LayerWeights(**_tiny_layer(rng, H, heads, F)) for _ in range(3)]
    mask = O.lengths_to_mask([2, 4], S)
    x = rng.normal(size=(2, S, H))
    y = x
    for w in layers:
        y = O.encoder_layer(y, mask, w)
    assert np.array_equal(O.encoder_stack(x, mask, layers), y)
    # final LN with gamma=1, beta=0 => rows have zero mean, unit variance
    p = _tiny_layer(rng, H, heads, F); p["ln1_g"] = np.ones(H); p["ln1_b"] = np.zeros(H); p["eps"] = 1e-12
    out = O.encoder_layer(x, mask, O.LayerWeights(**p))
    rows = out[mask == 1]
    assert np.abs(rows.mean(axis=1)).max() < 1e-12 and np.abs(rows.var(axis=1) - 1).max() < 1e-8


# ---------------------------------------------------------------- Table II
def test_table2_flops_from_shapes():
    """Table II closed forms against a count of multiply-adds from the shapes."""
    B, S, heads, d = 16, 256, 12, 64
    k = heads * d
    for alpha in (1.0, 0.6):
        rows = alpha * B * S                       # rows the GEMMs see
        L = alpha * S                              # per-sentence length seen by fused MHA
        want = {
            "GEMM0": 2 * rows * k * 3 * k,
            "GEMM1": 2 * rows * k * k,
            "GEMM2": 2 * rows * k * 4 * k,
            "GEMM3": 2 * rows * 4 * k * k,
        }
        got = O.table2_flops(B, S, k, alpha, "zero_padding_fmha")
        for name, val in want.items():
            assert got[name] == pytest.approx(val)
        assert got["MHA"] == pytest.approx(B * heads * (2 * L * L * d + 2 * L * L * d))
        zp = O.table2_flops(B, S, k, alpha, "zero_padding")
        assert zp["MHA"] == pytest.approx(B * heads * 4 * S * S * d)      # batched GEMM stays padded
        assert zp["GEMM2"] == pytest.approx(want["GEMM2"])
        base = O.table2_flops(B, S, k, alpha, "baseline")
        assert base["GEMM0"] == pytest.approx(6 * B * S * k * k)
