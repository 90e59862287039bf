"""Seeded synthetic inputs shaped like the paper's BERT workloads.

This module only draws random numbers (numpy ``default_rng``) and rounds them
to fp16 once; it contains none of the method's arithmetic.  It is the one
module that both the tests of the CPU oracle and the callers of the HIP
library (tests, bench, smoke) use, so that both sides see identical numbers.

Workloads follow the evaluation protocol of Sec. IV: fp16 tensors, sequence
lengths drawn uniformly at random, standard BERT shapes (12 heads x 64,
hidden 768, FFN 3072; the "large" shape is 16 x 64, hidden 1024, FFN 4096),
plus two of the stack variants of Table IV (cross-layer weight sharing with 16
heads, and a 6-layer stack).
The paper uses synthetic random lengths itself, so no dataset is stood in for.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 22100305


@dataclass(frozen=True)
class Workload:
    name: str
    index: int           # 1-based position in the list of configurations
    B: int               # batch size
    S: int               # maximum sequence length (padded length)
    H: int               # hidden size = heads * head_dim
    heads: int
    head_dim: int
    F: int               # FFN width
    layers: int          # 0 = attention alone
    length_law: str
    ln_eps: float = 1e-12
    shared_weights: bool = False   # every layer uses layer 0's parameters (cross-layer sharing, Table IV)

    @property
    def seed_lengths(self):
        return BASE_SEED + self.index

    @property
    def seed_tensors(self):
        return BASE_SEED + self.index + 100


WORKLOADS = {
    "layer_b4_s64": Workload("layer_b4_s64", 1, 4, 64, 768, 12, 64, 3072, 1, "U[8,64]"),
    "mha_b16_s256": Workload("mha_b16_s256", 2, 16, 256, 768, 12, 64, 3072, 0, "U[1,256]"),
    "bert_base_b16_s256": Workload("bert_base_b16_s256", 3, 16, 256, 768, 12, 64, 3072, 12, "U[51,256]"),
    "bert_base_b16_s1024": Workload("bert_base_b16_s1024", 4, 16, 1024, 768, 12, 64, 3072, 12, "U[128,1024]"),
    "bert_large_b32_s512": Workload("bert_large_b32_s512", 5, 32, 512, 1024, 16, 64, 4096, 24,
                                    "80% U[16,128] + 20% U[384,512], shuffled"),
    # Shape variants of Table IV (layers / heads / head size): same kernels, different stacks.
    "albert_b16_s256": Workload("albert_b16_s256", 6, 16, 256, 1024, 16, 64, 4096, 12, "U[51,256]",
                                shared_weights=True),                                        # 12 / 16 / 64, shared
    "distilbert_b16_s256": Workload("distilbert_b16_s256", 7, 16, 256, 768, 12, 64, 3072, 6, "U[51,256]"),  # 6 / 12 / 64
}


def draw_lengths(wl: Workload) -> np.ndarray:
    """Per-sequence valid lengths (int32[B]) for a workload, seeded."""
    rng = np.random.default_rng(wl.seed_lengths)
    if wl.index == 1:
        L = rng.integers(8, 64 + 1, wl.B)
    elif wl.index == 2:
        L = rng.integers(1, 256 + 1, wl.B)
    elif wl.index in (3, 6, 7):
        L = rng.integers(51, 256 + 1, wl.B)         # mean 153.5 = 0.6 * 256
    elif wl.index == 4:
        L = rng.integers(128, 1024 + 1, wl.B)
    elif wl.index == 5:
        n_long = int(round(0.2 * wl.B))
        short = rng.integers(16, 128 + 1, wl.B - n_long)
        long_ = rng.integers(384, 512 + 1, n_long)
        L = np.concatenate([short, long_])
        rng.shuffle(L)
    else:
        raise ValueError(wl.index)
    return L.astype(np.int32)


def uniform_lengths(B: int, lo: int, hi: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).integers(lo, hi + 1, B).astype(np.int32)


def _h(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16)


def make_layer_params(wl: Workload, layer: int, stress: bool = False) -> dict:
    """One layer's parameters as fp16 numpy arrays; weights are [out, in].

    Default: weights N(0, 0.02), biases 0, LN gamma 1, beta 0 (the stated
    initialisation).  ``stress=True`` draws non-trivial biases and LN affine
    parameters as well, so that a dropped bias or affine term cannot hide.
    """
    if wl.shared_weights:
        layer = 0
    rng = np.random.default_rng([wl.seed_tensors, layer, 1 if stress else 0])
    H, F = wl.H, wl.F
    p = {
        "w_qkv": _h(rng.normal(0, 0.02, (3 * H, H))),
        "w_o": _h(rng.normal(0, 0.02, (H, H))),
        "w_1": _h(rng.normal(0, 0.02, (F, H))),
        "w_2": _h(rng.normal(0, 0.02, (H, F))),
    }
    if stress:
        p.update(
            b_qkv=_h(rng.normal(0, 0.5, 3 * H)), b_o=_h(rng.normal(0, 0.5, H)),
            b_1=_h(rng.normal(0, 0.5, F)), b_2=_h(rng.normal(0, 0.5, H)),
            ln0_g=_h(rng.normal(1, 0.2, H)), ln0_b=_h(rng.normal(0, 0.2, H)),
            ln1_g=_h(rng.normal(1, 0.2, H)), ln1_b=_h(rng.normal(0, 0.2, H)),
        )
    else:
        z = lambda n: np.zeros(n, np.float16)
        o = lambda n: np.ones(n, np.float16)
        p.update(b_qkv=z(3 * H), b_o=z(H), b_1=z(F), b_2=z(H),
                 ln0_g=o(H), ln0_b=z(H), ln1_g=o(H), ln1_b=z(H))
    p["heads"] = wl.heads
    p["head_dim"] = wl.head_dim
    p["eps"] = wl.ln_eps
    return p


def make_hidden_packed(wl: Workload, T: int) -> np.ndarray:
    """Packed hidden states fp16[T,H] ~ N(0,1)."""
    rng = np.random.default_rng([wl.seed_tensors, 1000])
    return _h(rng.normal(0, 1, (T, wl.H)))


def make_qkv_packed(wl: Workload, T: int) -> np.ndarray:
    """Packed fused QKV buffer fp16[T,3H] ~ N(0,1), row = [q | k | v]."""
    rng = np.random.default_rng([wl.seed_tensors, 2000])
    return _h(rng.normal(0, 1, (T, 3 * wl.H)))


def pad_rows(x_packed: np.ndarray, lengths, S: int, fill=0.0) -> np.ndarray:
    """Place packed rows into a right-padded [B,S,H] array (pure indexing)."""
    lengths = np.asarray(lengths)
    B = lengths.size
    out = np.full((B, S, x_packed.shape[1]), fill, dtype=x_packed.dtype)
    o = 0
    for b in range(B):
        out[b, : lengths[b]] = x_packed[o : o + lengths[b]]
        o += lengths[b]
    return out
