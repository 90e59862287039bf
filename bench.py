#!/usr/bin/env python3
"""Benchmark of the padding-free BERT encoder forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path over one synthetic batch that is
already resident in HBM: bt_build_offsets (with its one host sync) -> bt_pack ->
bt_encoder_fwd (all layers) -> bt_unpack.  Prints ONE JSON line:
sequences/s (whole job), plus
  "roofline"     the dominant kernel's achieved rate against MI355X's published
                 peak, from HIP-event timing of that kernel in this process,
  "kernels"      the same figures for every kernel of the layer,
  "cpu_baseline" the fp64 numpy oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F16 = 2500.0   # TFLOP/s, dense fp16 MFMA, published
PEAK_HBM = 8000.0        # GB/s, published

# HBM bytes per launch (fetched + written) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script, scaled by the same counters' reading of a 1 GiB copy; see profiles/ for the runs.
MEASURED_TRAFFIC = {
    ("bert_base_b16_s256", "gemm0_qkv_bias"): 35989 * 1024,
    ("bert_base_b16_s256", "varlen_mha"): 20582 * 1024,
    ("bert_base_b16_s256", "gemm1_proj"): 16892 * 1024,
    ("bert_base_b16_s256", "bias_residual_ln0"): 10455 * 1024,
    ("bert_base_b16_s256", "gemm2_bias_gelu"): 41553 * 1024,
    ("bert_base_b16_s256", "gemm3_ffn_down"): 56984 * 1024,
    ("bert_base_b16_s256", "bias_residual_ln1"): 10455 * 1024,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="bert_base_b16_s256")
    ap.add_argument("--kernel-iters", type=int, default=200, help="launches per kernel for the roofline timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernels", action="store_true", help="skip the per-kernel timing pass")
    ap.add_argument("--fold", action="store_true",
                    help="LayerNorm folded into the GEMM epilogues (5 launches per layer) instead of the plain 7-launch layers")
    ap.add_argument("--no-pipelined", action="store_true", help="skip the two-batches-in-flight throughput point")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline run: BERT-base forward over batch {1,8,16} x max_seq 64..1024, "
                         "packed (mean length 0.6 max) against the same kernels on the padded batch, and the "
                         "single-layer batch-1 points of Table III, plus fused against separate element-wise launches "
                         "(LayerNorm, GELU) at the headline shape; prints one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run one 1 GiB device copy (counter scaling)")
    return ap.parse_args()


def time_launches(torch, fn, iters, warm=10):
    """Average duration of one launch: `iters` back-to-back launches between two
    HIP events on the launch stream (includes the inter-launch gap)."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters      # microseconds


def sweep(args):
    """Small-batch / variable-length regime (the axes of the end-to-end figure, Sec. IV-E), Table III, and the
    fused kernels against separate element-wise launches (the shape of the figures of Sec. IV-A and IV-B)."""
    import torch

    import paper_2210_03052_amd as bt
    from paper_2210_03052_amd import inputs as I

    bt.load_library()
    torch.cuda.set_device(0)
    base = I.WORKLOADS["bert_base_b16_s256"]
    layers = [bt.Layer(I.make_layer_params(base, i)) for i in range(base.layers)]
    H = base.H
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")

    def forward_ms(B, S, lengths, n_layers, iters):
        T = int(lengths.sum())
        x_padded = dev(I.pad_rows(I.make_hidden_packed(base, T), lengths, S))
        ld = dev(lengths.astype(np.int32))
        ws = torch.empty(bt.layer_workspace_bytes(layers[0], B * S, B, S), dtype=torch.uint8, device="cuda:0")
        xp, yp = (torch.empty((B * S, H), dtype=torch.float16, device="cuda:0") for _ in range(2))
        ypad = torch.empty((B, S, H), dtype=torch.float16, device="cuda:0")

        def step():
            cu, tok, t = bt.build_offsets(lengths=ld, S=S)
            x = bt.pack(x_padded, tok, out=xp[:t])
            y = bt.encoder_fwd(layers[:n_layers], x, cu, S, out=yp[:t], ws=ws)
            bt.unpack(y, tok, B, S, out=ypad)

        for _ in range(5):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / iters, T

    rows = []
    for B in (1, 8, 16):
        for S in (64, 128, 256, 384, 512, 1024):
            L = I.uniform_lengths(B, -(-S // 5), S, I.BASE_SEED + 1000 * B + S)       # mean 0.6 S
            ms_packed, T = forward_ms(B, S, L, base.layers, 50)
            ms_padded, _ = forward_ms(B, S, np.full(B, S, np.int32), base.layers, 50)
            rows.append({"batch": B, "max_seq": S, "valid_tokens": T, "alpha": round(T / (B * S), 3),
                         "ms_packed": round(ms_packed, 4), "ms_all_tokens_valid": round(ms_padded, 4),
                         "speedup_from_removing_padding": round(ms_padded / ms_packed, 3)})
    table3 = []
    for S, paper_ms in ((256, 0.07), (1024, 0.09)):                                    # Table III (A100, FP16)
        ms, _ = forward_ms(1, S, np.full(1, S, np.int32), 1, 200)
        x = dev(I.make_hidden_packed(base, S))
        cu = dev(np.array([0, S], np.int32))
        y = torch.empty_like(x)
        ws = torch.empty(bt.layer_workspace_bytes(layers[0], S, 1, S), dtype=torch.uint8, device="cuda:0")
        us = time_launches(torch, lambda: bt.encoder_layer_fwd(layers[0], x, cu, S, out=y, ws=ws), 200)
        table3.append({"batch": 1, "seq": S, "layers": 1, "ms_layer_only": round(us / 1e3, 4),
                       "ms_whole_step": round(ms, 4), "paper_a100_ms": paper_ms,
                       "note": "layer only = bt_encoder_layer_fwd (7 launches, HIP events); whole step adds "
                               "build_offsets + pack + unpack"})
    # Kernel fusion at the headline shape -- the shape of the add-bias + LayerNorm and add-bias + GELU figures
    # (Sec. IV-A, IV-B).  "Separate" runs the same arithmetic as one launch per element-wise operation, with
    # torch's element-wise kernels standing in for the unfused ones (they are not part of the library).
    wl = I.WORKLOADS["bert_base_b16_s256"]
    T = int(I.draw_lengths(wl).sum())
    F = wl.F
    rng = np.random.default_rng(I.BASE_SEED)
    h16 = lambda *shape, s=1.0: dev(rng.normal(0, s, shape).astype(np.float16))
    x, r, a = h16(T, H), h16(T, H), h16(T, H)
    b_h, g_h, be_h, b_f, w1 = h16(H, s=0.5), h16(H), h16(H), h16(F, s=0.5), h16(F, H, s=0.03)
    y_h, y_f = torch.empty_like(x), torch.empty((T, F), dtype=torch.float16, device="cuda:0")
    nn = torch.nn.functional
    def graph_us(fn, per_graph=20, replays=20):
        """GPU time of one call: `per_graph` calls captured in a HIP graph (no host launch cost in the
        timed region: both sides are a few microseconds of GPU work per launch) and replayed between events."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(per_graph):
                fn()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (per_graph * replays)

    ln_fused = graph_us(lambda: bt.add_bias_residual_layernorm(x, b_h, r, g_h, be_h, 1e-12, out=y_h))
    ln_separate = graph_us(lambda: nn.layer_norm((x + b_h) + r, (H,), g_h, be_h, 1e-12))
    gelu_fused = graph_us(lambda: bt.gemm_bias_act(a, w1, b_f, 1, out=y_f))
    gelu_separate = graph_us(lambda: nn.gelu(bt.gemm_bias_act(a, w1, None, 0, out=y_f) + b_f))
    # Attention (the shape of the fused-MHA figures, Sec. IV-C): the variable-length fused kernel on the packed
    # batch against padded attention through torch -- three launches with the S x S logits in memory
    # (batched product, masked softmax, batched product), and torch's own fused padded kernel where this
    # torch build has one.  Stand-ins again; same lengths, heads and head size.
    attention = []
    for wname in ("bert_base_b16_s256", "bert_base_b16_s1024"):
        w = I.WORKLOADS[wname]
        Lw = I.draw_lengths(w)
        Tw, S, B, nh = int(Lw.sum()), w.S, w.B, w.heads
        qkv = h16(Tw, 3 * nh * 64)
        cu = dev(np.concatenate([[0], np.cumsum(Lw)]).astype(np.int32))
        o = torch.empty((Tw, nh * 64), dtype=torch.float16, device="cuda:0")
        fused = graph_us(lambda: bt.varlen_mha(qkv, cu, S, nh, out=o), per_graph=10, replays=10)
        q, k, v = (torch.randn((B, nh, S, 64), dtype=torch.float16, device="cuda:0") for _ in range(3))
        keep = dev(np.arange(S)[None, :] < Lw[:, None])[:, None, None, :]          # [B,1,1,S] valid keys
        neg = torch.zeros((B, 1, 1, S), dtype=torch.float16, device="cuda:0").masked_fill(~keep, float("-inf"))
        three = graph_us(lambda: torch.matmul(torch.softmax(torch.matmul(q, k.transpose(-1, -2)) * 0.125 + neg, -1), v),
                         per_graph=10, replays=10)
        row = {"workload": wname, "valid_tokens": Tw, "fused_varlen_us": round(fused, 2),
               "padded_three_launches_us": round(three, 2)}
        try:
            sdpa = graph_us(lambda: nn.scaled_dot_product_attention(q, k, v, attn_mask=neg), per_graph=10, replays=10)
            row["padded_torch_fused_us"] = round(sdpa, 2)
        except Exception as e:                                                     # no such kernel in this build
            row["padded_torch_fused_us"] = None
        attention.append(row)
    fusion = {"tokens": T, "hidden": H, "ffn": F, "attention": attention,
              "add_bias_residual_layernorm_us": {"fused": round(ln_fused, 2), "separate_3_launches": round(ln_separate, 2),
                                                 "saved": round(1 - ln_fused / ln_separate, 3)},
              "gemm_add_bias_gelu_us": {"fused": round(gelu_fused, 2), "separate_3_launches": round(gelu_separate, 2),
                                        "saved": round(1 - gelu_fused / gelu_separate, 3)},
              "note": "separate = torch element-wise kernels as stand-ins for unfused ones; paper (A100): "
                      "LayerNorm fusion 61-69 % of that step, GELU fusion 24 % of GEMM+bias+GELU"}
    print(json.dumps({"metric": "ms per BERT-base forward (12 layers, fp16), packed vs all tokens valid",
                      "kernel_fusion": fusion,
                      "unit": "ms", "n_gpus": 1, "dtype": "f16", "data": "synthetic", "higher_is_better": False,
                      "length_law": "U[ceil(0.2 S), S] (mean 0.6 S)", "sweep": rows, "table3_single_layer": table3}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (sequences are independent, so more GPUs would be "
              "plain data parallelism with no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2210_03052_amd as bt
    from paper_2210_03052_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.sweep:
        return sweep(args)
    bt.load_library()                      # raises if libbt.so is not built: no fallback
    torch.cuda.set_device(0)
    wl = I.WORKLOADS[args.workload]
    if wl.layers < 1:
        print("bench.py: pick an encoder workload", file=sys.stderr)
        sys.exit(2)

    # ---------------- synthetic batch, resident in HBM before timing starts
    L = I.draw_lengths(wl)
    T = int(L.sum())
    sum_l2 = int((L.astype(np.int64) ** 2).sum())
    H, F, nl = wl.H, wl.F, wl.layers
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    x_packed_h = I.make_hidden_packed(wl, T)
    x_padded = dev(I.pad_rows(x_packed_h, L, wl.S))
    lengths_d = dev(L)
    params = [I.make_layer_params(wl, i) for i in range(nl)]
    layers = [bt.Layer(p) for p in params]
    fold = bt.encoder_prepare(layers) if args.fold else None   # depends on the parameters only: not timed
    ws = torch.empty(bt.layer_workspace_bytes(layers[0], wl.B * wl.S, wl.B, wl.S), dtype=torch.uint8, device="cuda:0")
    x_packed = torch.empty((wl.B * wl.S, H), dtype=torch.float16, device="cuda:0")
    y_packed = torch.empty((wl.B * wl.S, H), dtype=torch.float16, device="cuda:0")
    y_padded = torch.empty((wl.B, wl.S, H), dtype=torch.float16, device="cuda:0")

    def step():
        cu, tok, t = bt.build_offsets(lengths=lengths_d, S=wl.S)
        xp = bt.pack(x_padded, tok, out=x_packed[:t])
        yp = bt.encoder_fwd(layers, xp, cu, wl.S, out=y_packed[:t], ws=ws, fold=fold)
        bt.unpack(yp, tok, wl.B, wl.S, out=y_padded)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    seq_per_s = wl.B * args.steps / dt
    flops_step = nl * (24.0 * T * H * H + 4.0 * sum_l2 * H)

    out = {
        "metric": "sequences/s BERT-base fp16 varlen (b16, max256)" if args.workload == "bert_base_b16_s256"
                  else f"sequences/s {args.workload} fp16 varlen",
        "value": round(seq_per_s, 1), "unit": "sequences/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": args.workload, "batch": wl.B, "max_seq": wl.S, "hidden": H, "heads": wl.heads,
                   "ffn": F, "layers": nl, "length_law": wl.length_law, "valid_tokens": T, "sum_len_sq": sum_l2,
                   "step": "build_offsets+pack+encoder_fwd+unpack", "layernorm_folded": fold is not None},
        "useful_tflops_per_s": round(flops_step / (ms_per_step * 1e-3) / 1e12, 2),
    }

    # ---------------- the same step with pack / unpack fused into the first / last kernels (extra point)
    if fold is None:
        def step_fused():
            cu, tok, t = bt.build_offsets(lengths=lengths_d, S=wl.S)
            bt.encoder_fwd_padded(layers, x_padded, tok, cu, out=y_padded2, ws=ws)

        y_padded2 = torch.empty_like(y_padded)
        for _ in range(max(args.warmup // 2, 2)):
            step_fused()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_fused()
        torch.cuda.synchronize()
        dtf = time.perf_counter() - t0
        out["fused_pack_unpack"] = {"value": round(wl.B * args.steps / dtf, 1), "unit": "sequences/s",
                                    "ms_per_step": round(dtf * 1e3 / args.steps, 4),
                                    "step": "build_offsets+encoder_fwd_padded",
                                    "outputs_equal": bool(torch.equal(y_padded2, y_padded))}

    # ---------------- the same step with pack + encoder + unpack replayed from a HIP graph (extra point)
    # One graph launch instead of ~90 kernel launches per step: if this is faster than `value`, the host of
    # this box did not keep ahead of the GPU in the eager loop; on a quiet host the two agree.
    if fold is None:
        y_padded3 = torch.empty_like(y_padded)
        cu_g, tok_g, t_g = bt.build_offsets(lengths=lengths_d, S=wl.S)

        def body():
            xp = bt.pack(x_padded, tok_g, out=x_packed[:t_g])
            yp = bt.encoder_fwd(layers, xp, cu_g, wl.S, out=y_packed[:t_g], ws=ws)
            bt.unpack(yp, tok_g, wl.B, wl.S, out=y_padded3)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            body()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            body()

        def step_graph():
            bt.build_offsets(lengths=lengths_d, S=wl.S)      # same offsets every step here; still computed and waited for
            graph.replay()

        for _ in range(max(args.warmup // 2, 2)):
            step_graph()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_graph()
        torch.cuda.synchronize()
        dtg = time.perf_counter() - t0
        out["graph_replay"] = {"value": round(wl.B * args.steps / dtg, 1), "unit": "sequences/s",
                               "ms_per_step": round(dtg * 1e3 / args.steps, 4),
                               "step": "build_offsets + one HIP graph of pack+encoder_fwd+unpack",
                               "outputs_equal": bool(torch.equal(y_padded3, y_padded))}

    # ---------------- throughput with two batches in flight (extra point, not `value`)
    # One batch at a time leaves the GPU idle at every kernel boundary (~2.5 us per dependent launch) and
    # while the host waits for the token count in build_offsets.  A server keeps a second batch in flight
    # on another stream, which fills those holes; each batch has its own buffers and its own host thread,
    # the library keeps no state between calls.  Same steps, same kernels, same results.
    if not args.no_pipelined:
        import threading

        class Batch:
            def __init__(self):
                self.stream = torch.cuda.Stream()
                self.x_padded = x_padded.clone()
                self.lengths_d = lengths_d.clone()
                self.ws = torch.empty_like(ws)
                self.x_packed, self.y_packed, self.y_padded = (torch.empty_like(x_packed), torch.empty_like(y_packed),
                                                               torch.empty_like(y_padded))

            def run(self, n):
                torch.cuda.set_device(0)
                with torch.cuda.stream(self.stream):
                    for _ in range(n):
                        cu, tok, t = bt.build_offsets(lengths=self.lengths_d, S=wl.S)
                        xp = bt.pack(self.x_padded, tok, out=self.x_packed[:t])
                        yp = bt.encoder_fwd(layers, xp, cu, wl.S, out=self.y_packed[:t], ws=self.ws, fold=fold)
                        bt.unpack(yp, tok, wl.B, wl.S, out=self.y_padded)

        batches = [Batch(), Batch()]
        per = max(args.steps // 2, 1)

        def both(n):
            th = [threading.Thread(target=b.run, args=(n,)) for b in batches]
            for t_ in th:
                t_.start()
            for t_ in th:
                t_.join()
            torch.cuda.synchronize()

        both(max(args.warmup // 2, 2))
        t0 = time.perf_counter()
        both(per)
        dt2 = time.perf_counter() - t0
        same = bool(torch.equal(batches[0].y_padded, y_padded) and torch.equal(batches[1].y_padded, y_padded))
        out["two_batches_in_flight"] = {"value": round(wl.B * 2 * per / dt2, 1), "unit": "sequences/s",
                                        "steps": 2 * per, "ms_per_step": round(dt2 * 1e3 / (2 * per), 4),
                                        "streams": 2, "outputs_equal_single_stream": same}
        del batches

    # ---------------- per-kernel timing (HIP events on the launch stream)
    # Each kernel of the layer is launched `kernel_iters` times back to back through the C ABI (raw
    # ctypes calls with prebuilt arguments, ~1 us of host time each) between two HIP events recorded
    # on the stream the kernels run on; the average includes the inter-launch gap.
    if not args.no_kernels:
        import ctypes as C
        lib = bt.load_library()
        cu, tok, _ = bt.build_offsets(lengths=lengths_d, S=wl.S)
        xp = bt.pack(x_padded, tok)
        ly = layers[0]
        P = ly.tensors
        f16 = lambda *shape: torch.empty(shape, dtype=torch.float16, device="cuda:0")
        qkv, attn, proj, y1, g, y2 = f16(T, 3 * H), f16(T, H), f16(T, H), f16(T, H), f16(T, F), f16(T, H)
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        ptr = lambda t: C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)
        eps = C.c_float(ly.eps)
        HD = H
        def bind(fn, *a):            # marshal once; the timed loop only does the foreign call
            return lambda: fn(*a)
        gemm = lambda a, w, b, M, N, K, act, c: bind(lib.bt_gemm_bias_act, ptr(a), ptr(w), ptr(b), M, N, K, act, ptr(c), st)
        lnk = lambda x_, b, r, ga, be, y_: bind(lib.bt_add_bias_residual_layernorm, ptr(x_), ptr(b), ptr(r), ptr(ga),
                                                ptr(be), eps, T, H, ptr(y_), st)
        qb = qkv.data_ptr()
        mha = bind(lib.bt_varlen_mha, C.c_void_p(qb), C.c_void_p(qb + 2 * HD), C.c_void_p(qb + 4 * HD), 3 * HD, None, None,
                   None, ptr(cu), wl.B, T, wl.S, wl.heads, wl.head_dim, C.c_float(wl.head_dim ** -0.5), ptr(attn), None,
                   0, st)
        steps = [
            ("gemm0_qkv_bias", "mfma", 6.0 * T * H * H, gemm(xp, P["w_qkv"], P["b_qkv"], T, 3 * H, H, 0, qkv)),
            ("varlen_mha", "mfma", 4.0 * sum_l2 * H, mha),
            ("gemm1_proj", "mfma", 2.0 * T * H * H, gemm(attn, P["w_o"], None, T, H, H, 0, proj)),
            ("bias_residual_ln0", "hbm", 6.0 * T * H, lnk(proj, P["b_o"], xp, P["ln0_g"], P["ln0_b"], y1)),
            ("gemm2_bias_gelu", "mfma", 2.0 * T * H * F, gemm(y1, P["w_1"], P["b_1"], T, F, H, 1, g)),
            ("gemm3_ffn_down", "mfma", 2.0 * T * H * F, gemm(g, P["w_2"], None, T, H, F, 0, proj)),
            ("bias_residual_ln1", "hbm", 6.0 * T * H, lnk(proj, P["b_2"], y1, P["ln1_g"], P["ln1_b"], y2)),
            ("pack", "hbm", 4.0 * T * H, bind(lib.bt_pack, ptr(x_padded), ptr(tok), T, H, ptr(x_packed), st)),
            ("unpack", "hbm", 2.0 * T * H + 2.0 * wl.B * wl.S * H,
             bind(lib.bt_unpack, ptr(y2), ptr(tok), T, wl.B, wl.S, H, ptr(y_padded), st)),
        ]
        gemm_shapes = {"gemm0_qkv_bias": (T, 3 * H, H, 0), "gemm1_proj": (T, H, H, 0),
                       "gemm2_bias_gelu": (T, F, H, 1), "gemm3_ffn_down": (T, H, F, 0)}
        kernels = []
        for name, bound, work, fn in steps:
            if fn() != 0:
                raise RuntimeError(f"{name} failed")
            us = time_launches(torch, fn, args.kernel_iters)
            per_step = nl if name not in ("pack", "unpack") else 1
            if bound == "mfma":
                ach, peak, unit = work / us / 1e6, PEAK_MFMA_F16, "TFLOP/s"
            else:
                ach, peak, unit = work / us / 1e3, PEAK_HBM, "GB/s"
            kernels.append({"kernel": name, "bound": bound, "us": round(us, 2), "launches_per_step": per_step,
                            "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
                            "work_per_launch": work})
            if name in gemm_shapes:
                # tile-quantisation ceiling of this product: useful share of the tiles' area times the share of
                # the 256 compute units that the last round of tiles occupies
                M_, N_, K_, act_ = gemm_shapes[name]
                bm, bn = bt.gemm_tile_shape(M_, N_, K_, act_)
                tiles = -(-M_ // bm) * -(-N_ // bn)
                rounds = -(-tiles // 256)
                kernels[-1].update({"tile": f"{bm}x{bn}", "tiles": tiles, "rounds_of_256_cus": rounds,
                                    "tile_quantisation_ceiling": round(M_ * N_ / (tiles * bm * bn) * tiles / (rounds * 256), 4)})
        dom = max(kernels, key=lambda k: k["us"] * k["launches_per_step"])
        out["roofline"] = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"],
                           "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"],
                           "traffic": MEASURED_TRAFFIC.get((args.workload, dom["kernel"])),
                           "us_per_launch": dom["us"], "work_per_launch": dom["work_per_launch"]}
        out["kernels"] = kernels
        out["kernel_time_sum_ms_per_step"] = round(sum(k["us"] * k["launches_per_step"] for k in kernels) / 1e3, 4)

        # ---- two more measured points named by the metric ----------------------------------------
        # (a) variable-length MHA alone on the "attention alone" workload (b16, max 256, U[1,256])
        wm = I.WORKLOADS["mha_b16_s256"]
        Lm = I.draw_lengths(wm)
        Tm, s2m = int(Lm.sum()), int((Lm.astype(np.int64) ** 2).sum())
        qkv_m = dev(I.make_qkv_packed(wm, Tm))
        cu_m = dev(np.concatenate([[0], np.cumsum(Lm)]).astype(np.int32))
        out_m = f16(Tm, wm.H)
        qm = qkv_m.data_ptr()
        mha_m = bind(lib.bt_varlen_mha, C.c_void_p(qm), C.c_void_p(qm + 2 * wm.H), C.c_void_p(qm + 4 * wm.H), 3 * wm.H,
                     None, None, None, ptr(cu_m), wm.B, Tm, wm.S, wm.heads, wm.head_dim,
                     C.c_float(wm.head_dim ** -0.5), ptr(out_m), None, 0, st)
        us_m = time_launches(torch, mha_m, args.kernel_iters)
        out["varlen_mha_b16_s256"] = {"us": round(us_m, 2), "valid_tokens": Tm, "sum_len_sq": s2m,
                                      "tflops": round(4.0 * s2m * wm.H / us_m / 1e6, 2),
                                      "frac_mfma_peak": round(4.0 * s2m * wm.H / us_m / 1e6 / PEAK_MFMA_F16, 4)}
        # (b) the HBM-bound kernels at a streaming shape (tensors >> the 256 MB Infinity Cache), same code path
        Ts = 262144
        xs, rs, ys = f16(Ts, H), f16(Ts, H), f16(Ts, H)
        xs.normal_(); rs.normal_()
        ln_s = bind(lib.bt_add_bias_residual_layernorm, ptr(xs), ptr(P["b_o"]), ptr(rs), ptr(P["ln0_g"]), ptr(P["ln0_b"]),
                    eps, Ts, H, ptr(ys), st)
        us_ln = time_launches(torch, ln_s, 20, warm=3)
        tok_s = torch.arange(Ts, dtype=torch.int32, device="cuda:0")
        pk_s = bind(lib.bt_pack, ptr(xs), ptr(tok_s), Ts, H, ptr(ys), st)
        us_pk = time_launches(torch, pk_s, 20, warm=3)
        out["hbm_streaming"] = {
            "tokens": Ts, "hidden": H,
            "bias_residual_ln": {"us": round(us_ln, 1), "GBps": round(6.0 * Ts * H / us_ln / 1e3, 1),
                                 "frac_hbm_peak": round(6.0 * Ts * H / us_ln / 1e3 / PEAK_HBM, 4)},
            "pack": {"us": round(us_pk, 1), "GBps": round(4.0 * Ts * H / us_pk / 1e3, 1),
                     "frac_hbm_peak": round(4.0 * Ts * H / us_pk / 1e3 / PEAK_HBM, 4)}}
        del xs, rs, ys

    if args.calibrate_copy:
        # a plain device copy of known size (1 GiB read + 1 GiB written) for scaling rocprofv3's
        # FETCH_SIZE / WRITE_SIZE counters
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()

    # ---------------- CPU baseline: the oracle as it stands, on this machine's cores
    if not args.no_cpu_baseline:
        from oracle import bt_oracle as O
        cores = len(os.sched_getaffinity(0))
        try:                                                   # threads the BLAS behind numpy really uses
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [cores])
        except Exception:
            pass
        mask = O.lengths_to_mask(L, wl.S)
        xh = I.pad_rows(x_packed_h, L, wl.S).astype(np.float64)
        ow = [O.LayerWeights(**p) for p in params]
        n_base = min(nl, 12)
        O.encoder_layer(xh[:2], mask[:2], ow[0])            # warm the BLAS threads
        t0 = time.perf_counter()
        O.encoder_stack(xh, mask, ow[:n_base])
        cpu_s = (time.perf_counter() - t0) * nl / n_base
        out["cpu_baseline"] = {"value": round(wl.B / cpu_s, 3), "unit": "sequences/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"whole batch, {n_base} of {nl} layers timed once (scaled to {nl}), "
                                         f"numpy fp64 padded semantics", "seconds": round(cpu_s, 2)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
