#!/usr/bin/env python3
"""Benchmark of the padding-free BERT encoder forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path over one synthetic batch that is
already resident in HBM: bt_build_offsets (prefix sum; its token count is waited
for on the host) -> bt_encoder_fwd_padded (all layers; the pack is fused into
the first GEMM's operand load and the first residual read, the unpack into the
last LayerNorm's store), made as one call of the library (bt_encoder_fwd_masked:
the same two calls without host code of the caller between them).  Before the W warm-up steps the step is repeated for about
half a second, untimed, so that the device clocks have settled (--settle).  Prints ONE
JSON line: sequences/s (whole job; mean over the timed steps, with the median and the
minimum step beside it), plus
  "roofline"     the dominant kernel's achieved rate against MI355X's published
                 peak, from HIP-event timing of that kernel in this process
                 (--peaks adds the rates this GPU sustains in an MFMA-only loop
                 and a read-only stream as measured denominators),
  "kernels"      the same figures for every kernel of the layer,
  "cpu_baseline" the fp64 numpy oracle timed on this machine's host cores.
The attention-alone workload (mha_b16_s256) times bt_varlen_mha as the step.
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

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(workload, kernel):
    """HBM-side bytes per launch of `kernel` in `workload` from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary
    under profiles/ (written by paper_2210_03052_amd.profile_summary), or None when that pair was not profiled."""
    kernel = {"bias_residual_ln0": "bias_residual_ln", "bias_residual_ln1": "bias_residual_ln"}.get(kernel, kernel)
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) == 5 and f[0] == workload and f[1] == kernel:
                return int(f[4])
    except OSError:
        pass
    return None


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
                    help="hand the library the fold vectors of bt_encoder_prepare in the timed step: it then folds the "
                         "LayerNorms into the GEMM epilogues (5 launches per layer) where the token count makes that the "
                         "faster pipeline.  Without the flag the same run is reported as the extra point "
                         "`layernorm_fold_vectors`, and `value` is the default call (no fold vectors)")
    ap.add_argument("--no-pipelined", action="store_true", help="skip the two-batches-in-flight throughput point")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline run: BERT-base forward over batch {1,8,16} x max_seq 64..1024, "
                         "packed (mean length 0.6 max) against the same kernels on the padded batch, and the "
                         "single-layer batch-1 points of Table III, plus fused against separate element-wise launches "
                         "(LayerNorm, GELU) at the headline shape; prints one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run one 1 GiB device copy (counter scaling)")
    ap.add_argument("--settle", type=float, default=0.5,
                    help="seconds of untimed steps before the warm-up steps, to let the device clocks settle (0 = none)")
    ap.add_argument("--peaks", action="store_true",
                    help="also measure what this GPU sustains in an MFMA-only fp16 loop and in a read-only stream, and "
                         "report the roofline against those measured rates as well as the published ones")
    ap.add_argument("--separate-pack-unpack", action="store_true",
                    help="time bt_pack + bt_encoder_fwd + bt_unpack as the step instead of bt_encoder_fwd_padded")
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
        ypad = torch.empty((B, S, H), dtype=torch.float16, device="cuda:0")

        def step():
            bt.encoder_fwd_masked(layers[:n_layers], x_padded, lengths=ld, out=ypad, ws=ws)

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
                       "note": "layer only = bt_encoder_layer_fwd (HIP events); whole step = build_offsets + "
                               "encoder_fwd_padded (pack / unpack fused into the first / last kernels)"})
    # Kernel fusion at the headline shape -- the shape of the add-bias + LayerNorm and add-bias + GELU figures
    # (Sec. IV-A, IV-B) and of the step-wise encoder-layer figure (Sec. IV-D), all with this repository's own
    # kernels: "unfused" runs the same arithmetic with the element-wise steps as kernels of their own
    # (csrc/unfused.hip in the measurement library; never part of the encoder path).
    import ctypes as C
    aux = C.CDLL(os.path.join(ROOT, "paper_2210_03052_amd", "libbt_peaks.so"))
    vp = C.c_void_p
    aux.bt_unfused_add_bias_residual.argtypes = [vp, vp, vp, C.c_int, C.c_int, vp, vp]
    aux.bt_unfused_bias_gelu.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp]
    aux.bt_unfused_layernorm.argtypes = [vp, vp, vp, C.c_float, C.c_int, C.c_int, vp, vp]
    cur = lambda: vp(torch.cuda.current_stream().cuda_stream)
    P_ = lambda t: vp(t.data_ptr()) if t is not None else vp(0)

    def unfused_ln(x_, b_, r_, g_, be_, tmp, y_):            # two trips over memory (Sec. IV-A baseline)
        assert aux.bt_unfused_add_bias_residual(P_(x_), P_(b_), P_(r_), x_.shape[0], x_.shape[1], P_(tmp), cur()) == 0
        assert aux.bt_unfused_layernorm(P_(tmp), P_(g_), P_(be_), 1e-12, x_.shape[0], x_.shape[1], P_(y_), cur()) == 0

    def unfused_gelu(a_, w_, b_, tmp, y_):                    # GEMM, then bias + activation as its own kernel (Sec. IV-B)
        bt.gemm_bias_act(a_, w_, None, 0, out=tmp)
        assert aux.bt_unfused_bias_gelu(P_(tmp), P_(b_), tmp.shape[0], tmp.shape[1], P_(y_), cur()) == 0

    wl = I.WORKLOADS["bert_base_b16_s256"]
    Lh = I.draw_lengths(wl)
    T = int(Lh.sum())
    F = wl.F
    rng = np.random.default_rng(I.BASE_SEED)
    h16 = lambda *shape, s=1.0: dev(rng.normal(0, s, shape).astype(np.float16))
    x, r, a = h16(T, H), h16(T, H), h16(T, H)
    b_h, g_h, be_h, b_f, w1 = h16(H, s=0.5), h16(H), h16(H), h16(F, s=0.5), h16(F, H, s=0.03)
    y_h, y_f = torch.empty_like(x), torch.empty((T, F), dtype=torch.float16, device="cuda:0")
    t_h, t_f = torch.empty_like(x), torch.empty_like(y_f)
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
    ln_separate = graph_us(lambda: unfused_ln(x, b_h, r, g_h, be_h, t_h, y_h))
    gelu_fused = graph_us(lambda: bt.gemm_bias_act(a, w1, b_f, 1, out=y_f))
    gelu_separate = graph_us(lambda: unfused_gelu(a, w1, b_f, t_f, y_f))

    # One encoder layer step by step (the shape of the step-wise figure of Sec. IV-D), composed from C-ABI calls:
    #   padded, unfused -> + fused LayerNorm -> + fused GELU -> + zero padding (packed tokens, variable-length MHA)
    # "padded" runs every sequence at the full length S (what a padded pipeline computes); the attention of the
    # padded rungs is this library's fused kernel at full length (the paper's padded baseline has an unfused
    # attention on top of that, which is not rebuilt here).
    Pm = layers[0].tensors
    def layer_variant(Tn, cu_, S_, fused_ln, fused_gelu):
        xin = h16(Tn, H)
        qkv_, at_, pr_, y1_, g_, y2_ = (torch.empty((Tn, n_), dtype=torch.float16, device="cuda:0")
                                        for n_ in (3 * H, H, H, H, F, H))
        tmp_h, tmp_f = torch.empty_like(pr_), torch.empty_like(g_)
        def run():
            bt.gemm_bias_act(xin, Pm["w_qkv"], Pm["b_qkv"], 0, out=qkv_)
            bt.varlen_mha(qkv_, cu_, S_, base.heads, out=at_)
            bt.gemm_bias_act(at_, Pm["w_o"], None, 0, out=pr_)
            if fused_ln: bt.add_bias_residual_layernorm(pr_, Pm["b_o"], xin, Pm["ln0_g"], Pm["ln0_b"], 1e-12, out=y1_)
            else: unfused_ln(pr_, Pm["b_o"], xin, Pm["ln0_g"], Pm["ln0_b"], tmp_h, y1_)
            if fused_gelu: bt.gemm_bias_act(y1_, Pm["w_1"], Pm["b_1"], 1, out=g_)
            else: unfused_gelu(y1_, Pm["w_1"], Pm["b_1"], tmp_f, g_)
            bt.gemm_bias_act(g_, Pm["w_2"], None, 0, out=pr_)
            if fused_ln: bt.add_bias_residual_layernorm(pr_, Pm["b_2"], y1_, Pm["ln1_g"], Pm["ln1_b"], 1e-12, out=y2_)
            else: unfused_ln(pr_, Pm["b_2"], y1_, Pm["ln1_g"], Pm["ln1_b"], tmp_h, y2_)
        return graph_us(run, per_graph=5, replays=10)
    stepwise = []
    for wname in ("bert_base_b16_s256", "bert_base_b16_s1024"):
        w = I.WORKLOADS[wname]
        Lw = I.draw_lengths(w)
        cu_pad = dev((np.arange(w.B + 1) * w.S).astype(np.int32))
        cu_var = dev(np.concatenate([[0], np.cumsum(Lw)]).astype(np.int32))
        rungs = [("padded, unfused", layer_variant(w.B * w.S, cu_pad, w.S, False, False)),
                 ("+ fused add-bias/residual/LayerNorm", layer_variant(w.B * w.S, cu_pad, w.S, True, False)),
                 ("+ fused add-bias/GELU", layer_variant(w.B * w.S, cu_pad, w.S, True, True)),
                 ("+ zero padding and variable-length MHA", layer_variant(int(Lw.sum()), cu_var, w.S, True, True))]
        stepwise.append({"workload": wname, "padded_tokens": w.B * w.S, "valid_tokens": int(Lw.sum()),
                         "us_per_layer": [{"variant": n_, "us": round(u_, 1)} for n_, u_ in rungs],
                         "speedup_over_first_rung": round(rungs[0][1] / rungs[-1][1], 2)})
    # Attention (the shape of the fused-MHA figures, Sec. IV-C): the variable-length fused kernel on the packed
    # batch against padded attention through torch -- three launches with the S x S logits in memory
    # (batched product, masked softmax, batched product), and torch's own fused padded kernel where this
    # torch build has one.  torch is a stand-in here (a batched padded attention is not part of this library);
    # same lengths, heads and head size.
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
    fusion = {"tokens": T, "hidden": H, "ffn": F, "attention": attention, "encoder_layer_stepwise": stepwise,
              "add_bias_residual_layernorm_us": {"fused": round(ln_fused, 2), "unfused_2_launches": round(ln_separate, 2),
                                                 "saved": round(1 - ln_fused / ln_separate, 3)},
              "gemm_add_bias_gelu_us": {"fused": round(gelu_fused, 2), "unfused_2_launches": round(gelu_separate, 2),
                                        "saved": round(1 - gelu_fused / gelu_separate, 3)},
              "note": "unfused = this repository's own element-wise kernels (csrc/unfused.hip); padded attention "
                      "rows use torch as a stand-in; paper (A100): LayerNorm fusion 61-69 % of that step, GELU "
                      "fusion 24 % of GEMM+bias+GELU"}
    print(json.dumps({"metric": "ms per BERT-base forward (12 layers, fp16), packed vs all tokens valid",
                      "kernel_fusion": fusion,
                      "unit": "ms", "n_gpus": 1, "dtype": "f16", "data": "synthetic", "higher_is_better": False,
                      "length_law": "U[ceil(0.2 S), S] (mean 0.6 S)", "sweep": rows, "table3_single_layer": table3}))


def timed_steps(torch, step, steps, warmup):
    """Runs `warmup` untimed and `steps` timed steps.  Returns (seconds for all timed steps, per-step seconds).
    The total is the wall clock between two device synchronisations around exactly `steps` steps.
    Per-step durations need no extra synchronisation: every step begins with bt_build_offsets, which returns
    only when its kernel has run, i.e. when everything the previous step enqueued on the stream is complete;
    `step(mark)` calls mark() right after that call, so the differences of consecutive marks are the GPU's
    time for one whole step (forward of step i plus the prefix-sum kernel of step i+1)."""
    for _ in range(warmup):
        step(lambda: None)
    torch.cuda.synchronize()
    stamps, returned = [], []
    mark = lambda: stamps.append(time.perf_counter())
    t0 = time.perf_counter()
    for _ in range(steps):
        step(mark)
        returned.append(time.perf_counter())
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # host time from the mark (the token count is known) to the step's return (every launch enqueued)
    timed_steps.host_enqueue_s = sorted(r - m for m, r in zip(stamps, returned))[len(returned) // 2] if stamps else None
    stamps.append(t1)
    per = [b - a for a, b in zip(stamps[:-1], stamps[1:])]
    return t1 - t0, per


def step_stats(B, total_s, per_step_s, window=1):
    """window > 1: the time stamps were taken when the step's call returned (launches enqueued), not right after its
    wait for the device, so a single difference carries the jitter of the host's enqueue time; the fastest step is
    then taken as the fastest run of `window` consecutive steps, divided by `window`."""
    n = len(per_step_s)
    srt = sorted(per_step_s)
    med = srt[n // 2] if n % 2 else 0.5 * (srt[n // 2 - 1] + srt[n // 2])
    w = max(1, min(window, n))
    fastest = min(sum(per_step_s[i:i + w]) for i in range(n - w + 1)) / w
    return {"value": round(B * n / total_s, 1), "ms_per_step": round(total_s * 1e3 / n, 4),
            "ms_per_step_median": round(med * 1e3, 4), "ms_per_step_min": round(fastest * 1e3, 4)}


def measure_peaks(torch):
    """What this GPU sustains: an MFMA-only fp16 loop (constant operands; random operands, under which the clock
    settles lower) and a read-only stream over 2 GiB."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_2210_03052_amd", "libbt_peaks.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built: run `python -m paper_2210_03052_amd.build`")
    lib = C.CDLL(path)
    lib.bt_peak_mfma_f16.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.bt_peak_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p]
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    blocks, iters = 256 * 8, 4096
    sink = torch.empty(blocks * 256, dtype=torch.float32, device="cuda:0")
    flop = blocks * 4 * iters * 4 * 2.0 * 32 * 32 * 16
    out = {}
    for pattern, key in ((0, "mfma_f16_constant_operands_tflops"), (1, "mfma_f16_random_operands_tflops")):
        fn = lambda: lib.bt_peak_mfma_f16(iters, blocks, pattern, C.c_void_p(sink.data_ptr()), st)
        if fn() != 0:
            raise RuntimeError("bt_peak_mfma_f16 failed")
        us = time_launches(torch, fn, 10, warm=3)
        out[key] = round(flop / us / 1e6, 1)
    nbytes = 2 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    src.random_(0, 255)
    rb = 256 * 16
    rsink = torch.empty(rb * 256, dtype=torch.int32, device="cuda:0")
    fn = lambda: lib.bt_peak_stream_read(C.c_void_p(src.data_ptr()), C.c_size_t(nbytes), rb, C.c_void_p(rsink.data_ptr()), st)
    if fn() != 0:
        raise RuntimeError("bt_peak_stream_read failed")
    us = time_launches(torch, fn, 10, warm=3)
    out["hbm_read_stream_GBps"] = round(nbytes / us / 1e3, 1)
    out["note"] = ("MFMA: 2048 workgroups x 4 wavefronts x 4096 x 4 independent 32x32x16 fp16 MFMAs on register "
                   "operands; read: 2 GiB, 16 bytes per lane, non-temporal")
    del src
    return out


def calibrate_copy(torch):
    """A plain device copy of known size (1 GiB read + 1 GiB written) for scaling rocprofv3's FETCH_SIZE /
    WRITE_SIZE counters."""
    a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    b = torch.empty_like(a)
    b.copy_(a)
    torch.cuda.synchronize()


def cpu_baseline_encoder(wl, L, x_packed_h, params, nl):
    """The oracle as it stands on this machine's cores: whole batch, up to 12 layers timed once, scaled to nl."""
    from oracle import bt_oracle as O
    from paper_2210_03052_amd import inputs as I
    cores = len(os.sched_getaffinity(0))
    try:                                                   # threads the BLAS behind numpy really uses
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [cores])
    except Exception:
        pass
    mask = O.lengths_to_mask(L, wl.S)
    xh = I.pad_rows(x_packed_h, L, wl.S).astype(np.float64)
    ow = [O.LayerWeights(**p) for p in params]
    # a bounded sample: as many layers as fit ~20 s of CPU work, estimated from one warm layer on two sequences
    O.encoder_layer(xh[:2], mask[:2], ow[0])            # warm the BLAS threads
    t0 = time.perf_counter()
    O.encoder_layer(xh, mask, ow[0])
    one = time.perf_counter() - t0
    n_base = int(max(1, min(nl, 12, 20.0 // max(one, 1e-3))))
    t0 = time.perf_counter()
    O.encoder_stack(xh, mask, ow[:n_base])
    cpu_s = (time.perf_counter() - t0) * nl / n_base
    return {"value": round(wl.B / cpu_s, 3), "unit": "sequences/s", "cores": cores, "kind": "oracle",
            "sample": f"whole batch, {n_base} of {nl} layers timed once (scaled to {nl}), numpy fp64 padded semantics",
            "seconds": round(cpu_s, 2)}


def bench_mha_alone(args, torch, bt, I, wl):
    """The attention-alone workload: a step is one bt_varlen_mha over the packed fused QKV buffer."""
    import ctypes as C
    lib = bt.load_library()
    L = I.draw_lengths(wl)
    T, s2 = int(L.sum()), int((L.astype(np.int64) ** 2).sum())
    qkv_h = I.make_qkv_packed(wl, T)
    cu_h = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    qkv = torch.from_numpy(qkv_h).to("cuda:0")
    cu = torch.from_numpy(cu_h).to("cuda:0")
    o = torch.empty((T, wl.H), dtype=torch.float16, device="cuda:0")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    qb = qkv.data_ptr()
    fn = lambda: lib.bt_varlen_mha(C.c_void_p(qb), C.c_void_p(qb + 2 * wl.H), C.c_void_p(qb + 4 * wl.H), 3 * wl.H, None,
                                   None, None, C.c_void_p(cu.data_ptr()), wl.B, T, wl.S, wl.heads, wl.head_dim,
                                   C.c_float(wl.head_dim ** -0.5), C.c_void_p(o.data_ptr()), None, 0, st)
    if fn() != 0:
        raise RuntimeError("bt_varlen_mha failed")
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle:     # let the device clocks settle (see main)
        for _ in range(100):
            fn()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fn()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us = time_launches(torch, fn, args.kernel_iters)
    flop = 4.0 * s2 * wl.H
    ach = flop / us / 1e6
    out = {"metric": "sequences/s variable-length fused MHA alone (b16, max256, 12 heads x 64)",
           "value": round(wl.B * args.steps / dt, 1), "unit": "sequences/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt * 1e3 / args.steps, 5), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
           "config": {"workload": args.workload, "batch": wl.B, "max_seq": wl.S, "heads": wl.heads,
                      "head_dim": wl.head_dim, "length_law": wl.length_law, "valid_tokens": T, "sum_len_sq": s2,
                      "step": "bt_varlen_mha"},
           "roofline": {"kernel": "varlen_mha", "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_MFMA_F16,
                        "unit": "TFLOP/s", "frac": round(ach / PEAK_MFMA_F16, 4),
                        "traffic": measured_traffic(args.workload, "varlen_mha"), "us_per_launch": round(us, 2),
                        "work_per_launch": flop},
           "kernels": [{"kernel": "varlen_mha", "bound": "mfma", "us": round(us, 2), "launches_per_step": 1,
                        "achieved": round(ach, 2), "peak": PEAK_MFMA_F16, "unit": "TFLOP/s",
                        "frac": round(ach / PEAK_MFMA_F16, 4), "work_per_launch": flop}],
           "algorithmic_bytes": {"varlen_mha": 8 * T * wl.H},
           "hbm_fraction_of_the_same_launch": round(8.0 * T * wl.H / us / 1e3 / PEAK_HBM, 4)}
    if args.peaks:
        out["measured_peaks"] = measure_peaks(torch)
    if args.calibrate_copy:
        calibrate_copy(torch)
    if not args.no_cpu_baseline:
        from oracle import bt_oracle as O
        cores = len(os.sched_getaffinity(0))
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [cores])
        except Exception:
            pass
        t0 = time.perf_counter()
        O.varlen_mha_packed(qkv_h, cu_h, wl.heads, wl.head_dim)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(wl.B / cpu_s, 3), "unit": "sequences/s", "cores": cores, "kind": "oracle",
                               "sample": "whole batch, once, numpy fp64 padded attention", "seconds": round(cpu_s, 3)}
    print(json.dumps(out))


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
        return bench_mha_alone(args, torch, bt, I, wl)

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
    fold_vectors = bt.encoder_prepare(layers)     # depends on the parameters only: computed once, not timed
    fold = fold_vectors if args.fold else None
    ws = torch.empty(bt.layer_workspace_bytes(layers[0], wl.B * wl.S, wl.B, wl.S), dtype=torch.uint8, device="cuda:0")
    x_packed = torch.empty((wl.B * wl.S, H), dtype=torch.float16, device="cuda:0")
    y_packed = torch.empty((wl.B * wl.S, H), dtype=torch.float16, device="cuda:0")
    y_padded = torch.empty((wl.B, wl.S, H), dtype=torch.float16, device="cuda:0")
    y_padded_sep = torch.empty_like(y_padded)

    def step_separate(mark, out_=y_padded_sep):
        cu, tok, t = bt.build_offsets(lengths=lengths_d, S=wl.S)
        mark()
        xp = bt.pack(x_padded, tok, out=x_packed[:t])
        yp = bt.encoder_fwd(layers, xp, cu, wl.S, out=y_packed[:t], ws=ws, fold=fold)
        bt.unpack(yp, tok, wl.B, wl.S, out=out_)

    def step_two_calls(mark, out_=None):
        cu, tok, t = bt.build_offsets(lengths=lengths_d, S=wl.S)
        mark()
        bt.encoder_fwd_padded(layers, x_padded, tok, cu, out=y_padded if out_ is None else out_, ws=ws, fold=fold)

    def step_fused(mark):
        # the same two library calls behind one entry point: the token count goes from the prefix-sum kernel's
        # result into the launches of the layers without a trip through Python in between
        bt.encoder_fwd_masked(layers, x_padded, lengths=lengths_d, out=y_padded, ws=ws, fold=fold)
        mark()

    separate = args.separate_pack_unpack

    # ---------------- per-kernel timing (HIP events on the launch stream)
    # Each kernel of the layer is launched `kernel_iters` times back to back through the C ABI (raw
    # ctypes calls with prebuilt arguments, ~1 us of host time each) between two HIP events recorded
    # on the stream the kernels run on; the average includes the inter-launch gap.  Runs after the step timing.
    def kernel_leg():
        out = {}
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
        # GEMM #1 / #3 and the LayerNorms as the layer runs them: K slices (fp32) where the library splits K
        nsl = C.c_int(0)
        sl_bytes = max(int(lib.bt_gemm_kslices_bytes(T, H, H)), int(lib.bt_gemm_kslices_bytes(T, H, F)), 16)
        slices = torch.empty(sl_bytes // 4, dtype=torch.float32, device="cuda:0")
        def gemm_ks(a, w, K, c):
            return bind(lib.bt_gemm_kslices, ptr(a), ptr(w), T, H, K, ptr(c), ptr(slices), C.c_size_t(sl_bytes),
                        C.byref(nsl), st)
        def ln_after(gemm_fn, b, r, ga, be, y_):
            if gemm_fn() != 0:
                raise RuntimeError("bt_gemm_kslices failed")
            if nsl.value == 0:
                return lnk(proj, b, r, ga, be, y_), 0
            return bind(lib.bt_add_bias_residual_layernorm_kslices, ptr(slices), nsl.value, ptr(b), ptr(r), ptr(ga),
                        ptr(be), eps, T, H, ptr(y_), st), nsl.value
        g1, g3 = gemm_ks(attn, P["w_o"], H, proj), gemm_ks(g, P["w_2"], F, proj)
        ln0, ks1 = ln_after(g1, P["b_o"], xp, P["ln0_g"], P["ln0_b"], y1)
        ln1, ks3 = ln_after(g3, P["b_2"], y1, P["ln1_g"], P["ln1_b"], y2)
        out["k_slices"] = {"gemm1_proj": ks1, "gemm3_ffn_down": ks3}
        steps = [
            ("gemm0_qkv_bias", "mfma", 6.0 * T * H * H, gemm(xp, P["w_qkv"], P["b_qkv"], T, 3 * H, H, 0, qkv)),
            ("varlen_mha", "mfma", 4.0 * sum_l2 * H, mha),
            ("gemm1_proj", "mfma", 2.0 * T * H * H, g1),
            ("bias_residual_ln0", "hbm", 6.0 * T * H, ln0),
            ("gemm2_bias_gelu", "mfma", 2.0 * T * H * F, gemm(y1, P["w_1"], P["b_1"], T, F, H, 1, g)),
            ("gemm3_ffn_down", "mfma", 2.0 * T * H * F, g3),
            ("bias_residual_ln1", "hbm", 6.0 * T * H, ln1),
            ("pack", "hbm", 4.0 * T * H, bind(lib.bt_pack, ptr(x_padded), ptr(tok), T, H, ptr(x_packed), st)),
            ("unpack", "hbm", 2.0 * T * H + 2.0 * wl.B * wl.S * H,
             bind(lib.bt_unpack, ptr(y2), ptr(tok), T, wl.B, wl.S, H, ptr(y_padded_sep), st)),
        ]
        gemm_shapes = {"gemm0_qkv_bias": (T, 3 * H, H, 0), "gemm1_proj": (T, H, H, 0),
                       "gemm2_bias_gelu": (T, F, H, 1), "gemm3_ffn_down": (T, H, F, 0)}
        # operands read once + result written once, fp16 (what a launch must move at the least)
        out["algorithmic_bytes"] = {
            "gemm0_qkv_bias": 2 * (T * H + 3 * H * H + 3 * T * H + 3 * H), "varlen_mha": 8 * T * H,
            "gemm1_proj": 2 * (T * H + H * H + T * H), "bias_residual_ln": 6 * T * H + 6 * H,
            "gemm2_bias_gelu": 2 * (T * H + F * H + T * F + F), "gemm3_ffn_down": 2 * (T * F + H * F + T * H),
            "pack": 4 * T * H, "unpack": 2 * T * H + 2 * wl.B * wl.S * H}
        kernels = []
        for name, bound, work, fn in steps:
            if fn() != 0:
                raise RuntimeError(f"{name} failed")
            us = time_launches(torch, fn, args.kernel_iters)
            per_step = nl if name not in ("pack", "unpack") else (1 if separate else 0)
            if bound == "mfma":
                ach, peak, unit = work / us / 1e6, PEAK_MFMA_F16, "TFLOP/s"
            else:
                ach, peak, unit = work / us / 1e3, PEAK_HBM, "GB/s"
            kernels.append({"kernel": name, "bound": bound, "us": round(us, 2), "launches_per_step": per_step,
                            "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
                            "work_per_launch": work})
            if name in gemm_shapes and not out["k_slices"].get(name, 0):
                # tile-quantisation ceiling of this product: useful share of the tiles' area times the share of
                # the 256 compute units that the last round of tiles occupies
                M_, N_, K_, act_ = gemm_shapes[name]
                bm, bn = bt.gemm_tile_shape(M_, N_, K_, act_)
                tiles = -(-M_ // bm) * -(-N_ // bn)
                rounds = -(-tiles // 256)
                kernels[-1].update({"tile": f"{bm}x{bn}", "tiles": tiles, "rounds_of_256_cus": rounds,
                                    "tile_quantisation_ceiling": round(M_ * N_ / (tiles * bm * bn) * tiles / (rounds * 256), 4)})
                split_rows = bt.gemm_row_split(M_, N_, K_, act_)
                if split_rows:   # run as two launches over row ranges; the figures above describe one launch
                    kernels[-1]["rows_of_first_launch"] = split_rows
        dom = max(kernels, key=lambda k: k["us"] * k["launches_per_step"])
        out["roofline"] = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"],
                           "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"],
                           "traffic": measured_traffic(args.workload, dom["kernel"]),
                           "us_per_launch": dom["us"], "work_per_launch": dom["work_per_launch"]}
        out["kernels"] = kernels
        out["kernel_time_sum_ms_per_step"] = round(sum(k["us"] * k["launches_per_step"] for k in kernels) / 1e3, 4)

        # ---- two more measured points named by the metric ----------------------------------------
        if args.workload == "bert_base_b16_s256":
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


        return out

    step = (lambda mark: step_separate(mark, y_padded)) if separate else step_fused
    step_name = ("build_offsets+pack+encoder_fwd+unpack" if separate
                 else "encoder_fwd_masked (= build_offsets+encoder_fwd_padded in one library call)")
    # Device warm-up, before the W warm-up steps and outside every timed region: the GPU's power management takes
    # tens of milliseconds of sustained load to settle its clocks (20 timed steps right after 5 warm-up steps read
    # 5 % slower than the same steps later in the process), so the step is repeated for about `--settle` seconds
    # first.  It changes no result, only when the clock starts.
    n_settle = 0
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < args.settle:
        step(lambda: None)
        n_settle += 1
    torch.cuda.synchronize()
    dt, per = timed_steps(torch, step, args.steps, args.warmup)
    stats = step_stats(wl.B, dt, per, window=1 if separate else 8)
    flops_step = nl * (24.0 * T * H * H + 4.0 * sum_l2 * H)

    out = {
        "metric": "sequences/s BERT-base fp16 varlen (b16, max256)" if args.workload == "bert_base_b16_s256"
                  else f"sequences/s {args.workload} fp16 varlen",
        "value": stats["value"], "unit": "sequences/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": stats["ms_per_step"], "ms_per_step_median": stats["ms_per_step_median"],
        "ms_per_step_min": stats["ms_per_step_min"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": args.workload, "batch": wl.B, "max_seq": wl.S, "hidden": H, "heads": wl.heads,
                   "ffn": F, "layers": nl, "length_law": wl.length_law, "valid_tokens": T, "sum_len_sq": sum_l2,
                   "step": step_name, "layernorm_fold_vectors_given": fold is not None,
                   "device_settle_steps_before_warmup": n_settle},
        "useful_tflops_per_s": round(flops_step / (stats["ms_per_step"] * 1e-3) / 1e12, 2),
    }

    # ---------------- the same step with the fold vectors handed over (extra point; see --fold)
    if not separate and fold is None:
        y_padded_f = torch.empty_like(y_padded)

        def step_fold(mark):
            bt.encoder_fwd_masked(layers, x_padded, lengths=lengths_d, out=y_padded_f, ws=ws, fold=fold_vectors)
            mark()

        dtf, perf_ = timed_steps(torch, step_fold, args.steps, max(args.warmup // 2, 2))
        out["layernorm_fold_vectors"] = dict(
            step_stats(wl.B, dtf, perf_, window=8), unit="sequences/s", step="encoder_fwd_masked(d_fold)",
            max_abs_diff_to_value_path=round(float((y_padded_f.float() - y_padded.float()).abs().max()), 5),
            note="LayerNorms folded into the GEMM epilogues where the library finds that faster (a few hundred to "
                 "about 2 700 tokens at hidden 768), else the same kernels as `value`")

    # ---------------- the two library calls of the step made from Python one after the other (extra point; same bits)
    if not separate:
        y_two = torch.empty_like(y_padded)
        dt2, per2 = timed_steps(torch, lambda mark: step_two_calls(mark, y_two), args.steps, max(args.warmup // 2, 2))
        out["two_calls"] = dict(step_stats(wl.B, dt2, per2), unit="sequences/s",
                                step="build_offsets+encoder_fwd_padded", outputs_equal=bool(torch.equal(y_two, y_padded)),
                                # median host time from "the token count is known" to "every launch of the step
                                # is enqueued": when this approaches ms_per_step the machine's host paces the step
                                host_enqueue_ms_per_step=round(timed_steps.host_enqueue_s * 1e3, 4))

    # ---------------- the same work with pack / unpack as kernels of their own (extra point; same bits)
    if not separate:
        dts, pers = timed_steps(torch, step_separate, args.steps, max(args.warmup // 2, 2))
        out["separate_pack_unpack"] = dict(step_stats(wl.B, dts, pers), unit="sequences/s",
                                           step="build_offsets+pack+encoder_fwd+unpack",
                                           outputs_equal=bool(torch.equal(y_padded_sep, y_padded)))

    # ---------------- the same step with the forward replayed from a HIP graph (extra point)
    # One graph launch instead of ~85 kernel launches per step: if this is faster than `value`, the host of
    # this box did not keep ahead of the GPU in the eager loop; on a quiet host the two agree.
    if not separate:
        y_padded3 = torch.empty_like(y_padded)
        cu_g, tok_g, t_g = bt.build_offsets(lengths=lengths_d, S=wl.S)

        def body():
            bt.encoder_fwd_padded(layers, x_padded, tok_g, cu_g, out=y_padded3, ws=ws, fold=fold)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            body()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            body()

        def step_graph(mark):
            bt.build_offsets(lengths=lengths_d, S=wl.S)      # same offsets every step here; still computed and waited for
            mark()
            graph.replay()

        dtg, perg = timed_steps(torch, step_graph, args.steps, max(args.warmup // 2, 2))
        out["graph_replay"] = dict(step_stats(wl.B, dtg, perg), unit="sequences/s",
                                   step="build_offsets + one HIP graph of encoder_fwd_padded",
                                   outputs_equal=bool(torch.equal(y_padded3, y_padded)))

    # ---------------- throughput with two batches in flight (extra point, not `value`)
    # One batch at a time leaves the GPU idle at every kernel boundary (~2.5 us per dependent launch) and
    # while the host waits for the token count in build_offsets.  A server keeps a second batch in flight
    # on another stream, which fills those holes; each batch has its own buffers and its own host thread,
    # the library keeps no state between calls.  Same steps, same kernels, same results.
    if not args.no_pipelined and not separate:
        import threading

        class Batch:
            def __init__(self):
                self.stream = torch.cuda.Stream()
                self.x_padded = x_padded.clone()
                self.lengths_d = lengths_d.clone()
                self.ws = torch.empty_like(ws)
                self.y_padded = torch.empty_like(y_padded)

            def run(self, n):
                torch.cuda.set_device(0)
                with torch.cuda.stream(self.stream):
                    for _ in range(n):
                        cu, tok, t = bt.build_offsets(lengths=self.lengths_d, S=wl.S)
                        bt.encoder_fwd_padded(layers, self.x_padded, tok, cu, out=self.y_padded, ws=self.ws, fold=fold)

        batches = [Batch(), Batch()]
        per_b = max(args.steps // 2, 1)

        def both(n):
            th = [threading.Thread(target=b.run, args=(n,)) for b in batches]
            for t_ in th:
                t_.start()
            for t_ in th:
                t_.join()
            torch.cuda.synchronize()

        both(max(args.warmup // 2, 2))
        t0 = time.perf_counter()
        both(per_b)
        dt2 = time.perf_counter() - t0
        same = bool(torch.equal(batches[0].y_padded, y_padded) and torch.equal(batches[1].y_padded, y_padded))
        out["two_batches_in_flight"] = {"value": round(wl.B * 2 * per_b / dt2, 1), "unit": "sequences/s",
                                        "steps": 2 * per_b, "ms_per_step": round(dt2 * 1e3 / (2 * per_b), 4),
                                        "streams": 2, "outputs_equal_single_stream": same}
        del batches

    if not args.no_kernels:
        out.update(kernel_leg())

    if args.peaks:
        mp = measure_peaks(torch)
        out["measured_peaks"] = mp
        if "roofline" in out:
            r = out["roofline"]
            den = mp["mfma_f16_random_operands_tflops"] if r["bound"] == "mfma" else mp["hbm_read_stream_GBps"]
            r["frac_of_measured_peak"] = round(r["achieved"] / den, 4)
            r["measured_peak"] = den

    if args.calibrate_copy:
        calibrate_copy(torch)

    # ---------------- CPU baseline: the oracle as it stands, on this machine's cores
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_encoder(wl, L, x_packed_h, params, nl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
