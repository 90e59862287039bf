"""Turns rocprofv3 CSV output of `bench.py` runs into the short summaries kept under profiles/.

    python -m paper_2210_03052_amd.profile_summary --workload NAME [--stats DIR] [--pmc DIR ...]
           [--fetch DIR --write DIR] [--bench-json FILE] --out profiles/NAME.md [--traffic profiles/hbm_traffic.txt]

  --stats   directory of a `rocprofv3 --kernel-trace --stats` run        -> per-kernel call count, avg/min/max us
  --pmc     directories of `rocprofv3 --pmc <SQ counters>` runs          -> per-kernel counter averages and the
            MFMA figures derived from them (see `derive`)
  --fetch / --write  directories of the FETCH_SIZE and WRITE_SIZE runs (bench.py --calibrate-copy), scaled by what
            the same counter reads for the 1 GiB device copy of that run  -> HBM-side bytes per launch
  --traffic the machine-readable table bench.py reads its `roofline.traffic` from; the lines of this workload
            are replaced, other workloads' lines are kept.

Every kernel of the library is mapped to the step of the layer it implements by its name alone: the GEMM
kernel's template arguments spell out activation, epilogue and shape class, so the four products of a layer
are distinct kernels in a trace.  Reads CSV, writes text; nothing here touches a GPU.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re

COPY_KIB = 1048576.0     # bench.py --calibrate-copy: one 1 GiB device copy (1 GiB read + 1 GiB written)


def template_args(name: str):
    """Integer template arguments of a kernel name, mangled (`ILi64ELi128ELb0EE`) or demangled (`<64, 128, false>`)."""
    m = re.search(r"I((?:L[ib]\d+E)+)E", name)
    if m:
        return [int(x) for x in re.findall(r"L[ib](\d+)E", m.group(1))]
    m = re.search(r"<([^<>]*)>", name)
    if m:
        out = []
        for tok in m.group(1).split(","):
            tok = tok.strip().split("=")[-1].strip()
            out.append({"true": 1, "false": 0}.get(tok, None) if tok in ("true", "false") else int(re.sub(r"[^0-9-]", "", tok) or 0))
        return out
    return []


STREAMING_GRID = 20_000_000     # threads: bench.py's 262 144-token pack launches 25 M of them, the workloads < 2 M


def role_of(name: str, grid: int = 0):
    """(step of the layer, short label) for a kernel name of this library, else (None, None)."""
    a = template_args(name)
    if "unpack_kernel" not in name and "pack_kernel" in name and grid >= STREAMING_GRID:
        return "pack_streaming", "pack_kernel (262144 tokens)"
    if "gemm_pipe_kernel" in name and len(a) >= 8:
        bm, bn, wgm, wgn, ns, act, epi, shape = a[:8]
        label = f"gemm_pipe<{bm}x{bn},{wgm}x{wgn} waves,{ns} stages,act={act},epi={epi},shape={shape}>"
        if epi == 3:
            return ("gemm3_ffn_down" if shape == 2 else "gemm1_proj"), label
        if epi == 1:   # LayerNorm of the input folded into the epilogue (5-launch pipeline)
            return ("gemm2_bias_gelu_folded" if act != 0 else ("gemm0_qkv_folded" if shape == 0 else "gemm_folded")), label
        if act != 0:
            return "gemm2_bias_gelu", label
        if epi == 2:   # bias + residual + row sums in the epilogue (5-launch pipeline)
            return ("gemm3_ffn_down_resid" if shape == 2 else "gemm1_proj_resid"), label
        return {0: "gemm0_qkv_bias", 1: "gemm1_proj", 2: "gemm3_ffn_down"}.get(shape, "gemm"), label
    if "gemm_simple_kernel" in name:
        return "gemm_fallback", "gemm_simple"
    if "varlen_mha_splitkey_kernel" in name:
        return "varlen_mha", f"varlen_mha_splitkey<{','.join(map(str, a[:2]))}>"
    if "varlen_mha_kernel" in name:
        return "varlen_mha", f"varlen_mha<{','.join(map(str, a[:2]))}>"
    if "bias_residual_ln_kernel" in name:
        stream = len(a) >= 3 and a[2] == 1
        return ("bias_residual_ln_streaming" if stream else "bias_residual_ln"), f"bias_residual_ln<{','.join(map(str, a[:3]))}>"
    for key, role in (("ln_finalize_kernel", "ln_finalize"), ("unpack_kernel", "unpack"), ("pack_kernel", "pack"),
                      ("offsets_kernel", "offsets"), ("fold_vectors_kernel", "fold_vectors"),
                      ("peak_mfma_kernel", "peak_mfma"), ("peak_read_kernel", "peak_read"),
                      ("copyBuffer", "device_copy")):
        if key in name:
            return role, key
    return None, None


def _csv(dirname, suffix):
    files = glob.glob(os.path.join(dirname, "**", f"*{suffix}"), recursive=True)
    if not files:
        raise SystemExit(f"no *{suffix} under {dirname}")
    rows = []
    for f in files:
        rows.extend(csv.DictReader(open(f, newline="")))
    return rows


def read_trace(dirname):
    """{label: [durations in us]} and {label: role} from a kernel trace."""
    dur, roles = collections.defaultdict(list), {}
    for r in _csv(dirname, "kernel_trace.csv"):
        role, label = role_of(r["Kernel_Name"], int(r.get("Grid_Size_X") or 0))
        if role is None:
            continue
        dur[label].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
        roles[label] = role
    return dur, roles


def read_counters(dirname):
    """{label: {counter: average over the dispatches of that kernel}}, {label: role}, {label: dispatches}."""
    acc, roles, n = collections.defaultdict(lambda: collections.defaultdict(list)), {}, collections.Counter()
    for r in _csv(dirname, "counter_collection.csv"):
        role, label = role_of(r["Kernel_Name"], int(r.get("Grid_Size") or 0))
        if role is None:
            continue
        acc[label][r["Counter_Name"]].append(float(r["Counter_Value"]))
        roles[label] = role
    out = {}
    for label, cs in acc.items():
        out[label] = {c: sum(v) / len(v) for c, v in cs.items()}
        n[label] = max(len(v) for v in cs.values())
    return out, roles, n


def derive(c):
    """MFMA figures from raw SQ counters of one kernel (averages per dispatch).
    SQ_INSTS_VALU_MFMA_MOPS_F16 counts units of 512 FLOP; SQ_VALU_MFMA_BUSY_CYCLES adds up, over the chip's
    1024 SIMDs, the cycles their matrix pipe is busy (32 per 32x32x16 fp16 instruction); SQ_BUSY_CU_CYCLES adds
    up the cycles each compute unit has a wave resident."""
    d = {}
    if not c.get("SQ_INSTS_VALU_MFMA_MOPS_F16") and not c.get("SQ_VALU_MFMA_BUSY_CYCLES") and not c.get("SQ_INSTS_MFMA"):
        if c.get("SQ_WAVE_CYCLES") and "SQ_WAIT_INST_ANY" in c:
            d["wave_cycles_waiting_on_an_instruction"] = c["SQ_WAIT_INST_ANY"] / c["SQ_WAVE_CYCLES"]
        return d
    if "SQ_INSTS_VALU_MFMA_MOPS_F16" in c:
        d["executed_gflop"] = c["SQ_INSTS_VALU_MFMA_MOPS_F16"] * 512 / 1e9
    if "SQ_VALU_MFMA_BUSY_CYCLES" in c and c.get("SQ_BUSY_CU_CYCLES"):
        d["mfma_busy_share_of_busy_simd_cycles"] = c["SQ_VALU_MFMA_BUSY_CYCLES"] / (4.0 * c["SQ_BUSY_CU_CYCLES"])
    if "SQ_VALU_MFMA_BUSY_CYCLES" in c:
        d["mfma_pipe_us_at_2.4GHz_all_simds"] = c["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024.0 / 2400.0
    if "SQ_BUSY_CU_CYCLES" in c:
        d["cu_busy_us_at_2.4GHz_all_cus"] = c["SQ_BUSY_CU_CYCLES"] / 256.0 / 2400.0
    if c.get("SQ_WAVE_CYCLES") and "SQ_WAIT_INST_ANY" in c:
        d["wave_cycles_waiting_on_an_instruction"] = c["SQ_WAIT_INST_ANY"] / c["SQ_WAVE_CYCLES"]
    if c.get("SQ_INSTS_MFMA") and "SQ_INSTS_VALU" in c:
        d["valu_instructions_per_mfma"] = (c["SQ_INSTS_VALU"] - c["SQ_INSTS_MFMA"]) / c["SQ_INSTS_MFMA"]
    return d


def traffic_from(fetch_dir, write_dir):
    """{role: (fetch KiB, write KiB, HBM bytes)} per launch, scaled by the 1 GiB copy of the same runs."""
    out = {}
    scale = {}
    per = {}
    for kind, d in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        cs, roles, counts = read_counters(d)
        # the calibration copy is by far the largest copyBuffer dispatch; averages would be polluted by small ones
        big = 0.0
        for r in _csv(d, "counter_collection.csv"):
            if "copyBuffer" in r["Kernel_Name"] and r["Counter_Name"] == kind:
                big = max(big, float(r["Counter_Value"]))
        scale[kind] = COPY_KIB / big if big > 1000 else 1.0
        # one figure per step: the kernel with the most dispatches -- or, for a product that runs as two launches
        # over row ranges (two GEMM kernels of one step, dispatched equally often), the two added
        by_role = {}
        for lab, v in cs.items():
            if kind in v:
                by_role.setdefault(roles[lab], []).append((counts[lab], v[kind]))
        for role, items in by_role.items():
            top = max(c for c, _ in items)
            same = [x for c, x in items if abs(c - top) <= 0.02 * top]
            per.setdefault(role, {})[kind] = sum(same) if role.startswith("gemm") and len(same) == 2 else same[0]
    for role, v in per.items():
        if "FETCH_SIZE" in v and "WRITE_SIZE" in v:
            hbm = (v["FETCH_SIZE"] * scale["FETCH_SIZE"] + v["WRITE_SIZE"] * scale["WRITE_SIZE"]) * 1024.0
            out[role] = (v["FETCH_SIZE"], v["WRITE_SIZE"], hbm)
    return out, scale


def update_traffic_file(path, workload, table):
    head = ["# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py, each scaled by the",
            "# same counter's reading of a 1 GiB device copy in the same run.  Written by",
            "# `python -m paper_2210_03052_amd.profile_summary`; read by bench.py (roofline.traffic).",
            "# workload kernel fetch_kib write_kib hbm_bytes"]
    keep = []
    if os.path.exists(path):
        for line in open(path):
            line = line.rstrip("\n")
            if line and not line.startswith("#") and line.split()[0] != workload:
                keep.append(line)
    new = [f"{workload} {role} {f:.1f} {w:.1f} {int(round(h))}" for role, (f, w, h) in sorted(table.items())
           if role not in ("device_copy",)]
    with open(path, "w") as fh:
        fh.write("\n".join(head + sorted(keep + new)) + "\n")


def sweep_summary(path_json: str, out: str) -> None:
    """`bench.py --sweep > sweep.json` as tables (profiles/bench_sweep_small_batch_and_table3.md)."""
    d = {}
    for line in open(path_json):
        line = line.strip()
        if line.startswith("{"):
            d = json.loads(line)
    rows, kf, t3 = d["sweep"], d["kernel_fusion"], d["table3_single_layer"]
    small = [r["ms_packed"] for r in rows if r["valid_tokens"] < 600]
    md = ["# bench.py --sweep: BERT-base forward (12 layers, fp16) over batch and maximum length, one MI355X", "",
          "Command (from the repository root): `python3 bench.py --sweep > sweep.json`, then",
          "`python -m paper_2210_03052_amd.profile_summary --sweep-json sweep.json --out <this file>` (this is the JSON line as tables).",
          f"Lengths are drawn `{d['length_law']}`, the end-to-end protocol of Sec. IV-E, seeded. \"all tokens valid\" runs the",
          "same kernels on the same batch with every sequence at full length, i.e. what a padded pipeline computes;",
          "the ratio is the gain from removing padding (Sec. III-D; the paper reports +24 % per layer at mean 0.6 max on A100).",
          "Each figure is the whole step (`bt_encoder_fwd_masked` = `bt_build_offsets` + `bt_encoder_fwd_padded`: 12 layers with pack / unpack fused into the",
          "first / last kernels), 50 timed iterations.", "",
          "| batch | max_seq | valid tokens | ms packed | ms all tokens valid | gain |", "|---|---|---|---|---|---|"]
    for r in rows:
        md.append(f"| {r['batch']} | {r['max_seq']} | {r['valid_tokens']} | {r['ms_packed']:.3f} | "
                  f"{r['ms_all_tokens_valid']:.3f} | {r['speedup_from_removing_padding']:.2f}x |")
    md += ["",
           f"Below about 600 tokens the forward is bound by its 85 dependent launches (offsets + 12 x 7): {min(small):.2f}-{max(small):.2f} ms, "
           f"about {1e3 * min(small) / 85:.1f} us",
           "per launch, of which about 2.5 us is the gap between dependent launches and the rest a kernel whose K loop a few dozen",
           "tiles walk alone (a HIP-graph replay of the same launches takes the same time: the gaps are on the GPU side). The",
           "output projection and FFN-down run split over K there (2-6 slices, added by the LayerNorm kernel that follows).",
           "What remains per layer: GEMM #0, attention, GEMM #1, add-bias+residual+LayerNorm, GEMM #2 (+GELU), GEMM #3,",
           "add-bias+residual+LayerNorm. The LayerNorm-folded pipeline (5 launches) does not help here: its residual epilogue has no",
           "split-K form, so FFN-down walks K = 3072 on a dozen tiles (measured +1.5 % at 186 tokens); a whole-layer persistent",
           "kernel needs grid-wide barriers, which cost more than the launch gaps they would replace.", "",
           "## Single encoder layer, batch 1 (the two absolute times the paper prints, Table III, A100 FP16)", "",
           "| seq | ms, layer only (`bt_encoder_layer_fwd`, HIP events, 200 launches) | ms, whole step (+ build_offsets, pack / unpack fused) | paper, A100 |",
           "|---|---|---|---|"]
    for r in t3:
        md.append(f"| {r['seq']} | {r['ms_layer_only']:.4f} | {r['ms_whole_step']:.4f} | {r['paper_a100_ms']} |")
    ln, ge = kf["add_bias_residual_layernorm_us"], kf["gemm_add_bias_gelu_us"]
    md += ["", f"## Fused kernels against unfused ones (headline shape: {kf['tokens']} tokens, hidden {kf['hidden']}, FFN {kf['ffn']})", "",
           "The shape of the add-bias + LayerNorm and add-bias + GELU comparisons of Sec. IV-A / IV-B, with this repository's own",
           "unfused kernels (`csrc/unfused.hip`, measurement library only): add-bias+residual then LayerNorm as two trips over",
           "memory; GEMM then add-bias+GELU as a kernel of its own. Both sides are captured in a HIP graph (20 calls, 20 replays)",
           "so that the host launch path is outside the timed region.", "",
           "| step | fused us | unfused us (2 launches) | saved | paper (A100) |", "|---|---|---|---|---|",
           f"| add bias + residual + LayerNorm | {ln['fused']} | {ln['unfused_2_launches']} | {100 * ln['saved']:.0f} % | 61-69 % |",
           f"| GEMM + add bias + GELU | {ge['fused']} | {ge['unfused_2_launches']} | {100 * ge['saved']:.0f} % | 24 % |", "",
           "One encoder layer step by step (the shape of the step-wise figure of Sec. IV-D), composed from C-ABI calls and timed",
           "from a HIP graph. \"padded\" runs every sequence at the full length S; the attention of the padded rungs is this",
           "library's fused kernel at full length (the paper's padded baseline has an unfused attention on top of that, which is not",
           "rebuilt here).", ""]
    for w in kf["encoder_layer_stepwise"]:
        md += [f"`{w['workload']}` ({w['padded_tokens']} padded / {w['valid_tokens']} valid tokens):", "",
               "| variant | us per layer |", "|---|---|"]
        md += [f"| {v['variant']} | {v['us']} |" for v in w["us_per_layer"]]
        md += ["", f"First to last rung: {w['speedup_over_first_rung']}x.", ""]
    md += ["Attention alone (the shape of the fused-MHA comparisons of Sec. IV-C; 12 heads of 64, lengths of the two BERT-base",
           "workloads): the variable-length fused kernel on the packed batch against padded attention through torch (a stand-in:",
           "a batched padded attention is not part of this library): three launches with the S x S logits in memory, and torch's",
           "own fused padded kernel (`scaled_dot_product_attention` with the padding mask).", "",
           "| workload | valid tokens | variable-length fused us | padded, three launches us | padded, torch fused us |",
           "|---|---|---|---|---|"]
    for a in kf["attention"]:
        f = a["fused_varlen_us"]
        md.append(f"| {a['workload']} | {a['valid_tokens']} | {f} | {a['padded_three_launches_us']} "
                  f"({a['padded_three_launches_us'] / f:.1f}x) | {a['padded_torch_fused_us']} ({a['padded_torch_fused_us'] / f:.1f}x) |")
    with open(out, "w") as fh:
        fh.write("\n".join(md) + "\n")
    print("wrote", out)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--sweep-json", help="the JSON line of `bench.py --sweep`: write it out as tables to --out and stop")
    ap.add_argument("--workload")
    ap.add_argument("--stats")
    ap.add_argument("--pmc", nargs="*", default=[])
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--bench-json", help="the JSON line bench.py printed in the --stats run (useful FLOPs per kernel)")
    ap.add_argument("--commands", help="text file with the commands that produced the inputs (copied into the summary)")
    ap.add_argument("--out", required=True)
    ap.add_argument("--traffic")
    args = ap.parse_args()
    if args.sweep_json:
        return sweep_summary(args.sweep_json, args.out)
    if not args.workload:
        ap.error("--workload is required without --sweep-json")

    bench = {}
    if args.bench_json and os.path.exists(args.bench_json):
        for line in open(args.bench_json):
            line = line.strip()
            if line.startswith("{"):
                bench = json.loads(line)
    work = {k["kernel"]: k for k in bench.get("kernels", [])}
    if "bias_residual_ln0" in work:
        work["bias_residual_ln"] = work["bias_residual_ln0"]
    # the folded pipeline's GEMMs do the same products as the plain ones
    for folded, plain in (("gemm0_qkv_folded", "gemm0_qkv_bias"), ("gemm2_bias_gelu_folded", "gemm2_bias_gelu"),
                          ("gemm1_proj_resid", "gemm1_proj"), ("gemm3_ffn_down_resid", "gemm3_ffn_down")):
        if plain in work:
            work[folded] = work[plain]

    md = [f"# rocprofv3 summary: bench.py, workload `{args.workload}`", ""]
    if bench.get("config"):
        c = bench["config"]
        md += [f"Batch {c.get('batch')} x max {c.get('max_seq')}, hidden {c.get('hidden')}, {c.get('layers')} layers, "
               f"{c.get('valid_tokens')} valid tokens, sum of squared lengths {c.get('sum_len_sq')}.", ""]
    if args.commands and os.path.exists(args.commands):
        md += ["Commands (on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", ""]
        md += ["    " + l.rstrip() for l in open(args.commands) if l.strip()] + [""]

    if args.stats:
        dur, roles = read_trace(args.stats)
        md += ["## Kernel trace (`--kernel-trace --stats`)", "",
               "| step | kernel | calls | avg us | min us | max us | useful work / avg time | of peak |", "|---|---|---|---|---|---|---|---|"]
        tot = sum(sum(v) for v in dur.values())
        # A product that the library runs as two launches over row ranges shows up as two GEMM kernels of one
        # step with the same number of calls: the step's work belongs to the two together, not to either.
        by_role = collections.defaultdict(list)
        for label in dur:
            by_role[roles[label]].append(label)
        halves = {}
        for role, labels in by_role.items():
            if role.startswith("gemm") and len(labels) > 1:
                top = max(labels, key=lambda l: len(dur[l]))
                pair = [l for l in labels if abs(len(dur[l]) - len(dur[top])) <= 0.02 * len(dur[top])]
                if len(pair) == 2:
                    both = sum(sum(dur[l]) / len(dur[l]) for l in pair)
                    for l in pair:
                        halves[l] = both
        for label, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
            role = roles[label]
            avg = sum(v) / len(v)
            w = work.get(role)
            rate = frac = ""
            if label in halves and w:
                r_ = w["work_per_launch"] / halves[label] / 1e6
                rate = f"two row ranges, {halves[label]:.2f} us together: {r_:.0f} TFLOP/s"
                frac = f"{r_ / w['peak']:.3f}"
            elif w and role not in ("bias_residual_ln_streaming", "pack_streaming"):
                if w["bound"] == "mfma":
                    r_ = w["work_per_launch"] / avg / 1e6
                    rate, frac = f"{r_:.0f} TFLOP/s", f"{r_ / w['peak']:.3f}"
                else:
                    r_ = w["work_per_launch"] / avg / 1e3
                    rate, frac = f"{r_:.0f} GB/s", f"{r_ / w['peak']:.3f}"
            md.append(f"| {role} | `{label}` | {len(v)} | {avg:.2f} | {min(v):.2f} | {max(v):.2f} | {rate} | {frac} |")
        md += ["", f"Total GPU time of these kernels in the run: {tot / 1e3:.1f} ms.", ""]

    for d in args.pmc:
        cs, roles, n = read_counters(d)
        names = sorted({c for v in cs.values() for c in v})
        md += [f"## Counters (`--pmc {' '.join(names)}`), averages per dispatch", "",
               "| step | kernel | dispatches | " + " | ".join(names) + " |", "|---|---|---|" + "---|" * len(names)]
        derived = []
        for label in sorted(cs, key=lambda l: roles[l]):
            if roles[label] in ("device_copy", "offsets", "fold_vectors"):
                continue
            v = cs[label]
            md.append(f"| {roles[label]} | `{label}` | {n[label]} | " + " | ".join(f"{v.get(c, float('nan')):.0f}" for c in names) + " |")
            dv = derive(v)
            w = work.get(roles[label])
            if w and w["bound"] == "mfma" and "executed_gflop" in dv:
                dv["useful_gflop"] = w["work_per_launch"] / 1e9
                dv["useful_share_of_executed"] = dv["useful_gflop"] / dv["executed_gflop"]
            if dv:
                derived.append((roles[label], label, dv))
        # a product run as two launches over row ranges: its useful FLOPs are to be set against the two together
        pairs = collections.defaultdict(list)
        for role, label, dv in derived:
            if role.startswith("gemm") and "useful_gflop" in dv:
                pairs[role].append((label, dv))
        for role, items in pairs.items():
            top = max(n[l] for l, _ in items)
            both = [(l, dv) for l, dv in items if abs(n[l] - top) <= 0.02 * top]
            if len(both) == 2:
                executed = sum(dv["executed_gflop"] for _, dv in both)
                for _, dv in both:
                    dv["executed_gflop_of_both_row_ranges"] = executed
                    dv["useful_share_of_executed"] = dv["useful_gflop"] / executed
        if derived:
            md += ["", "Derived:", ""]
            for role, label, dv in derived:
                md.append(f"- {role} `{label}`: " + ", ".join(f"{k} = {x:.3f}" for k, x in dv.items()))
        md.append("")

    if args.fetch and args.write:
        table, scale = traffic_from(args.fetch, args.write)
        md += ["## HBM-side traffic (`--pmc FETCH_SIZE`, `--pmc WRITE_SIZE`, one run each)", "",
               f"Scale factors from the 1 GiB device copy of the same runs: FETCH_SIZE x{scale['FETCH_SIZE']:.3f}, "
               f"WRITE_SIZE x{scale['WRITE_SIZE']:.3f}.", "",
               "| step | FETCH_SIZE KiB | WRITE_SIZE KiB | bytes beyond L2 per launch | algorithmic bytes | ratio |", "|---|---|---|---|---|---|"]
        for role, (f, w_, h) in sorted(table.items()):
            if role == "device_copy":
                continue
            alg = bench.get("algorithmic_bytes", {}).get(role)
            md.append(f"| {role} | {f:.1f} | {w_:.1f} | {h:.0f} | {alg if alg else ''} | {h / alg:.2f} |" if alg else
                      f"| {role} | {f:.1f} | {w_:.1f} | {h:.0f} | | |")
        md.append("")
        if args.traffic:
            update_traffic_file(args.traffic, args.workload, table)

    with open(args.out, "w") as fh:
        fh.write("\n".join(md) + "\n")
    print(f"wrote {args.out}")


if __name__ == "__main__":
    main()
