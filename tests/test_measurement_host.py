"""Host-side checks of the measurement plumbing (no GPU): kernel-name -> layer-step mapping of the profile
summariser, and bench.py's lookup of measured traffic in profiles/hbm_traffic.txt."""
import importlib.util
import os

from paper_2210_03052_amd import profile_summary as PS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_kernel_names_map_to_layer_steps():
    g = "_ZN2bt16gemm_pipe_kernelILi{}ELi{}ELi{}ELi{}ELi{}ELi{}ELi{}ELi{}EEEvPKDF16_S2_PKiS2_iiiiiiPDF16_NS_7GemmEpiE"
    assert PS.role_of(g.format(192, 128, 2, 4, 3, 0, 0, 0))[0] == "gemm0_qkv_bias"
    assert PS.role_of(g.format(64, 128, 2, 4, 4, 0, 0, 1))[0] == "gemm1_proj"
    assert PS.role_of(g.format(256, 128, 4, 2, 3, 1, 0, 1))[0] == "gemm2_bias_gelu"
    assert PS.role_of(g.format(64, 128, 2, 4, 4, 0, 0, 2))[0] == "gemm3_ffn_down"
    assert PS.role_of(g.format(64, 64, 2, 2, 4, 0, 3, 2))[0] == "gemm3_ffn_down"      # split over K, deep
    assert PS.role_of(g.format(192, 128, 2, 4, 3, 0, 1, 0))[0] == "gemm0_qkv_folded"   # folded pipeline
    assert PS.role_of(g.format(256, 128, 4, 2, 3, 1, 1, 1))[0] == "gemm2_bias_gelu_folded"
    assert PS.role_of(g.format(64, 128, 2, 4, 4, 0, 2, 1))[0] == "gemm1_proj_resid"
    assert PS.role_of(g.format(64, 128, 2, 4, 4, 0, 2, 2))[0] == "gemm3_ffn_down_resid"
    assert PS.role_of(g.format(64, 64, 2, 2, 4, 0, 3, 1))[0] == "gemm1_proj"          # split over K, square
    assert PS.role_of("_ZN2bt17varlen_mha_kernelILi4ELi2EEEvPKiiifPKDF16_S4_S4_lPDF16_S4_S4_") == \
        ("varlen_mha", "varlen_mha<4,2>")
    assert PS.role_of("_ZN2bt23bias_residual_ln_kernelILi2ELb0ELb1EEEvPKDF16_S2_S2_iiif")[0] == "bias_residual_ln_streaming"
    assert PS.role_of("_ZN2bt23bias_residual_ln_kernelILi2ELb1ELb0EEEvPKDF16_S2_S2_iiif")[0] == "bias_residual_ln"
    assert PS.role_of("bt::pack_kernel(unsigned int __vector(4) const*, int const*, unsigned long, int)", 221568)[0] == "pack"
    assert PS.role_of("bt::pack_kernel(unsigned int __vector(4) const*, int const*, unsigned long, int)", 25165824)[0] == "pack_streaming"
    assert PS.role_of("bt::unpack_kernel(unsigned int __vector(4) const*, int const*, int, int, int)")[0] == "unpack"
    assert PS.role_of("void at::native::vectorized_elementwise_kernel<4, foo>") == (None, None)
    assert PS.template_args("gemm_pipe_kernel<64, 128, 2, 4, 4, 0, 0, 2>") == [64, 128, 2, 4, 4, 0, 0, 2]


def test_derived_mfma_figures():
    # 1000 MFMAs of 32x32x16: 32 busy cycles and 64 units of 512 FLOP each
    d = PS.derive({"SQ_INSTS_VALU_MFMA_MOPS_F16": 64000.0, "SQ_VALU_MFMA_BUSY_CYCLES": 32000.0,
                   "SQ_BUSY_CU_CYCLES": 20000.0, "SQ_INSTS_MFMA": 1000.0, "SQ_INSTS_VALU": 6000.0,
                   "SQ_WAVE_CYCLES": 100.0, "SQ_WAIT_INST_ANY": 25.0})
    assert abs(d["executed_gflop"] - 1000 * 2 * 32 * 32 * 16 / 1e9) < 1e-12
    assert abs(d["mfma_busy_share_of_busy_simd_cycles"] - 0.4) < 1e-12
    assert abs(d["valu_instructions_per_mfma"] - 5.0) < 1e-12
    assert abs(d["wave_cycles_waiting_on_an_instruction"] - 0.25) < 1e-12
    assert PS.derive({"SQ_WAVE_CYCLES": 10.0, "SQ_WAIT_INST_ANY": 1.0}) == {"wave_cycles_waiting_on_an_instruction": 0.1}


def test_bench_reads_traffic_table(tmp_path):
    spec = importlib.util.spec_from_file_location("bench_mod", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    table = tmp_path / "t.txt"
    table.write_text("# workload kernel fetch_kib write_kib hbm_bytes\nw1 gemm3_ffn_down 10.0 20.0 12345\n"
                     "w1 bias_residual_ln 1.0 1.0 777\n")
    bench.TRAFFIC_FILE = str(table)
    assert bench.measured_traffic("w1", "gemm3_ffn_down") == 12345
    assert bench.measured_traffic("w1", "bias_residual_ln1") == 777        # both LayerNorms are one kernel
    assert bench.measured_traffic("w1", "gemm0_qkv_bias") is None
    assert bench.measured_traffic("w2", "gemm3_ffn_down") is None
    bench.TRAFFIC_FILE = str(tmp_path / "missing.txt")
    assert bench.measured_traffic("w1", "gemm3_ffn_down") is None
    # the committed table covers the dominant kernels of the workloads the bench is run on
    bench.TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    for w, k in (("bert_base_b16_s256", "gemm3_ffn_down"), ("bert_base_b16_s1024", "gemm2_bias_gelu"),
                 ("bert_large_b32_s512", "gemm2_bias_gelu"), ("mha_b16_s256", "varlen_mha")):
        assert bench.measured_traffic(w, k) > 0
