"""The cost model of Section 5.2 against the numbers the paper prints
(tests/golden/paper_tables.txt)."""
from paper_2503_21817_amd import flopmodel as M
from paper_2503_21817_amd import workloads as W


def test_table1_ffn_share(golden):
    C, I, L = int(golden["llama3_8b_C"]), int(golden["llama3_8b_M"]), int(golden["llama3_8b_layers"])
    assert abs(M.ffn_params(C, I, L) / 1e9 - golden["ffn_params_billion"]) < 0.005
    # 10.5 L N C^2 = 3 N C M L with M = 3.5 C
    assert 3 * I / C == golden["ffn_complexity_coeff"]
    assert M.ffn_macs(1, C, I) * L == golden["ffn_complexity_coeff"] * L * C * C


def test_table3_flops_column(golden):
    # SV-LLaVA: N1 = N_r + N_s tokens in attention, N2 = N_r in the FFN, baseline 576
    assert round(100 * M.flops_ratio(256, 100, 576)) == golden["sv_llava_100_156_flops_pct"]
    assert abs(100 * M.flops_ratio(576, 256, 576) - golden["sv_llava_256_320_flops_pct"]) < 1.0
    # SV-CoS: 272 + 256 tokens in attention, 272 in the FFN, baseline 1296 (within a point)
    assert abs(100 * M.flops_ratio(528, 272, 1296) - golden["sv_cos_272_256_flops_pct"]) < 1.5


def test_bench_flops_are_the_ffn_term():
    w = W.config(2)
    assert w.flops() == 2 * M.ffn_macs(w.R, w.C, w.I) == M.skipffn_flops(w.R, w.C, w.I, False)
    assert abs(w.flops() / 1e12 - 0.5186) < 1e-3
    w3 = W.config(3)
    assert w3.flops() == M.skipffn_flops(w3.R, w3.C, w3.I, True)
    assert abs(w3.flops() / 1e12 - 2.706) < 2e-3
    w5 = W.config(5)
    assert abs(w5.flops() / 1e12 - 99.57) < 0.05
