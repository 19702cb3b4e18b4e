"""The cost-model helper against the figures the paper prints (tests/golden/paper_cost_figures.txt)."""
import os

from paper_2506_17286_amd import costmodel as cm


def _golden():
    vals = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_cost_figures.txt")
    for line in open(path):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


def test_cache_columns_of_tables_1_and_2():
    g = _golden()
    assert cm.gta_cache_elems_per_token(1, 1, 64, 128) == g["gta1_cache_per_layer"] == g["gta3_cache_per_layer"]
    assert cm.gta_cache_elems_per_token(1, 2, 64, 128) == g["gta4_cache_per_layer"]
    assert cm.gqa_cache_elems_per_token(3, 64) == g["gqa160m_cache_per_layer"]
    assert cm.gqa_cache_elems_per_token(4, 64) == g["gqa500m_cache_per_layer"]
    assert cm.gqa_cache_elems_per_token(12, 64) == g["mha160m_cache_per_layer"]
    assert cm.gqa_cache_elems_per_token(20, 64) == g["mha500m_cache_per_layer"]
    assert cm.gta_cache_elems_per_token(1, 2, 64, 128) / cm.gqa_cache_elems_per_token(20, 64) == g["gta4_over_mha500m_cache"]


def test_gta1b_ratios():
    g = _golden()
    N = 2048
    cache = cm.gta_cache_elems_per_token(1, 1, 64, 128) / cm.gqa_cache_elems_per_token(5, 64)
    attn = cm.gta_attention_ops(5, 64, 128, N) / cm.mha_attention_ops(20, 64, N)
    assert abs(cache - g["gta1b_over_gqa1b_cache"]) < 1e-12
    assert abs(attn - g["gta1b_over_gqa1b_attention"]) < 1e-12


def test_benchmark_counters():
    from paper_2506_17286_amd.workloads import WORKLOADS
    w2 = WORKLOADS[1]
    f = cm.prefill_flops(w2, [4096] * 4)
    assert f["attn"] == 2 * 4 * 640 * 4 * (4096 * 4097 // 2)
    assert f["proj"] == 2 * 16384 * 2048 * 3584
    assert f["decoder"] == 2 * 16384 * 16 * 512 * 128
    w4 = WORKLOADS[3]
    assert cm.decode_cache_bytes(w4, [32768] * 8) == 8 * 32768 * 1024 * 2
