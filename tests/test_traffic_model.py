"""The byte/flop model against the counts the paper prints (no GPU needed)."""
import os

from paper_2105_04779_amd import traffic_model as tm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_counts.txt")


def _rows():
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                yield line


def test_table4_cache_sizes_and_ratio():
    # BART-large: 12 decoder layers, d_m 1024, beam 4, half precision.
    seen = 0
    for row in _rows():
        if row[0] == "cache":
            B, n, mha_gb, el_gb = int(row[1]), int(row[2]), float(row[3]), float(row[4])
            el = tm.el_state_bytes(B, n, 1024) / tm.GiB
            mha = tm.mha_cache_bytes(B, n, 1024, layers=12, beam=4) / tm.GiB
            assert abs(mha - mha_gb) < 1e-9          # printed exactly
            assert abs(el - el_gb) <= 0.01           # printed with two decimals
            seen += 1
        if row[0] == "cache_ratio":
            assert tm.mha_cache_bytes(32, 256, 1024, 12, 4) == int(row[1]) * tm.el_state_bytes(32, 256, 1024)
            seen += 1
    assert seen == 7


def test_section_4_1_1_counts():
    vals = {r[0]: float(r[1]) for r in _rows() if r[0] != "cache"}
    B, x, n, d_m = 32, 4, 1024, 1024
    assert tm.build_kv_flops(B, x, n, d_m) / 1e9 > vals["build_kv_gflop_more_than"]
    assert tm.build_kv_flops(B, x, n, d_m) / 1e9 < 1.2 * vals["build_kv_gflop_more_than"]
    assert abs(tm.mha_group3_bytes(B, x, n, d_m) / 1e9 - vals["mha_group3_gb_about"]) < 0.05
    assert abs(tm.el_group3_bytes_two_reads(B, n, d_m) / 1e9 - vals["el_group3_gb_about"]) < 0.02
    # the fused kernel reads H once: half of the two-call figure
    assert tm.core_algorithmic_bytes(B * n, d_m, 2) * 2 == tm.el_group3_bytes_two_reads(B, n, d_m)


def test_step_totals_at_bart_large_shape():
    # mean length 768, B 64, beam 4: about 110 MB and 15 GFLOP per step
    sum_len = 64 * 768
    b = tm.step_algorithmic_bytes(sum_len, 64, 4, 1024, 1024, 2, out_bytes=4)
    f = tm.step_flops(sum_len, 64, 4, 16, 1024, 64)
    assert 108e6 < b < 112e6
    assert 14.9e9 < f < 15.1e9
