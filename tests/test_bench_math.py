"""The algorithmic work bench.py prices a step at (the numerators of its roofline figures), against the figures worked out
by hand from the model shape: per layer 385.9 MFLOP per row, vocabulary projection 1.245 GFLOP per row, 4096 B of K/V per
cached token and layer (8B shape: hidden 4096, 32 q / 8 kv heads x 128, ffn 12288, vocabulary 151 936)."""
import importlib.util
import os

import focus_inputs as fi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(spec)
spec.loader.exec_module(bench)


def test_projection_flops_of_the_batch256_configuration():
    wl = fi.workload("c4_batch256")
    per_row_layer = 2 * (6144 * 4096 + 4096 * 4096 + 3 * 12288 * 4096)
    assert per_row_layer == 385_875_968
    head = 2 * 151936 * 4096
    T0 = 8192
    for Tp, tflop in ((8192, 124.0), (4096, 63.8), (2048, 33.7), (1024, 18.6)):
        # layer 0 complete and layer 1's QKV on all rows; the rest of layer 1, layers 2..35 and the vocabulary projection on T' rows
        by_hand = T0 * (per_row_layer + 2 * 6144 * 4096) + Tp * (per_row_layer - 2 * 6144 * 4096 + 34 * per_row_layer + head)
        assert bench.gemm_flops_per_step(wl, T0, Tp) == by_hand
        assert abs(by_hand / 1e12 - tflop) < 0.05


def test_kv_and_phase_bytes():
    wl = fi.workload("c4_batch256")
    lens = wl.prefix_lens()
    assert bench.kv_bytes_per_step(wl, lens) == sum(l + 32 for l in lens) * 4096 * 36
    pb = bench.phase_bytes(wl, 8192, 2048)
    assert pb["gather"] == 2048 * 49152                       # fp32 residual row and bf16 query row, read and written
    assert pb["kv_write"] == (2 * 8192 + 34 * 2048) * (12288 + 10240 + 4096)
    moe = fi.workload("c6_moe_mini")
    assert bench.expert_bytes_per_step(moe) == 19 * 256 * 3 * 2048 * 512 * 2
