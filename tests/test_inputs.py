"""The seeded input generator: tensor hash equals the big-integer definition, sub-ranges agree,
statistics are as documented, workload recipes have the stated shapes."""
import numpy as np
import torch

import focus_inputs as fi


def test_tensor_hash_equals_python_integers():
    key = fi.stream_key(3, 17)
    idx = [0, 1, 2, 12345, (1 << 31) + 5, (1 << 40) + 123, 43_000_000_000]
    h = fi.hash_t(key, torch.tensor(idx, dtype=torch.int64)).tolist()
    for i, v in zip(idx, h):
        assert v % (1 << 64) == fi.hash_py(key, i)


def test_subrange_equals_whole_and_bf16_rounding():
    whole = fi.normal_values(1, 5, 0, 5000, 0.02)
    part = fi.normal_values(1, 5, 1234, 100, 0.02)
    assert torch.equal(whole[1234:1334], part)
    b = fi.normal_values(1, 5, 0, 5000, 0.02, dtype=torch.bfloat16)
    assert torch.equal(b, whole.to(torch.bfloat16))
    assert not torch.equal(fi.normal_values(2, 5, 0, 100, 0.02), whole[:100])      # seed matters
    assert not torch.equal(fi.normal_values(1, 6, 0, 100, 0.02), whole[:100])      # tensor id matters


def test_statistics():
    z = fi.normal_values(0, 1, 0, 400000, 1.0).double()
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert z.abs().max() <= 3.47


def test_fill_matches_values_and_page_view():
    wl = fi.workload("c1_tiny")
    lens = wl.prefix_lens()
    assert len(lens) == 4 and all(32 <= l <= 64 for l in lens)
    tables, n_pages = wl.page_tables(lens)
    assert sum(len(t) for t in tables) == n_pages and all(len(t) * wl.page_size >= l + wl.block_size for t, l in zip(tables, lens))
    pool = torch.empty((wl.n_layers, n_pages, 2, wl.n_kv_heads, wl.page_size, wl.head_dim))
    wl.kv_pool_fill_(pool)
    page = wl.kv_page(1, 3, n_pages)
    assert torch.equal(pool[1, 3, 0], page[0]) and torch.equal(pool[1, 3, 1].reshape(wl.n_kv_heads, wl.head_dim, wl.page_size).transpose(1, 2), page[1])
    w = wl.layer_weight(1, "w_o")
    assert w.shape == (256, 256) and abs(float(w.std()) - 0.02) < 1e-3


def test_workload_recipes():
    c4 = fi.workload("c4_batch256")
    lens = c4.prefix_lens()
    assert len(lens) == 256 and min(lens) >= 512 and max(lens) <= 4096 and 2000 < np.mean(lens) < 2600
    c5 = fi.workload("c5_ragged")
    l5 = c5.prefix_lens()
    assert len(l5) == 64 and min(l5) >= 1024 and max(l5) <= 32768
    ks = c5.k_overrides()
    assert ks[0] == 0 and ks[1] == 64 and all(0 <= k <= 64 for k in ks)
    t5, n5 = c5.page_tables(l5)
    flat = [p for t in t5 for p in t]
    assert sorted(flat) == list(range(n5)) and flat != sorted(flat)                 # a real permutation
    toks = fi.workload("c1_tiny").prompt_tokens()
    assert all(1 <= t < 1024 for row in toks for t in row)


def test_expert_weights_and_forced_routes():
    wl = fi.workload("c1_tiny", n_experts=8, experts_per_token=3, expert_ffn=16, shared_ffn=8, first_moe_layer=1, n_layers=3)
    assert [wl.is_moe_layer(l) for l in range(3)] == [False, True, True]
    shapes = wl.moe_weight_shapes()
    assert shapes["w_expert_gate_up"] == (8, 32, wl.hidden) and shapes["w_expert_down"] == (8, wl.hidden, 16)
    w1, w2 = wl.moe_weight(1, "w_expert_gate_up"), wl.moe_weight(2, "w_expert_gate_up")
    assert torch.equal(w1, wl.moe_weight(1, "w_expert_gate_up")) and not torch.equal(w1, w2)       # pure function of (seed, layer, tensor)
    assert abs(float(w1.std()) - fi.WEIGHT_STD) < 0.1 * fi.WEIGHT_STD
    # an expert's slice is the same stream whichever way it is generated (flat index = row-major offset)
    e = 5
    per = 32 * wl.hidden
    part = fi.normal_values(wl.seed, fi.TID_MOE0 + 8 * 1 + 1, e * per, per, fi.WEIGHT_STD).view(32, wl.hidden)
    assert torch.equal(part, w1[e])
    routes = wl.route_override(2)
    assert len(routes) == 3 and len(routes[0]) == 2 * wl.block_size
    assert all(len(set(r)) == 3 and all(0 <= x < 8 for x in r) for layer in routes for r in layer)
    assert routes == wl.route_override(2) and routes[1] != routes[2]
    counts = np.bincount([x for layer in routes for r in layer for x in r], minlength=8)
    assert counts.min() > 0                                                                        # every expert gets rows
