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
