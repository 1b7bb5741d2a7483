"""Pins of the CPU oracle against things other than itself: library routines, closed forms,
brute force on tiny inputs, invariants the paper states, hand-worked values."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import focus_oracle as fo

RNG = np.random.default_rng(1234)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(**kw):
    base = dict(n_layers=3, hidden=32, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn=48, vocab=40, block_size=8,
                mask_token_id=0, page_size=4, rope_base=10000.0, evict_layer=1, budget_mode=1, keep_ratio=0.25)
    base.update(kw)
    return fo.OracleConfig(**base)


def tiny_weights(cfg, seed=0, scale=0.3):
    r = np.random.default_rng(seed)
    qkv = (cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim
    layers = [dict(w_qkv=r.normal(0, scale, (qkv, cfg.hidden)),
                   w_o=r.normal(0, scale, (cfg.hidden, cfg.n_q_heads * cfg.head_dim)),
                   w_gate_up=r.normal(0, scale, (2 * cfg.ffn, cfg.hidden)),
                   w_down=r.normal(0, scale, (cfg.hidden, cfg.ffn)),
                   attn_norm=r.uniform(0.5, 1.5, cfg.hidden), mlp_norm=r.uniform(0.5, 1.5, cfg.hidden))
              for _ in range(cfg.n_layers)]
    return fo.Weights(r.normal(0, 1.0, (cfg.vocab, cfg.hidden)), r.normal(0, scale, (cfg.vocab, cfg.hidden)),
                      r.uniform(0.5, 1.5, cfg.hidden), lambda l: layers[l])


def tiny_batch(cfg, W, prefix_lens, seed=0, page_offset=0, page_order=None):
    """Prefilled oracle batch from random prompts."""
    r = np.random.default_rng(seed + 77)
    pool = fo.KVPool(cfg)
    states, prompts, at = [], [], 0
    for L in prefix_lens:
        npg = (L + cfg.block_size + cfg.page_size - 1) // cfg.page_size
        pages = list(range(page_offset + at, page_offset + at + npg))
        if page_order is not None:
            pages = [page_order[p] for p in pages]
        at += npg
        states.append(fo.new_seq_state(cfg, L, pages))
        prompts.append(list(r.integers(1, cfg.vocab, L)))
    fo.prefill(cfg, W, pool, states, prompts)
    return pool, states, prompts


# ---------------------------------------------------------------------------------------------
# textbook pieces against library routines

def test_maxpool_matches_torch_maxpool1d():
    s = RNG.normal(size=(5, 7, 11))
    for k in (1, 3, 5):
        ref = F.max_pool1d(torch.from_numpy(s), kernel_size=k, stride=1, padding=(k - 1) // 2).numpy()
        assert np.array_equal(fo.maxpool1d_same(s, k), ref)


def test_rmsnorm_matches_torch():
    x, w = RNG.normal(size=(6, 32)), RNG.uniform(0.5, 2.0, 32)
    ref = F.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(w), eps=1e-6).numpy()
    np.testing.assert_allclose(fo.rmsnorm(x, w, 1e-6), ref, rtol=1e-13, atol=1e-14)


def test_rope_is_complex_rotation_and_relative():
    D, H = 16, 3
    x = RNG.normal(size=(5, H, D))
    pos = np.array([0, 1, 7, 100, 4095])
    out = fo.rope(x, pos, 10000.0)
    # pair (i, i + D/2) as a complex number rotated by pos * base^(-2i/D)
    z = x[..., :D // 2] + 1j * x[..., D // 2:]
    theta = pos[:, None] * 10000.0 ** (-2.0 * np.arange(D // 2) / D)
    zr = z * np.exp(1j * theta)[:, None, :]
    np.testing.assert_allclose(out[..., :D // 2], zr.real, atol=1e-12)
    np.testing.assert_allclose(out[..., D // 2:], zr.imag, atol=1e-12)
    # position 0 is the identity; the norm is preserved
    np.testing.assert_allclose(out[0], x[0], atol=0)
    np.testing.assert_allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # inner products depend on the position difference only
    q, k = RNG.normal(size=(1, 1, D)), RNG.normal(size=(1, 1, D))
    a = (fo.rope(q, np.array([13]), 1e4) * fo.rope(k, np.array([9]), 1e4)).sum()
    b = (fo.rope(q, np.array([104]), 1e4) * fo.rope(k, np.array([100]), 1e4)).sum()
    assert abs(a - b) < 1e-10


def test_softmax_rows_sum_to_one_and_attention_of_ones():
    s = RNG.normal(size=(9, 33)) * 5
    assert np.max(np.abs(fo.softmax_rows(s).sum(-1) - 1)) < 1e-12
    cfg = tiny_cfg()
    q = RNG.normal(size=(5, 4, 8))
    K = RNG.normal(size=(17, 2, 8))
    out = fo._attention(cfg, q, K, np.ones((17, 2, 8)))
    np.testing.assert_allclose(out, 1.0, atol=1e-12)       # rows of attention weights sum to one


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (4, 1)])
def test_attention_matches_torch_sdpa(Hq, Hkv):
    cfg = tiny_cfg(n_q_heads=Hq, n_kv_heads=Hkv)
    D = 8
    for r, t in [(1, 1), (1, 19), (6, 6), (5, 23)]:
        q, K, V = RNG.normal(size=(r, Hq, D)), RNG.normal(size=(t, Hkv, D)), RNG.normal(size=(t, Hkv, D))
        g = Hq // Hkv
        Kr, Vr = np.repeat(K, g, axis=1), np.repeat(V, g, axis=1)     # key head h // g
        ref = F.scaled_dot_product_attention(torch.from_numpy(q).transpose(0, 1)[None],
                                             torch.from_numpy(Kr).transpose(0, 1)[None],
                                             torch.from_numpy(Vr).transpose(0, 1)[None])[0].transpose(0, 1).numpy()
        np.testing.assert_allclose(fo._attention(cfg, q, K, V), ref, rtol=1e-11, atol=1e-12)


def test_confidence_matches_torch_softmax_and_lowest_index_tie():
    lg = RNG.normal(size=(7, 50)) * 3
    lg[2, 10] = lg[2, 30] = 99.0
    conf, am = fo.confidence(lg)
    p = torch.softmax(torch.from_numpy(lg), -1)
    np.testing.assert_allclose(conf, p.max(-1).values.numpy(), rtol=1e-12)
    assert am[2] == 10
    assert np.array_equal(np.delete(am, 2), np.delete(p.argmax(-1).numpy(), 2))


# ---------------------------------------------------------------------------------------------
# Eq. 2

def importance_brute(q, k, pool_k):
    """Triple-loop statement of Eq. 2 with python floats."""
    B, Hq, D = q.shape
    g = Hq // k.shape[1]
    r = (pool_k - 1) // 2
    I = [0.0] * B
    for h in range(Hq):
        for i in range(B):
            S = [sum(q[i, h, d] * k[j, h // g, d] for d in range(D)) / math.sqrt(D) for j in range(B)]
            pooled = [max(S[jj] for jj in range(max(0, j - r), min(B, j + r + 1))) for j in range(B)]
            m = max(pooled)
            ex = [math.exp(v - m) for v in pooled]
            z = sum(ex)
            for j in range(B):
                I[j] += ex[j] / z
    return np.array(I)


@pytest.mark.parametrize("B,Hq,Hkv,D", [(5, 2, 1, 4), (8, 4, 2, 8), (16, 4, 4, 8)])
def test_importance_brute_force_and_total_mass(B, Hq, Hkv, D):
    q, k = RNG.normal(size=(B, Hq, D)) * 2, RNG.normal(size=(B, Hkv, D)) * 2
    for pk in (1, 3):
        I = fo.importance(q, k, pk)
        np.testing.assert_allclose(I, importance_brute(q, k, pk), rtol=1e-12, atol=1e-12)
        assert abs(I.sum() - B * Hq) < 1e-9              # every (query, head) row adds one unit of mass


def test_importance_without_pooling_is_softmax_column_sum_and_constant_scores():
    B, Hq, D = 6, 3, 4
    q, k = RNG.normal(size=(B, Hq, D)), RNG.normal(size=(B, Hq, D))
    S = torch.einsum("ihd,jhd->hij", torch.from_numpy(q), torch.from_numpy(k)) / math.sqrt(D)
    ref = torch.softmax(S, -1).sum(dim=(0, 1)).numpy()
    np.testing.assert_allclose(fo.importance(q, k, 1), ref, rtol=1e-12)
    # all scores equal -> every key gets 1/B from each of the B*Hq rows
    np.testing.assert_allclose(fo.importance(np.zeros((B, Hq, D)), k, 3), np.full(B, Hq), rtol=1e-13)


def test_importance_pooling_spreads_a_peak_to_its_neighbours():
    # one key (j = 3) with a dominant score for every query: with k = 3 positions 2, 3, 4 share the mass
    B, D = 8, 4
    q = np.ones((B, 1, D))
    k = np.zeros((B, 1, D))
    k[3] = 20.0
    I = fo.importance(q, k, 3)
    np.testing.assert_allclose(I[2:5], B / 3.0, rtol=1e-9)
    assert I[[0, 1, 5, 6, 7]].max() < 1e-9


# ---------------------------------------------------------------------------------------------
# Eq. 4-5, budget

def test_budget_golden_cases():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq4_budget_cases.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 8
    for a, ts, st, ns, B, K in rows:
        B, ns = int(B), int(ns)
        cfg = tiny_cfg(block_size=B, budget_mode=2, alpha=float(a))
        # a delta vector with exactly `ns` masked entries above mean + std: ns + 1 spikes, one of them on a
        # position that is no longer masked, the rest flat
        dI = [0.0] * B
        masked = [True] * B
        for j in range(ns + 1):
            dI[j] = 10.0
        masked[ns] = False
        mu, sd = np.mean(dI), np.std(dI)
        assert 10.0 >= mu + sd and 0.0 < mu + sd
        assert fo.budget(cfg, dI, masked, int(ts), int(st)) == int(K)


def test_n_sigma_hand_vector_and_mask():
    dI = [3.0, -1.0, -1.0, -1.0, 2.0, -1.0, -1.0, 0.0]            # mean 0, population std = sqrt(18/8) = 1.5
    assert abs(np.std(dI) - 1.5) < 1e-15
    assert fo.n_sigma(dI, [True] * 8) == 2                          # 3.0 and 2.0 are >= 1.5
    assert fo.n_sigma(dI, [False] + [True] * 7) == 1                # only masked positions are counted
    dI2 = [1.5 + 0.5, -0.5, -0.5, -0.5, 1.5 + 0.5 - 1.0, -0.5, -0.5, 0.5 - 1.0 + 0.5]
    # threshold is mean + std (not std alone): shift everything by +10 and the count must not change
    assert fo.n_sigma([v + 10 for v in dI], [True] * 8) == 2
    # ">=": a value sitting exactly on the threshold counts (two-point vector: mean 0, std 1)
    assert fo.n_sigma([1.0, -1.0], [True, True]) == 1


def test_fixed_budget_modes():
    B = 32
    assert fo.budget(tiny_cfg(block_size=B, budget_mode=0, topk=2), [0] * B, [True] * B, 0, 0) == 2
    for rho, K in [(1.0, 32), (0.5, 16), (0.25, 8), (0.125, 4), (0.3, 10)]:
        assert fo.budget(tiny_cfg(block_size=B, budget_mode=1, keep_ratio=rho), [0] * B, [True] * B, 0, 0) == K
    assert fo.budget(tiny_cfg(block_size=B, budget_mode=3), [0] * B, [True] * B, 0, 0, k_override=77) == B
    assert fo.budget(tiny_cfg(block_size=B, budget_mode=3), [0] * B, [True] * B, 0, 0, k_override=0) == 0


def test_running_mean_recurrence_three_steps():
    # App. E.3.1: token_sum += n_decoded, total_steps += 1, Nbar = token_sum / total_steps
    cfg = tiny_cfg(conf_threshold=0.5)
    st = fo.new_seq_state(cfg, 4, [0, 1, 2])
    S = [0, 1, 2, 3]
    assert fo.commit(cfg, st, S, [0.9, 0.6, 0.1, 0.2], [11, 12, 13, 14]) == [0, 1]      # two pass the threshold
    assert (st.token_sum, st.total_steps) == (2, 1)
    assert fo.commit(cfg, st, S, [0.99, 0.99, 0.3, 0.4], [21, 22, 23, 24]) == [3]        # none passes: best masked one
    assert (st.token_sum, st.total_steps) == (3, 2)
    assert st.tokens[:4] == [11, 12, cfg.mask_token_id, 24] and st.masked[:4] == [False, False, True, False]
    assert fo.commit(cfg, st, S, [0.0, 0.0, 0.5, 0.0], [31, 32, 33, 34]) == [2]          # ">=": exactly on threshold
    assert (st.token_sum, st.total_steps) == (4, 3)
    assert abs(st.token_sum / st.total_steps - 4 / 3) < 1e-15
    # forced commit tie -> lower position; empty S leaves the counters alone
    st2 = fo.new_seq_state(cfg, 4, [0, 1, 2])
    assert fo.commit(cfg, st2, [2, 5], [0.25, 0.25], [7, 8]) == [2]
    assert fo.commit(cfg, st2, [], [], []) == [] and (st2.token_sum, st2.total_steps) == (1, 1)


# ---------------------------------------------------------------------------------------------
# Alg. 1 phase 3: selection, brute force

def select_brute(dI, masked, K, B, constraints):
    """Set algebra of Alg. 1 phase 3, with top-K found by exhaustive search over subsets."""
    if K >= B:
        return list(range(B))
    M = [j for j in range(B) if masked[j]]
    k = min(K, len(M))
    if k <= 0:
        return []

    def before(i, j):         # i ranks ahead of j
        return dI[i] > dI[j] or (dI[i] == dI[j] and i < j)
    tops = [set(T) for T in itertools.combinations(M, k)
            if all(before(i, j) for i in T for j in M if j not in T)]
    assert len(tops) == 1
    S = set(tops[0])
    if constraints & 1:
        S = S | {i - 1 for i in tops[0] if i - 1 >= 0}
    if constraints & 2:
        S = S | {j for j in range(B) if j < max(S) and masked[j]}
    return sorted(S)


@pytest.mark.parametrize("constraints", [0, 1, 2, 3])
def test_select_brute_force(constraints):
    r = np.random.default_rng(5 + constraints)
    B = 8
    cfg = tiny_cfg(block_size=B, constraints=constraints)
    for trial in range(300):
        dI = list(np.round(r.normal(size=B), 1))                   # coarse values -> frequent ties
        masked = list(r.random(B) < 0.7)
        for K in range(0, B + 1):
            assert fo.select(cfg, dI, masked, [False] * B, K) == select_brute(dI, masked, K, B, constraints)


def test_select_hand_cases():
    B = 8
    dI = [0.1, 0.9, 0.2, 0.9, -0.5, 0.3, 0.0, 0.8]
    allm = [True] * B
    assert fo.select(tiny_cfg(block_size=B), dI, allm, [False] * B, 2) == [1, 3]               # tie -> lower index
    assert fo.select(tiny_cfg(block_size=B), dI, allm, [False] * B, 3) == [1, 3, 7]
    m = list(allm)
    m[1] = False                                                                                # unmasked is no candidate
    assert fo.select(tiny_cfg(block_size=B), dI, m, [False] * B, 2) == [3, 7]
    assert fo.select(tiny_cfg(block_size=B, constraints=1), dI, m, [False] * B, 2) == [2, 3, 6, 7]
    assert fo.select(tiny_cfg(block_size=B, constraints=2), dI, m, [False] * B, 1) == [0, 2, 3]
    assert fo.select(tiny_cfg(block_size=B, constraints=3), dI, m, [False] * B, 1) == [0, 2, 3]
    assert fo.select(tiny_cfg(block_size=B), dI, [False] * B, [False] * B, 3) == []            # nothing masked
    assert fo.select(tiny_cfg(block_size=B), dI, allm, [False] * B, 8) == list(range(8))       # K = B: keep all
    assert fo.select(tiny_cfg(block_size=B), dI, m, [False] * B, 8) == list(range(8))          # ... decoded ones too
    nan = float("nan")
    assert fo.select(tiny_cfg(block_size=B), [nan, 0.0, nan, -1.0] + [-2.0] * 4, allm, [False] * B, 2) == [1, 3]
    # minimum retention: K >= 1 and a masked token exist -> at least one row
    assert len(fo.select(tiny_cfg(block_size=B), dI, [False] * 7 + [True], [False] * B, 1)) == 1


# ---------------------------------------------------------------------------------------------
# Sec. 5.2: Top / Random / Bottom pick of the K candidates

def test_selection_key_is_the_published_splitmix64_stream():
    # first outputs of SplitMix64 started at 0 (test vector circulated with the generator's reference code)
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [fo.selection_key(0, 0, 0, j) for j in range(3)] == want
    # the counter is (slot * 2^32 + step) * 64 + j: a step moves 64 outputs ahead, a slot 2^38
    assert fo.selection_key(0, 0, 1, 0) != fo.selection_key(0, 0, 0, 0)
    state, outs = 0, []
    for _ in range(64 + 3):
        state = (state + 0x9E3779B97F4A7C15) & (2 ** 64 - 1)
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & (2 ** 64 - 1)
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & (2 ** 64 - 1)
        outs.append(z ^ (z >> 31))
    assert [fo.selection_key(0, 0, 1, j) for j in range(3)] == outs[64:67]
    # a different seed is a different start of the same stream
    assert fo.selection_key(0x9E3779B97F4A7C15, 0, 0, 0) == outs[1]


@pytest.mark.parametrize("constraints", [0, 3])
def test_bottom_pick_is_the_top_pick_of_the_negated_delta(constraints):
    r = np.random.default_rng(31 + constraints)
    B = 8
    top, bot = tiny_cfg(block_size=B, constraints=constraints), tiny_cfg(block_size=B, constraints=constraints, selection=2)
    for trial in range(300):
        dI = list(np.round(r.normal(size=B), 1))
        masked = list(r.random(B) < 0.7)
        for K in range(0, B + 1):
            neg = [-x + 0.0 for x in dI]
            assert fo.select(bot, dI, masked, [False] * B, K) == select_brute(neg, masked, K, B, constraints)
            assert fo.select(bot, dI, masked, [False] * B, K) == fo.select(top, neg, masked, [False] * B, K)
    nan = float("nan")
    allm = [True] * B
    assert fo.select(tiny_cfg(block_size=B, selection=2), [nan, 0.0, nan, -1.0] + [2.0] * 4, allm, [False] * B, 2) == [1, 3]
    assert fo.select(tiny_cfg(block_size=B, selection=2), [0.5, 0.1, 0.1, 0.9, 0.1, 3, 3, 3], allm, [False] * B, 2) == [1, 2]


def test_random_pick_is_a_uniform_k_subset_of_the_masked_positions():
    B, K = 8, 3
    cfg = tiny_cfg(block_size=B, selection=1, selection_seed=7)
    masked = [True, True, False, True, True, True, False, True]
    M = [j for j in range(B) if masked[j]]
    dI = [float(j) for j in range(B)]                          # the delta must play no part
    counts = np.zeros(B)
    n = 6000
    for step in range(n):
        rk = [fo.selection_key(cfg.selection_seed, 5, step, j) for j in range(B)]
        S = fo.select(cfg, dI, masked, [False] * B, K, None, rk)
        assert len(S) == K and set(S) <= set(M)
        assert S == sorted(sorted(M, key=lambda j: (-rk[j], j))[:K])
        counts[S] += 1
    # every masked position is picked with probability K / |M| = 1/2: binomial std 0.0065, allow 5 sigma
    assert np.all(np.abs(counts[M] / n - K / len(M)) < 0.033) and counts[2] == counts[6] == 0
    # K beyond the candidates keeps them all, like the other strategies
    rk = [fo.selection_key(7, 0, 0, j) for j in range(B)]
    for sel in (0, 1, 2):
        assert fo.select(tiny_cfg(block_size=B, selection=sel), dI, masked, [False] * B, 7, None, rk) == M
    # ties in the key go to the lower position
    assert fo.select(cfg, dI, [True] * B, [False] * B, 2, None, [5, 9, 9, 1, 9, 0, 0, 0]) == [1, 2]


def test_random_pick_inside_a_step_uses_slot_and_step_counters():
    cfg = tiny_cfg(selection=1, selection_seed=3, keep_ratio=0.25)
    W = tiny_weights(cfg)
    pool, seqs, _ = tiny_batch(cfg, W, [6, 9])
    seqs[0].slot, seqs[1].slot = 4, 2
    B = cfg.block_size
    for step in range(3):
        before = [(list(st.masked), st.total_steps) for st in seqs]
        tr = fo.focus_step(cfg, W, pool, seqs)
        for b, st in enumerate(seqs):
            masked, steps = before[b]
            M = [j for j in range(B) if masked[j]]
            rk = [fo.selection_key(3, st.slot, steps, j) for j in range(B)]
            assert tr.keep[b] == sorted(sorted(M, key=lambda j: (-rk[j], j))[:min(tr.K[b], len(M))])


def test_compact_order_and_permutation_invariance():
    keep = [[1, 5], [], [0, 2, 7], [3]]
    cu, rm = fo.compact(keep, 8)
    assert cu == [0, 2, 2, 5, 6]
    assert rm == [1, 5, 16, 18, 23, 27]
    perm = [2, 0, 3, 1]
    cu2, rm2 = fo.compact([keep[i] for i in perm], 8)
    assert [cu2[i + 1] - cu2[i] for i in range(4)] == [len(keep[i]) for i in perm]
    for newb, oldb in enumerate(perm):
        assert [r % 8 for r in rm2[cu2[newb]:cu2[newb + 1]]] == keep[oldb]


# ---------------------------------------------------------------------------------------------
# whole step against an independently written dense forward (torch, full sequence, block-causal mask)

def dense_reference(cfg, W, prompt, block_ids):
    """Block-diffusion forward of one whole sequence at once: token t attends to every token whose block
    index is <= its own (blocks of B counted from position 0).  Returns logits of the last B rows and the
    per-layer K/V of all positions.  Written with torch library ops only."""
    B = cfg.block_size
    ids = torch.tensor(list(prompt) + list(block_ids))
    T = len(ids)
    X = torch.from_numpy(W.embed)[ids]
    blk = torch.arange(T) // B
    mask = blk[None, :] <= blk[:, None]
    Hq, Hkv, D = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    inv = cfg.rope_base ** (-torch.arange(0, D, 2, dtype=torch.float64) / D)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None]
    cos, sin = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

    def rot(x):
        a, b = x[..., :D // 2], x[..., D // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], -1)
    kvs = []
    for l in range(cfg.n_layers):
        w = {k: torch.from_numpy(np.asarray(v)) for k, v in W.layer(l).items()}
        u = F.rms_norm(X, (cfg.hidden,), w["attn_norm"], eps=cfg.rms_eps)
        q, k, v = F.linear(u, w["w_qkv"]).split([Hq * D, Hkv * D, Hkv * D], dim=-1)
        q, k, v = rot(q.view(T, Hq, D)), rot(k.view(T, Hkv, D)), v.view(T, Hkv, D)
        kvs.append((k.numpy().copy(), v.numpy().copy()))
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           attn_mask=mask, enable_gqa=True)[0].transpose(0, 1).reshape(T, Hq * D)
        X = X + F.linear(o, w["w_o"])
        u = F.rms_norm(X, (cfg.hidden,), w["mlp_norm"], eps=cfg.rms_eps)
        g, up = F.linear(u, w["w_gate_up"]).split([cfg.ffn, cfg.ffn], dim=-1)
        X = X + F.linear(F.silu(g) * up, w["w_down"])
    logits = F.linear(F.rms_norm(X, (cfg.hidden,), torch.from_numpy(W.final_norm), eps=cfg.rms_eps),
                      torch.from_numpy(W.lm_head))
    return logits[-B:].numpy(), kvs


@pytest.mark.parametrize("Hkv", [2, 4])
def test_keep_all_step_equals_dense_block_forward_and_prefill_is_exact(Hkv):
    cfg = tiny_cfg(n_kv_heads=Hkv, keep_ratio=1.0)                  # K = B: no eviction
    W = tiny_weights(cfg, seed=3)
    lens = [16, 8]                                                  # multiples of B so blocks line up
    pool, states, prompts = tiny_batch(cfg, W, lens, seed=1)
    tr = fo.focus_step(cfg, W, pool, states)
    B = cfg.block_size
    assert tr.keep == [list(range(B))] * 2 and tr.cu == [0, B, 2 * B]
    for b, L in enumerate(lens):
        ref_logits, kvs = dense_reference(cfg, W, prompts[b], [cfg.mask_token_id] * B)
        np.testing.assert_allclose(tr.logits[b * B:(b + 1) * B], ref_logits, rtol=1e-9, atol=1e-10)
        for l in range(cfg.n_layers):                               # prefix and block K/V, every layer
            Kc, Vc = pool.read(l, states[b].pages, list(range(L + B)))
            np.testing.assert_allclose(Kc, kvs[l][0], rtol=1e-9, atol=1e-10)
            np.testing.assert_allclose(Vc, kvs[l][1], rtol=1e-9, atol=1e-10)
        # commit took the arg-max of the most confident row (nothing passes 0.9 with random weights)
        p = torch.softmax(torch.from_numpy(ref_logits), -1)
        best = int(p.max(-1).values.argmax())
        assert tr.committed[b] == [best] and states[b].tokens[best] == int(p[best].argmax())


def test_second_step_after_commit_equals_dense_forward_with_committed_token():
    cfg = tiny_cfg(keep_ratio=1.0)
    W = tiny_weights(cfg, seed=4)
    pool, states, prompts = tiny_batch(cfg, W, [8], seed=2)
    fo.focus_step(cfg, W, pool, states)
    st = states[0]
    ids = [cfg.mask_token_id if st.masked[p] else st.tokens[p] for p in range(cfg.block_size)]
    assert sum(st.masked) == cfg.block_size - 1
    tr = fo.focus_step(cfg, W, pool, states)
    ref_logits, _ = dense_reference(cfg, W, prompts[0], ids)
    np.testing.assert_allclose(tr.logits, ref_logits, rtol=1e-9, atol=1e-10)


def test_no_prefix_block_is_plain_bidirectional_attention():
    cfg = tiny_cfg(keep_ratio=1.0)
    W = tiny_weights(cfg, seed=6)
    pool, states, _ = tiny_batch(cfg, W, [0], seed=3)
    tr = fo.focus_step(cfg, W, pool, states)
    ref_logits, _ = dense_reference(cfg, W, [], [cfg.mask_token_id] * cfg.block_size)
    np.testing.assert_allclose(tr.logits, ref_logits, rtol=1e-9, atol=1e-10)


# ---------------------------------------------------------------------------------------------
# eviction semantics

def evicted_reference(cfg, W, prompt, block_ids, keep):
    """First step of a block with eviction after layer e, written as masked dense attention over the whole
    sequence (torch): layers <= e see everything; in layers > e only retained block rows exist (as queries and
    as keys).  Returns logits of the retained rows."""
    B, e = cfg.block_size, cfg.evict_layer
    L = len(prompt)
    ids = torch.tensor(list(prompt) + list(block_ids))
    T = len(ids)
    X = torch.from_numpy(W.embed)[ids]
    blk = torch.arange(T) // B
    mask_full = blk[None, :] <= blk[:, None]
    alive = torch.ones(T, dtype=torch.bool)
    alive[L:] = False
    alive[[L + p for p in keep]] = True
    Hq, Hkv, D = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    inv = cfg.rope_base ** (-torch.arange(0, D, 2, dtype=torch.float64) / D)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None]
    cos, sin = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

    def rot(x):
        a, b = x[..., :D // 2], x[..., D // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], -1)
    for l in range(cfg.n_layers):
        w = {k: torch.from_numpy(np.asarray(v)) for k, v in W.layer(l).items()}
        u = F.rms_norm(X, (cfg.hidden,), w["attn_norm"], eps=cfg.rms_eps)
        q, k, v = F.linear(u, w["w_qkv"]).split([Hq * D, Hkv * D, Hkv * D], dim=-1)
        q, k, v = rot(q.view(T, Hq, D)), rot(k.view(T, Hkv, D)), v.view(T, Hkv, D)
        mask = mask_full if l <= e else (mask_full & alive[None, :])
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           attn_mask=mask, enable_gqa=True)[0].transpose(0, 1).reshape(T, Hq * D)
        X = X + F.linear(o, w["w_o"])
        u = F.rms_norm(X, (cfg.hidden,), w["mlp_norm"], eps=cfg.rms_eps)
        g, up = F.linear(u, w["w_gate_up"]).split([cfg.ffn, cfg.ffn], dim=-1)
        X = X + F.linear(F.silu(g) * up, w["w_down"])
    logits = F.linear(F.rms_norm(X, (cfg.hidden,), torch.from_numpy(W.final_norm), eps=cfg.rms_eps),
                      torch.from_numpy(W.lm_head))
    return logits[[L + p for p in keep]].numpy()


@pytest.mark.parametrize("e", [1, 2])
def test_first_step_with_eviction_matches_masked_dense_reference(e):
    cfg = tiny_cfg(n_layers=4, evict_layer=e, keep_ratio=0.375)
    W = tiny_weights(cfg, seed=8)
    pool, states, prompts = tiny_batch(cfg, W, [16, 8, 24], seed=5)
    tr = fo.focus_step(cfg, W, pool, states)
    assert all(len(S) == 3 for S in tr.keep)
    for b in range(3):
        ref = evicted_reference(cfg, W, prompts[b], [cfg.mask_token_id] * cfg.block_size, tr.keep[b])
        np.testing.assert_allclose(tr.logits[tr.cu[b]:tr.cu[b + 1]], ref, rtol=1e-9, atol=1e-10)
        assert abs(tr.I_evict[b].sum() - cfg.block_size * cfg.n_q_heads) < 1e-9
        assert abs(tr.delta_I[b].sum()) < 1e-9                      # deltas are zero-sum (Sec. 4.1)
        # the retained set is the top-3 of the delta
        order = sorted(range(cfg.block_size), key=lambda j: (-tr.delta_I[b][j], j))
        assert tr.keep[b] == sorted(order[:3])


def run_steps(cfg, W, lens, steps, seed, **kw):
    pool, states, prompts = tiny_batch(cfg, W, lens, seed=seed, **kw)
    return [fo.focus_step(cfg, W, pool, states) for _ in range(steps)], states, pool


def test_stale_and_never_processed_slots():
    """Layers above e: a row evicted now but retained earlier stays visible with its old K/V; a position never
    retained is invisible, whatever its slot holds."""
    cfg = tiny_cfg(n_layers=3, keep_ratio=0.25)
    W = tiny_weights(cfg, seed=9)
    trs, states, pool = run_steps(cfg, W, [12], 3, seed=6)
    st = states[0]
    never = [p for p in range(cfg.block_size) if not st.processed[p]]
    assert never, "test needs a never-retained position"
    # rerun with garbage in the never-processed slots of the top layer: nothing may change
    pool2, states2, _ = tiny_batch(cfg, W, [12], seed=6)
    out2 = []
    for s in range(3):
        for p in never:
            pool2.write(2, states2[0].pages, 12 + p, np.full((cfg.n_kv_heads, cfg.head_dim), 1e6),
                        np.full((cfg.n_kv_heads, cfg.head_dim), -1e6))
        out2.append(fo.focus_step(cfg, W, pool2, states2))
    for a, b in zip(trs, out2):
        assert a.keep == b.keep and np.array_equal(a.logits, b.logits)
    # a processed-but-not-retained position is read: perturbing its stale slot changes the output
    union = set(trs[0].keep[0]) | set(trs[1].keep[0])
    stale = sorted(union - set(trs[2].keep[0]))
    if stale:
        pool3, states3, _ = tiny_batch(cfg, W, [12], seed=6)
        fo.focus_step(cfg, W, pool3, states3)
        fo.focus_step(cfg, W, pool3, states3)
        pool3.write(2, states3[0].pages, 12 + stale[0], np.full((cfg.n_kv_heads, cfg.head_dim), 3.0),
                    np.full((cfg.n_kv_heads, cfg.head_dim), 3.0))
        t3 = fo.focus_step(cfg, W, pool3, states3)
        assert not np.array_equal(t3.logits, trs[2].logits)


def test_batch_permutation_and_page_placement_invariance():
    cfg = tiny_cfg(n_layers=3, keep_ratio=0.25, constraints=3)
    W = tiny_weights(cfg, seed=10)
    lens = [12, 5, 9]
    trs, states, _ = run_steps(cfg, W, lens, 2, seed=7)
    # other physical pages (reversed order, offset): bitwise the same results
    npg = sum((L + cfg.block_size + cfg.page_size - 1) // cfg.page_size for L in lens)
    order = {p: 1000 + (npg - 1 - p) for p in range(npg)}
    trs2, states2, _ = run_steps(cfg, W, lens, 2, seed=7, page_order=order)
    for a, b in zip(trs, trs2):
        assert a.keep == b.keep and a.row_map == b.row_map and np.array_equal(a.logits, b.logits)
    assert [s.tokens for s in states] == [s.tokens for s in states2]
    # permuted batch: per-sequence results move with the sequence
    perm = [2, 0, 1]
    r = np.random.default_rng(7 + 77)
    prompts = [list(r.integers(1, cfg.vocab, L)) for L in lens]
    pool3 = fo.KVPool(cfg)
    st3, at = [], 0
    for i in perm:
        n = (lens[i] + cfg.block_size + cfg.page_size - 1) // cfg.page_size
        st3.append(fo.new_seq_state(cfg, lens[i], list(range(at, at + n))))
        at += n
    fo.prefill(cfg, W, pool3, st3, [prompts[i] for i in perm])
    t3 = fo.focus_step(cfg, W, pool3, st3)
    for newb, oldb in enumerate(perm):
        assert t3.keep[newb] == trs[0].keep[oldb]
        np.testing.assert_array_equal(t3.logits[t3.cu[newb]:t3.cu[newb + 1]],
                                      trs[0].logits[trs[0].cu[oldb]:trs[0].cu[oldb + 1]])


def test_dynamic_budget_first_step_keeps_two_and_counters_feed_next_step():
    cfg = tiny_cfg(n_layers=2, budget_mode=2, alpha=1.5)
    W = tiny_weights(cfg, seed=11)
    pool, states, _ = tiny_batch(cfg, W, [8], seed=8)
    tr = fo.focus_step(cfg, W, pool, states)
    ns = fo.n_sigma(tr.delta_I[0], [True] * cfg.block_size)
    assert tr.K[0] == max(2, ns)                                    # first step: ceil(1.5 * 1) = 2
    st = states[0]
    assert st.total_steps == 1 and st.token_sum == tr.n_decoded[0] >= 1
    tr2 = fo.focus_step(cfg, W, pool, states)
    exp = max(int(math.ceil(1.5 * st.token_sum / 1)) if False else int(math.ceil(1.5 * tr.n_decoded[0])),
              fo.n_sigma(tr2.delta_I[0], [p not in tr.committed[0] for p in range(cfg.block_size)]))
    assert tr2.K[0] == min(cfg.block_size, exp)


def test_override_budget_zero_and_full():
    cfg = tiny_cfg(n_layers=2, budget_mode=3)
    W = tiny_weights(cfg, seed=12)
    pool, states, _ = tiny_batch(cfg, W, [8, 8, 8], seed=9)
    tr = fo.focus_step(cfg, W, pool, states, k_override=[0, cfg.block_size, 3])
    assert tr.keep[0] == [] and tr.keep[1] == list(range(cfg.block_size)) and len(tr.keep[2]) == 3
    assert tr.cu == [0, 0, 8, 11]
    assert states[0].total_steps == 0 and states[0].token_sum == 0 and tr.n_decoded[0] == 0
    assert states[1].total_steps == 1 and tr.n_decoded[1] == 1


# ---------------------------------------------------------------------------------------------
# multi-block generation: finalized blocks leave the exact K/V of their tokens

@pytest.mark.parametrize("keep_ratio", [1.0, 0.25])
def test_finalized_block_kv_equals_prefill_of_the_generated_tokens(keep_ratio):
    cfg = tiny_cfg(n_layers=3, keep_ratio=keep_ratio)
    W = tiny_weights(cfg, seed=21)
    B = cfg.block_size
    lens = [8, 16]                                                # block-aligned prefixes
    r = np.random.default_rng(5)
    pool = fo.KVPool(cfg)
    states, prompts, at = [], [], 0
    for L in lens:
        npg = (L + 3 * B) // cfg.page_size                        # room for two more blocks
        states.append(fo.new_seq_state(cfg, L, list(range(at, at + npg))))
        at += npg
        prompts.append(list(r.integers(1, cfg.vocab, L)))
    fo.prefill(cfg, W, pool, states, prompts)
    generated = [[], []]
    for block in range(2):
        steps = 0
        while any(any(st.masked) for st in states):
            assert fo.finalize_blocks(cfg, W, pool, states) == [False, False]     # nothing to finalize yet
            fo.focus_step(cfg, W, pool, states)
            steps += 1
            assert steps <= B
        toks = [list(st.tokens) for st in states]
        stats = [(st.token_sum, st.total_steps) for st in states]
        assert fo.finalize_blocks(cfg, W, pool, states) == [True, True]
        for i, st in enumerate(states):
            generated[i] += toks[i]
            assert st.prefix_len == lens[i] + (block + 1) * B and all(st.masked) and not any(st.processed)
            assert (st.token_sum, st.total_steps) == stats[i] and st.token_sum == (block + 1) * B
    # the cache now equals a fresh prefill of prompt + generated tokens (and the torch dense reference)
    for i, st in enumerate(states):
        full = prompts[i] + generated[i]
        pool2 = fo.KVPool(cfg)
        st2 = fo.new_seq_state(cfg, len(full), list(range(100, 100 + len(st.pages))))
        fo.prefill(cfg, W, pool2, [st2], [full])
        _, kvs = dense_reference(cfg, W, full[:-B], full[-B:])
        for l in range(cfg.n_layers):
            K1, V1 = pool.read(l, st.pages, list(range(len(full))))
            K2, V2 = pool2.read(l, st2.pages, list(range(len(full))))
            np.testing.assert_allclose(K1, K2, rtol=1e-9, atol=1e-10)
            np.testing.assert_allclose(V1, V2, rtol=1e-9, atol=1e-10)
            np.testing.assert_allclose(K1, kvs[l][0], rtol=1e-9, atol=1e-10)
            np.testing.assert_allclose(V1, kvs[l][1], rtol=1e-9, atol=1e-10)


def test_finalize_needs_room_and_a_complete_block():
    cfg = tiny_cfg(n_layers=2, keep_ratio=1.0)
    W = tiny_weights(cfg, seed=22)
    pool, states, _ = tiny_batch(cfg, W, [8], seed=3)            # pages for exactly one block
    for _ in range(cfg.block_size):
        fo.focus_step(cfg, W, pool, states)
    assert not any(states[0].masked)
    assert fo.finalize_blocks(cfg, W, pool, states) == [False] and states[0].prefix_len == 8


# ---------------------------------------------------------------------------------------------
# intra-block K/V cache with the neighbour-aware stability criterion (Sec. 4.3, App. E.3.1)

def snapshot_block_kv(cfg, pool, st):
    toks = [st.prefix_len + p for p in range(cfg.block_size)]
    return [tuple(a.copy() for a in pool.read(l, st.pages, toks)) for l in range(cfg.n_layers)]


def reference_step_rows(cfg, W, prefix_kv, block_kv_before, st_before, U, S, processed_after):
    """Independent (torch) statement of one step for one sequence, given as INPUTS the prefix K/V and the block's K/V
    before the step: rows U go through layers <= e, rows S through the rest; a row's keys are the prefix, the fresh
    K/V of the rows of its layer, and the given (old) K/V of every other visible block position.  Returns the logits
    of the rows S."""
    B, e, D, Hq, Hkv = cfg.block_size, cfg.evict_layer, cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    L = st_before["prefix_len"]
    ids = [cfg.mask_token_id if st_before["masked"][p] else st_before["tokens"][p] for p in U]
    X = torch.from_numpy(W.embed)[torch.tensor(ids)]
    inv = cfg.rope_base ** (-torch.arange(0, D, 2, dtype=torch.float64) / D)

    def rot(x, pos):
        ang = torch.tensor(pos, dtype=torch.float64)[:, None] * inv[None]
        c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
        a, b = x[..., :D // 2], x[..., D // 2:]
        return torch.cat([a * c - b * s, b * c + a * s], -1)
    rows = list(U)
    for l in range(cfg.n_layers):
        w = {k: torch.from_numpy(np.asarray(v)) for k, v in W.layer(l).items()}
        if l > e and rows is not S:
            X = X[[rows.index(p) for p in S]]
            rows = list(S)
        u = F.rms_norm(X, (cfg.hidden,), w["attn_norm"], eps=cfg.rms_eps)
        q, k, v = F.linear(u, w["w_qkv"]).split([Hq * D, Hkv * D, Hkv * D], dim=-1)
        pos = [L + p for p in rows]
        q, k, v = rot(q.view(-1, Hq, D), pos), rot(k.view(-1, Hkv, D), pos), v.view(-1, Hkv, D)
        if l == e:                                    # layer e: projections for U, attention only for S
            keep_idx = [rows.index(p) for p in S]
        visible = list(range(B)) if l <= e else [p for p in range(B) if processed_after[p]]
        Kb = torch.from_numpy(block_kv_before[l][0]).clone()
        Vb = torch.from_numpy(block_kv_before[l][1]).clone()
        for i, p in enumerate(rows):
            Kb[p], Vb[p] = k[i], v[i]
        Kall = torch.cat([torch.from_numpy(prefix_kv[l][0]), Kb[visible]])
        Vall = torch.cat([torch.from_numpy(prefix_kv[l][1]), Vb[visible]])
        if l == e:
            X, q, rows = X[keep_idx], q[keep_idx], list(S)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], Kall.transpose(0, 1)[None], Vall.transpose(0, 1)[None],
                                           enable_gqa=True)[0].transpose(0, 1).reshape(len(rows), Hq * D)
        X = X + F.linear(o, w["w_o"])
        u = F.rms_norm(X, (cfg.hidden,), w["mlp_norm"], eps=cfg.rms_eps)
        g, up = F.linear(u, w["w_gate_up"]).split([cfg.ffn, cfg.ffn], dim=-1)
        X = X + F.linear(F.silu(g) * up, w["w_down"])
    return F.linear(F.rms_norm(X, (cfg.hidden,), torch.from_numpy(W.final_norm), eps=cfg.rms_eps), torch.from_numpy(W.lm_head)).numpy()


def test_intra_block_cache_rows_freezing_and_reference():
    cfg = tiny_cfg(n_layers=3, keep_ratio=0.25, conf_threshold=0.05, intra_block_cache=1)    # low threshold: several commits per step
    W = tiny_weights(cfg, seed=31, scale=0.6)
    B = cfg.block_size
    pool, states, _ = tiny_batch(cfg, W, [12], seed=11)
    st = states[0]
    frozen = {}
    saw_cached_step = False
    for step in range(2 * B):
        if not any(st.masked):
            break
        before = dict(prefix_len=st.prefix_len, masked=list(st.masked), tokens=list(st.tokens), cached=list(st.cached))
        prefix_kv = [pool.read(l, st.pages, list(range(st.prefix_len))) for l in range(cfg.n_layers)]
        block_kv = snapshot_block_kv(cfg, pool, st)
        tr = fo.focus_step(cfg, W, pool, states)
        U, S = tr.uncached[0], tr.keep[0]
        # rows: exactly the positions that were not frozen; decoded-but-not-frozen positions are always retained
        assert U == [p for p in range(B) if not before["cached"][p]]
        assert set(S) <= set(U) and {p for p in U if not before["masked"][p]} <= set(S)
        assert abs(tr.I_evict[0].sum() - len(U) * cfg.n_q_heads) < 1e-9
        # neighbour-aware rule, written out
        unm = [not m for m in before["masked"]]
        expect = [before["cached"][p] or (p in S and unm[p] and (p == B - 1 or unm[p + 1])) for p in range(B)]
        assert st.cached == expect
        # frozen K/V never changes again
        after = snapshot_block_kv(cfg, pool, st)
        for p, kv in frozen.items():
            for l in range(cfg.n_layers):
                assert np.array_equal(after[l][0][p], kv[l][0]) and np.array_equal(after[l][1][p], kv[l][1])
        for p in range(B):
            if st.cached[p] and p not in frozen:
                frozen[p] = [(after[l][0][p].copy(), after[l][1][p].copy()) for l in range(cfg.n_layers)]
        # the step's logits against the independent statement (the K/V before the step are inputs)
        if S:
            ref = reference_step_rows(cfg, W, prefix_kv, block_kv, before, U, S, st.processed)
            np.testing.assert_allclose(tr.logits, ref, rtol=1e-9, atol=1e-10)
        saw_cached_step = saw_cached_step or len(U) < B
    assert saw_cached_step and frozen, "the scenario must reach steps with frozen positions"
    assert not any(st.masked)
    # finalisation forwards only what is not frozen, then clears the state
    block_kv = snapshot_block_kv(cfg, pool, st)
    was_cached = list(st.cached)
    st.pages = st.pages + [900, 901]                              # room for another block
    L0 = st.prefix_len
    assert fo.finalize_blocks(cfg, W, pool, states) == [True]
    toks = [L0 + p for p in range(B)]
    for l in range(cfg.n_layers):
        Kc, Vc = pool.read(l, st.pages, toks)
        for p in range(B):
            if was_cached[p]:
                assert np.array_equal(Kc[p], block_kv[l][0][p]) and np.array_equal(Vc[p], block_kv[l][1][p])
    assert st.cached == [False] * B and st.prefix_len == L0 + B


def test_intra_block_cache_off_or_idle_changes_nothing():
    # with nothing decoded before a step the cache cannot freeze anything: first steps equal the plain method
    for ratio in (0.25, 1.0):
        outs = []
        for flag in (0, 1):
            cfg = tiny_cfg(n_layers=3, keep_ratio=ratio, intra_block_cache=flag)
            W = tiny_weights(cfg, seed=32)
            pool, states, _ = tiny_batch(cfg, W, [8, 12], seed=12)
            outs.append(fo.focus_step(cfg, W, pool, states))
        assert outs[0].keep == outs[1].keep and np.array_equal(outs[0].logits, outs[1].logits)


# ---------------------------------------------------------------------------------------------
# mixture-of-experts feed-forward (second model of Sec. 5.1; the layer is the common token-choice one)

def torch_swiglu(u, w_gate_up, w_down):
    F_ = w_gate_up.shape[0] // 2
    u, wg, wu, wd = (torch.from_numpy(np.asarray(a)) for a in (u, w_gate_up[:F_], w_gate_up[F_:], w_down))
    return ((F.silu(u @ wg.T) * (u @ wu.T)) @ wd.T).numpy()


def moe_weights(cfg, r, same_experts=False):
    E, Fe, h = cfg.n_experts, cfg.expert_ffn, cfg.hidden
    w = dict(w_router=r.normal(0, 1.0, (E, h)), w_expert_gate_up=r.normal(0, 0.3, (E, 2 * Fe, h)),
             w_expert_down=r.normal(0, 0.3, (E, h, Fe)))
    if same_experts:
        w["w_expert_gate_up"][:] = w["w_expert_gate_up"][0]
        w["w_expert_down"][:] = w["w_expert_down"][0]
    if cfg.shared_ffn:
        w["w_shared_gate_up"] = r.normal(0, 0.3, (2 * cfg.shared_ffn, h))
        w["w_shared_down"] = r.normal(0, 0.3, (h, cfg.shared_ffn))
    return w


def test_swiglu_matches_torch():
    r = np.random.default_rng(3)
    u, wgu, wd = r.normal(size=(5, 16)), r.normal(size=(24, 16)), r.normal(size=(16, 12))
    np.testing.assert_allclose(fo.swiglu(u, wgu, wd), torch_swiglu(u, wgu, wd), rtol=1e-12, atol=1e-12)


def test_route_hand_cases():
    cfg = tiny_cfg(n_experts=4, experts_per_token=2, expert_ffn=8, route_scale=1.0)
    ch, wt = fo.route(cfg, np.log(np.array([0.5, 0.25, 0.125, 0.125])))
    assert ch == [0, 1] and np.allclose(wt, [2 / 3, 1 / 3])
    ch, wt = fo.route(cfg, np.array([0.0, 1.0, 1.0, 1.0]))                   # ties: lower expert first
    assert ch == [1, 2] and np.allclose(wt, [0.5, 0.5])
    cfg.route_scale = 2.5
    ch, wt = fo.route(cfg, np.log(np.array([0.5, 0.25, 0.125, 0.125])), forced=[3, 0])
    assert ch == [3, 0] and np.allclose(wt, [2.5 * 0.2, 2.5 * 0.8])           # forced list, in its own order
    cfg.experts_per_token = 4
    ch, wt = fo.route(cfg, np.array([0.3, -2.0, 5.0, 0.1]))
    assert ch == [2, 0, 3, 1] and abs(sum(wt) - 2.5) < 1e-12                  # k = E: the plain softmax, scaled


@pytest.mark.parametrize("E,k,Fs", [(1, 1, 0), (6, 2, 0), (8, 3, 12), (4, 4, 8)])
def test_moe_ffn_against_masked_dense_formulation_in_torch(E, k, Fs):
    """Independent statement: gates = top-k of the softmax (torch.topk), renormalised; every expert runs on every row and
    the outputs are mixed with the gate matrix."""
    r = np.random.default_rng(10 * E + k)
    cfg = tiny_cfg(n_experts=E, experts_per_token=k, expert_ffn=12, shared_ffn=Fs, route_scale=1.7)
    w = moe_weights(cfg, r)
    u = r.normal(size=(9, cfg.hidden))
    y, experts, weights, _ = fo.moe_ffn(cfg, w, u)
    tu = torch.from_numpy(u)
    probs = torch.softmax(tu @ torch.from_numpy(w["w_router"]).T, dim=-1)
    val, idx = torch.topk(probs, k, dim=-1)
    gates = torch.zeros_like(probs).scatter(1, idx, val / val.sum(-1, keepdim=True)) * float(np.float32(1.7))
    want = sum(gates[:, e:e + 1].numpy() * torch_swiglu(u, w["w_expert_gate_up"][e], w["w_expert_down"][e]) for e in range(E))
    if Fs:
        want = want + torch_swiglu(u, w["w_shared_gate_up"], w["w_shared_down"])
    np.testing.assert_allclose(y, want, rtol=1e-10, atol=1e-10)
    assert all(sorted(experts[i]) == sorted(idx[i].tolist()) for i in range(9))
    assert all(abs(sum(wt) - float(np.float32(1.7))) < 1e-12 and all(a >= b for a, b in zip(wt, wt[1:])) for wt in weights)
    if E == 1:   # one expert: the dense feed-forward with that expert's weights
        np.testing.assert_allclose(y, float(np.float32(1.7)) * torch_swiglu(u, w["w_expert_gate_up"][0], w["w_expert_down"][0]), rtol=1e-10)


def test_moe_forced_routing_uses_the_given_experts():
    r = np.random.default_rng(77)
    cfg = tiny_cfg(n_experts=5, experts_per_token=2, expert_ffn=12)
    w = moe_weights(cfg, r)
    u = r.normal(size=(4, cfg.hidden))
    forced = [[4, 0], [1, 2], [3, 4], [0, 1]]
    y, experts, weights, _ = fo.moe_ffn(cfg, w, u, forced)
    assert experts == forced
    p = torch.softmax(torch.from_numpy(u @ w["w_router"].T), dim=-1).numpy()
    for i in range(4):
        a, b = forced[i]
        g = p[i, [a, b]] / p[i, [a, b]].sum()
        want = g[0] * torch_swiglu(u[i:i + 1], w["w_expert_gate_up"][a], w["w_expert_down"][a]) + \
            g[1] * torch_swiglu(u[i:i + 1], w["w_expert_gate_up"][b], w["w_expert_down"][b])
        np.testing.assert_allclose(y[i], want[0], rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("first", [0, 1])
def test_step_with_identical_experts_equals_the_dense_model(first):
    """Experts that share one set of weights make the routing irrelevant (the weights sum to one): the whole step,
    decisions included, must equal the step of the dense model with that feed-forward."""
    dense = tiny_cfg(ffn=24, keep_ratio=0.5)
    moe = tiny_cfg(ffn=24, keep_ratio=0.5, n_experts=4, experts_per_token=2, expert_ffn=24, first_moe_layer=first)
    Wd = tiny_weights(dense, seed=5)
    layers = []
    for l in range(dense.n_layers):
        w = dict(Wd.layer(l))
        w["w_router"] = np.random.default_rng(l).normal(size=(4, dense.hidden))
        w["w_expert_gate_up"] = np.stack([w["w_gate_up"]] * 4)
        w["w_expert_down"] = np.stack([w["w_down"]] * 4)
        layers.append(w)
    Wm = fo.Weights(Wd.embed, Wd.lm_head, Wd.final_norm, lambda l: layers[l])
    pd, sd, _ = tiny_batch(dense, Wd, [5, 11])
    pm, sm, _ = tiny_batch(moe, Wm, [5, 11])
    for step in range(3):
        td, tm = fo.focus_step(dense, Wd, pd, sd), fo.focus_step(moe, Wm, pm, sm)
        assert td.keep == tm.keep and td.committed == tm.committed
        np.testing.assert_allclose(tm.logits, td.logits, rtol=1e-9, atol=1e-9)
        assert sorted(tm.route) == list(range(first, 3)) and all(len(v[0]) == 2 for v in tm.route[2].values())
        assert first or len(tm.route[0]) == 2 * moe.block_size           # layers below e run on the whole block
        assert set(tm.route[2]) == set(tm.row_map) == set(tm.route[1])      # the feed-forward of layer e runs after the gather


# ---------------------------------------------------------------------------------------------
# freeze criterion of the delayed intra-block cache: a hand-worked trace (tests/golden/r17_freeze_trace.txt)

def test_intra_block_cache_freeze_trace_worked_by_hand():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "r17_freeze_trace.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    B = 6
    as_set = lambda s: set() if s == "-" else {int(c) for c in s}
    cfg = tiny_cfg(n_layers=3, block_size=B, intra_block_cache=1, conf_threshold=2.0)     # threshold above 1: only forced commits
    W = tiny_weights(cfg, seed=5)
    pool, states, _ = tiny_batch(cfg, W, [9], seed=3)
    st = states[0]
    for masked, S, before, after in rows:
        M, S, C0, C1 = as_set(masked), sorted(as_set(S)), as_set(before), as_set(after)
        assert st.cached == [p in C0 for p in range(B)]           # the trace's steps chain: what a step froze is the next one's input
        st.masked = [p in M for p in range(B)]
        st.tokens = [cfg.mask_token_id if p in M else 1 + p for p in range(B)]
        tr = fo.focus_step(cfg, W, pool, states, keep_override=[S])
        assert tr.uncached[0] == [p for p in range(B) if p not in C0]
        assert st.cached == [p in C1 for p in range(B)], (masked, S, st.cached)


# ---------------------------------------------------------------------------------------------
# storage-format model (OracleConfig.store_cast): off = the oracle; identity = the oracle (pins the un-normalised softmax
# form it uses); bf16 = a small, non-zero distance

def test_store_cast_identity_is_the_oracle_and_bf16_is_close():
    from oracle.harness import bf16_store_cast, round_bf16
    outs = {}
    for name, cast in (("off", None), ("identity", lambda n, x: x), ("bf16", bf16_store_cast())):
        cfg = tiny_cfg(n_layers=3, keep_ratio=0.5)
        cfg.store_cast = cast
        W = tiny_weights(cfg, seed=41)
        pool, states, _ = tiny_batch(fo.OracleConfig(**{**cfg.__dict__, "store_cast": None}), W, [7, 12], seed=9)
        outs[name] = fo.focus_step(cfg, W, pool, states, keep_override=[[0, 2, 5, 6], [1, 2, 3, 7]])
    np.testing.assert_allclose(outs["identity"].logits, outs["off"].logits, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(outs["identity"].delta_I[0], outs["off"].delta_I[0], rtol=1e-12, atol=1e-12)
    err = np.max(np.abs(outs["bf16"].logits - outs["off"].logits)) / np.max(np.abs(outs["off"].logits))
    assert 1e-4 < err < 2e-2, err
    # the rounding itself: nearest-even to 8 significant bits
    assert round_bf16(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -3.14159, 1e-40])).tolist()[:2] == [1.0, 1.0 + 2.0 ** -6]
