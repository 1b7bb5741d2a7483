"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Integer results (budget, retained sets, packing offsets, row map, committed ids, mask bits, counters) must be
bit-exact given identical scores; floating point within max|gpu - oracle| / max|oracle| <= 1e-3 (fp32 model)
or 2e-2 (bf16 model).  Where a bf16 score decides an integer, the GPU's decision is accepted only if it is a
valid decision for the oracle's scores within that tolerance, and the oracle then continues from the GPU's
decision (teacher forcing) so that later stages stay comparable.
"""
import math

import numpy as np
import pytest
import torch

import focus_inputs as fi
from oracle import focus_oracle as fo
from oracle.harness import oracle_batch, oracle_config

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _pk():
    import paper_2601_23278_amd as pk
    from paper_2601_23278_amd import runner
    return pk, runner


def bits_of(positions):
    v = 0
    for p in positions:
        v |= 1 << p
    return v


def positions_of(bits, B):
    return [p for p in range(B) if (bits >> p) & 1]


def relerr(gpu, ora):
    ora = np.asarray(ora, dtype=np.float64)
    gpu = np.asarray(gpu, dtype=np.float64)
    if ora.size == 0:
        return 0.0
    return float(np.max(np.abs(gpu - ora)) / max(np.max(np.abs(ora)), 1e-30))


def row_relerr(gpu, ora):
    return max([relerr(g, o) for g, o in zip(gpu, ora)] + [0.0])


class Outs:
    def __init__(self, pk, wl, n):
        B, h, V = wl.block_size, wl.hidden, wl.vocab
        d = DEV
        z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=d)
        self.t = dict(tokens=z(n, B, dt=torch.int32), mask_bits=z(n, dt=torch.int64), n_decoded=z(n, dt=torch.int32),
                      importance_prev=z(n, B), importance=z(n, B), delta_I=z(n, B), K=z(n, dt=torch.int32),
                      keep_bits=z(n, dt=torch.int64), cu_seqlens=z(n + 1, dt=torch.int32), row_map=z(n * B, dt=torch.int32),
                      conf=z(n * B), argmax=z(n * B, dt=torch.int32), hidden_full=z(n * B, h), hidden_packed=z(n * B, h),
                      logits=z(n * B, V))
        if wl.n_experts:
            k = wl.experts_per_token
            self.t["route_experts"] = torch.full((wl.n_layers, n * B, k), -1, dtype=torch.int32, device=d)
            self.t["route_weights"] = z(wl.n_layers, n * B, k)
        self.struct = pk.make_step_out(**self.t)

    def host(self):
        torch.cuda.synchronize()
        return {k: v.cpu().numpy() for k, v in self.t.items()}


def u64(x):
    return int(x) & ((1 << 64) - 1)


def check_selection_valid(dI_ora, masked, keep_gpu, K, B, tol):
    """The GPU's top-K is a valid top-K of the oracle's scores up to `tol`."""
    cand = [j for j in range(B) if masked[j]]
    k = min(K, len(cand))
    if k == 0 or K >= B:
        return
    srt = sorted((dI_ora[j] for j in cand), reverse=True)
    kth = srt[k - 1]
    for j in cand:
        if j in keep_gpu:
            assert dI_ora[j] >= kth - tol, (j, dI_ora[j], kth)
        else:
            assert dI_ora[j] <= kth + tol, (j, dI_ora[j], kth)


def check_routes(wl, g, tr, tol, exact):
    """Experts and mixing weights of every row that ran in a mixture-of-experts layer."""
    for l, rows in tr.route.items():
        for rid, (experts, weights, logits) in rows.items():
            got_e = [int(x) for x in g["route_experts"][l, rid]]
            got_w = g["route_weights"][l, rid].astype(np.float64)
            if exact:
                assert got_e == experts, (l, rid, got_e, experts)
            else:
                assert got_e == experts, (l, rid)          # forced routing: the given list in its order
            assert np.max(np.abs(got_w - np.asarray(weights))) <= tol * max(1.0, wl.route_scale), (l, rid, got_w, weights)
    ran = {l: set(rows) for l, rows in tr.route.items()}
    for l in range(wl.n_layers):                           # rows that did not run in a layer are left untouched
        idle = [r for r in range(g["route_experts"].shape[1]) if r not in ran.get(l, ())]
        assert np.all(g["route_experts"][l, idle] == -1), l


def compare_steps(wl, steps, tol, exact, seq_ids=None, k_override=None, forced_routes=False, row_hint=None):
    pk, runner = _pk()
    cfg, W, pool, states, lens, tables, n_pages = oracle_batch(wl, seq_ids)
    sess = runner.open_session(wl, DEV, seq_ids)
    if row_hint is not None:
        sess.focus.focus_set_row_hint(*row_hint)
    n, B = len(states), wl.block_size
    outs = Outs(pk, wl, n)
    routes = None
    if forced_routes:
        routes = wl.route_override(n)
        sess.focus.focus_set_route_override(torch.tensor(routes, dtype=torch.int32, device=DEV))
    ko_dev = None if k_override is None else torch.tensor(k_override, dtype=torch.int32, device=DEV)
    stats = []
    for step in range(steps):
        print("step", step, flush=True)
        masked_before = [list(st.masked) for st in states]
        pre = [(list(st.masked), list(st.processed), list(st.cached) if st.cached else [False] * B, st.token_sum, st.total_steps, st.slot)
               for st in states]
        if wl.n_experts:
            outs.t["route_experts"].fill_(-1)
        sess.focus.focus_step(n, k_override=ko_dev, out=outs.struct)
        g = outs.host()
        keep_gpu = [positions_of(u64(g["keep_bits"][b]), B) for b in range(n)]
        if exact:
            tr = fo.focus_step(cfg, W, pool, states, k_override=k_override,
                               score_cast=lambda d: d.astype(np.float32).astype(np.float64),
                               conf_cast=lambda c: c.astype(np.float32).astype(np.float64), route_override=routes)
        else:
            tr = fo.focus_step(cfg, W, pool, states, keep_override=keep_gpu, route_override=routes)
        if wl.n_experts:
            check_routes(wl, g, tr, tol, exact)
        # scores
        e_dI = max(relerr(g["delta_I"][b], tr.delta_I[b]) for b in range(n))
        e_I = max(relerr(g["importance"][b], tr.I_evict[b]) for b in range(n))
        # the delta is a difference of two importances that are each within the tolerance of their own scale: its error is
        # bounded on that scale (relative to the delta's own size it can be anything when the two layers nearly agree)
        a_dI = max(float(np.max(np.abs(g["delta_I"][b] - tr.delta_I[b]))) / max(float(np.max(np.abs(tr.I_evict[b]))), 1e-30) for b in range(n))
        assert e_I <= tol and a_dI <= 2 * tol, (e_I, a_dI, e_dI)
        if tr.I_prev:           # Eq. 2 of the layer below the eviction layer (computed inside that layer's attention launch where possible)
            e_Ip = max(relerr(g["importance_prev"][b], tr.I_prev[b]) for b in range(n))
            assert e_Ip <= tol, e_Ip
        for b in range(n):      # Eq. 2 sums to (query rows) x H_q: all B positions, or those not frozen (Sec. 4.3)
            assert abs(float(g["importance"][b].sum()) - len(tr.uncached[b]) * wl.n_q_heads) < 1e-2 * B * wl.n_q_heads * tol + 1e-3
        # decisions
        if exact:
            assert [int(k) for k in g["K"]] == tr.K
            assert keep_gpu == tr.keep
        else:
            for b in range(n):
                # the integer logic on the GPU's own scores: budget and retained set must be exactly what the oracle's rules
                # give for those fp32 values (whatever the switches); the scores themselves were compared above
                Kb = int(g["K"][b])
                d = g["delta_I"][b].astype(np.float64)
                m, pr, ca, ts, tsteps, slot = pre[b]
                assert Kb == fo.budget(cfg, d, m, ts, tsteps, None if k_override is None else k_override[b]), b
                rk = [fo.selection_key(cfg.selection_seed, slot, tsteps, j) for j in range(B)] if cfg.selection == 1 else None
                assert keep_gpu[b] == fo.select(cfg, d, m, pr, Kb, ca, rk), b
                if cfg.constraints == 0 and not cfg.intra_block_cache and cfg.selection == 0:
                    scale = float(np.max(np.abs(tr.delta_I[b])))
                    check_selection_valid(tr.delta_I[b], masked_before[b], set(keep_gpu[b]), Kb, B, 5 * tol * scale)
        assert [int(x) for x in g["cu_seqlens"]] == tr.cu
        T = tr.cu[-1]
        assert [int(x) for x in g["row_map"][:T]] == tr.row_map
        # floats
        e_hf = relerr(g["hidden_full"][:len(tr.hidden_full)], tr.hidden_full)
        e_hp = relerr(g["hidden_packed"][:T], tr.hidden_packed)
        e_lg = row_relerr(g["logits"][:T], tr.logits)
        e_cf = relerr(g["conf"][:T], np.asarray(tr.conf)) if T else 0.0
        stats.append(dict(step=step, T=T, dI=e_dI, hidden_full=e_hf, hidden_packed=e_hp, logits=e_lg, conf=e_cf))
        print(stats[-1], flush=True)
        assert e_hf <= tol and e_hp <= tol and e_lg <= tol, stats[-1]
        # commit
        gm = [u64(x) for x in g["mask_bits"]]
        if exact:
            assert np.array_equal(g["argmax"][:T], tr.argmax)
            assert e_cf <= tol
            for b, st in enumerate(states):
                assert gm[b] == bits_of([p for p in range(B) if st.masked[p]])
                assert [int(t) for t in g["tokens"][b]] == st.tokens
                assert int(g["n_decoded"][b]) == tr.n_decoded[b]
        else:
            # accept the GPU's commit if it is valid for the oracle's logits within tolerance, then adopt it
            for b, st in enumerate(states):
                sl = slice(tr.cu[b], tr.cu[b + 1])
                newly = [p for p in range(B) if masked_before[b][p] and not (gm[b] >> p) & 1]
                assert len(newly) == int(g["n_decoded"][b])
                cand = [(i, p) for i, p in enumerate(tr.keep[b]) if masked_before[b][p]]
                if cand:
                    assert len(newly) >= 1
                    best = max(float(tr.conf[sl][i]) for i, _ in cand)
                    thr = float(np.float32(wl.conf_threshold))
                    for p in newly:
                        i = tr.keep[b].index(p)
                        c = float(tr.conf[sl][i])
                        assert c >= thr * (1 - 5 * tol) or c >= best * (1 - 5 * tol), (b, p, c, best)
                        lg = tr.logits[sl][i]
                        tok = int(g["tokens"][b][p])
                        assert lg[tok] >= lg.max() - 5 * tol * np.max(np.abs(lg)), (b, p)
                        st.tokens[p] = tok
                    # undo the oracle's own commit where it differs, adopt the GPU's
                    for p in range(B):
                        st.masked[p] = bool((gm[b] >> p) & 1)
                        if st.masked[p]:
                            st.tokens[p] = cfg.mask_token_id
                    st.token_sum += len(newly) - tr.n_decoded[b]
        for b in range(n):
            s = sess.focus.focus_get_state(b)
            assert (s.token_sum, s.total_steps, s.prefix_len) == (states[b].token_sum, states[b].total_steps, lens[sess.seq_ids[b]])
            assert s.processed_bits == bits_of([p for p in range(B) if states[b].processed[p]])
            assert s.cached_bits == bits_of([p for p in range(B) if states[b].cached[p]])
        stats[-1]["frozen"] = sum(sum(st.cached) for st in states)
        stats[-1]["rows_full"] = len(tr.hidden_full)
    sess.focus.focus_free()
    return stats


# ---------------------------------------------------------------------------------------------

def test_c1_tiny_fp32_four_steps_exact():
    """BASELINE configs[0]: real prefill, four denoising steps, fp32 on both sides, zero divergences."""
    wl = fi.workload("c1_tiny")
    pk, runner = _pk()
    # prefix K/V written by the GPU prefill equals the oracle's
    cfg, W, pool, states, lens, tables, n_pages = oracle_batch(wl)
    sess = runner.open_session(wl, DEV)
    kv = sess.kv_pool.cpu().numpy()
    for l in range(wl.n_layers):
        for b, st in enumerate(states):
            for t in range(st.prefix_len):
                pg = pool.layers[l][st.pages[t // wl.page_size]]
                page = kv[l, st.pages[t // wl.page_size]]
                got_k = page[0][:, t % wl.page_size, :]
                got_v = page[1].reshape(wl.n_kv_heads, wl.head_dim, wl.page_size)[:, :, t % wl.page_size]
                assert relerr(got_k, pg[0, :, t % wl.page_size, :]) <= 1e-3, (l, b, t)
                assert relerr(got_v, pg[1, :, t % wl.page_size, :]) <= 1e-3, (l, b, t)
    sess.focus.focus_free()
    stats = compare_steps(wl, wl.steps, 1e-3, exact=True)
    assert len(stats) == 4 and all(s["T"] == 16 for s in stats)


@pytest.mark.parametrize("variant", ["dynamic", "constraints", "evict2", "override", "dense", "rawI"])
def test_c1_variants_fp32_exact(variant):
    over = dict(dynamic=dict(budget_mode=2, alpha=1.5, steps=3),
                constraints=dict(constraints=3, steps=3),
                evict2=dict(n_layers=4, evict_layer=2, steps=2),
                override=dict(budget_mode=3, steps=2),
                dense=dict(keep_ratio=1.0, steps=2),
                rawI=dict(importance_mode=1, maxpool_k=1, steps=2))[variant]
    wl = fi.workload("c1_tiny", **over)
    ko = wl.k_overrides() if variant == "override" else None
    compare_steps(wl, wl.steps, 1e-3, exact=True, k_override=ko)


@pytest.mark.parametrize("selection,topk", [(1, 2), (1, 4), (2, 2), (2, 8)])
def test_c1_random_and_bottom_selection_fp32_exact(selection, topk):
    """Controls of the selection validation (Sec. 5.2): fixed K, the pick replaced by Random / Bottom."""
    wl = fi.workload("c1_tiny", budget_mode=0, topk=topk, selection=selection, selection_seed=20260123, steps=4,
                     constraints=1 if topk == 4 else 0)
    compare_steps(wl, wl.steps, 1e-3, exact=True)


def test_c1_intra_block_cache_fp32_exact():
    """Delayed intra-block K/V cache with the neighbour-aware stability criterion (Sec. 4.3): a low threshold makes
    several tokens commit per step, so positions freeze, leave the rows of the early layers and keep their K/V."""
    wl = fi.workload("c1_tiny", intra_block_cache=1, conf_threshold=0.0013, keep_ratio=0.5, steps=7)
    stats = compare_steps(wl, wl.steps, 1e-3, exact=True)
    assert stats[-1]["frozen"] > 0 and min(s["rows_full"] for s in stats) < wl.batch * wl.block_size, stats


def test_c1_intra_block_cache_with_constraints_and_dynamic_budget():
    wl = fi.workload("c1_tiny", intra_block_cache=1, conf_threshold=0.0013, budget_mode=2, constraints=3, steps=6)
    stats = compare_steps(wl, wl.steps, 1e-3, exact=True)
    assert stats[-1]["frozen"] > 0, stats


MOE_TINY = dict(n_experts=8, experts_per_token=2, expert_ffn=64, shared_ffn=32, route_scale=2.5)


@pytest.mark.parametrize("first,forced", [(0, False), (1, False), (0, True)])
def test_c1_moe_fp32_exact(first, forced):
    """Mixture-of-experts feed-forward (second model of Sec. 5.1) on the tiny fp32 configuration: the router's own picks
    must equal the oracle's, layer by layer and row by row; with forced routing the given experts are used."""
    wl = fi.workload("c1_tiny", n_layers=3, first_moe_layer=first, steps=3, **MOE_TINY)
    compare_steps(wl, wl.steps, 1e-3, exact=True, forced_routes=forced)


def test_c1_moe_single_choice_without_shared_expert_and_intra_block_cache():
    wl = fi.workload("c1_tiny", n_layers=3, n_experts=5, experts_per_token=1, expert_ffn=40, first_moe_layer=1,
                     intra_block_cache=1, conf_threshold=0.0013, keep_ratio=0.5, steps=5)
    compare_steps(wl, wl.steps, 1e-3, exact=True)


def test_c1_everything_at_once_fp32_exact():
    """Mixture of experts from layer 0, delayed intra-block cache, dynamic budget, both structural constraints, eviction
    after layer 2: every switch of the step in one run."""
    wl = fi.workload("c1_tiny", n_layers=4, evict_layer=2, first_moe_layer=0, intra_block_cache=1, conf_threshold=0.0013,
                     budget_mode=2, alpha=1.5, constraints=3, steps=6, **MOE_TINY)
    stats = compare_steps(wl, wl.steps, 1e-3, exact=True)
    assert stats[-1]["frozen"] > 0, stats


def test_no_prefix_and_single_sequence():
    """A block with nothing before it (the attention sees the block alone) and a batch of one.  Without a prefix all rows are
    the mask token and differ by their position only, so confidences come out nearly equal: decisions are checked for validity
    within the tolerance there, not for identity."""
    compare_steps(fi.workload("c1_tiny", prefix_lo=0, prefix_hi=0, prefix_dist="fixed", steps=3), 3, 1e-3, exact=False)
    compare_steps(fi.workload("c1_tiny", batch=1, steps=2), 2, 1e-3, exact=True)
    compare_steps(small_bf16(prefix_lo=0, prefix_hi=0, prefix_dist="fixed", batch=2, steps=2), 2, 2e-2, exact=False)
    compare_steps(small_bf16(batch=1, steps=2), 2, 2e-2, exact=False)


def small_bf16(**over):
    base = dict(n_layers=3, hidden=512, n_q_heads=8, n_kv_heads=2, ffn=1024, vocab=4096, mask_token_id=4095,
                batch=5, prefix_lo=70, prefix_hi=200, prefix_dist="uniform", block_size=32, budget_mode=1,
                keep_ratio=0.25, steps=3, shuffle_pages=True)
    base.update(over)
    return fi.workload("c3_llada36", **base)


def test_small_bf16_teacher_forced():
    compare_steps(small_bf16(), 3, 2e-2, exact=False)


@pytest.mark.parametrize("hint", [(8, 2), (48, 8), (100000, 64)])
def test_small_bf16_dynamic_budget_and_constraints_with_row_hints(hint):
    """The method's own operating mode (Eq. 4-5 budget with alpha 1.5, both constraints of Sec. 4.2): the packed row count is
    known on the device only.  A launch-shape hint that is too small (sequences then take several attention passes and the
    projections more workgroups than planned), about right, or far too large must not change what is computed."""
    compare_steps(small_bf16(budget_mode=2, constraints=3, batch=7), 3, 2e-2, exact=False, row_hint=hint)


def test_small_bf16_block64_dense_with_a_one_row_hint():
    """Nothing is evicted (ratio 1.0, 64 rows per sequence and 4 query heads per kv head: 256 (row, head) pairs) while the hint
    promises one row per sequence: the packed layers' attention runs with one wavefront and eight passes per sequence."""
    compare_steps(small_bf16(block_size=64, keep_ratio=1.0, batch=3, prefix_lo=100, prefix_hi=300), 2, 2e-2, exact=False, row_hint=(3, 1))


def test_small_bf16_intra_block_cache_teacher_forced():
    stats = compare_steps(small_bf16(intra_block_cache=1, conf_threshold=0.0004, keep_ratio=0.5, steps=6), 6, 2e-2, exact=False)
    assert stats[-1]["frozen"] > 0, stats


MOE_SMALL = dict(n_experts=16, experts_per_token=4, expert_ffn=128, shared_ffn=128, route_scale=1.5)


@pytest.mark.parametrize("first", [0, 1])
def test_small_bf16_moe_forced_routes_teacher_forced(first):
    """bf16 model on the matrix-core grouped projections; both sides use the same seeded routing (a bf16 router logit can
    flip a near-tie against the float64 oracle, so the pick itself is checked separately below)."""
    compare_steps(small_bf16(first_moe_layer=first, **MOE_SMALL), 3, 2e-2, exact=False, forced_routes=True)


def test_small_bf16_moe_several_row_tiles_per_expert():
    """Few experts and many rows: an expert's rows span two tiles of the grouped projections, the second one ragged."""
    wl = small_bf16(batch=12, n_experts=4, experts_per_token=2, expert_ffn=192, shared_ffn=0, first_moe_layer=0, steps=2)
    compare_steps(wl, 2, 2e-2, exact=False, forced_routes=True)


def test_small_bf16_moe_router_picks_are_valid_for_the_oracle_logits():
    """Free routing in bf16: the oracle is run with the GPU's picks; every pick must be among the oracle's k best experts
    up to the tolerance on the logits, in descending order up to that tolerance, and the weights must agree."""
    pk, runner = _pk()
    wl = small_bf16(first_moe_layer=0, steps=1, **MOE_SMALL)
    cfg, W, pool, states, lens, tables, n_pages = oracle_batch(wl)
    sess = runner.open_session(wl, DEV)
    n, B, k = len(states), wl.block_size, wl.experts_per_token
    outs = Outs(pk, wl, n)
    sess.focus.focus_step(n, out=outs.struct)
    g = outs.host()
    keep_gpu = [positions_of(u64(g["keep_bits"][b]), B) for b in range(n)]
    routes = [[[int(x) for x in g["route_experts"][l, r]] for r in range(n * B)] for l in range(wl.n_layers)]
    tr = fo.focus_step(cfg, W, pool, states, keep_override=keep_gpu, route_override=routes)
    seen = 0
    for l, rows in tr.route.items():
        for rid, (experts, weights, logits) in rows.items():
            assert len(set(experts)) == k and all(0 <= e < wl.n_experts for e in experts)
            tol = 2e-2 * max(1.0, float(np.max(np.abs(logits))))
            kth = np.sort(logits)[-k]
            assert all(logits[e] >= kth - tol for e in experts), (l, rid)
            assert all(logits[a] >= logits[b] - tol for a, b in zip(experts, experts[1:])), (l, rid)
            assert np.max(np.abs(g["route_weights"][l, rid] - np.asarray(weights))) <= 2e-2 * wl.route_scale
            seen += 1
    assert seen >= n * B
    assert relerr(g["hidden_packed"][:tr.cu[-1]], tr.hidden_packed) <= 2e-2
    sess.focus.focus_free()


@pytest.mark.parametrize("B", [4, 24, 40])
def test_small_bf16_block_sizes_below_the_key_tile(B):
    """Block sizes that do not fill the 32-key tiles of the matrix-core importance kernel (pooling at the block's edge)."""
    compare_steps(small_bf16(block_size=B, batch=6, keep_ratio=0.5, steps=2), 2, 2e-2, exact=False)


def test_small_bf16_large_vocabulary_few_rows():
    """Few rows and a large vocabulary: the confidence of a row is computed in column ranges and merged."""
    compare_steps(small_bf16(vocab=20008, mask_token_id=20007, batch=3, steps=2), 2, 2e-2, exact=False)


def test_small_bf16_confidence_fused_into_the_vocabulary_projection():
    """Without a logits output the vocabulary projection reduces its tiles to (max, sum exp, arg-max) triples and the logits are
    never written (Alg. 1 Decode_and_Verify).  Same step twice from the same state, with and without the logits output: arg-max
    tokens identical, confidences equal up to the order of the exp sums, commits identical; and the fused result against the
    oracle's confidences.  40 sequences x 8 rows and 33000 tokens give the projection enough tiles for the fused kernel; the odd
    vocabulary leaves a partly filled last column tile."""
    pk, runner = _pk()
    wl = small_bf16(vocab=33000, mask_token_id=32999, batch=40, prefix_lo=40, prefix_hi=90)
    cfg, W, pool, states, lens, tables, n_pages = oracle_batch(wl)
    sess = runner.open_session(wl, DEV)
    n, B = wl.batch, wl.block_size
    full = Outs(pk, wl, n)
    sess.focus.focus_step(n, out=full.struct)
    g1 = full.host()
    sess.focus.focus_prefill_kv(sess.prefix_lens, sess.page_tables, None)          # same block again
    lean = {k: torch.zeros_like(v) for k, v in full.t.items() if k in ("tokens", "mask_bits", "n_decoded", "keep_bits", "cu_seqlens", "conf", "argmax")}
    sess.focus.focus_step(n, out=pk.make_step_out(**lean))
    torch.cuda.synchronize()
    g2 = {k: v.cpu().numpy() for k, v in lean.items()}
    T = int(g1["cu_seqlens"][n])
    assert T == n * 8 and np.array_equal(g1["keep_bits"], g2["keep_bits"])
    assert np.array_equal(g1["argmax"][:T], g2["argmax"][:T])
    assert np.max(np.abs(g1["conf"][:T] - g2["conf"][:T]) / g1["conf"][:T]) < 1e-5
    assert np.array_equal(g1["tokens"], g2["tokens"]) and np.array_equal(g1["mask_bits"], g2["mask_bits"])
    keep = [positions_of(u64(k), B) for k in g2["keep_bits"]]
    tr = fo.focus_step(cfg, W, pool, states, keep_override=keep)
    assert relerr(g2["conf"][:T], tr.conf) <= 5 * 2e-2
    top = np.sort(tr.logits, axis=1)
    for r in range(T):        # the fused arg-max is (nearly) the oracle's
        assert tr.logits[r][int(g2["argmax"][r])] >= top[r, -1] - 5 * 2e-2 * np.max(np.abs(tr.logits[r]))
    sess.focus.focus_free()


def test_small_bf16_block64_override_empty_and_full():
    wl = small_bf16(block_size=64, budget_mode=3, batch=4, steps=2)
    compare_steps(wl, 2, 2e-2, exact=False, k_override=[0, 64, 17, 1])


# ---------------------------------------------------------------------------------------------
# stage tests: identical scores in, identical integers out

def install_states(pk, sess, wl, masks, sums, steps):
    for b, (m, ts, st) in enumerate(zip(masks, sums, steps)):
        s = sess.focus.focus_get_state(b)
        s.mask_bits, s.token_sum, s.total_steps = m, ts, st
        sess.focus.focus_set_state(b, s)


@pytest.mark.parametrize("mode,constraints,selection", [(0, 0, 0), (1, 0, 0), (2, 0, 0), (2, 3, 0), (3, 1, 0), (1, 2, 0),
                                                        (0, 0, 1), (3, 3, 1), (0, 0, 2), (2, 3, 2)])
def test_select_compact_stage_bit_exact(mode, constraints, selection):
    pk, runner = _pk()
    B, n = 32, 37
    wl = fi.workload("c1_tiny", block_size=B, batch=n, budget_mode=mode, topk=3, keep_ratio=0.2, constraints=constraints,
                     prefill="synthetic", n_layers=2, selection=selection, selection_seed=0xC0FFEE)
    sess = runner.open_session(wl, DEV)
    cfg = oracle_config(wl)
    r = np.random.default_rng(100 + mode * 10 + constraints)
    for trial in range(4):
        dI = r.normal(size=(n, B)).astype(np.float32)
        dI = np.round(dI * 4) / 4 if trial % 2 else dI                     # coarse values: many exact ties
        if trial == 3:
            dI[0, :] = 0.0
            dI[1, 5] = np.nan
        masks = [int(r.integers(0, 1 << B)) for _ in range(n)]
        masks[2] = 0
        masks[3] = (1 << B) - 1
        sums = [int(r.integers(0, 40)) for _ in range(n)]
        stp = [int(r.integers(0, 9)) for _ in range(n)]
        ko = [int(r.integers(0, B + 1)) for _ in range(n)]
        install_states(pk, sess, wl, masks, sums, stp)
        outs = Outs(pk, wl, n)
        sess.focus.focus_select_compact(n, torch.from_numpy(dI).to(DEV), outs.struct,
                                        k_override=torch.tensor(ko, dtype=torch.int32, device=DEV) if mode == 3 else None)
        g = outs.host()
        keep = []
        for b in range(n):
            masked = [bool((masks[b] >> p) & 1) for p in range(B)]
            K = fo.budget(cfg, dI[b].astype(np.float64), masked, sums[b], stp[b], ko[b])
            assert int(g["K"][b]) == K, (trial, b)
            rk = [fo.selection_key(cfg.selection_seed, b, stp[b], j) for j in range(B)]
            S = fo.select(cfg, dI[b].astype(np.float64), masked, [False] * B, K, None, rk)
            assert positions_of(u64(g["keep_bits"][b]), B) == S, (trial, b)
            keep.append(S)
        cu, rm = fo.compact(keep, B)
        assert [int(x) for x in g["cu_seqlens"]] == cu
        assert [int(x) for x in g["row_map"][:cu[-1]]] == rm
    sess.focus.focus_free()


def test_commit_stage_bit_exact():
    pk, runner = _pk()
    B, n = 32, 41
    wl = fi.workload("c1_tiny", block_size=B, batch=n, conf_threshold=0.6, prefill="synthetic")
    sess = runner.open_session(wl, DEV)
    cfg = oracle_config(wl)
    r = np.random.default_rng(7)
    for trial in range(3):
        masks = [int(r.integers(0, 1 << B)) for _ in range(n)]
        keeps = [sorted(r.choice(B, size=int(r.integers(0, B + 1)), replace=False).tolist()) for _ in range(n)]
        keeps[0], masks[1] = [], 0
        install_states(pk, sess, wl, masks, [3] * n, [2] * n)
        cu, _ = fo.compact(keeps, B)
        conf = r.random(cu[-1]).astype(np.float32)
        conf = np.round(conf * 8) / 8 if trial == 1 else conf            # ties in the forced-commit path
        if trial == 2:
            conf = conf * 0.5                                             # nothing passes: forced commits only
        am = r.integers(1, wl.vocab, cu[-1]).astype(np.int32)
        outs = Outs(pk, wl, n)
        sess.focus.focus_commit(n, torch.tensor([bits_of(k) for k in keeps], dtype=torch.int64, device=DEV),
                                torch.tensor(cu, dtype=torch.int32, device=DEV), torch.from_numpy(conf).to(DEV),
                                torch.from_numpy(am).to(DEV), outs.struct)
        g = outs.host()
        for b in range(n):
            st = fo.new_seq_state(cfg, 0, [])
            st.masked = [bool((masks[b] >> p) & 1) for p in range(B)]
            st.token_sum, st.total_steps = 3, 2
            D = fo.commit(cfg, st, keeps[b], conf[cu[b]:cu[b + 1]], am[cu[b]:cu[b + 1]])
            assert u64(g["mask_bits"][b]) == bits_of([p for p in range(B) if st.masked[p]]), (trial, b)
            assert int(g["n_decoded"][b]) == len(D)
            got = [int(t) for t in g["tokens"][b]]
            assert [got[p] for p in D] == [st.tokens[p] for p in D]
            s = sess.focus.focus_get_state(b)
            assert (s.token_sum, s.total_steps) == (st.token_sum, st.total_steps)
    sess.focus.focus_free()


@pytest.mark.parametrize("moe", [False, True])
def test_run_twice_bitwise_and_slot_permutation(moe):
    """Same call, same bits; and a permuted batch order moves the rows without changing a bit of them (with experts: the rows
    then sit in other tiles of the grouped projections, next to other rows)."""
    pk, runner = _pk()
    wl = small_bf16(batch=4, steps=1, **(dict(first_moe_layer=0, **MOE_SMALL) if moe else {}))
    res = []
    for perm in (None, None, [2, 0, 3, 1]):
        sess = runner.open_session(wl, DEV)
        n = wl.batch
        outs = Outs(pk, wl, n)
        slot = None if perm is None else torch.tensor(perm, dtype=torch.int32, device=DEV)
        sess.focus.focus_step(n, seq_slot=slot, out=outs.struct)
        res.append(outs.host())
        sess.focus.focus_free()
    a, b, c = res
    for k in a:
        assert np.array_equal(a[k], b[k]), k                              # same call, same bits
    B = wl.block_size
    for newb, oldb in enumerate([2, 0, 3, 1]):                            # batch order permuted: rows move with it
        assert c["keep_bits"][newb] == a["keep_bits"][oldb]
        ra = slice(a["cu_seqlens"][oldb], a["cu_seqlens"][oldb + 1])
        rc = slice(c["cu_seqlens"][newb], c["cu_seqlens"][newb + 1])
        assert np.array_equal(c["logits"][rc], a["logits"][ra])
        assert np.array_equal(c["tokens"][newb], a["tokens"][oldb])


def test_step_argument_errors():
    pk, runner = _pk()
    wl = fi.workload("c1_tiny", budget_mode=3)
    sess = runner.open_session(wl, DEV)
    with pytest.raises(pk.FocusError):
        sess.focus.focus_step(wl.batch)                    # OVERRIDE without budgets
    with pytest.raises(pk.FocusError):
        sess.focus.focus_step(wl.batch + 1)                # more sequences than slots
    with pytest.raises(pk.FocusError):
        sess.focus.focus_prefill_kv([10_000], [[0]])       # prefix longer than planned
    with pytest.raises(pk.FocusError):
        sess.focus.focus_prefill_kv([8], [[999]])          # page outside the pool
    sess.focus.focus_step(0, k_override=torch.zeros(1, dtype=torch.int32, device=DEV))   # an empty batch is a no-op
    sess.focus.focus_finalize_blocks(0)
    with pytest.raises(pk.FocusError):
        sess.focus.focus_run_steps(wl.batch, 2)            # per-step budgets cannot be looped
    with pytest.raises(pk.FocusError):
        sess.focus.focus_set_route_override(torch.zeros(8, dtype=torch.int32, device=DEV))   # dense model
    sess.focus.focus_free()


@pytest.mark.parametrize("intra_block_cache,moe", [(0, False), (1, False), (0, True)])
def test_multi_block_generation_with_finalize_fp32(intra_block_cache, moe):
    """Two blocks generated back to back: steps until a block has no masked position, focus_finalize_blocks, next
    block.  Tokens, masks, counters and prefix lengths must equal the oracle's at every step; at the end the whole
    cache (prompt + both generated blocks, every layer) must equal the oracle's.  With the delayed intra-block cache
    (Sec. 4.3) frozen positions take no part in the last forward and keep the K/V they have."""
    pk, runner = _pk()
    wl = fi.workload("c1_tiny", keep_ratio=0.5, extra_blocks=2, intra_block_cache=intra_block_cache,
                     **(dict(n_layers=3, first_moe_layer=1, **MOE_TINY) if moe else {}))      # (prefill and finalisation route on their own)
    cfg, W, pool, states, lens, tables, n_pages = oracle_batch(wl)
    sess = runner.open_session(wl, DEV)
    n, B = wl.batch, wl.block_size
    outs = Outs(pk, wl, n)
    fin = torch.zeros(n, dtype=torch.int32, device=DEV)
    frozen_seen = False
    for block in range(2):
        for step in range(B + 1):
            sess.focus.focus_finalize_blocks(n, fin)
            done_gpu = fin.cpu().tolist()
            done_ora = fo.finalize_blocks(cfg, W, pool, states)
            assert [bool(x) for x in done_gpu] == done_ora, (block, step)
            if all(done_ora):
                break
            assert not any(done_ora)                             # equal commit counts: the sequences finish together
            sess.focus.focus_step(n, out=outs.struct)
            g = outs.host()
            tr = fo.focus_step(cfg, W, pool, states, score_cast=lambda d: d.astype(np.float32).astype(np.float64),
                               conf_cast=lambda c: c.astype(np.float32).astype(np.float64))
            T = tr.cu[-1]
            assert [positions_of(u64(k), B) for k in g["keep_bits"]] == tr.keep
            assert row_relerr(g["logits"][:T], tr.logits) <= 1e-3
            for b, st in enumerate(states):
                assert [int(t) for t in g["tokens"][b]] == st.tokens
                assert u64(g["mask_bits"][b]) == bits_of([p for p in range(B) if st.masked[p]])
                assert sess.focus.focus_get_state(b).cached_bits == bits_of([p for p in range(B) if st.cached[p]])
            frozen_seen = frozen_seen or any(any(st.cached) for st in states)
        else:
            raise AssertionError("block did not finish")
        for b, st in enumerate(states):
            s = sess.focus.focus_get_state(b)
            assert (s.prefix_len, s.token_sum, s.total_steps, s.processed_bits) == (lens[b] + (block + 1) * B, st.token_sum, st.total_steps, 0)
            assert s.mask_bits == (1 << B) - 1 and st.prefix_len == s.prefix_len and s.cached_bits == 0
    assert frozen_seen == bool(intra_block_cache)
    kv = sess.kv_pool.cpu().numpy()
    P = wl.page_size
    for l in range(wl.n_layers):
        for b, st in enumerate(states):
            for t in range(st.prefix_len):
                pg = pool.layers[l][st.pages[t // P]]
                page = kv[l, st.pages[t // P]]
                got_k = page[0][:, t % P, :]
                got_v = page[1].reshape(wl.n_kv_heads, wl.head_dim, P)[:, :, t % P]
                assert relerr(got_k, pg[0, :, t % P, :]) <= 1e-3 and relerr(got_v, pg[1, :, t % P, :]) <= 1e-3, (l, b, t)
    # no room for a third block beyond the planned two extra ones is needed here; a sequence without room is left alone
    sess.focus.focus_free()


def test_finalize_skips_incomplete_blocks_and_sequences_without_room():
    pk, runner = _pk()
    wl = fi.workload("c1_tiny", keep_ratio=1.0)                  # pages for the current block only
    sess = runner.open_session(wl, DEV)
    n, B = wl.batch, wl.block_size
    fin = torch.ones(n, dtype=torch.int32, device=DEV)
    sess.focus.focus_finalize_blocks(n, fin)
    assert fin.cpu().tolist() == [0] * n                         # all masked: nothing to finalize
    for _ in range(B):
        sess.focus.focus_step(n)
    assert all(sess.focus.focus_get_state(b).mask_bits == 0 for b in range(n))
    before = [sess.focus.focus_get_state(b).prefix_len for b in range(n)]
    sess.focus.focus_finalize_blocks(n, fin)
    assert fin.cpu().tolist() == [0] * n                         # complete, but no pages / positions planned for another block
    assert [sess.focus.focus_get_state(b).prefix_len for b in range(n)] == before
    sess.focus.focus_free()


@pytest.mark.parametrize("budget_mode,intra_block_cache", [(1, 0), (2, 1)])
def test_run_steps_equals_separate_steps_with_finalisation(budget_mode, intra_block_cache):
    """Several steps per host call with the state updated on the device (App. E.3.4): bit-identical to the same steps
    enqueued one call at a time, across a block boundary, with the dynamic budget reading the fresh statistics."""
    pk, runner = _pk()
    wl = fi.workload("c1_tiny", budget_mode=budget_mode, keep_ratio=0.5, conf_threshold=0.0013, extra_blocks=2,
                     intra_block_cache=intra_block_cache, constraints=3 if budget_mode == 2 else 0)
    n, B, steps = wl.batch, wl.block_size, 5

    def snapshot(sess, outs):
        torch.cuda.synchronize()
        st = [sess.focus.focus_get_state(b) for b in range(n)]
        return ([(s.prefix_len, s.total_steps, s.token_sum, s.mask_bits, s.processed_bits, s.cached_bits, list(s.tokens)[:B]) for s in st],
                {k: v.cpu().numpy().copy() for k, v in outs.t.items()})

    sess = runner.open_session(wl, DEV)
    outs = Outs(pk, wl, n)
    total = np.zeros(n, dtype=np.int64)
    for i in range(steps):
        sess.focus.focus_step(n, out=outs.struct)
        total += outs.host()["n_decoded"]
        sess.focus.focus_finalize_blocks(n)
    want_state, want_out = snapshot(sess, outs)
    kv_want = sess.kv_pool.cpu()
    sess.focus.focus_free()

    sess = runner.open_session(wl, DEV)
    outs = Outs(pk, wl, n)
    decoded = torch.zeros(n, dtype=torch.int64, device=DEV)
    sess.focus.focus_run_steps(n, 2, finalize=True, decoded=decoded)
    sess.focus.focus_run_steps(n, steps - 2, finalize=True, decoded=decoded, out=outs.struct)
    got_state, got_out = snapshot(sess, outs)
    assert got_state == want_state
    assert max(s[0] for s in got_state) > max(sess.prefix_lens)            # some block was finalised on the way
    T = int(want_out["cu_seqlens"][-1])
    assert T > 0
    for k in want_out:          # (the separate calls wrote every step's outputs: beyond the last step's T' rows theirs are older)
        rows = T if k in ("row_map", "conf", "argmax", "hidden_packed", "logits") else len(want_out[k])
        assert np.array_equal(got_out[k][:rows], want_out[k][:rows]), k
    assert decoded.cpu().numpy().tolist() == total.tolist()
    assert torch.equal(sess.kv_pool.cpu(), kv_want)
    sess.focus.focus_free()


def _random_workload(seed, bf16):
    """A small configuration drawn from the seed: shapes and switches that the fixed tests do not visit."""
    r = np.random.default_rng(1000 + seed)
    pick = lambda xs: xs[int(r.integers(0, len(xs)))]
    n_layers = int(r.integers(2, 5))
    importance_mode = pick([0, 0, 1])
    evict = int(r.integers(1 if importance_mode == 0 else 0, n_layers))
    B = pick([1, 2, 3, 8, 16, 31, 33, 64]) if not bf16 else pick([2, 5, 17, 32, 48, 64])
    budget_mode = pick([0, 1, 1, 2])
    over = dict(n_layers=n_layers, evict_layer=evict, importance_mode=importance_mode, maxpool_k=pick([1, 3]), block_size=B,
                budget_mode=budget_mode, topk=int(r.integers(0, B + 1)), keep_ratio=float(pick([0.1, 0.25, 0.5, 0.75, 1.0])),
                alpha=float(pick([1.0, 1.5, 2.5])), constraints=int(r.integers(0, 4)), intra_block_cache=pick([0, 1]),
                conf_threshold=float(pick([0.9, 0.002, 0.0005])), batch=int(r.integers(1, 7)), steps=3,
                selection=pick([0, 0, 1, 2]), selection_seed=int(r.integers(0, 1 << 30)))
    if r.integers(0, 3) == 0:        # a mixture-of-experts model every third draw
        E = pick([3, 8, 16])
        over.update(n_experts=E, experts_per_token=int(r.integers(1, min(4, E) + 1)), expert_ffn=pick([64, 128]), shared_ffn=pick([0, 64]),
                    first_moe_layer=int(r.integers(0, n_layers)), route_scale=float(pick([1.0, 2.5])))
    if bf16:
        hkv = pick([1, 2, 4, 8])
        lo = int(r.integers(0, 150))
        over.update(hidden=pick([256, 512]), n_q_heads=8, n_kv_heads=hkv, ffn=pick([256, 768]), vocab=4096, mask_token_id=4095,
                    prefix_lo=lo, prefix_hi=lo + int(r.integers(0, 200)), prefix_dist="uniform", shuffle_pages=bool(r.integers(0, 2)))
        return fi.workload("c3_llada36", **over)
    hq = pick([2, 4, 8])
    lo = int(r.integers(0, 40))
    over.update(n_q_heads=hq, n_kv_heads=pick([h for h in (1, 2, 4, 8) if hq % h == 0]), head_dim=pick([64, 128]), hidden=pick([64, 256]),
                ffn=pick([128, 320]), page_size=pick([16, 32, 64]), prefix_lo=lo, prefix_hi=lo + int(r.integers(0, 60)),
                prefill=pick(["prompt", "synthetic"]), shuffle_pages=bool(r.integers(0, 2)))
    return fi.workload("c1_tiny", **over)


@pytest.mark.parametrize("seed", range(16))
def test_random_small_configurations_fp32_exact(seed):
    wl = _random_workload(seed, bf16=False)
    print(wl, flush=True)
    compare_steps(wl, wl.steps, 1e-3, exact=True)


@pytest.mark.parametrize("seed", range(16))
def test_random_small_configurations_bf16(seed):
    wl = _random_workload(seed, bf16=True)
    print(wl, flush=True)
    compare_steps(wl, wl.steps, 2e-2, exact=False, forced_routes=wl.n_experts > 0)
