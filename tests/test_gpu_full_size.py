"""Full-size parity: the benchmark configurations run on the GPU at their real batch, lengths, depth and shapes, in
the launch configuration bench.py times; a few sampled sequences are recomputed by the CPU oracle (sequences are
independent, so the oracle can take them one by one), the rest is covered by properties that hold at any size.
Retained sets are teacher-forced from the GPU into the oracle after checking that they are a valid top-K of the
oracle's own scores within tolerance.

Floating point, bf16 models.  The stated bound is 2e-2 (max|gpu - oracle| / max|oracle|).  It is checked
  (a) on the layers up to the eviction layer, from the embeddings (identical inputs);
  (b) on EVERY window of two deep layers, fed the float64 oracle's own residual stream through focus_run_layers.
End to end, free-running through 36 layers, the bound is NOT met against the float64 oracle and cannot be by anything that
keeps its activations in bf16: the storage format alone, with exact arithmetic everywhere, moves the result by 3-4 %
(tests/golden/bf16_drift_c4_batch256.txt, CPU only), because every layer of this random-init model amplifies what the
roundings of the layers before it left, and two runs whose roundings differ in a few places decorrelate (the GPU is
2.8 % from the format model while both are 3.4-3.9 % from float64).  So the end-to-end check is made against that
yardstick, computed in the same test from the CPU oracle alone:
  (c) the oracle is run a second time with the bf16 storage format switched on (OracleConfig.store_cast: the activations
      a bf16 model keeps in memory are rounded, all arithmetic stays float64); the GPU's distance from the float64 oracle
      must be at most max(2e-2, 1.5 x the format run's distance from the float64 oracle), for the final residual stream and
      for the logits.  At the depths where the format costs less than 1.3 % (the 4- and 6-layer cases) that is 2e-2."""
import copy
import time

import numpy as np
import pytest
import torch

import focus_inputs as fi
from oracle import focus_oracle as fo
from oracle.harness import _f64, bf16_store_cast, oracle_config, oracle_weights_from_tensors
from test_gpu_parity import DEV, _pk, bits_of, check_selection_valid, positions_of, relerr, u64

pytestmark = pytest.mark.gpu
TOL = 2e-2


def signed64(v):
    return v - (1 << 64) if v >= (1 << 63) else v


def gpu_step(pk, sess, wl, sample_ids, k_override=None, keep_rows_of=None):
    """One focus_step of the whole batch.  Returns the small outputs of every sequence and, for the sampled sequences,
    their rows of the residual streams and logits (the big tensors stay on the device)."""
    n, B, h, V = wl.batch, wl.block_size, wl.hidden, wl.vocab
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=DEV)
    t = dict(tokens=z(n, B, dt=torch.int32), mask_bits=z(n, dt=torch.int64), n_decoded=z(n, dt=torch.int32),
             importance=z(n, B), importance_prev=z(n, B), delta_I=z(n, B), K=z(n, dt=torch.int32), keep_bits=z(n, dt=torch.int64),
             cu_seqlens=z(n + 1, dt=torch.int32), row_map=z(n * B, dt=torch.int32), conf=z(n * B),
             argmax=z(n * B, dt=torch.int32), hidden_full=z(n * B, h), hidden_packed=z(n * B, h), logits=z(n * B, V))
    if wl.n_experts:
        t["route_experts"] = torch.full((wl.n_layers, n * B, wl.experts_per_token), -1, dtype=torch.int32, device=DEV)
        t["route_weights"] = z(wl.n_layers, n * B, wl.experts_per_token)
    ko = None if k_override is None else torch.tensor(k_override, dtype=torch.int32, device=DEV)
    mask_before = [sess.focus.focus_get_state(b).mask_bits for b in sample_ids]
    sess.focus.focus_step(n, k_override=ko, out=pk.make_step_out(**t))
    torch.cuda.synchronize()
    g = {k: v.cpu().numpy() for k, v in t.items() if k != "logits" and not k.startswith("hidden")}
    cu = [int(x) for x in g["cu_seqlens"]]
    g["cu"] = cu
    g["keep"] = [positions_of(u64(g["keep_bits"][b]), B) for b in range(n)]
    g["mask_before"] = dict(zip(sample_ids, mask_before))
    g["rows"] = {}
    for b in sample_ids:
        g["rows"][b] = dict(hidden_full=t["hidden_full"][b * B:(b + 1) * B].cpu().numpy(),
                            hidden_packed=t["hidden_packed"][cu[b]:cu[b + 1]].cpu().numpy(),
                            logits=t["logits"][cu[b]:cu[b + 1]].cpu().numpy())
    g["route_dev"] = t.get("route_experts")
    return g


def check_whole_batch(wl, g, k_override=None, first_step=True):
    """Properties that hold for every sequence of the batch, at any size."""
    n, B = wl.batch, wl.block_size
    cu, keep = g["cu"], g["keep"]
    exp_k = [min(B, max(0, int(k))) for k in (k_override if k_override is not None else [int(g["K"][0])] * n)]
    assert [int(k) for k in g["K"]] == exp_k
    if first_step:
        assert [len(s) for s in keep] == exp_k                              # all masked, no constraints: |S| = K
    assert cu == [int(x) for x in np.concatenate([[0], np.cumsum([len(s) for s in keep])])]
    assert [int(r) for r in g["row_map"][:cu[-1]]] == [b * B + p for b in range(n) for p in keep[b]]
    assert np.allclose(g["importance"].sum(axis=1), B * wl.n_q_heads, rtol=2e-3)
    assert np.all(np.abs(g["delta_I"].sum(axis=1)) < 2e-3 * B * wl.n_q_heads)
    for b in range(n):
        nd = int(g["n_decoded"][b])
        if first_step:
            assert nd == (1 if exp_k[b] > 0 else 0)                         # random-init weights: the forced single commit
            newly = [p for p in range(B) if not (u64(g["mask_bits"][b]) >> p) & 1]
            assert len(newly) == nd and set(newly) <= set(keep[b])
            for p in newly:
                row = cu[b] + keep[b].index(p)
                assert int(g["tokens"][b][p]) == int(g["argmax"][row])
                assert g["conf"][row] == g["conf"][cu[b]:cu[b + 1]].max()
    if wl.n_experts:
        re_, rw = g["route_experts"], g["route_weights"]
        for l in range(wl.n_layers):
            ran = re_[l][:, 0] >= 0
            assert ran.sum() == (0 if not wl.is_moe_layer(l) else (n * B if l < wl.evict_layer else cu[-1])), l
            if ran.any():
                srt = np.sort(re_[l][ran], axis=1)
                assert np.all(srt[:, 1:] > srt[:, :-1]) and srt.min() >= 0 and srt.max() < wl.n_experts
                assert np.allclose(rw[l][ran].sum(axis=1), wl.route_scale, rtol=1e-4)
                assert np.all(rw[l][ran][:, :-1] >= rw[l][ran][:, 1:])
    return exp_k


class OraclePair:
    """The float64 oracle and the oracle with the bf16 storage format, on the same sampled sequences (own K/V pools and
    block states), sharing one set of float64 weights widened from the tensors the GPU session generated."""

    def __init__(self, wl, sess, sample_ids):
        self.wl, self.ids = wl, list(sample_ids)
        embed, lm_head, norm, layers = sess.weights
        # the device tensors come from the same seeded recipe the CPU uses; spot-check one of them against a CPU generation
        assert torch.equal(wl.layer_weight(wl.n_layers - 1, "w_o"), layers[wl.n_layers - 1]["w_o"].cpu())
        self.W = oracle_weights_from_tensors(wl, lm_head, layers)
        lens = wl.prefix_lens()
        tables, n_pages = wl.page_tables(lens)
        self.lens = lens
        self.cfg = oracle_config(wl)
        self.cfg_fmt = oracle_config(wl)
        self.cfg_fmt.store_cast = bf16_store_cast()
        self.pool = fo.KVPool(self.cfg)
        for l in range(wl.n_layers):
            for b in self.ids:
                for pid in tables[b]:
                    self.pool.layers[l][pid] = _f64(wl.kv_page(l, pid, n_pages))
        self.pool_fmt = copy.deepcopy(self.pool)
        self.states = [fo.new_seq_state(self.cfg, lens[b], tables[b], slot=b) for b in self.ids]
        self.states_fmt = copy.deepcopy(self.states)

    def step(self, keeps, record=None, routes=None):
        t0 = time.time()
        tr = fo.focus_step(self.cfg, self.W, self.pool, self.states, keep_override=keeps, record_layers=record, route_override=routes)
        t1 = time.time()
        tf = fo.focus_step(self.cfg_fmt, self.W, self.pool_fmt, self.states_fmt, keep_override=keeps, route_override=routes)
        print("oracle passes: %.0f s float64, %.0f s bf16 storage format" % (t1 - t0, time.time() - t1), flush=True)
        return tr, tf


def compare_sample(wl, g, b, i, tr, tf, exp_k, label):
    """Sampled sequence b of GPU step g against row segment i of the oracle traces (tr float64, tf bf16 storage format)."""
    B = wl.block_size
    rows = g["rows"][b]
    assert relerr(g["importance"][b], tr.I_evict[i]) <= TOL
    assert relerr(g["importance_prev"][b], tr.I_prev[i]) <= TOL
    scale = float(np.max(np.abs(tr.delta_I[i])))
    assert float(np.max(np.abs(g["delta_I"][b] - tr.delta_I[i]))) <= 2 * TOL * float(np.max(np.abs(tr.I_evict[i])))
    masked = [bool((g["mask_before"][b] >> p) & 1) for p in range(B)]
    check_selection_valid(tr.delta_I[i], masked, set(g["keep"][b]), exp_k, B, 5 * TOL * scale)
    assert relerr(rows["hidden_full"], tr.hidden_full[i * B:(i + 1) * B]) <= TOL            # (a)
    lo, hi = tr.cu[i], tr.cu[i + 1]
    if hi == lo:
        return None
    fmt_hp = relerr(tf.hidden_packed[lo:hi], tr.hidden_packed[lo:hi])                      # what the format alone costs
    fmt_lg = max(relerr(tf.logits[lo + r], tr.logits[lo + r]) for r in range(hi - lo))
    e_hp_f = relerr(rows["hidden_packed"], tf.hidden_packed[lo:hi])                         # (c) GPU vs format oracle
    e_lg_f = max(relerr(rows["logits"][r], tf.logits[lo + r]) for r in range(hi - lo))
    e_hp = relerr(rows["hidden_packed"], tr.hidden_packed[lo:hi])                           # GPU vs float64 oracle
    e_lg = max(relerr(rows["logits"][r], tr.logits[lo + r]) for r in range(hi - lo))
    cu = g["cu"]
    e_cf_f = relerr(g["conf"][cu[b]:cu[b + 1]], tf.conf[lo:hi])
    rec = dict(case=label, seq=b, rows=hi - lo, gpu_vs_format=dict(hidden=e_hp_f, logits=e_lg_f, conf=e_cf_f),
               gpu_vs_float64=dict(hidden=e_hp, logits=e_lg), format_vs_float64=dict(hidden=fmt_hp, logits=fmt_lg))
    print(rec, flush=True)
    assert e_hp <= max(TOL, 1.5 * fmt_hp) and e_lg <= max(TOL, 1.5 * fmt_lg), rec                  # (c)
    assert e_cf_f <= 5 * max(TOL, 1.5 * fmt_lg), rec
    # the committed position is (nearly) the most confident one for the oracle too, and its token (nearly) the arg-max
    newly = [p for p in range(B) if masked[p] and not (u64(g["mask_bits"][b]) >> p) & 1]
    for p in newly:
        r = g["keep"][b].index(p)
        cand = [j for j, q in enumerate(g["keep"][b]) if masked[q]]
        best = max(float(tf.conf[lo + j]) for j in cand)
        assert tf.conf[lo + r] >= best * (1 - 5 * TOL) or tf.conf[lo + r] >= float(np.float32(wl.conf_threshold)) * (1 - 5 * TOL)
        tok = int(g["tokens"][b][p])
        assert tf.logits[lo + r][tok] >= tf.logits[lo + r].max() - 5 * TOL * np.max(np.abs(tf.logits[lo + r]))
    return rec


def all_windows(wl, sess, pairs, tr, step=2):
    """(b): every window of `step` deep layers from the float64 oracle's own residual stream.  pairs = [(sequence id,
    retained positions)] in the order of the oracle's batch."""
    B, h, L, e = wl.block_size, wl.hidden, wl.n_layers, wl.evict_layer
    ns, Tp = len(pairs), tr.cu[-1]
    if not Tp:
        return
    kb = torch.tensor([signed64(bits_of(k)) for _, k in pairs], dtype=torch.int64, device=DEV)
    slots = torch.tensor([b for b, _ in pairs], dtype=torch.int32, device=DEV)
    worst = 0.0
    for l in range(e + 1, L, step):
        l1 = min(l + step, L)
        hid = torch.zeros(ns * B, h, device=DEV)
        hid[:Tp] = torch.from_numpy(tr.hidden_entering[l]).to(DEV, torch.float32)
        sess.focus.focus_run_layers(ns, kb, kb, l, l1, hid, seq_slot=slots)
        torch.cuda.synchronize()
        ref = tr.hidden_entering[l1] if l1 < L else tr.hidden_packed
        err = relerr(hid[:Tp].cpu().numpy(), ref)
        worst = max(worst, err)
        assert err <= TOL, (l, l1, err)
    print(dict(windows="layers %d..%d in steps of %d from the oracle's stream" % (e + 1, L, step), worst=worst), flush=True)


def run_full_and_compare(wl, sample_ids, k_override=None):
    pk, runner = _pk()
    sess = runner.open_session(wl, DEV)
    print("gpu step", flush=True)
    g = gpu_step(pk, sess, wl, sample_ids, k_override)
    exp_k = check_whole_batch(wl, g, k_override)
    routes = None
    B, L = wl.block_size, wl.n_layers
    if wl.n_experts:
        # the oracle is teacher-forced with the GPU's picks for the sampled sequences (checked against its own logits below);
        # oracle row ids are i * B + p for the i-th sampled sequence
        re_ = g["route_experts"]
        routes = [[[int(x) for x in re_[l, b * B + p]] for b in sample_ids for p in range(B)] for l in range(L)]
    print("oracle on sequences", sample_ids, flush=True)
    op = OraclePair(wl, sess, sample_ids)
    keeps = [g["keep"][b] for b in sample_ids]
    tr, tf = op.step(keeps, record=set(range(L)), routes=routes)
    for l, rows in tr.route.items():
        for rid, (experts, weights, logits) in rows.items():
            tol = TOL * max(1.0, float(np.max(np.abs(logits))))
            kth = np.sort(logits)[-wl.experts_per_token]
            assert all(logits[x] >= kth - tol for x in experts), (l, rid)
            grid = sample_ids[rid // B] * B + rid % B
            assert np.max(np.abs(g["route_weights"][l, grid] - np.asarray(weights))) <= 2 * TOL * wl.route_scale, (l, rid)
    for i, b in enumerate(sample_ids):
        compare_sample(wl, g, b, i, tr, tf, exp_k[b], wl.name)
    if wl.n_experts:                 # the windows use the step's picks (rows are named by their place in the window's batch)
        forced = torch.zeros_like(g["route_dev"])
        for i, b in enumerate(sample_ids):
            forced[:, i * B:(i + 1) * B] = g["route_dev"][:, b * B:(b + 1) * B]
        sess.focus.focus_set_route_override(forced)
    all_windows(wl, sess, list(zip(sample_ids, keeps)), tr)
    sess.focus.focus_free()


def test_c4_batch256_full_size_all_keep_ratios():
    """BASELINE configs[3] at full size (36 layers, batch 256, prefix U[512,4096], block 32) at every keep ratio of its sweep:
    the GPU runs the whole batch once per ratio; five sampled sequences (two at ratio 0.25, one at each other ratio) go
    through ONE pass of the oracle, each with the retained set of its own GPU run."""
    pk, runner = _pk()
    wl = fi.workload("c4_batch256", keep_ratio=0.25)
    lens = wl.prefix_lens()
    order = [int(i) for i in np.argsort(lens)]
    plan = [(0.25, order[0]), (0.25, 137), (1.0, order[1]), (0.5, order[2]), (0.125, order[len(order) // 2])]
    assert len({b for _, b in plan}) == len(plan)
    sess = runner.open_session(wl, DEV)
    runs = {}
    for ratio in (0.25, 1.0, 0.5, 0.125):
        sess.reopen(keep_ratio=ratio)
        ids = [b for r, b in plan if r == ratio]
        print("gpu step at keep ratio", ratio, flush=True)
        runs[ratio] = gpu_step(pk, sess, wl, ids)
        exp = check_whole_batch(wl, runs[ratio])
        assert exp[0] == int(np.ceil(ratio * wl.block_size))
    ids = [b for _, b in plan]
    op = OraclePair(wl, sess, ids)
    keeps = [runs[r]["keep"][b] for r, b in plan]
    tr, tf = op.step(keeps, record=set(range(wl.n_layers)))
    for i, (r, b) in enumerate(plan):
        compare_sample(wl, runs[r], b, i, tr, tf, len(keeps[i]), "%s keep ratio %g" % (wl.name, r))
    all_windows(wl, sess, list(zip(ids, keeps)), tr)
    sess.focus.focus_free()


def test_c3_llada36_batch128_eight_steps():
    """BASELINE configs[2] at its full batch, lengths and depth (36 layers, batch 128, prefix U[256,2048], block 32, keep ratio
    0.25, threshold 0.9): the 8 denoising steps of a block, free-running on the GPU; one sampled sequence is followed by both
    oracles step by step (retained sets and commits taken over from the GPU after they were checked against the oracle's
    own values), so stale K/V of evicted positions and the growing set of decoded tokens are compared at full depth."""
    pk, runner = _pk()
    wl = fi.workload("c3_llada36")
    lens = wl.prefix_lens()
    b = int(np.argsort(lens)[len(lens) // 2])
    sess = runner.open_session(wl, DEV)
    op = OraclePair(wl, sess, [b])
    B = wl.block_size
    for step in range(wl.steps):
        print("step", step, flush=True)
        g = gpu_step(pk, sess, wl, [b])
        check_whole_batch(wl, g, first_step=step == 0)
        tr, tf = op.step([g["keep"][b]], record=set(range(wl.n_layers)) if step in (0, wl.steps - 1) else None)
        compare_sample(wl, g, b, 0, tr, tf, int(g["K"][b]), "%s step %d" % (wl.name, step))
        if step in (0, wl.steps - 1):
            # windows see the K/V state of this step: the retained rows rewrite theirs, earlier retained positions are visible
            vis = [p for p in range(B) if op.states[0].processed[p]]
            kb = torch.tensor([signed64(bits_of(g["keep"][b]))], dtype=torch.int64, device=DEV)
            vb = torch.tensor([signed64(bits_of(vis))], dtype=torch.int64, device=DEV)
            slots = torch.tensor([b], dtype=torch.int32, device=DEV)
            Tp = tr.cu[-1]
            for l in range(wl.evict_layer + 1, wl.n_layers, 2):
                hid = torch.zeros(B, wl.hidden, device=DEV)
                hid[:Tp] = torch.from_numpy(tr.hidden_entering[l]).to(DEV, torch.float32)
                sess.focus.focus_run_layers(1, kb, vb, l, min(l + 2, wl.n_layers), hid, seq_slot=slots)
                torch.cuda.synchronize()
                ref = tr.hidden_entering[l + 2] if l + 2 < wl.n_layers else tr.hidden_packed
                err = relerr(hid[:Tp].cpu().numpy(), ref)
                assert err <= TOL, (step, l, err)
        # both oracles go on from the GPU's commit (it was checked against the format oracle's confidences in compare_sample)
        toks, mb = [int(x) for x in g["tokens"][b]], u64(g["mask_bits"][b])
        for st in (op.states[0], op.states_fmt[0]):
            st.masked = [bool((mb >> p) & 1) for p in range(B)]
            st.tokens = [toks[p] if not st.masked[p] else st.tokens[p] for p in range(B)]
            st.token_sum = sess.focus.focus_get_state(b).token_sum
    sess.focus.focus_free()


def test_c5_ragged_36_layers_shortest_and_full_segment():
    """BASELINE configs[4] at its full batch, lengths (log-uniform up to 32768), shuffled 64-token pages, block 64 and depth,
    per-sequence budgets 0..64: the shortest sequence and the one with the forced full segment (K = 64) through all 36
    layers of both oracles; the empty segment (K = 0) is checked by the whole-batch properties."""
    wl = fi.workload("c5_ragged")
    ks = wl.k_overrides()
    lens = wl.prefix_lens()
    assert ks[0] == 0 and ks[1] == wl.block_size
    short = int(np.argmin(lens))
    run_full_and_compare(wl, [short] + ([1] if short != 1 and lens[1] <= 12000 else []), k_override=ks)


def test_c5_ragged_longest_sequence_six_layers():
    """The same configuration with the layer count cut to 6 to bound the oracle's time on the LONGEST sequence (tens of
    thousands of cached tokens, hundreds of shuffled pages), plus the empty and the full segment."""
    wl = fi.workload("c5_ragged", n_layers=6)
    ks = wl.k_overrides()
    lens = wl.prefix_lens()
    run_full_and_compare(wl, [0, 1, int(np.argmax(lens))], k_override=ks)


def test_c6_moe_mini_full_depth():
    """Second workload (mixture-of-experts, 256 experts of which 8 per token, one shared expert, dense first layer) at its
    full batch, lengths, expert shapes and depth (20 layers).  Routing runs free on the GPU; the oracles are teacher-forced
    with the picks of the sampled sequence after checking them against the float64 oracle's router logits."""
    wl = fi.workload("c6_moe_mini")
    run_full_and_compare(wl, [int(np.argmin(wl.prefix_lens()))])


def test_c2_sdar4_small_batch_block4_topk2():
    """BASELINE configs[1] as given (4 layers of the 8B shape, batch 32, prefix 512, block 4, top-k 2, one step): 128 rows
    in the full-block phase and 64 after eviction, the regime where the projections are K-split."""
    wl = fi.workload("c2_sdar4")
    run_full_and_compare(wl, [0, 13, 31])
