"""focus_step under HIP graph capture (the paper's App. E.4 captures the reduced forward pass in CUDA graphs).

A step only enqueues kernels on the caller's stream: no allocation, no host synchronisation, no memset nodes, and
every kernel reads the packed row count from device memory, so one captured graph serves every step whatever the
number of retained rows (no shape buckets).  The test captures one step, replays it for several consecutive
denoising steps with eager work and synchronisations between the replays, and checks every replay bit for bit
against the same steps run eagerly.
"""
import numpy as np
import pytest
import torch

import focus_inputs as fi

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _small_bf16(**over):
    base = dict(n_layers=3, hidden=512, n_q_heads=8, n_kv_heads=2, ffn=1024, vocab=4096, mask_token_id=4095,
                batch=5, prefix_lo=70, prefix_hi=200, prefix_dist="uniform", block_size=32, budget_mode=1,
                keep_ratio=0.25, steps=4, shuffle_pages=True)
    base.update(over)
    return fi.workload("c3_llada36", **base)


def _outs(pk, wl, n):
    B, V = wl.block_size, wl.vocab
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=DEV)
    t = dict(tokens=z(n, B, dt=torch.int32), mask_bits=z(n, dt=torch.int64), n_decoded=z(n, dt=torch.int32),
             delta_I=z(n, B), keep_bits=z(n, dt=torch.int64), cu_seqlens=z(n + 1, dt=torch.int32),
             row_map=z(n * B, dt=torch.int32), conf=z(n * B), argmax=z(n * B, dt=torch.int32), logits=z(n * B, V))
    return t, pk.make_step_out(**t)


def _snapshot(t):
    torch.cuda.synchronize()
    return {k: v.cpu().numpy().copy() for k, v in t.items()}


@pytest.mark.parametrize("dtype", ["bf16", "fp32", "bf16-moe"])
def test_captured_step_replays_match_eager(dtype):
    import paper_2601_23278_amd as pk
    from paper_2601_23278_amd import runner
    wl = fi.workload("c1_tiny") if dtype == "fp32" else _small_bf16() if dtype == "bf16" else \
        _small_bf16(n_experts=16, experts_per_token=4, expert_ffn=128, shared_ffn=128, route_scale=1.5, first_moe_layer=0)
    n, steps = wl.batch, 4

    sess = runner.open_session(wl, DEV)
    t, out = _outs(pk, wl, n)
    eager = []
    for _ in range(steps):
        sess.focus.focus_step(n, out=out)
        eager.append(_snapshot(t))
    sess.focus.focus_free()

    sess = runner.open_session(wl, DEV)
    t, out = _outs(pk, wl, n)
    side = torch.cuda.Stream()
    # first calls of a kernel set its LDS attribute, which cannot be captured: run one step eagerly, then start the block again
    sess.focus.focus_step(n, out=out)
    torch.cuda.synchronize()
    sess.focus.focus_prefill_kv(sess.prefix_lens, sess.page_tables, None if wl.prefill != "prompt" else
                                [wl.prompt_tokens(wl.prefix_lens())[b] for b in sess.seq_ids])
    graph = torch.cuda.CUDAGraph()
    scratch = torch.zeros(1 << 20, device=DEV)
    with torch.cuda.graph(graph, stream=side):
        sess.focus.focus_step(n, out=out, stream=side)
    # capture does not execute: the block is still at its first step
    for i in range(steps):
        graph.replay()
        got = _snapshot(t)
        for k in got:
            assert np.array_equal(got[k], eager[i][k]), (i, k)
        scratch.add_(1.0)                      # the program's own eager work between replays
        assert float(scratch[0].item()) == i + 1
    sess.focus.focus_free()


@pytest.mark.parametrize("prefix", [224, 992])
def test_captured_step_matches_the_oracle_also_after_the_prefix_grew(prefix):
    """A step is captured while prefix + block is exactly one K/V split (224 + 32 = 256 tokens: one split per sequence) or
    two (992 + 32 = 1024 with few sequences), replayed and compared with the CPU oracle; then the block is completed and
    finalised, which makes it prefix (prefix_len += B, one token range more than the captured launch was sized for), and
    the SAME graph is replayed for the first step of the next block and compared with the oracle again."""
    import paper_2601_23278_amd as pk
    from paper_2601_23278_amd import runner
    from oracle import focus_oracle as fo
    from oracle.harness import oracle_batch
    wl = _small_bf16(batch=3, prefix_lo=prefix, prefix_hi=prefix, prefix_dist="fixed", extra_blocks=1)
    n, B = wl.batch, wl.block_size
    cfg, W, pool, states, lens, tables, n_pages = oracle_batch(wl)
    sess = runner.open_session(wl, DEV)
    t, out = _outs(pk, wl, n)
    side = torch.cuda.Stream()
    sess.focus.focus_step(n, out=out)                       # first launches set LDS attributes: not capturable
    torch.cuda.synchronize()
    sess.focus.focus_prefill_kv(sess.prefix_lens, sess.page_tables, None)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sess.focus.focus_step(n, out=out, stream=side)

    def replay_and_compare(tag):
        graph.replay()
        g = _snapshot(t)
        keep = [[p for p in range(B) if (int(k) >> p) & 1] for k in g["keep_bits"]]
        assert all(len(s) == 8 for s in keep), (tag, keep)
        tr = fo.focus_step(cfg, W, pool, states, keep_override=keep)
        assert [int(x) for x in g["cu_seqlens"]] == tr.cu, tag
        T = tr.cu[-1]
        for b in range(n):
            ref = tr.delta_I[b]
            assert np.max(np.abs(g["delta_I"][b] - ref)) <= 4e-2 * np.max(np.abs(tr.I_evict[b])), tag
        err = max(float(np.max(np.abs(g["logits"][r] - tr.logits[r])) / np.max(np.abs(tr.logits[r]))) for r in range(T))
        print(tag, "logits max rel err", err, flush=True)
        assert err <= 2e-2, (tag, err)
        return g

    g = replay_and_compare("captured prefix")
    # complete the block on both sides with the same tokens, finalise: the block becomes prefix
    toks = [[1 + (7 * b + 13 * p) % (wl.vocab - 2) for p in range(B)] for b in range(n)]
    for b in range(n):
        s = sess.focus.focus_get_state(b)
        s.mask_bits = 0
        for p in range(B):
            s.tokens[p] = toks[b][p]
        sess.focus.focus_set_state(b, s)
        states[b].tokens, states[b].masked = list(toks[b]), [False] * B
    fin = torch.zeros(n, dtype=torch.int32, device=DEV)
    sess.focus.focus_finalize_blocks(n, fin)
    assert fin.cpu().tolist() == [1] * n
    assert fo.finalize_blocks(cfg, W, pool, states) == [True] * n
    assert all(sess.focus.focus_get_state(b).prefix_len == prefix + B for b in range(n))
    replay_and_compare("prefix grown by one block")
    sess.focus.focus_free()
