"""Glue between the seeded input recipes and the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Builds oracle configs, float64 weights and the oracle's paged K/V pool from a `focus_inputs.Workload`.
The same recipes feed the HIP library in the GPU tests, so both sides see identical bits.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

from focus_inputs import Workload
from . import focus_oracle as fo


def oracle_config(wl: Workload, **over) -> fo.OracleConfig:
    cfg = fo.OracleConfig(
        n_layers=wl.n_layers, hidden=wl.hidden, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
        head_dim=wl.head_dim, ffn=wl.ffn, vocab=wl.vocab, block_size=wl.block_size,
        mask_token_id=wl.mask_token_id, page_size=wl.page_size, rms_eps=wl.rms_eps, rope_base=wl.rope_base,
        evict_layer=wl.evict_layer, importance_mode=wl.importance_mode, maxpool_k=wl.maxpool_k,
        budget_mode=wl.budget_mode, topk=wl.topk, keep_ratio=wl.keep_ratio, alpha=wl.alpha,
        constraints=wl.constraints, conf_threshold=wl.conf_threshold, intra_block_cache=wl.intra_block_cache,
        selection=wl.selection, selection_seed=wl.selection_seed, n_experts=wl.n_experts,
        experts_per_token=wl.experts_per_token, expert_ffn=wl.expert_ffn, shared_ffn=wl.shared_ffn,
        first_moe_layer=wl.first_moe_layer, route_scale=wl.route_scale)
    for k, v in over.items():
        setattr(cfg, k, v)
    return cfg


def _f64(t) -> np.ndarray:
    return t.to(dtype=__import__("torch").float64).numpy()


class LazyRows:
    """Embedding table whose rows are generated when they are indexed (a 150k x 4096 table is 5 GB in
    float64 and a step only looks up a handful of ids)."""

    def __init__(self, wl: Workload):
        self.wl = wl

    def __getitem__(self, ids) -> np.ndarray:
        from focus_inputs import TID_EMBED, WEIGHT_STD, normal_values
        h = self.wl.hidden
        rows = [_f64(normal_values(self.wl.seed, TID_EMBED, int(i) * h, h, WEIGHT_STD, dtype=self.wl.torch_dtype))
                for i in np.asarray(ids).reshape(-1)]
        return np.stack(rows) if rows else np.zeros((0, h))


def oracle_weights(wl: Workload, cache_layers: bool = True, lazy_embed: bool = False) -> fo.Weights:
    """Float64 copies of the workload's weights (bf16 workloads: the bf16 bit patterns widened).
    Layers are generated on first use; with cache_layers=False each fetch regenerates (large models)."""
    cache: Dict[int, Dict[str, np.ndarray]] = {}
    ones = np.ones(wl.hidden)

    def layer(l: int):
        if l in cache:
            return cache[l]
        moe = wl.is_moe_layer(l)
        w = {k: _f64(wl.layer_weight(l, k)) for k in (("w_qkv", "w_o") if moe else ("w_qkv", "w_o", "w_gate_up", "w_down"))}
        if moe:
            w.update({k: _f64(wl.moe_weight(l, k)) for k in wl.moe_weight_shapes()})
        w["attn_norm"] = ones
        w["mlp_norm"] = ones
        if cache_layers:
            cache[l] = w
        return w

    return fo.Weights(LazyRows(wl) if lazy_embed else _f64(wl.embed()), _f64(wl.lm_head()), ones, layer)


def oracle_batch(wl: Workload, seq_ids: Optional[Sequence[int]] = None, lazy_embed: bool = False):
    """Oracle pool + per-sequence states for the listed sequences of the workload's batch (default all),
    with the prefix K/V in place: seeded synthetic pages, or a real prefill of the seeded prompts.
    Returns (cfg, weights, pool, states, prefix_lens, page_tables, n_pages_total)."""
    cfg = oracle_config(wl)
    W = oracle_weights(wl, cache_layers=wl.n_layers <= 8, lazy_embed=lazy_embed)
    lens = wl.prefix_lens()
    tables, n_pages = wl.page_tables(lens)
    ids = list(range(wl.batch)) if seq_ids is None else list(seq_ids)
    pool = fo.KVPool(cfg)
    states = [fo.new_seq_state(cfg, lens[b], tables[b], slot=i) for i, b in enumerate(ids)]
    if wl.prefill == "synthetic":
        for l in range(wl.n_layers):
            for b in ids:
                for pid in tables[b]:
                    pool.layers[l][pid] = _f64(wl.kv_page(l, pid, n_pages))
    else:
        prompts = wl.prompt_tokens(lens)
        fo.prefill(cfg, W, pool, states, [prompts[b] for b in ids])
    return cfg, W, pool, states, lens, tables, n_pages


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to nearest-even bf16, returned as float64 (the format model of OracleConfig.store_cast)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


BF16_STORE_POINTS = ("normed", "qkv", "rope", "p", "attn", "act")


def bf16_store_cast(points: Sequence[str] = BF16_STORE_POINTS):
    """store_cast that rounds the named activation stores to bf16 and leaves the rest in float64."""
    pts = set(points)
    return lambda name, x: round_bf16(x) if name in pts else x


def oracle_weights_from_tensors(wl: Workload, lm_head, layers, max_cached_bytes: float = 8e10) -> fo.Weights:
    """Float64 weights widened from already generated tensors of the workload (any device; e.g. the ones a GPU test
    generated with the same seeded recipe, which saves generating 16 GB a second time on the host).  A widened layer
    is kept for later passes over the model while the kept layers stay below max_cached_bytes."""
    cache: Dict[int, Dict[str, np.ndarray]] = {}
    used = [0.0]
    ones = np.ones(wl.hidden)

    def layer(l: int):
        if l in cache:
            return cache[l]
        w = {k: _f64(v.cpu()) for k, v in layers[l].items() if k.startswith("w_") and not k.startswith("w_expert")}
        for k, v in layers[l].items():
            if k.startswith("w_expert"):
                w[k] = LazyExperts(v)
        w["attn_norm"] = ones
        w["mlp_norm"] = ones
        size = sum(a.nbytes for a in w.values() if isinstance(a, np.ndarray))
        if used[0] + size <= max_cached_bytes:
            cache[l] = w
            used[0] += size
        return w

    return fo.Weights(LazyRows(wl), _f64(lm_head.cpu()), ones, layer)


class LazyExperts:
    """Per-expert weight stack [E, ...] whose experts are widened to float64 when they are indexed (a step touches a few
    experts of the hundreds a mixture-of-experts layer has)."""

    def __init__(self, t):
        self.t = t
        self.cache: Dict[int, np.ndarray] = {}

    def __getitem__(self, e):
        e = int(e)
        if e not in self.cache:
            self.cache[e] = _f64(self.t[e].cpu())
        return self.cache[e]
