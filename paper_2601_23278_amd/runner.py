"""Sets up a libfocus context for a seeded synthetic workload: weights and K/V pool generated on the device
from the input recipes, sequences installed.  Used by the GPU tests, the smoke check and the benchmark."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from focus_inputs import Workload
from .binding import FOCUS_BF16, FOCUS_F32, Focus, focus_config, focus_kv_pool_bytes


def config_from_workload(wl: Workload, max_batch: int, max_prefix_len: int, n_pages: int) -> focus_config:
    c = focus_config()
    c.n_layers, c.hidden, c.n_q_heads, c.n_kv_heads, c.head_dim = wl.n_layers, wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    c.ffn, c.vocab = wl.ffn, wl.vocab
    c.dtype = FOCUS_F32 if wl.dtype == "fp32" else FOCUS_BF16
    c.rms_eps, c.rope_base = wl.rms_eps, wl.rope_base
    c.block_size, c.mask_token_id = wl.block_size, wl.mask_token_id
    c.max_batch, c.max_prefix_len, c.page_size, c.n_pages = max_batch, max_prefix_len, wl.page_size, n_pages
    c.evict_layer, c.importance_mode, c.maxpool_k = wl.evict_layer, wl.importance_mode, wl.maxpool_k
    c.budget_mode, c.topk, c.keep_ratio, c.alpha = wl.budget_mode, wl.topk, wl.keep_ratio, wl.alpha
    c.constraints, c.conf_threshold = wl.constraints, wl.conf_threshold
    c.intra_block_cache = wl.intra_block_cache
    c.selection, c.selection_seed = wl.selection, wl.selection_seed
    c.n_experts, c.experts_per_token, c.expert_ffn = wl.n_experts, wl.experts_per_token, wl.expert_ffn
    c.shared_ffn, c.first_moe_layer, c.route_scale = wl.shared_ffn, wl.first_moe_layer, wl.route_scale
    return c


@dataclass
class Session:
    wl: Workload
    focus: Focus
    prefix_lens: List[int]
    page_tables: List[List[int]]
    n_pages: int
    kv_pool: torch.Tensor
    seq_ids: List[int]
    weights: tuple = ()

    def reopen(self, **cfg_over) -> "Session":
        """Frees the context and creates a new one over the same weights, K/V pool and workspace with some
        configuration members replaced (e.g. keep_ratio), then re-installs the sequences (new block)."""
        cfg = self.focus.cfg
        for k, v in cfg_over.items():
            setattr(cfg, k, v)
        ws = self.focus.workspace
        self.focus.focus_free()
        embed, lm_head, norm, layers = self.weights
        self.focus = Focus(cfg, embed, lm_head, norm, layers, self.kv_pool, ws)
        self.focus.focus_prefill_kv(self.prefix_lens, self.page_tables, None)
        return self


def open_session(wl: Workload, device="cuda:0", seq_ids: Optional[Sequence[int]] = None, **cfg_over) -> Session:
    """Generates the workload's weights and prefix K/V on `device`, creates the context and installs the listed
    sequences of the workload's batch (default: all) in slots 0..n-1."""
    lens_all = wl.prefix_lens()
    tables_all, n_pages = wl.page_tables(lens_all)
    ids = list(range(wl.batch)) if seq_ids is None else list(seq_ids)
    lens = [lens_all[b] for b in ids]
    tables = [tables_all[b] for b in ids]
    cfg = config_from_workload(wl, max_batch=len(ids), max_prefix_len=max(lens) + wl.extra_blocks * wl.block_size, n_pages=n_pages)
    for k, v in cfg_over.items():
        setattr(cfg, k, v)
    dev = torch.device(device)
    embed, lm_head, norm = wl.embed(dev), wl.lm_head(dev), wl.norm_weight(dev)
    layers = []
    for l in range(wl.n_layers):
        moe = wl.is_moe_layer(l)
        w = {k: wl.layer_weight(l, k, dev) for k in (("w_qkv", "w_o") if moe else ("w_qkv", "w_o", "w_gate_up", "w_down"))}
        if moe:
            w.update({k: wl.moe_weight(l, k, dev) for k in wl.moe_weight_shapes()})
        w["attn_norm"], w["mlp_norm"] = norm, norm
        layers.append(w)
    pool = torch.empty((wl.n_layers, n_pages, 2, wl.n_kv_heads, wl.page_size, wl.head_dim), dtype=wl.torch_dtype, device=dev)
    assert pool.numel() * pool.element_size() == focus_kv_pool_bytes(cfg)
    if wl.prefill == "synthetic":
        wl.kv_pool_fill_(pool)
    else:
        pool.zero_()
    f = Focus(cfg, embed, lm_head, norm, layers, pool)
    prompts = None
    if wl.prefill == "prompt":
        all_prompts = wl.prompt_tokens(lens_all)
        prompts = [all_prompts[b] for b in ids]
    f.focus_prefill_kv(lens, tables, prompts)
    return Session(wl, f, lens, tables, n_pages, pool, ids, (embed, lm_head, norm, layers))
