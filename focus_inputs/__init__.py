"""Seeded synthetic inputs for the FOCUS decode step (weights, prefix KV, prompts, lengths).

This module is shared by the CPU oracle's tests and by the GPU tests / benchmark.  It holds
no arithmetic of the method itself: only a counter-based integer hash, the mapping from hash
bits to values, and the named workload recipes.  Every value is a pure function of
(seed, tensor id, flat element index), so any sub-range of any tensor can be regenerated
independently on the CPU or on the GPU and the bits agree.

Value recipe: one 64-bit hash per element; its four 16-bit fields are summed (an Irwin-Hall
sum of four uniforms), centred, and multiplied once in fp32 by a constant that gives the
requested standard deviation.  |z| <= 3.47 sigma.  bf16 tensors are the fp32 value rounded to
nearest-even once.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB


def _s64(c: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant (torch has no uint64 arithmetic)."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def _mix_py(x: int) -> int:
    x &= _M64
    x = ((x ^ (x >> 30)) * _MUL1) & _M64
    x = ((x ^ (x >> 27)) * _MUL2) & _M64
    return x ^ (x >> 31)


def stream_key(seed: int, tensor_id: int) -> int:
    """Per-(seed, tensor) 64-bit key, computed with Python integers."""
    return _mix_py(_mix_py(seed * _GOLD + 0x1234567) ^ (tensor_id * _MUL2 + 0x7654321))


def hash_py(key: int, index: int) -> int:
    """Reference big-integer form of the element hash (used by tests and for scalars)."""
    return _mix_py((index * _GOLD + key) & _M64)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def hash_t(key: int, index: torch.Tensor) -> torch.Tensor:
    """Element hash on an int64 tensor of flat indices (wrap-around arithmetic), any device."""
    x = index * _s64(_GOLD) + _s64(key)
    x = (x ^ _lsr(x, 30)) * _s64(_MUL1)
    x = (x ^ _lsr(x, 27)) * _s64(_MUL2)
    return x ^ _lsr(x, 31)


_IH_MEAN = 2 * 65535
_IH_STD = math.sqrt(4 * (65536.0 ** 2 - 1.0) / 12.0)


def normal_values(seed: int, tensor_id: int, start: int, count: int, std: float,
                  device="cpu", dtype=torch.float32) -> torch.Tensor:
    """`count` values of the stream (seed, tensor_id) starting at flat index `start`."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    h = hash_t(stream_key(seed, tensor_id), idx)
    s = (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)
    z = (s - _IH_MEAN).to(torch.float32) * float(np.float32(std / _IH_STD))
    return z.to(dtype)


def fill_normal_(out: torch.Tensor, seed: int, tensor_id: int, std: float,
                 chunk: Optional[int] = None) -> torch.Tensor:
    """Fill a contiguous tensor in place, flat index = row-major element offset.  The chunk size only
    shapes the temporaries (cache-sized on the CPU, large on the GPU); values do not depend on it."""
    flat = out.view(-1)
    n = flat.numel()
    if chunk is None:
        chunk = (1 << 18) if out.device.type == "cpu" else (1 << 26)
    for i, s in enumerate(range(0, n, chunk)):
        c = min(chunk, n - s)
        flat[s:s + c] = normal_values(seed, tensor_id, s, c, std, device=out.device, dtype=out.dtype)
        if out.device.type != "cpu" and i % 32 == 31:
            torch.cuda.synchronize(out.device)     # bounds the queue of pending launches (a profiler that counts every dispatch needs that)
    return out


def uniform_ints(seed: int, tensor_id: int, count: int, lo: int, hi: int) -> List[int]:
    """`count` integers uniform in [lo, hi] (Python ints)."""
    key = stream_key(seed, tensor_id)
    return [lo + hash_py(key, i) % (hi - lo + 1) for i in range(count)]


def log_uniform_ints(seed: int, tensor_id: int, count: int, lo: int, hi: int) -> List[int]:
    key = stream_key(seed, tensor_id)
    out = []
    for i in range(count):
        u = hash_py(key, i) / float(1 << 64)
        out.append(min(hi, max(lo, int(math.floor(math.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))))))))
    return out


def permutation(seed: int, tensor_id: int, n: int) -> List[int]:
    """Seeded permutation of range(n): argsort of per-index hashes."""
    key = stream_key(seed, tensor_id)
    return sorted(range(n), key=lambda i: (hash_py(key, i), i))


# ---------------------------------------------------------------------------------------------
# tensor ids
TID_EMBED, TID_LM_HEAD, TID_KV, TID_PROMPT, TID_PREFIX_LEN, TID_K_OVERRIDE, TID_PAGE_PERM = 1, 2, 3, 4, 5, 6, 7
TID_LAYER0 = 16           # + 8*layer + {0: w_qkv, 1: w_o, 2: w_gate_up, 3: w_down}
TID_ROUTE_OVERRIDE = 8
TID_MOE0 = 1 << 20        # + 8*layer + {0: w_router, 1: w_expert_gate_up, 2: w_expert_down, 3: w_shared_gate_up, 4: w_shared_down}
WEIGHT_STD = 0.02
KV_STD = 1.0


@dataclass(frozen=True)
class Workload:
    """Model shape, method switches and batch recipe of one named configuration."""
    name: str
    seed: int
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str                  # "fp32" | "bf16"
    rope_base: float
    rms_eps: float
    block_size: int
    mask_token_id: int
    page_size: int
    batch: int
    prefix_lo: int
    prefix_hi: int
    prefix_dist: str            # "uniform" | "loguniform" | "fixed"
    prefill: str                # "prompt" (real block-causal prefill) | "synthetic" (seeded K/V)
    evict_layer: int = 1
    importance_mode: int = 0    # 0 = I(e) - I(e-1), 1 = raw I(e)
    maxpool_k: int = 3
    budget_mode: int = 1        # 0 TOPK, 1 RATIO, 2 DYNAMIC, 3 OVERRIDE
    topk: int = 0
    keep_ratio: float = 0.25
    alpha: float = 1.5
    constraints: int = 0        # bit0 AR-context, bit1 placeholder integrity
    conf_threshold: float = 0.9
    intra_block_cache: int = 0  # 1 = delayed intra-block K/V cache with the neighbour-aware stability criterion
    selection: int = 0          # 0 TOP, 1 RANDOM, 2 BOTTOM pick of the K candidates
    selection_seed: int = 0
    n_experts: int = 0          # mixture-of-experts feed-forward from first_moe_layer on (0 = dense model)
    experts_per_token: int = 0
    expert_ffn: int = 0
    shared_ffn: int = 0
    first_moe_layer: int = 0
    route_scale: float = 1.0
    steps: int = 1
    shuffle_pages: bool = False
    extra_blocks: int = 0       # further blocks each sequence will generate (pages and positions are planned for them)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    def prefix_lens(self) -> List[int]:
        if self.prefix_dist == "fixed":
            return [self.prefix_lo] * self.batch
        if self.prefix_dist == "loguniform":
            return log_uniform_ints(self.seed, TID_PREFIX_LEN, self.batch, self.prefix_lo, self.prefix_hi)
        return uniform_ints(self.seed, TID_PREFIX_LEN, self.batch, self.prefix_lo, self.prefix_hi)

    def pages_per_seq(self, prefix_len: int) -> int:
        return (prefix_len + self.block_size * (1 + self.extra_blocks) + self.page_size - 1) // self.page_size

    def page_tables(self, prefix_lens: Optional[List[int]] = None):
        """(tables, n_pages): consecutive logical page ids per sequence, optionally mapped
        through a seeded permutation of the physical pages."""
        lens = self.prefix_lens() if prefix_lens is None else prefix_lens
        counts = [self.pages_per_seq(l) for l in lens]
        total = sum(counts)
        phys = permutation(self.seed, TID_PAGE_PERM, total) if self.shuffle_pages else list(range(total))
        tables, at = [], 0
        for c in counts:
            tables.append(phys[at:at + c])
            at += c
        return tables, total

    def k_overrides(self) -> List[int]:
        """Per-sequence budgets for budget_mode 3: uniform in [0, B], first forced 0, second forced B."""
        ks = uniform_ints(self.seed, TID_K_OVERRIDE, self.batch, 0, self.block_size)
        if self.batch >= 1:
            ks[0] = 0
        if self.batch >= 2:
            ks[1] = self.block_size
        return ks

    def prompt_tokens(self, prefix_lens: Optional[List[int]] = None) -> List[List[int]]:
        lens = self.prefix_lens() if prefix_lens is None else prefix_lens
        key = stream_key(self.seed, TID_PROMPT)
        out, at = [], 0
        for l in lens:
            out.append([1 + hash_py(key, at + i) % (self.vocab - 1) for i in range(l)])
            at += l
        return out

    # -- tensors ------------------------------------------------------------------------------
    def weight_shapes(self) -> Dict[str, tuple]:
        qkv = (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim
        return {"w_qkv": (qkv, self.hidden), "w_o": (self.hidden, self.n_q_heads * self.head_dim),
                "w_gate_up": (2 * self.ffn, self.hidden), "w_down": (self.hidden, self.ffn)}

    def layer_weight(self, layer: int, which: str, device="cpu") -> torch.Tensor:
        order = {"w_qkv": 0, "w_o": 1, "w_gate_up": 2, "w_down": 3}
        shape = self.weight_shapes()[which]
        out = torch.empty(shape, dtype=self.torch_dtype, device=device)
        return fill_normal_(out, self.seed, TID_LAYER0 + 8 * layer + order[which], WEIGHT_STD)

    def is_moe_layer(self, layer: int) -> bool:
        return self.n_experts > 0 and layer >= self.first_moe_layer

    def moe_weight_shapes(self) -> Dict[str, tuple]:
        E, Fe, Fs, h = self.n_experts, self.expert_ffn, self.shared_ffn, self.hidden
        shapes = {"w_router": (E, h), "w_expert_gate_up": (E, 2 * Fe, h), "w_expert_down": (E, h, Fe)}
        if Fs:
            shapes.update({"w_shared_gate_up": (2 * Fs, h), "w_shared_down": (h, Fs)})
        return shapes

    def moe_weight(self, layer: int, which: str, device="cpu") -> torch.Tensor:
        order = {"w_router": 0, "w_expert_gate_up": 1, "w_expert_down": 2, "w_shared_gate_up": 3, "w_shared_down": 4}
        out = torch.empty(self.moe_weight_shapes()[which], dtype=self.torch_dtype, device=device)
        return fill_normal_(out, self.seed, TID_MOE0 + 8 * layer + order[which], WEIGHT_STD)

    def route_override(self, n_seq: Optional[int] = None) -> List[List[List[int]]]:
        """Seeded forced routing [layer][row id b * B + p] -> experts_per_token distinct experts (teacher forcing)."""
        n = (self.batch if n_seq is None else n_seq) * self.block_size
        key = stream_key(self.seed, TID_ROUTE_OVERRIDE)
        out = []
        for l in range(self.n_layers):
            rows = []
            for r in range(n):
                base = (l * n + r) * self.n_experts
                ranked = sorted(range(self.n_experts), key=lambda e: (hash_py(key, base + e), e))
                rows.append(ranked[:self.experts_per_token])
            out.append(rows)
        return out

    def embed(self, device="cpu") -> torch.Tensor:
        out = torch.empty((self.vocab, self.hidden), dtype=self.torch_dtype, device=device)
        return fill_normal_(out, self.seed, TID_EMBED, WEIGHT_STD)

    def lm_head(self, device="cpu") -> torch.Tensor:
        out = torch.empty((self.vocab, self.hidden), dtype=self.torch_dtype, device=device)
        return fill_normal_(out, self.seed, TID_LM_HEAD, WEIGHT_STD)

    def norm_weight(self, device="cpu") -> torch.Tensor:
        return torch.ones((self.hidden,), dtype=self.torch_dtype, device=device)

    def kv_page_elems(self) -> int:
        return 2 * self.n_kv_heads * self.page_size * self.head_dim

    def kv_pool_fill_(self, pool: torch.Tensor) -> torch.Tensor:
        """Fill a whole pool [layer, page, page_elems] with seeded K/V.  A page holds K as [H_kv, page_size, D]
        followed by V transposed, [H_kv, D, page_size] (the library's cache layout)."""
        return fill_normal_(pool, self.seed, TID_KV, KV_STD)

    def kv_page(self, layer: int, page: int, n_pages: int, device="cpu") -> torch.Tensor:
        """One page of the seeded pool as (K, V), both [H_kv, page_size, D], same bits as kv_pool_fill_."""
        e = self.kv_page_elems()
        v = normal_values(self.seed, TID_KV, (layer * n_pages + page) * e, e, KV_STD, device=device,
                          dtype=self.torch_dtype)
        k = v[:e // 2].view(self.n_kv_heads, self.page_size, self.head_dim)
        vt = v[e // 2:].view(self.n_kv_heads, self.head_dim, self.page_size)
        return torch.stack([k, vt.transpose(1, 2)])


_SHAPE_8B = dict(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=12288, vocab=151936,
                 dtype="bf16", rope_base=1.0e6, rms_eps=1e-6, mask_token_id=151935, page_size=64,
                 prefill="synthetic")

WORKLOADS: Dict[str, Workload] = {}


def _add(w: Workload):
    WORKLOADS[w.name] = w


# benchmark configs[0]: tiny fp32 model, real prefill, 4 denoising steps.
_add(Workload(name="c1_tiny", seed=0, n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=1024,
              vocab=1024, dtype="fp32", rope_base=10000.0, rms_eps=1e-6, block_size=16, mask_token_id=0,
              page_size=16, batch=4, prefix_lo=32, prefix_hi=64, prefix_dist="uniform", prefill="prompt",
              budget_mode=1, keep_ratio=0.25, steps=4))
# configs[1]: SDAR-8B-shaped 4-layer stack, batch 32, prefix 512, B=4, top-k 2, one step.
_add(Workload(name="c2_sdar4", seed=1, n_layers=4, block_size=4, batch=32, prefix_lo=512, prefix_hi=512,
              prefix_dist="fixed", budget_mode=0, topk=2, steps=1, **_SHAPE_8B))
# configs[2]: 36 layers, batch 128, prefix U[256,2048], B=32, ratio .25, tau .9, 8 steps.
_add(Workload(name="c3_llada36", seed=2, n_layers=36, block_size=32, batch=128, prefix_lo=256, prefix_hi=2048,
              prefix_dist="uniform", budget_mode=1, keep_ratio=0.25, conf_threshold=0.9, steps=8, **_SHAPE_8B))
# configs[3]: batch 256, prefix U[512,4096], B=32, keep-ratio sweep (ratio set by the caller).
_add(Workload(name="c4_batch256", seed=3, n_layers=36, block_size=32, batch=256, prefix_lo=512, prefix_hi=4096,
              prefix_dist="uniform", budget_mode=1, keep_ratio=0.25, steps=1, **_SHAPE_8B))
# configs[4]: batch 64, prefix log-uniform [1024,32768], paged (64) with shuffled pages, B=64, per-seq K.
_add(Workload(name="c5_ragged", seed=4, n_layers=36, block_size=64, batch=64, prefix_lo=1024, prefix_hi=32768,
              prefix_dist="loguniform", budget_mode=3, keep_ratio=0.25, steps=1, shuffle_pages=True, **_SHAPE_8B))


# Second workload (Sec. 5.1): a mixture-of-experts model with the parameter counts the paper states for it, 16B in
# total and 1.4B active per token: 20 layers, hidden 2048, 256 experts of inner width 512 with 8 active plus one shared
# expert, a dense first layer; same batch recipe as the batch-256 configuration.
_add(Workload(name="c6_moe_mini", seed=5, n_layers=20, hidden=2048, n_q_heads=16, n_kv_heads=4, head_dim=128, ffn=5120,
              vocab=157184, dtype="bf16", rope_base=6.0e5, rms_eps=1e-6, mask_token_id=157183, page_size=64,
              prefill="synthetic", block_size=32, batch=256, prefix_lo=512, prefix_hi=4096, prefix_dist="uniform",
              budget_mode=1, keep_ratio=0.25, steps=1, n_experts=256, experts_per_token=8, expert_ffn=512, shared_ffn=512,
              first_moe_layer=1, route_scale=2.5))


def workload(name: str, **overrides) -> Workload:
    """A named workload, optionally with fields replaced (e.g. fewer layers or sequences)."""
    return replace(WORKLOADS[name], **overrides) if overrides else WORKLOADS[name]
