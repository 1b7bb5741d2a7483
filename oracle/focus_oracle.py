"""CPU oracle for one FOCUS block-diffusion decode step.  TEST INFRASTRUCTURE ONLY.

This file is the plain, slow, float64 statement of what the decode step computes, written from
the paper (FOCUS, arXiv 2601.23278).  It shares no code with the HIP library and is imported only
by tests, by the smoke check and by the benchmark's CPU-baseline leg; the product path never
calls it.

What follows the paper directly (each function cites its passage):
  * token importance, Eq. 2 / App. E.2.1            -> importance()
  * importance delta, Eq. 3                          -> focus_step()
  * dynamic budget, Eq. 4-5, Alg. 1 phase 2          -> n_sigma(), budget()
  * top-K + AR-context + placeholder integrity,
    Alg. 1 phase 3, Sec. 4.2, App. E.2.2             -> select()
  * gather to the reduced set, packed order          -> compact()
  * reduced forward of the remaining layers          -> focus_step()
  * confidence decoding and the running mean of
    decoded tokens, Alg. 1 last lines, App. E.3.1    -> confidence(), commit()
  * Top / Random / Bottom pick of the candidates,
    Sec. 5.2                                         -> select(), selection_key()
The transformer layer itself (RMSNorm, rotate-half RoPE, grouped-query attention over an exact
prefix KV cache that is bidirectional inside the block, SwiGLU) is the textbook definition, and so
is the mixture-of-experts feed-forward of the paper's second model (Sec. 5.1): route(), moe_ffn().

Readings taken where the paper is silent are listed next to the code that takes them.

All floating point is float64.  Matrix products use numpy's matmul as a library step; there is
no blocking or fusion.  Decisions that floating point feeds (top-K order, thresholds, arg-max)
are taken on the values handed in, so a caller can hand in float32 bit patterns and get the
decision in that precision.

Parity pins (tests/test_oracle_*.py): softmax rows sum to one; sum of importance equals
B * H_q and the delta sums to zero; importance with pooling off equals a column sum of the
block-local softmax; brute-force set algebra for select(); identity of keep-all with an
independently written dense block decode; permutation invariance of compaction; page-placement
invariance; Eq. 4 hand values (alpha 1.5, mean 1 gives K 2); the running-mean recurrences; the
random pick's generator against SplitMix64's published outputs and a frequency test; the
mixture-of-experts layer against a masked dense formulation built on torch.topk, hand-worked routes,
and the dense model when all experts share one set of weights.
Whether the delta predicts decodability on trained weights is parity unpinned (no weights here).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

NEG_INF = -np.inf


# ---------------------------------------------------------------------------------------------
# configuration and state

@dataclass
class OracleConfig:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    block_size: int
    mask_token_id: int
    page_size: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0
    evict_layer: int = 1          # e: importance of layers e-1 and e decides eviction after layer e's K/V fill
    importance_mode: int = 0      # 0: delta I(e) - I(e-1) (Eq. 3); 1: raw I(e) (App. B comparison)
    maxpool_k: int = 3            # MaxPool1D window of Eq. 2 (App. F.1 fixes 3); 1 = off
    budget_mode: int = 1          # 0 TOPK, 1 RATIO, 2 DYNAMIC (Eq. 4), 3 OVERRIDE (K per sequence)
    topk: int = 0
    keep_ratio: float = 0.25
    alpha: float = 1.5
    constraints: int = 0          # bit0 AR-context preservation, bit1 placeholder integrity
    conf_threshold: float = 0.9
    placeholder_unprocessed_only: bool = False   # alternative reading of placeholder integrity
    intra_block_cache: int = 0    # 1: delayed intra-block K/V cache with the neighbour-aware stability criterion (Sec. 4.3)
    selection: int = 0            # which K masked positions are picked: 0 TOP (the method), 1 RANDOM, 2 BOTTOM (Sec. 5.2)
    selection_seed: int = 0       # RANDOM: seed of the counter-based generator
    # mixture-of-experts feed-forward (the paper's second model, Sec. 5.1, is an MoE; it gives no formulas, see moe_ffn)
    n_experts: int = 0            # E; 0 = every layer has the dense SwiGLU feed-forward
    experts_per_token: int = 0    # k
    expert_ffn: int = 0           # F_e, inner width of a routed expert
    shared_ffn: int = 0           # F_s, inner width of the always-on shared expert; 0 = none
    first_moe_layer: int = 0      # layers below it keep the dense feed-forward
    route_scale: float = 1.0      # factor on the routed experts' sum
    # Optional model of a reduced-precision activation format.  None (the default) leaves every value in float64: that is
    # the oracle.  A function (name, array) -> array is applied where an implementation that keeps activations in the
    # model's 16-bit type (the benchmark configurations fix bf16) has to round them: "normed" (RMSNorm output, the operand
    # of a projection), "qkv" (projection output), "rope" (rotated q and k), "p" (un-normalised softmax probabilities as the
    # operand of P V), "attn" (attention output), "act" (SiLU(gate) * up).  The residual stream, the softmax statistics and
    # the logits are never passed through it.  Used by oracle/drift_study.py and by the end-to-end parity tests of the
    # bf16 configurations to tell format rounding from implementation error.
    store_cast: Optional[Callable] = None


@dataclass
class SeqState:
    """Per-sequence block state (App. E.3.1): what the scheduler keeps between steps."""
    prefix_len: int
    pages: List[int]                       # physical page ids covering prefix_len + B tokens
    tokens: List[int]                      # committed id per block position (meaningless where masked)
    masked: List[bool]                     # M: position still holds the mask token
    processed: List[bool]                  # P: position has K/V in the layers above the eviction layer
    cached: Optional[List[bool]] = None    # C: position's K/V is frozen in every layer (Sec. 4.3); None = none
    token_sum: int = 0                     # running sum of tokens decoded per step
    total_steps: int = 0                   # number of steps this sequence took part in
    slot: int = 0                          # the scheduler's slot of the sequence (names its random stream)


def new_seq_state(cfg: OracleConfig, prefix_len: int, pages: Sequence[int], slot: int = 0) -> SeqState:
    B = cfg.block_size
    return SeqState(prefix_len, list(pages), [cfg.mask_token_id] * B, [True] * B, [False] * B, [False] * B, slot=slot)


class Weights:
    """Weights as float64 arrays, [out, in] row-major.  Layers are fetched through a callback so
    that a large model can be generated layer by layer; `fetch_seconds` accumulates the time the
    callback took (the benchmark subtracts it: producing inputs is not part of the step)."""

    def __init__(self, embed, lm_head, final_norm, layer_fn: Callable[[int], Dict[str, np.ndarray]]):
        self.embed, self.lm_head, self.final_norm = embed, lm_head, final_norm
        self._layer_fn = layer_fn
        self.fetch_seconds = 0.0

    def layer(self, l: int) -> Dict[str, np.ndarray]:
        import time
        t0 = time.perf_counter()
        w = self._layer_fn(l)
        self.fetch_seconds += time.perf_counter() - t0
        return w


class KVPool:
    """Paged K/V store: per layer a dict page id -> array [2, H_kv, page_size, D] (0 = K, 1 = V)."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self.layers: List[Dict[int, np.ndarray]] = [dict() for _ in range(cfg.n_layers)]

    def page(self, l: int, pid: int) -> np.ndarray:
        d = self.layers[l]
        if pid not in d:
            c = self.cfg
            d[pid] = np.zeros((2, c.n_kv_heads, c.page_size, c.head_dim))
        return d[pid]

    def write(self, l: int, pages: Sequence[int], tok: int, k: np.ndarray, v: np.ndarray):
        P = self.cfg.page_size
        pg = self.page(l, pages[tok // P])
        pg[0, :, tok % P, :] = k
        pg[1, :, tok % P, :] = v

    def read(self, l: int, pages: Sequence[int], toks: Sequence[int]):
        """K, V of the listed token slots: two arrays [len(toks), H_kv, D]."""
        P = self.cfg.page_size
        c = self.cfg
        K = np.empty((len(toks), c.n_kv_heads, c.head_dim))
        V = np.empty_like(K)
        for i, t in enumerate(toks):
            pg = self.page(l, pages[t // P])
            K[i] = pg[0, :, t % P, :]
            V[i] = pg[1, :, t % P, :]
        return K, V


# ---------------------------------------------------------------------------------------------
# textbook pieces

def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * w over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half rotary embedding.  x [r, H, D], pos [r] absolute positions.
    Pair (i, i + D/2) is rotated by pos * base^(-2i/D)."""
    D = x.shape[-1]
    half = D // 2
    inv_freq = base ** (-(np.arange(half, dtype=np.float64) * 2.0) / D)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]           # [r, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def maxpool1d_same(s: np.ndarray, k: int) -> np.ndarray:
    """Stride-1 max pooling along the last axis with window k (odd), padded with -inf so the
    length is kept: out[..., j] = max(s[..., j-(k-1)/2 .. j+(k-1)/2])."""
    if k <= 1:
        return s
    r = (k - 1) // 2
    n = s.shape[-1]
    out = np.full_like(s, NEG_INF)
    for d in range(-r, r + 1):
        lo, hi = max(0, -d), min(n, n - d)
        out[..., lo:hi] = np.maximum(out[..., lo:hi], s[..., lo + d:hi + d])
    return out


# ---------------------------------------------------------------------------------------------
# Eq. 2: token importance

def importance(q: np.ndarray, k: np.ndarray, maxpool_k: int = 3) -> np.ndarray:
    """Eq. 2 (and its restatement in App. E.2.1): I_j = sum_i sum_h Softmax_j(MaxPool1D_j(S^h_ij)).

    q [B, H_q, D], k [B, H_kv, D] are the block's (rotated) queries and keys of one layer.
    S^h_ij = q_i^h . k_j^(h // g) / sqrt(D).  Readings: i and j both run over all B positions of
    the block; the softmax normalises over the B block keys only (so each row contributes one
    unit of mass and the deltas are zero-sum, as Sec. 4.1 says of them); pooling runs along the
    key index on the pre-softmax scores, stride 1, same length."""
    Hq, D = q.shape[1], q.shape[2]
    B = k.shape[0]                      # keys: every block position; queries: the rows that are forwarded (all B unless
    g = Hq // k.shape[1]                # some positions are cached, Sec. 4.3)
    I = np.zeros(B)
    for h in range(Hq):
        S = q[:, h, :] @ k[:, h // g, :].T / math.sqrt(D)          # [i, j]
        I += softmax_rows(maxpool1d_same(S, maxpool_k)).sum(axis=0)
    return I


# ---------------------------------------------------------------------------------------------
# Eq. 4-5: budget

def mean_std_sequential(x: Sequence[float]):
    """Population mean and standard deviation, accumulated left to right in float64."""
    n = len(x)
    s = 0.0
    for v in x:
        s = s + float(v)
    mu = s / n
    ss = 0.0
    for v in x:
        d = float(v) - mu
        ss = ss + d * d
    return mu, math.sqrt(ss / n)


def n_sigma(dI: Sequence[float], masked: Sequence[bool]) -> int:
    """Eq. 5: number of masked positions whose delta is at least one standard deviation above the
    block mean.  Reading: mean and (population) std over all B positions (App. E.2.2 calls them
    block-wise; Eq. 5 omits the mean because the deltas are zero-mean)."""
    mu, sd = mean_std_sequential(dI)
    thr = mu + sd
    return sum(1 for j, m in enumerate(masked) if m and float(dI[j]) >= thr)


def budget(cfg: OracleConfig, dI: Sequence[float], masked: Sequence[bool], token_sum: int, total_steps: int,
           k_override: Optional[int] = None) -> int:
    """Retention budget K.  Mode 2 is Eq. 4 / Alg. 1 phase 2: K = min(B, max(ceil(alpha * Nbar), N_sigma)),
    Nbar = token_sum / total_steps, or 1 on a sequence's first step.  Modes 0, 1, 3 are the fixed budgets
    of the benchmark configurations (top-k; ceil(ratio * B); a per-sequence value)."""
    B = cfg.block_size
    if cfg.budget_mode == 0:
        K = cfg.topk
    elif cfg.budget_mode == 1:
        K = int(math.ceil(float(np.float32(cfg.keep_ratio)) * B))
    elif cfg.budget_mode == 3:
        K = int(k_override)
    else:
        nbar = (float(token_sum) / float(total_steps)) if total_steps > 0 else 1.0
        k_hist = int(math.ceil(float(np.float32(cfg.alpha)) * nbar))
        K = max(k_hist, n_sigma(dI, masked))
    return max(0, min(B, K))


# ---------------------------------------------------------------------------------------------
# Alg. 1 phase 3: selection

_MASK64 = (1 << 64) - 1


def selection_key(seed: int, slot: int, step: int, j: int) -> int:
    """64-bit random key of block position j for the RANDOM strategy: output number c + 1 of the SplitMix64
    generator (Steele, Lea, Flood 2014) started at `seed`, with the counter c = (slot * 2^32 + step) * 64 + j,
    step = the sequence's total_steps before this step.  Reading: the paper only says K candidates are drawn at
    random; a counter-based stream keeps the draw a pure function of (seed, slot, step, position)."""
    c = ((((slot << 32) + step) << 6) + j) & _MASK64
    z = (seed + (c + 1) * 0x9E3779B97F4A7C15) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def select(cfg: OracleConfig, dI: Sequence[float], masked: Sequence[bool], processed: Sequence[bool],
           K: int, cached: Optional[Sequence[bool]] = None, rand_keys: Optional[Sequence[int]] = None) -> List[int]:
    """The retained set S of one sequence, ascending.

    K >= B keeps the whole block (no eviction: the step is the dense block decode).  Otherwise the
    min(K, |M|) masked positions with the largest delta are taken (ties: lower index first; NaN
    ranks below every number), then, per Alg. 1: predecessors i-1 of those picks (bit0), then every
    masked j below max(S) (bit1).  The predecessor of position 0 lies in the prefix; predecessors are
    added once, for the top-K picks only.

    cfg.selection swaps the pick for the validation of Sec. 5.2: BOTTOM takes the min(K, |M|) masked positions
    with the smallest delta (ties: lower index first; NaN still ranks last), RANDOM the ones with the largest
    rand_keys (ties: lower index first).  Everything after the pick is unchanged."""
    B = cfg.block_size
    cached = [False] * B if cached is None else cached
    uncached = [j for j in range(B) if not cached[j]]
    # with the intra-block cache, decoded tokens that are not frozen yet stay in: they are owed the forward with
    # their final token in every layer (Sec. 4.3 "decoded and forwarded one additional time")
    owed = [j for j in uncached if not masked[j]] if cfg.intra_block_cache else []
    if K >= B:
        return uncached
    cand = [j for j in range(B) if masked[j]]
    if K <= 0 or not cand:
        return owed

    def key(j):
        if cfg.selection == 1:
            return (-int(rand_keys[j]), j)
        v = float(dI[j])
        if cfg.selection == 2:
            return ((v if v == v else -NEG_INF), j)
        return (-(v if v == v else NEG_INF), j)
    top = sorted(cand, key=key)[:min(K, len(cand))]
    S = set(top)
    if cfg.constraints & 1:
        S |= {i - 1 for i in top if i >= 1 and not cached[i - 1]}
    if cfg.constraints & 2:
        mx = max(S)
        for j in range(mx):
            if masked[j] and (not cfg.placeholder_unprocessed_only or not processed[j]):
                S.add(j)
    return sorted(S | set(owed))


def compact(keep: Sequence[Sequence[int]], B: int):
    """Packed order of the survivors: sequences ascending, positions ascending inside a sequence.
    Returns cu (exclusive prefix sum of the counts, length n+1) and row_map[r] = b * B + p."""
    cu = [0]
    row_map = []
    for b, S in enumerate(keep):
        cu.append(cu[-1] + len(S))
        row_map.extend(b * B + p for p in S)
    return cu, row_map


# ---------------------------------------------------------------------------------------------
# decode and verify

def confidence(logits: np.ndarray):
    """Per row: probability of the most likely token (1 / sum exp(logit - max)) and its id
    (lowest id on ties)."""
    m = np.max(logits, axis=-1, keepdims=True)
    conf = 1.0 / np.sum(np.exp(logits - m), axis=-1)
    return conf, np.argmax(logits, axis=-1)


def commit(cfg: OracleConfig, st: SeqState, S: Sequence[int], conf: Sequence[float], tok: Sequence[int]) -> List[int]:
    """Confidence-based parallel decoding on the retained rows of one sequence (Alg. 1 Decode_and_Verify)
    and the running statistics of App. E.3.1.  conf/tok are aligned with S.

    Masked survivors with confidence >= threshold are unmasked with their arg-max token.  If none
    passes, the single most confident masked survivor is unmasked (ties: lower position) so that a
    block always finishes.  token_sum += number unmasked, total_steps += 1 whenever S is not empty."""
    if len(S) == 0:
        return []
    thr = float(np.float32(cfg.conf_threshold))
    cand = [(i, p) for i, p in enumerate(S) if st.masked[p]]
    D = [(i, p) for i, p in cand if float(conf[i]) >= thr]
    if not D and cand:
        best = cand[0]
        for i, p in cand[1:]:
            if float(conf[i]) > float(conf[best[0]]):
                best = (i, p)
        D = [best]
    for i, p in D:
        st.tokens[p] = int(tok[i])
        st.masked[p] = False
    st.token_sum += len(D)
    st.total_steps += 1
    return [p for _, p in D]


# ---------------------------------------------------------------------------------------------
# transformer layer on a set of rows

def _cast(cfg: OracleConfig, name: str, x: np.ndarray) -> np.ndarray:
    return x if cfg.store_cast is None else cfg.store_cast(name, x)


def _attention(cfg: OracleConfig, q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """q [r, H_q, D] over keys/values [t, H_kv, D]: one ordinary softmax per (row, head) over all t
    keys (prefix and visible block positions alike; no mask inside the block)."""
    r, Hq, D = q.shape
    g = Hq // K.shape[1]
    out = np.empty((r, Hq, D))
    for h in range(Hq):
        S = q[:, h, :] @ K[:, h // g, :].T / math.sqrt(D)
        if cfg.store_cast is None:
            out[:, h, :] = softmax_rows(S) @ V[:, h // g, :]
        else:       # format model: the probabilities are rounded as an operand, their sum is not
            E = np.exp(S - np.max(S, axis=-1, keepdims=True))
            out[:, h, :] = (cfg.store_cast("p", E) @ V[:, h // g, :]) / np.sum(E, axis=-1, keepdims=True)
    return _cast(cfg, "attn", out)


def _project_qkv(cfg: OracleConfig, w: Dict[str, np.ndarray], X: np.ndarray, abs_pos: np.ndarray):
    u = _cast(cfg, "normed", rmsnorm(X, w["attn_norm"], cfg.rms_eps))
    qkv = _cast(cfg, "qkv", u @ w["w_qkv"].T)
    Hq, Hkv, D = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    q = qkv[:, :Hq * D].reshape(-1, Hq, D)
    k = qkv[:, Hq * D:(Hq + Hkv) * D].reshape(-1, Hkv, D)
    v = qkv[:, (Hq + Hkv) * D:].reshape(-1, Hkv, D)
    return _cast(cfg, "rope", rope(q, abs_pos, cfg.rope_base)), _cast(cfg, "rope", rope(k, abs_pos, cfg.rope_base)), v


def swiglu(u: np.ndarray, w_gate_up: np.ndarray, w_down: np.ndarray, act_cast=None) -> np.ndarray:
    """SwiGLU feed-forward: (silu(u Wg^T) * (u Wu^T)) Wd^T with w_gate_up = [Wg; Wu] stacked by rows.
    act_cast: optional format model applied to silu(gate) * up (OracleConfig.store_cast)."""
    F = w_gate_up.shape[0] // 2
    gu = u @ w_gate_up.T
    act = silu(gu[:, :F]) * gu[:, F:]
    return (act if act_cast is None else act_cast("act", act)) @ w_down.T


def route(cfg: OracleConfig, logits: np.ndarray, forced: Optional[Sequence[int]] = None):
    """Experts and mixing weights of one row from its router logits [E].

    The k experts with the largest router probability p = softmax(logits), taken in descending order (ties: lower
    expert first; the decision is made on the logits, which order the same way), or the `forced` list in its own
    order (teacher forcing).  Weights: p over the chosen experts, renormalised to sum to one, times route_scale."""
    E = logits.shape[0]
    p = softmax_rows(logits[None, :])[0]
    chosen = list(forced) if forced is not None else \
        sorted(range(E), key=lambda i: (-float(logits[i]), i))[:cfg.experts_per_token]
    tot = sum(float(p[i]) for i in chosen)
    return chosen, [float(np.float32(cfg.route_scale)) * float(p[i]) / tot for i in chosen]


def moe_ffn(cfg: OracleConfig, w: Dict[str, np.ndarray], u: np.ndarray, forced=None):
    """Mixture-of-experts feed-forward on normalised rows u [r, h].

    Reading (the paper evaluates an MoE diffusion model, Sec. 5.1, without stating its layer): the common
    token-choice layer.  A linear router scores E experts per row, route() picks k of them with weights, each
    expert is a SwiGLU feed-forward of inner width F_e, the row's output is the weighted sum of its experts'
    outputs plus, when F_s > 0, a shared SwiGLU expert that every row goes through.
    forced[i]: expert list to use for row i instead of the router's pick.  Returns (y, experts, weights, router logits)."""
    r = u.shape[0]
    logits = u @ w["w_router"].T
    y = np.zeros((r, cfg.hidden))
    experts, weights = [], []
    for i in range(r):
        ch, wt = route(cfg, logits[i], None if forced is None else forced[i])
        experts.append(ch)
        weights.append(wt)
        for e, g in zip(ch, wt):
            y[i] += g * swiglu(u[i:i + 1], w["w_expert_gate_up"][e], w["w_expert_down"][e], cfg.store_cast)[0]
    if cfg.shared_ffn > 0:
        y += swiglu(u, w["w_shared_gate_up"], w["w_shared_down"], cfg.store_cast)
    return y, experts, weights, logits


def _finish_layer(cfg: OracleConfig, w: Dict[str, np.ndarray], X: np.ndarray, attn: np.ndarray,
                  layer: int = 0, row_ids: Optional[Sequence[int]] = None, route_override=None, route_log=None) -> np.ndarray:
    """Output projection, residual, then the feed-forward (dense, or mixture-of-experts from first_moe_layer on) and its
    residual.  row_ids[i] = b * B + p names row i for route_override[layer][row id] and for route_log[layer]."""
    X = X + attn.reshape(X.shape[0], cfg.n_q_heads * cfg.head_dim) @ w["w_o"].T      # explicit width: a step may have no rows
    u = _cast(cfg, "normed", rmsnorm(X, w["mlp_norm"], cfg.rms_eps))
    if cfg.n_experts > 0 and layer >= cfg.first_moe_layer:
        forced = None if route_override is None else [route_override[layer][rid] for rid in row_ids]
        y, experts, weights, logits = moe_ffn(cfg, w, u, forced)
        if route_log is not None:
            for i, rid in enumerate(row_ids):
                route_log.setdefault(layer, {})[rid] = (experts[i], weights[i], logits[i])
        return X + y
    return X + swiglu(u, w["w_gate_up"], w["w_down"], cfg.store_cast)


@dataclass
class StepTrace:
    """Everything a step decided or produced, for stage-by-stage comparison."""
    I_prev: List[np.ndarray] = field(default_factory=list)    # per sequence, importance at layer e-1
    I_evict: List[np.ndarray] = field(default_factory=list)   # per sequence, importance at layer e
    delta_I: List[np.ndarray] = field(default_factory=list)
    K: List[int] = field(default_factory=list)
    keep: List[List[int]] = field(default_factory=list)
    uncached: List[List[int]] = field(default_factory=list)  # per sequence, the positions forwarded through layers <= e
    cu: List[int] = field(default_factory=list)
    row_map: List[int] = field(default_factory=list)
    hidden_full: Optional[np.ndarray] = None                   # [n*B, h] residual stream entering layer e
    hidden_packed: Optional[np.ndarray] = None                 # [T', h] residual stream after the last layer
    hidden_entering: Dict[int, np.ndarray] = field(default_factory=dict)   # layer l > e -> [T', h] stream entering it
    logits: Optional[np.ndarray] = None                        # [T', V]
    conf: Optional[np.ndarray] = None
    argmax: Optional[np.ndarray] = None
    committed: List[List[int]] = field(default_factory=list)  # per sequence, positions unmasked this step
    n_decoded: List[int] = field(default_factory=list)
    route: Dict[int, Dict[int, tuple]] = field(default_factory=dict)   # MoE layer -> row id b * B + p -> (experts, weights, router logits)


def focus_step(cfg: OracleConfig, W: Weights, pool: KVPool, seqs: List[SeqState],
               k_override: Optional[Sequence[int]] = None,
               keep_override: Optional[Sequence[Sequence[int]]] = None,
               score_cast=None, conf_cast=None, record_layers=None, route_override=None) -> StepTrace:
    """One FOCUS inference step (Alg. 1) for a batch of sequences, in place on `seqs` and `pool`.

    Order of work, as in Alg. 1 and App. C: layers below the eviction layer e run on the whole
    block; layer e projects q, k, v for the whole block and fills its K/V before eviction; the
    importance of layers e-1 and e gives the delta; budget; selection; gather; the rest of layer e
    and all later layers run on the retained rows only; decode and verify; statistics.

    Which in-block keys a retained row sees: in layers <= e all B (they were just refreshed); in
    layers > e the positions retained now or in an earlier step of this block (their K/V there
    is the latest one written; positions never retained have none and are left out).

    keep_override: per-sequence retained sets to use instead of budget()+select() (teacher forcing).
    score_cast / conf_cast: optional functions applied to the delta and to the confidences before
    the integer decisions (e.g. rounding to float32 so both sides decide in the same precision).
    record_layers: layers (> e) whose incoming residual stream is kept in the trace.
    route_override: mixture-of-experts layers only: route_override[l][b * B + p] = the experts row (b, p) uses in layer l
    instead of the router's pick (teacher forcing); the trace's `route` records what every row used."""
    B, e = cfg.block_size, cfg.evict_layer
    n = len(seqs)
    tr = StepTrace()
    if cfg.importance_mode == 0 and e < 1:
        raise ValueError("importance delta needs an eviction layer >= 1")
    if e >= cfg.n_layers:
        raise ValueError("eviction layer outside the model")

    # rows of the layers up to e: the positions whose K/V is not frozen (all B without the intra-block cache)
    for st in seqs:
        if st.cached is None:
            st.cached = [False] * B
    U = [[p for p in range(B) if not st.cached[p]] for st in seqs]
    tr.uncached = U
    cuU = [0]
    for u in U:
        cuU.append(cuU[-1] + len(u))
    # block input: mask embedding where masked, committed token's embedding elsewhere
    ids = [[cfg.mask_token_id if st.masked[p] else st.tokens[p] for p in U[b]] for b, st in enumerate(seqs)]
    X = np.concatenate([W.embed[np.array(row, dtype=np.int64)].reshape(len(row), cfg.hidden) for row in ids], axis=0) \
        if n else np.zeros((0, cfg.hidden))
    abs_pos = np.array([st.prefix_len + p for b, st in enumerate(seqs) for p in U[b]], dtype=np.int64)
    full_ids = [b * B + p for b in range(n) for p in U[b]]

    def block_keys(l, st):
        Kc, _ = pool.read(l, st.pages, [st.prefix_len + p for p in range(B)])
        return Kc

    # layers 0 .. e-1 on those rows; they see the prefix and all B in-block keys (frozen ones from the cache)
    for l in range(e):
        w = W.layer(l)
        q, k, v = _project_qkv(cfg, w, X, abs_pos)
        attn = np.empty_like(q)
        for b, st in enumerate(seqs):
            sl = slice(cuU[b], cuU[b + 1])
            for i, p in enumerate(U[b]):
                pool.write(l, st.pages, st.prefix_len + p, k[sl.start + i], v[sl.start + i])
            if l == e - 1 and cfg.importance_mode == 0:
                tr.I_prev.append(importance(q[sl], block_keys(l, st), cfg.maxpool_k))
            Kc, Vc = pool.read(l, st.pages, list(range(st.prefix_len + B)))
            attn[sl] = _attention(cfg, q[sl], Kc, Vc)
        X = _finish_layer(cfg, w, X, attn, l, full_ids, route_override, tr.route)
    tr.hidden_full = X.copy()

    # layer e: projections and K/V fill for those rows, importance, delta
    w = W.layer(e)
    q, k, v = _project_qkv(cfg, w, X, abs_pos)
    for b, st in enumerate(seqs):
        sl = slice(cuU[b], cuU[b + 1])
        for i, p in enumerate(U[b]):
            pool.write(e, st.pages, st.prefix_len + p, k[sl.start + i], v[sl.start + i])
        Ie = importance(q[sl], block_keys(e, st), cfg.maxpool_k)
        tr.I_evict.append(Ie)
        d = Ie - tr.I_prev[b] if cfg.importance_mode == 0 else Ie.copy()
        tr.delta_I.append(score_cast(d) if score_cast is not None else d)

    # budget and selection
    for b, st in enumerate(seqs):
        if keep_override is not None:
            S = sorted(int(p) for p in keep_override[b])
            tr.K.append(len(S))
        else:
            K = budget(cfg, tr.delta_I[b], st.masked, st.token_sum, st.total_steps,
                       None if k_override is None else k_override[b])
            tr.K.append(K)
            rk = [selection_key(cfg.selection_seed, st.slot, st.total_steps, j) for j in range(B)] \
                if cfg.selection == 1 else None
            S = select(cfg, tr.delta_I[b], st.masked, st.processed, K, st.cached, rk)
        tr.keep.append(S)
        for p in S:
            st.processed[p] = True
    tr.cu, tr.row_map = compact(tr.keep, B)
    rows = np.array([cuU[b] + U[b].index(p) for b in range(n) for p in tr.keep[b]], dtype=np.int64)

    # gather; rest of layer e on the retained rows (they see all B keys of layer e)
    Xp, qp = X[rows], q[rows]
    attn = np.empty_like(qp)
    for b, st in enumerate(seqs):
        sl = slice(tr.cu[b], tr.cu[b + 1])
        if sl.stop > sl.start:
            Kc, Vc = pool.read(e, st.pages, list(range(st.prefix_len + B)))
            attn[sl] = _attention(cfg, qp[sl], Kc, Vc)
    Xp = _finish_layer(cfg, w, Xp, attn, e, tr.row_map, route_override, tr.route)

    # layers e+1 .. on the retained rows
    for l in range(e + 1, cfg.n_layers):
        if record_layers is not None and l in record_layers:
            tr.hidden_entering[l] = Xp.copy()
        w = W.layer(l)
        abs_pos = np.array([seqs[r // B].prefix_len + r % B for r in tr.row_map], dtype=np.int64)
        q, k, v = _project_qkv(cfg, w, Xp, abs_pos)
        attn = np.empty_like(q)
        for b, st in enumerate(seqs):
            sl = slice(tr.cu[b], tr.cu[b + 1])
            if sl.stop == sl.start:
                continue
            for i, p in enumerate(tr.keep[b]):
                pool.write(l, st.pages, st.prefix_len + p, k[sl.start + i], v[sl.start + i])
            vis = list(range(st.prefix_len)) + [st.prefix_len + p for p in range(B) if st.processed[p]]
            Kc, Vc = pool.read(l, st.pages, vis)
            attn[sl] = _attention(cfg, q[sl], Kc, Vc)
        Xp = _finish_layer(cfg, w, Xp, attn, l, tr.row_map, route_override, tr.route)
    tr.hidden_packed = Xp

    # decode and verify
    logits = _cast(cfg, "normed", rmsnorm(Xp, W.final_norm, cfg.rms_eps)) @ W.lm_head.T
    tr.logits = logits
    conf, am = confidence(logits) if len(rows) else (np.zeros(0), np.zeros(0, dtype=np.int64))
    tr.conf = conf_cast(conf) if conf_cast is not None else conf
    tr.argmax = am
    for b, st in enumerate(seqs):
        sl = slice(tr.cu[b], tr.cu[b + 1])
        unmasked_before = [not m for m in st.masked]
        D = commit(cfg, st, tr.keep[b], tr.conf[sl], am[sl])
        tr.committed.append(D)
        tr.n_decoded.append(len(D))
        if cfg.intra_block_cache:
            # neighbour-aware stability (Sec. 4.3, App. E.3.1): a position is frozen once it and its right neighbour
            # were both decoded before this step, i.e. both went through this forward with their final tokens
            for p in tr.keep[b]:
                if unmasked_before[p] and (p == B - 1 or unmasked_before[p + 1]):
                    st.cached[p] = True
    return tr


# ---------------------------------------------------------------------------------------------
# prefix cache

def prefill(cfg: OracleConfig, W: Weights, pool: KVPool, seqs: List[SeqState], prompts: Sequence[Sequence[int]]):
    """Exact prefix K/V of a block-diffusion model: the prompt is cut into consecutive blocks of B
    tokens (the last may be short); a block attends to all earlier blocks and, bidirectionally, to
    itself.  Writes K/V of token t at slot t of every layer."""
    B = cfg.block_size
    for st, toks in zip(seqs, prompts):
        assert len(toks) == st.prefix_len
        for c0 in range(0, len(toks), B):
            blk = list(toks[c0:c0 + B])
            X = W.embed[np.array(blk)]
            pos = c0 + np.arange(len(blk))
            for l in range(cfg.n_layers):
                w = W.layer(l)
                q, k, v = _project_qkv(cfg, w, X, pos)
                for i in range(len(blk)):
                    pool.write(l, st.pages, c0 + i, k[i], v[i])
                Kc, Vc = pool.read(l, st.pages, list(range(c0 + len(blk))))
                X = _finish_layer(cfg, w, X, _attention(cfg, q, Kc, Vc), l)


def finalize_blocks(cfg: OracleConfig, W: Weights, pool: KVPool, seqs: List[SeqState]) -> List[bool]:
    """Multi-block generation (the engine loop around Alg. 1, App. E.3.1 "state persistence and reset"): a
    sequence whose block has no masked position left gets one last forward of the whole block with its
    committed tokens through every layer, so that the K/V the block leaves behind is the exact K/V of those
    tokens (each saw the final tokens of its block); then the block becomes part of the prefix
    (prefix_len += B) and a new all-masked block starts.  The running statistics persist.  Sequences that
    still have masked positions, or whose page list has no room for another block, are left untouched.
    Returns which sequences were finalized."""
    B = cfg.block_size
    done = []
    for st in seqs:
        room = (st.prefix_len + 2 * B) <= len(st.pages) * cfg.page_size
        if any(st.masked) or not room:
            done.append(False)
            continue
        rows_p = [p for p in range(B) if not (st.cached and st.cached[p])]      # frozen positions keep their K/V
        X = W.embed[np.array([st.tokens[p] for p in rows_p], dtype=np.int64)].reshape(len(rows_p), cfg.hidden)
        pos = st.prefix_len + np.array(rows_p, dtype=np.int64)
        for l in range(cfg.n_layers):
            w = W.layer(l)
            q, k, v = _project_qkv(cfg, w, X, pos)
            for i, p in enumerate(rows_p):
                pool.write(l, st.pages, st.prefix_len + p, k[i], v[i])
            Kc, Vc = pool.read(l, st.pages, list(range(st.prefix_len + B)))
            X = _finish_layer(cfg, w, X, _attention(cfg, q, Kc, Vc), l)
        st.prefix_len += B
        st.tokens = [cfg.mask_token_id] * B
        st.masked = [True] * B
        st.processed = [False] * B
        st.cached = [False] * B
        done.append(True)
    return done
