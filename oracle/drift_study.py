"""How much of the bf16 model's distance from the float64 oracle is the number format itself.  TEST INFRASTRUCTURE ONLY.

Runs the oracle's FOCUS step (Alg. 1) on one sequence of a benchmark workload several times: once in float64
(the reference), once with every activation that a bf16 implementation keeps in memory rounded to bf16
(OracleConfig.store_cast), and once per rounding point with only that one switched on.  For every layer it
prints  max|variant - reference| / max|reference|  of the residual stream entering the layer, and the same
for the final stream, the logits (worst row) and the confidences.  Nothing here touches the HIP library: the
numbers say what ANY implementation with bf16 activations and exact arithmetic would show.

    python -m oracle.drift_study --workload c4_batch256 --seq shortest --out tests/golden/bf16_drift_c4_batch256.txt
"""
from __future__ import annotations

import argparse
import sys
import time

import numpy as np

import focus_inputs as fi
from oracle import focus_oracle as fo
from oracle.harness import BF16_STORE_POINTS, LazyRows, _f64, bf16_store_cast, oracle_config

POINTS = list(BF16_STORE_POINTS)


def relerr(a, b):
    return float(np.max(np.abs(a - b)) / max(float(np.max(np.abs(b))), 1e-300))


class CachedWeights:
    """The workload's weights kept as bf16 tensors (2 bytes per element) and widened per use, so that several runs
    share one generation."""

    def __init__(self, wl):
        self.wl, self.layers, self.head = wl, {}, None

    def weights(self) -> fo.Weights:
        wl, ones = self.wl, np.ones(self.wl.hidden)

        def layer(l):
            if l not in self.layers:
                self.layers[l] = {k: wl.layer_weight(l, k) for k in ("w_qkv", "w_o", "w_gate_up", "w_down")}
            w = {k: _f64(v) for k, v in self.layers[l].items()}
            w["attn_norm"] = w["mlp_norm"] = ones
            return w
        if self.head is None:
            self.head = wl.lm_head()
        return fo.Weights(LazyRows(wl), _f64(self.head), ones, layer)


def run(wl, cw, seq, keep, points, n_pages, lens, tables):
    cfg = oracle_config(wl)
    cfg.store_cast = bf16_store_cast(points) if points else None
    pool = fo.KVPool(cfg)
    for l in range(wl.n_layers):
        for pid in tables[seq]:
            pool.layers[l][pid] = _f64(wl.kv_page(l, pid, n_pages))
    st = fo.new_seq_state(cfg, lens[seq], tables[seq], slot=0)
    return fo.focus_step(cfg, cw.weights(), pool, [st], keep_override=keep, record_layers=set(range(wl.n_layers)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c4_batch256")
    ap.add_argument("--seq", default="shortest", help="'shortest', 'longest' or an index into the batch")
    ap.add_argument("--layers", type=int, default=0, help="run only the first layers of the model (0 = all)")
    ap.add_argument("--out", default="")
    args = ap.parse_args()
    wl = fi.workload(args.workload, **({"n_layers": args.layers} if args.layers else {}))
    assert not wl.n_experts, "dense models only"
    lens = wl.prefix_lens()
    tables, n_pages = wl.page_tables(lens)
    seq = int(np.argmin(lens)) if args.seq == "shortest" else int(np.argmax(lens)) if args.seq == "longest" else int(args.seq)
    cw = CachedWeights(wl)
    t0 = time.time()
    ref = run(wl, cw, seq, None if wl.budget_mode != 3 else [list(range(wl.block_size // 4))], [], n_pages, lens, tables)
    keep = [ref.keep[0]]                       # every variant runs on the reference's retained set
    print("reference done in %.0f s, retained %s" % (time.time() - t0, keep[0]), file=sys.stderr, flush=True)
    variants = [("all", POINTS)] + [(p, [p]) for p in POINTS]
    L, e = wl.n_layers, wl.evict_layer
    cols = {}
    for name, pts in variants:
        t0 = time.time()
        tr = run(wl, cw, seq, keep, pts, n_pages, lens, tables)
        col = [relerr(tr.hidden_full, ref.hidden_full)]
        col += [relerr(tr.hidden_entering[l], ref.hidden_entering[l]) for l in range(e + 1, L)]
        col.append(relerr(tr.hidden_packed, ref.hidden_packed))
        col.append(max(relerr(tr.logits[r], ref.logits[r]) for r in range(len(ref.logits))))
        col.append(relerr(tr.conf, ref.conf))
        col.append(float(np.max(np.abs(tr.delta_I[0] - ref.delta_I[0])) / np.max(np.abs(ref.I_evict[0]))))
        cols[name] = col
        print("variant %s done in %.0f s" % (name, time.time() - t0), file=sys.stderr, flush=True)
    rows = ["entering layer %d" % e] + ["entering layer %d" % l for l in range(e + 1, L)] + \
           ["after the last layer", "logits (worst row)", "confidence", "importance delta / max importance"]
    lines = ["# bf16 activation format against float64, CPU oracle only (python -m oracle.drift_study --workload %s --seq %s%s)"
             % (args.workload, args.seq, " --layers %d" % args.layers if args.layers else ""),
             "# workload %s, sequence %d (prefix %d), block %d, retained positions %s" % (wl.name, seq, lens[seq], wl.block_size, keep[0]),
             "# max|variant - float64| / max|float64| of the residual stream; column = which stored activations are rounded to bf16",
             "%-34s" % "where" + "".join("%10s" % n for n, _ in variants)]
    for i, r in enumerate(rows):
        lines.append("%-34s" % r + "".join("%10.2e" % cols[n][i] for n, _ in variants))
    text = "\n".join(lines) + "\n"
    sys.stdout.write(text)
    if args.out:
        open(args.out, "w").write(text)


if __name__ == "__main__":
    main()
