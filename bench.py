#!/usr/bin/env python3
"""Benchmark of the FOCUS decode step on one MI355X.

A "step" is one call of focus_step: the whole hot path (full-block layers up to the eviction layer,
importance, selection, packing, packed layers, logits, confidence, commit) over the batch of the named
workload.  The default workload is the batch-256 configuration of the benchmark spec (36 layers, 8B shape, bf16,
prefix lengths uniform in [512, 4096], block 32), keep ratio 0.25; weights and prefix K/V are seeded synthetic
values generated on the device before the timed region.

Prints one JSON line.  `value` = decoded tokens / second over the timed steps (with random-init weights no
confidence reaches the threshold, so every sequence commits exactly its one forced token per step).
`roofline` is the GEMM kernel class (dominant at this keep ratio): algorithmic flops of all projections of a
step divided by their summed device time, measured with HIP event pairs around every launch in a separate
pass.  `cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def gemm_flops_per_step(wl, T0: int, Tp: int) -> float:
    """Algorithmic flops of the dense projections of one step: 2*M*N*K per projection."""
    h, F, V = wl.hidden, wl.ffn, wl.vocab
    qkv = (wl.n_q_heads + 2 * wl.n_kv_heads) * wl.head_dim
    qd = wl.n_q_heads * wl.head_dim

    def ffn(l):        # dense feed-forward, or router + shared expert of a mixture-of-experts layer (the routed experts are counted apart)
        return (wl.n_experts * h + 3 * wl.shared_ffn * h) if wl.is_moe_layer(l) else 3 * F * h
    e = wl.evict_layer
    full = sum(qkv * h + qd * h + ffn(l) for l in range(e)) + qkv * h          # layers < e complete, layer e's QKV
    packed = qd * h + ffn(e) + sum(qkv * h + qd * h + ffn(l) for l in range(e + 1, wl.n_layers)) + V * h
    return 2.0 * (T0 * full + Tp * packed)


def expert_bytes_per_step(wl) -> float:
    """Weights of the routed experts, read once per mixture-of-experts layer and step (every expert has rows at these batch
    sizes); activations are not counted."""
    n_moe = sum(1 for l in range(wl.n_layers) if wl.is_moe_layer(l))
    return float(n_moe) * wl.n_experts * 3 * wl.hidden * wl.expert_ffn * 2


def kv_bytes_per_step(wl, lens) -> float:
    """K/V bytes the attention of one step has to read once per (sequence, layer)."""
    per_tok = 2 * wl.n_kv_heads * wl.head_dim * (4 if wl.dtype == "fp32" else 2)
    return float(sum(l + wl.block_size for l in lens)) * per_tok * wl.n_layers


def cpu_baseline(wl, n_seq_sample: int, n_layers_sample: int):
    """Times the CPU oracle on the first sequences of the batch through the first layers of the model and
    extrapolates the packed-layer time to the full depth."""
    import numpy as np
    import torch
    from oracle import focus_oracle as fo
    from oracle.harness import oracle_batch
    import focus_inputs as fi

    from dataclasses import replace
    small = replace(wl, n_layers=n_layers_sample)
    cfg, W, pool, states, lens, tables, n_pages = oracle_batch(small, list(range(n_seq_sample)), lazy_embed=True)
    marks = []
    inner = W._layer_fn

    def stamped(l):
        t_in = time.perf_counter()
        w = inner(l)
        marks.append((l, t_in, time.perf_counter()))
        return w
    W._layer_fn = stamped
    t0 = time.perf_counter()
    tr = fo.focus_step(cfg, W, pool, states)
    t1 = time.perf_counter()
    # compute time of layer l = start of fetch(l+1) - end of fetch(l)
    ends = [m[1] for m in marks[1:]] + [t1]
    per_layer = [ends[i] - marks[i][2] for i in range(len(marks))]
    e = small.evict_layer
    pre = (marks[0][1] - t0) + sum(per_layer[:e + 1])                 # embed, layers 0..e incl. selection and layer e's packed part
    packed = per_layer[e + 1:-1]
    t_packed = sum(packed) / len(packed)
    t_last = per_layer[-1]                                            # last packed layer + logits + confidence + commit
    total = pre + t_packed * (wl.n_layers - e - 2) + t_last
    decoded = sum(tr.n_decoded)
    return dict(value=decoded / total, unit="tokens/s", cores=torch.get_num_threads(), kind="oracle",
                sample="first %d of %d sequences, keep ratio %.3f, oracle run through layers 0..%d of %d plus logits/commit "
                       "(%.1f s measured, input generation excluded); the mean time of the packed layers stands in for the "
                       "%d layers not run: %.1f s per step for the sample"
                       % (n_seq_sample, wl.batch, wl.keep_ratio, n_layers_sample - 1, wl.n_layers, t1 - t0 - W.fetch_seconds,
                          wl.n_layers - n_layers_sample, total))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c4_batch256")
    ap.add_argument("--keep-ratio", type=float, default=None, help="fixed-ratio budget (default: the workload's own budget rule)")
    ap.add_argument("--sweep", action="store_true", help="also time keep ratios 1.0, 0.5, 0.125")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debug only; the JSON says so)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch (debug only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=96)
    ap.add_argument("--cpu-layers", type=int, default=6)
    ap.add_argument("--constant-weights", action="store_true",
                    help="diagnostic: overwrite every weight with one constant, so that the matrix cores see operands that do not "
                         "toggle (shows how much of the projection time is the chip's power limit); the JSON says so")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also launch one 1 GiB device-to-device copy (a dispatch of known size for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (sequences are independent, so the path shards by "
              "sequence with replicated weights); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import focus_inputs as fi
    import paper_2601_23278_amd as pk
    from paper_2601_23278_amd import runner

    over = {} if args.keep_ratio is None else dict(keep_ratio=args.keep_ratio, budget_mode=1)
    if args.layers:
        over["n_layers"] = args.layers
    if args.batch:
        over["batch"] = args.batch
    wl = fi.workload(args.workload, **over)
    if wl.budget_mode not in (0, 1):
        print("bench.py: workload %s has a per-sequence budget; give --keep-ratio" % wl.name, file=sys.stderr)
        sys.exit(2)
    ratio0 = wl.keep_ratio if wl.budget_mode == 1 else wl.topk / wl.block_size      # fraction of the block that is retained
    t_setup = time.time()
    sess = runner.open_session(wl, "cuda:0")
    if args.constant_weights:
        embed, lm_head, norm, layers = sess.weights
        for t in [embed, lm_head] + [w for layer in layers for k, w in layer.items() if k.startswith("w_")]:
            t.fill_(0.01)
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup
    n, B = wl.batch, wl.block_size
    stream = torch.cuda.current_stream()
    n_dec = torch.zeros(n, dtype=torch.int32, device="cuda:0")
    cu = torch.zeros(n + 1, dtype=torch.int32, device="cuda:0")
    out = pk.make_step_out(n_decoded=n_dec, cu_seqlens=cu)

    def reinstall():
        sess.focus.focus_prefill_kv(sess.prefix_lens, sess.page_tables, None)

    def run(ratio: float, steps: int, warmup: int):
        """Times `steps` consecutive denoising steps of one block at the given keep ratio."""
        if wl.budget_mode == 1:
            sess.reopen(keep_ratio=ratio)
        else:
            sess.reopen()
        f = sess.focus
        K = min(B, max(0, int(math.ceil(float(torch.tensor(ratio, dtype=torch.float32)) * B)))) if wl.budget_mode == 1 else wl.topk
        period = max(1, B - K) if K < B else B          # steps before a block runs out of masked tokens
        reinstall()
        for _ in range(warmup):
            f.focus_step(n, out=out)
        reinstall()
        decoded = torch.zeros((), dtype=torch.int64, device="cuda:0")
        decoded += n_dec.sum()          # first use loads torch's reduction kernel: keep that out of the timed region
        decoded.zero_()
        torch.cuda.synchronize()
        dt, t0 = 0.0, time.perf_counter()
        for i in range(steps):
            if i and i % period == 0:
                # the block has run out of masked tokens: install a fresh one (host-side set-up of inputs, not a step: the
                # clock stops around it)
                torch.cuda.synchronize()
                dt += time.perf_counter() - t0
                reinstall()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            f.focus_step(n, out=out)
            decoded += n_dec.sum()
        torch.cuda.synchronize()
        dt += time.perf_counter() - t0
        return dict(keep_ratio=ratio, ms_per_step=1e3 * dt / steps, decoded_tokens_per_s=float(decoded.item()) / dt,
                    decoded_per_step=float(decoded.item()) / steps, rows_full=n * B, rows_packed=int(cu[-1].item()))

    head = run(ratio0, args.steps, args.warmup)

    # per-class device time of one step (event pairs around every launch; separate pass)
    sess.reopen()
    f = sess.focus
    f.focus_set_timing(True)
    f.focus_step(n, out=out)
    classes = {}
    for k, name in enumerate(pk.binding.KC_NAMES):
        ms, cnt = f.focus_get_kernel_time(k)
        classes[name] = dict(ms=round(ms, 4), launches=cnt)
    f.focus_set_timing(False)
    Tp = int(cu[-1].item())
    flops = gemm_flops_per_step(wl, n * B, Tp)
    gemm_ms = classes["gemm"]["ms"]
    achieved = flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    kvb = kv_bytes_per_step(wl, sess.prefix_lens)
    attn_ms = classes["attention"]["ms"]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic_%s_keep%03d.json" % (wl.name, int(round(1000 * ratio0))))
    if os.path.exists(tpath) and not (args.layers or args.batch):
        traffic = json.load(open(tpath)).get("gemm_hbm_bytes_per_step")
    roofline = dict(bound="mfma", kernel="gemm (all dense projections of a step)", achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS,
                    unit="TFLOP/s", frac=round(achieved / PEAK_BF16_TFLOPS, 4), traffic=traffic,
                    flops_per_step=flops, launches=classes["gemm"]["launches"], avg_launch_ms=round(gemm_ms / max(1, classes["gemm"]["launches"]), 5))
    dense_gemm = None
    if not wl.n_experts and n * B < 312:
        # fewer rows than the ridge point (about 312 flop per byte): the projections are bound by streaming every weight once
        dense_gemm = roofline
        qkv_w = (wl.n_q_heads + 2 * wl.n_kv_heads) * wl.head_dim
        wbytes = 2.0 * (wl.n_layers * (qkv_w * wl.hidden + wl.n_q_heads * wl.head_dim * wl.hidden + 3 * wl.ffn * wl.hidden) + wl.vocab * wl.hidden)
        gbs = wbytes / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else 0.0
        roofline = dict(bound="hbm", kernel="gemm (all dense projections of a step; every weight is read once)", achieved=round(gbs, 1),
                        peak=PEAK_HBM_GBS, unit="GB/s", frac=round(gbs / PEAK_HBM_GBS, 4), traffic=None, bytes_per_step=wbytes,
                        launches=classes["gemm"]["launches"], avg_launch_ms=round(gemm_ms / max(1, classes["gemm"]["launches"]), 5))
    if wl.n_experts:
        # mixture-of-experts model: the grouped expert projections stream the expert weights once per layer and dominate
        dense_gemm = roofline
        ex_ms, ex_n = classes["experts"]["ms"], classes["experts"]["launches"]
        eb = expert_bytes_per_step(wl)
        gbs = eb / (ex_ms * 1e-3) / 1e9 if ex_ms > 0 else 0.0
        roofline = dict(bound="hbm", kernel="grouped expert projections (gate/up + down of every mixture-of-experts layer)",
                        achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s", frac=round(gbs / PEAK_HBM_GBS, 4), traffic=None,
                        bytes_per_step=eb, launches=ex_n, avg_launch_ms=round(ex_ms / max(1, ex_n), 5))
    attention = dict(bound="hbm", achieved=round(kvb / (attn_ms * 1e-3) / 1e9, 1) if attn_ms > 0 else 0.0, peak=PEAK_HBM_GBS, unit="GB/s",
                     frac=round(kvb / (attn_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if attn_ms > 0 else 0.0, kv_bytes_per_step=kvb)

    if args.pmc_calibrate:
        a_ = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        b_ = torch.empty_like(a_)
        a_.fill_(1)
        torch.cuda.synchronize()
        b_.copy_(a_)
        torch.cuda.synchronize()

    # achievable ceilings measured in the same run: a device copy for HBM, the vendor library's bf16 GEMM on the gate/up shape as
    # an outside yardstick for the matrix cores (torch.matmul; nothing of it is linked into the library)
    def timed_ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    src.fill_(1)
    copy_ms = timed_ms(lambda: dst.copy_(src), 5)
    ga = torch.randn(2048, wl.hidden, device="cuda:0").to(torch.bfloat16)
    gw = (torch.randn(2 * wl.ffn, wl.hidden, device="cuda:0") * 0.02).to(torch.bfloat16)
    mm_ms = timed_ms(lambda: torch.matmul(ga, gw.t()), 10)
    ceilings = dict(hbm_copy_GBs=round(2.0 * (1 << 30) / (copy_ms * 1e-3) / 1e9, 1),
                    library_gemm_TFLOPs=round(2.0 * 2048 * 2 * wl.ffn * wl.hidden / (mm_ms * 1e-3) / 1e12, 1),
                    note="1 GiB device-to-device copy (read + write bytes); torch.matmul bf16 2048 x %d x %d with random operands" % (2 * wl.ffn, wl.hidden))
    del src, dst, ga, gw

    sweep = None
    if args.sweep:
        sweep = [head] + [run(r, args.steps, args.warmup) for r in (1.0, 0.5, 0.125) if abs(r - ratio0) > 1e-9 and wl.budget_mode == 1]

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, min(args.cpu_seqs, wl.batch), min(args.cpu_layers, wl.n_layers))

    sess.focus.focus_free()
    line = {
        "metric": "decoded tokens/s at batch %d (%s, bf16, 1 GPU)" % (n, "8B-shaped" if not wl.n_experts else "mixture-of-experts, 16B total / 1.4B active shape"), "value": round(head["decoded_tokens_per_s"], 2),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(head["ms_per_step"], 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic" if not args.constant_weights else "synthetic, every weight overwritten with 0.01 (diagnostic run)",
        "config": {"workload": "%s: %d layers, hidden %d, %dq/%dkv x %d, ffn %d, vocab %d, batch %d, prefix %s[%d,%d], block %d, keep ratio %.3f"
                               % (wl.name, wl.n_layers, wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.vocab, n,
                                  wl.prefix_dist, wl.prefix_lo, wl.prefix_hi, B, ratio0),
                   "rows_full": n * B, "rows_packed": head["rows_packed"], "decoded_per_step": head["decoded_per_step"],
                   "experts": None if not wl.n_experts else "%d experts x %d, %d per token, shared %d, dense below layer %d"
                              % (wl.n_experts, wl.expert_ffn, wl.experts_per_token, wl.shared_ffn, wl.first_moe_layer),
                   "debug_overrides": {k: v for k, v in (("layers", args.layers), ("batch", args.batch)) if v}},
        "roofline": roofline, "dense_gemm": dense_gemm, "attention_hbm": attention, "kernel_classes_ms": classes, "ceilings": ceilings, "cpu_baseline": cpu, "sweep": sweep,
        "setup_s": round(t_setup, 1),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
