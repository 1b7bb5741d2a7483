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
pass.  `phases` gives the HBM-bound phases (K/V read of the attention, gather, selection + packing, rotary + K/V
scatter) the same way, in GB/s of algorithmic bytes.  `cpu_baseline` is the CPU oracle timed on a bounded sample
of the same workload.  Unless --no-extras is given the line also carries, each measured the same way in the same
run: the keep-ratio sweep of the batch-256 configuration (`sweep`), the method's own budget rule on it (Eq. 4-5 with
alpha 1.5, without and with the structural constraints of Sec. 4.2: `method_budget`), and the batch-128 and the
long-context ragged configurations of the benchmark spec (`other_workloads`).

`bench.py --pmc-summary FETCH.csv WRITE.csv` does not touch the GPU: it condenses the counter files of two
`rocprofv3 --pmc` runs of this benchmark into profiles/ (see profiles/*hbm_traffic.txt for the commands).
"""
from __future__ import annotations

import argparse
import csv
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def gemm_flops_per_step(wl, T0: int, Tp: float) -> float:
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


def phase_bytes(wl, T0: int, Tp: float):
    """Algorithmic bytes per step of the small HBM-bound phases (read + write, every byte once)."""
    es = 4 if wl.dtype == "fp32" else 2
    n, B, h, Hq, Hkv, D = wl.batch, wl.block_size, wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    e, L = wl.evict_layer, wl.n_layers
    gather = Tp * (2 * h * 4 + 2 * Hq * D * es)                              # residual row (fp32) and layer-e queries, in and out
    select = (2 * n * Hq * B * 4 + n * (8 + 8 + 8 + 4)                        # per-head importance sums of two layers, block state
              + n * B * 4 + n * (4 + 8 + 4 + 8) + (n + 1) * 4 + Tp * 4)      # delta, K, sets, offsets, row map
    per_row = (Hq + 2 * Hkv) * D * es + (Hq + Hkv) * D * es + 2 * Hkv * D * es   # qkv row in, rotated q, k back, k and v into the cache
    kv_write = ((e + 1) * T0 + (L - e - 1) * Tp) * per_row
    return dict(gather=float(gather), select=float(select), kv_write=float(kv_write))


def cpu_baseline(wl, n_seq_sample: int, n_layers_sample: int):
    """Times the CPU oracle on the first sequences of the batch through the first layers of the model and
    extrapolates the packed-layer time to the full depth."""
    import torch
    from oracle import focus_oracle as fo
    from oracle.harness import oracle_batch

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


# ---------------------------------------------------------------------------------------------
# one measured configuration

class Runner:
    def __init__(self, wl, pk, runner, torch, constant_weights=False):
        self.wl, self.pk, self.torch = wl, pk, torch
        t0 = time.time()
        self.sess = runner.open_session(wl, "cuda:0")
        if constant_weights:
            embed, lm_head, norm, layers = self.sess.weights
            for t in [embed, lm_head] + [w for layer in layers for k, w in layer.items() if k.startswith("w_")]:
                t.fill_(0.01)
        torch.cuda.synchronize()
        self.setup_s = time.time() - t0
        n = wl.batch
        self.n_dec = torch.zeros(n, dtype=torch.int32, device="cuda:0")
        self.cu = torch.zeros(n + 1, dtype=torch.int32, device="cuda:0")
        self.K = torch.zeros(n, dtype=torch.int32, device="cuda:0")
        self.keep = torch.zeros(n, dtype=torch.int64, device="cuda:0")
        self.out = pk.make_step_out(n_decoded=self.n_dec, cu_seqlens=self.cu, K=self.K, keep_bits=self.keep)

    def reinstall(self):
        self.sess.focus.focus_prefill_kv(self.sess.prefix_lens, self.sess.page_tables, None)

    def measure(self, steps: int, warmup: int, label: str, **cfg_over):
        """Times `steps` consecutive denoising steps with the configuration members in cfg_over replaced, then runs one more
        step with an event pair around every launch for the per-class times."""
        torch, wl, pk = self.torch, self.wl, self.pk
        n, B = wl.batch, wl.block_size
        self.sess.reopen(**cfg_over)
        f = self.sess.focus
        cfg = f.cfg
        ko = None
        if cfg.budget_mode == 3:
            ks = wl.k_overrides()
            ko = torch.tensor(ks, dtype=torch.int32, device="cuda:0")
        fixed = cfg.budget_mode in (0, 1) and not cfg.constraints
        if cfg.budget_mode in (0, 1):
            K = wl.topk if cfg.budget_mode == 0 else min(B, max(0, int(math.ceil(float(torch.tensor(cfg.keep_ratio, dtype=torch.float32)) * B))))
            period = max(1, B - K) if K < B else B          # steps before a block has fewer masked positions than the budget
        else:
            period = max(1, B // 2)
        hint = None
        if not fixed:
            # the packed row count is known on the device only: one probe step tells the launch shapes what to expect
            self.reinstall()
            f.focus_step(n, k_override=ko, out=self.out)
            torch.cuda.synchronize()
            counts = (self.cu[1:] - self.cu[:-1])
            hint = (int(self.cu[-1].item()), int(counts.max().item()))
            f.focus_set_row_hint(*hint)
        self.reinstall()
        for _ in range(warmup):
            f.focus_step(n, k_override=ko, out=self.out)
        self.reinstall()
        acc = torch.zeros(2, dtype=torch.int64, device="cuda:0")            # decoded tokens, packed rows
        acc[0] += self.n_dec.sum()          # first use loads torch's reduction kernel: keep that out of the timed region
        acc.zero_()
        torch.cuda.synchronize()
        dt, t0 = 0.0, time.perf_counter()
        for i in range(steps):
            if i and i % period == 0:
                # the block is running out of masked tokens: install a fresh one (host-side set-up of inputs, not a step: the
                # clock stops around it)
                torch.cuda.synchronize()
                dt += time.perf_counter() - t0
                self.reinstall()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            f.focus_step(n, k_override=ko, out=self.out)
            acc[0] += self.n_dec.sum()
            acc[1] += self.cu[-1]
        torch.cuda.synchronize()
        dt += time.perf_counter() - t0
        decoded, rows = (float(x) for x in acc.cpu().tolist())
        res = dict(label=label, ms_per_step=round(1e3 * dt / steps, 3), decoded_tokens_per_s=round(decoded / dt, 2),
                   decoded_per_step=decoded / steps, rows_full=n * B, rows_packed=rows / steps, steps=steps, row_hint=hint)
        # per-class device time of one step (first step of a fresh block; event pairs around every launch)
        self.reinstall()
        f.focus_set_timing(True)
        f.focus_step(n, k_override=ko, out=self.out)
        classes = {}
        for k, name in enumerate(pk.binding.KC_NAMES):
            ms, cnt = f.focus_get_kernel_time(k)
            classes[name] = dict(ms=round(ms, 4), launches=cnt)
        f.focus_set_timing(False)
        Tp = int(self.cu[-1].item())
        res["classes"] = classes
        res["rows_packed_timing_pass"] = Tp
        flops = gemm_flops_per_step(wl, n * B, Tp)
        g_ms = classes["gemm"]["ms"]
        res["gemm"] = dict(TFLOPs=round(flops / (g_ms * 1e-3) / 1e12, 1) if g_ms > 0 else 0.0, ms=g_ms, flops_per_step=flops,
                           launches=classes["gemm"]["launches"])
        res["gemm"]["frac_of_mfma_peak"] = round(res["gemm"]["TFLOPs"] / PEAK_BF16_TFLOPS, 4)
        kvb = kv_bytes_per_step(wl, self.sess.prefix_lens)
        pb = phase_bytes(wl, n * B, Tp)
        pb["attention"] = kvb
        phases = {}
        for name, nbytes in pb.items():
            ms = classes[name]["ms"]
            gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
            phases[name] = dict(GBs=round(gbs, 1), frac_of_hbm_peak=round(gbs / PEAK_HBM_GBS, 4), ms=ms, bytes_per_step=nbytes,
                                launches=classes[name]["launches"])
        # matrix work of the attention: QK^T and PV, 4 * D flop per (query row, query head, visible token)
        counts = (self.cu[1:] - self.cu[:-1]).cpu().tolist()
        e, L = wl.evict_layer, wl.n_layers
        lens = self.sess.prefix_lens
        fl_att = 4.0 * wl.n_q_heads * wl.head_dim * sum((e * B + (L - e) * q) * (l + B) for q, l in zip(counts, lens))
        a_ms = classes["attention"]["ms"]
        phases["attention"]["TFLOPs"] = round(fl_att / (a_ms * 1e-3) / 1e12, 1) if a_ms > 0 else 0.0
        phases["attention"]["frac_of_mfma_peak"] = round(phases["attention"]["TFLOPs"] / PEAK_BF16_TFLOPS, 4)
        res["phases"] = phases
        return res


def workload_text(wl, ratio_text):
    return "%s: %d layers, hidden %d, %dq/%dkv x %d, ffn %d, vocab %d, batch %d, prefix %s[%d,%d], block %d, %s" % (
        wl.name, wl.n_layers, wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.vocab, wl.batch,
        wl.prefix_dist, wl.prefix_lo, wl.prefix_hi, wl.block_size, ratio_text)


# ---------------------------------------------------------------------------------------------
# rocprofv3 byte counters -> profiles/

def pmc_summary(fetch_csv: str, write_csv: str, workload: str, ratio: float):
    """Condenses two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE) of `bench.py --workload W --keep-ratio R --steps 1
    --warmup 0 --no-extras --no-cpu-baseline --pmc-calibrate` into profiles/: per (kernel, grid) launch counts and bytes, the
    projection class total per step, and the JSON bench.py reads for roofline.traffic.  The run holds two passes over the
    model (the timed step and the per-class timing pass), the counters of both are averaged."""
    def short(n):
        m = re.match(r"_ZN2fk\d+(k_[a-z0-9_]+)", n)
        if m:
            return m.group(1)
        s = re.sub(r"^void ", "", n)
        s = re.sub(r"\(.*", "", s)
        return s.replace("fk::", "")

    def load(path, counter):
        per, cal = {}, None
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            name, v = r["Kernel_Name"], float(r["Counter_Value"])
            if ("copyBuffer" in name or "direct_copy" in name) and v > 4e5:
                cal = v                                            # the 1 GiB calibration copy: the largest copy of the run
            if "fk::" in name or "_ZN2fk" in name:
                per.setdefault((short(name), int(r["Grid_Size"])), []).append(v)
        return per, cal
    fetch, fcal = load(fetch_csv, "FETCH_SIZE")
    write, wcal = load(write_csv, "WRITE_SIZE")
    if not fcal or not wcal:
        raise SystemExit("no calibration copy found: run bench.py with --pmc-calibrate")
    fs, ws = 1048576.0 / fcal, 1048576.0 / wcal
    passes = 2.0
    lines = ["rocprofv3 byte counters of one benchmark step, workload %s, keep ratio %g, one MI355X; one counter per run:" % (workload, ratio)]
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        lines.append("  rocprofv3 --pmc %s --output-format csv -d gpurun_out/pmc_%s -o p -- python3 /root/repo/bench.py --workload %s --keep-ratio %g "
                     "--steps 1 --warmup 0 --no-extras --no-cpu-baseline --pmc-calibrate" % (c, c, workload, ratio))
    lines.append("  python3 bench.py --workload %s --keep-ratio %g --pmc-summary gpurun_out/pmc_FETCH_SIZE/.../p_counter_collection.csv "
                 "gpurun_out/pmc_WRITE_SIZE/.../p_counter_collection.csv" % (workload, ratio))
    lines.append("Calibration: the 1 GiB device-to-device copy of --pmc-calibrate reads FETCH_SIZE = %.0f KiB and WRITE_SIZE = %.0f KiB, "
                 "so FETCH_SIZE is scaled by %.4f and WRITE_SIZE by %.4f." % (fcal, wcal, fs, ws))
    lines.append("The counters sit behind the L2: they count what the memory-side cache and HBM serve together.  The run holds %g passes over "
                 "the model (one step, one per-class timing pass); launches/step = launches of the run / %g.  MB = 1e6 bytes, per launch.\n" % (passes, passes))
    lines.append("%-44s %8s %14s %12s %12s" % ("kernel", "grid", "launches/step", "fetch MB", "write MB"))
    tot = {"gemm": 0.0, "attention": 0.0, "other": 0.0}
    for k in sorted(fetch, key=lambda k: (k[0], -k[1])):
        f = sum(fetch[k]) / len(fetch[k]) * fs * 1024 / 1e6
        w = sum(write.get(k, [0.0])) / max(1, len(write.get(k, [0.0]))) * ws * 1024 / 1e6
        n = len(fetch[k]) / passes
        cls = "gemm" if "k_gemm" in k[0] or "k_splitk" in k[0] else "attention" if "k_attn" in k[0] else "other"
        tot[cls] += (f + w) * n
        lines.append("%-44s %8d %14.1f %12.1f %12.1f" % (k[0][:44], k[1], n, f, w))
    lines.append("\nper step, beyond the L2: projections %.1f GB, attention %.1f GB, everything else %.2f GB." % (tot["gemm"] / 1e3, tot["attention"] / 1e3, tot["other"] / 1e3))
    tag = "%s_keep%03d" % (workload, int(round(1000 * ratio)))
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    open(os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % tag), "w").write("\n".join(lines) + "\n")
    json.dump({"workload": workload, "keep_ratio": ratio, "gemm_hbm_bytes_per_step": tot["gemm"] * 1e6,
               "attention_hbm_bytes_per_step": tot["attention"] * 1e6,
               "method": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on the full benchmark step, scaled by a 1 GiB copy; see %s_hbm_traffic.txt" % tag},
              open(os.path.join(ROOT, "profiles", "pmc_traffic_%s.json" % tag), "w"))
    print("\n".join(lines[-3:]))


def trace_summary(stats_csv: str, bench_log: str, tag: str, command: str):
    """Condenses `rocprofv3 --kernel-trace --stats` of one benchmark run into profiles/bench_<tag>_kernel_stats.txt: the
    library's kernels with calls, total and average duration, and the projection / attention rates that follow from them.
    bench_log = the stdout of that same run (its JSON line supplies steps, flops and bytes)."""
    line = json.loads([l for l in open(bench_log).read().splitlines() if l.startswith("{")][-1])

    def short(n):
        m = re.match(r"_ZN2fk\d+(k_[a-z0-9_]+)", n)
        if m:
            return m.group(1)
        s = re.sub(r"^void ", "", n)
        s = re.sub(r"\(.*", "", s)
        return s.replace("fk::", "")
    rows = [r for r in csv.DictReader(open(stats_csv)) if "fk::" in r["Name"] or "_ZN2fk" in r["Name"]]
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    # per-dispatch durations (a kernel that serves two shapes, e.g. the O and the down projection, shows both in its quantiles)
    per = {}
    trace_csv = stats_csv.replace("_kernel_stats.csv", "_kernel_trace.csv")
    if os.path.exists(trace_csv):
        for r in csv.DictReader(open(trace_csv)):
            per.setdefault(short(r["Kernel_Name"]), []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)

    def quant(n):
        d = sorted(per.get(n, []))
        return "%9.1f %9.1f %9.1f" % (d[len(d) // 10], d[len(d) // 2], d[(9 * len(d)) // 10]) if d else ""
    passes = line["steps"] + line["warmup"] + 1 + (1 if line["config"].get("row_hint") else 0)
    out = ["rocprofv3 kernel trace of bench.py, %s, one MI355X." % line["config"]["workload"],
           "Command (from /tmp, TMPDIR=/tmp):", "  " + command,
           "The run executes %d steps (%d warm-up, %d timed, 1 per-class timing pass%s); bench.py reported %.2f ms per step in the same run."
           % (passes, line["warmup"], line["steps"], ", 1 probe step for the row hint" if line["config"].get("row_hint") else "", line["ms_per_step"]),
           "Source: *_kernel_stats.csv (Calls, TotalDurationNs, AverageNs); library kernels only.\n",
           "%-64s %8s %12s %10s %9s %9s %9s" % ("kernel", "calls", "total_ms", "avg_us", "p10_us", "p50_us", "p90_us")]
    tot = gemm = attn = 0.0
    for r in rows:
        n, t = short(r["Name"]), float(r["TotalDurationNs"])
        tot += t
        gemm += t if ("k_gemm" in n or "k_splitk" in n) else 0.0
        attn += t if "k_attn" in n else 0.0
        out.append("%-64s %8s %12.3f %10.2f %s" % (n[:64], r["Calls"], t / 1e6, float(r["AverageNs"]) / 1e3, quant(n)))
    out.append("library kernels total: %.3f ms over %d steps = %.3f ms per step\n" % (tot / 1e6, passes, tot / 1e6 / passes))
    fl, nl = line["roofline"].get("flops_per_step"), line["roofline"]["launches"]
    kvb = line["attention_hbm"]["kv_bytes_per_step"]
    if fl:
        out.append("Projection class (k_gemm_*, %d launches per step): %.2f ms per step for %.2f TFLOP (timing pass rows) -> %.0f TFLOP/s = %.1f %% of the "
                   "2.5 PFLOP/s bf16 MFMA peak; average launch %.1f us.  bench.py's event pairs in the same run: %.2f ms, %.0f TFLOP/s, average launch %.1f us."
                   % (nl, gemm / 1e6 / passes, fl / 1e12, fl / (gemm / 1e9 / passes) / 1e12, 100 * fl / (gemm / 1e9 / passes) / 2.5e15,
                      gemm / 1e3 / passes / nl, line["kernel_classes_ms"]["gemm"]["ms"], line["roofline"]["achieved"], 1e3 * line["roofline"]["avg_launch_ms"]))
    rl = line["roofline"]
    if rl["bound"] == "hbm":
        grp = sum(float(r["TotalDurationNs"]) for r in rows if "k_group_gemm" in r["Name"])
        out.append("bench.py's roofline of this run (event pairs): %s: %.1f GB per step in %.2f ms over %d launches -> %.0f GB/s = %.1f %% of the 8 TB/s HBM peak."
                   % (rl["kernel"], rl["bytes_per_step"] / 1e9, rl["avg_launch_ms"] * rl["launches"], rl["launches"], rl["achieved"], 100 * rl["frac"]))
        if line["config"].get("experts"):
            out.append("Kernel trace of the same class (k_group_gemm<1> = gate/up + SiLU*up, <0> = down): %.2f ms per step -> %.0f GB/s."
                       % (grp / 1e6 / passes, rl["bytes_per_step"] / (grp / 1e9 / passes) / 1e9))
    out.append("Attention class (k_attn_*): %.2f ms per step for %.1f GB of K/V -> %.2f TB/s = %.1f %% of the 8 TB/s HBM peak (event pairs: %.2f ms)."
               % (attn / 1e6 / passes, kvb / 1e9, kvb / (attn / 1e9 / passes) / 1e12, 100 * kvb / (attn / 1e9 / passes) / 8e12, line["kernel_classes_ms"]["attention"]["ms"]))
    for name, ph in line["phases"].items():
        if name != "attention":
            out.append("%s (event pairs): %.1f MB in %.1f us over %d launches = %.0f GB/s = %.1f %% of the HBM peak."
                       % (name, ph["bytes_per_step"] / 1e6, 1e3 * ph["ms"], ph["launches"], ph["GBs"], 100 * ph["frac_of_hbm_peak"]))
    open(os.path.join(ROOT, "profiles", "bench_%s_kernel_stats.txt" % tag), "w").write("\n".join(out) + "\n")
    print("\n".join(out[-8:]))


def mfma_summary(counter_csv: str, workload: str, ratio: float):
    """Condenses `rocprofv3 --pmc MfmaUtil MfmaFlopsBF16` of one benchmark step into profiles/: per (kernel, grid) the share of
    cycles in which the matrix cores were busy (SQ_VALU_MFMA_BUSY_CYCLES over active cycles x SIMDs: a figure in the chip's
    ACTUAL clock cycles, unlike the TFLOP/s fractions, which are against the peak at the nominal clock) and the bf16 flops the
    hardware counted, next to the algorithmic flops bench.py prices the launch at."""
    def short(n):
        m = re.match(r"_ZN2fk\d+(k_[a-z0-9_]+)", n)
        if m:
            return m.group(1)
        s = re.sub(r"^void ", "", n)
        s = re.sub(r"\(.*", "", s)
        return s.replace("fk::", "")
    per = {}
    for r in csv.DictReader(open(counter_csv)):
        name = r["Kernel_Name"]
        if not ("fk::" in name or "_ZN2fk" in name):
            continue
        e = per.setdefault((short(name), int(r["Grid_Size"])), {"MfmaUtil": [], "MfmaFlopsBF16": [], "us": []})
        if r["Counter_Name"] in e:
            e[r["Counter_Name"]].append(float(r["Counter_Value"]))
        if r["Counter_Name"] == "MfmaUtil":
            e["us"].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    lines = ["rocprofv3 matrix-core counters of one benchmark step, workload %s, keep ratio %g, one MI355X:" % (workload, ratio),
             "  rocprofv3 --pmc MfmaUtil MfmaFlopsBF16 --kernel-include-regex fk --output-format csv -d gpurun_out/pmc_mfma -o p -- python3 /root/repo/bench.py "
             "--workload %s --keep-ratio %g --steps 1 --warmup 0 --no-extras --no-cpu-baseline" % (workload, ratio),
             "  python3 bench.py --workload %s --keep-ratio %g --mfma-summary gpurun_out/pmc_mfma/.../p_counter_collection.csv" % (workload, ratio),
             "MfmaUtil = 100 * SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE * number of SIMDs): the share of the chip's ACTUAL cycles in which a SIMD's matrix",
             "core was busy.  The TFLOP/s fractions elsewhere are against the peak at the nominal 2.4 GHz; busy share x (actual clock / 2.4 GHz) = that fraction,",
             "so e.g. 61 % busy at 0.50 of the nominal peak means the chip ran at about 2.0 GHz under this load.  Durations are under the profiler (serialised).",
             "MfmaFlopsBF16 = what the hardware counted; it equals 2*M*N*K of the launch (no padded or wasted MFMA work beyond the tile edges).\n",
             "%-40s %9s %9s %12s %14s %10s" % ("kernel", "grid", "launches", "MFMA busy %", "bf16 GFLOP", "avg us")]
    for k in sorted(per, key=lambda k: -sum(per[k]["MfmaFlopsBF16"])):
        e = per[k]
        if not e["MfmaUtil"] or sum(e["MfmaFlopsBF16"]) == 0:
            continue
        lines.append("%-40s %9d %9d %12.1f %14.1f %10.1f" % (k[0][:40], k[1], len(e["MfmaUtil"]), sum(e["MfmaUtil"]) / len(e["MfmaUtil"]),
                                                              sum(e["MfmaFlopsBF16"]) / len(e["MfmaFlopsBF16"]) / 1e9, sum(e["us"]) / len(e["us"])))
    gem = [(sum(e["MfmaUtil"]) / len(e["MfmaUtil"]), sum(e["us"])) for k, e in per.items() if "k_gemm" in k[0] and e["MfmaUtil"]]
    att = [(sum(e["MfmaUtil"]) / len(e["MfmaUtil"]), sum(e["us"])) for k, e in per.items() if "k_attn" in k[0] and e["MfmaUtil"]]
    for name, g in (("projection", gem), ("attention", att)):
        if g:
            lines.append("%s class, time-weighted: matrix cores busy %.1f %% of the cycles" % (name, sum(u * t for u, t in g) / sum(t for _, t in g)))
    tag = "%s_keep%03d" % (workload, int(round(1000 * ratio)))
    open(os.path.join(ROOT, "profiles", "%s_mfma_util.txt" % tag), "w").write("\n".join(lines) + "\n")
    json.dump({"workload": workload, "keep_ratio": ratio,
               "gemm_mfma_busy_pct": sum(u * t for u, t in gem) / sum(t for _, t in gem) if gem else None,
               "attention_mfma_busy_pct": sum(u * t for u, t in att) / sum(t for _, t in att) if att else None,
               "method": "rocprofv3 --pmc MfmaUtil, time-weighted over the launches of the class; see %s_mfma_util.txt" % tag},
              open(os.path.join(ROOT, "profiles", "pmc_mfma_%s.json" % tag), "w"))
    print("\n".join(lines[-14:]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c4_batch256")
    ap.add_argument("--keep-ratio", type=float, default=None, help="fixed-ratio budget (default: the workload's own budget rule)")
    ap.add_argument("--budget", default="workload", choices=["workload", "dynamic", "dynamic-constrained"],
                    help="dynamic: Eq. 4-5 with alpha 1.5; dynamic-constrained: plus AR-context and placeholder integrity (Sec. 4.2)")
    ap.add_argument("--no-extras", action="store_true", help="only the headline measurement (no sweep, no other budget rules or workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=96)
    ap.add_argument("--cpu-layers", type=int, default=6)
    ap.add_argument("--constant-weights", action="store_true",
                    help="diagnostic: overwrite every weight with one constant, so that the matrix cores see operands that do not "
                         "toggle (shows how much of the projection time is the chip's power limit); the JSON says so")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also launch one 1 GiB device-to-device copy (a dispatch of known size for scaling rocprofv3 byte counters)")
    ap.add_argument("--trace-summary", nargs=4, metavar=("STATS_CSV", "BENCH_LOG", "TAG", "COMMAND"),
                    help="no GPU: write profiles/bench_TAG_kernel_stats.txt from a rocprofv3 --kernel-trace --stats run of this benchmark")
    ap.add_argument("--mfma-summary", metavar="COUNTER_CSV", help="no GPU: write profiles/*_mfma_util.txt from a rocprofv3 --pmc MfmaUtil MfmaFlopsBF16 run")
    ap.add_argument("--pmc-summary", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"), help="no GPU: write profiles/ summaries from two rocprofv3 --pmc runs")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (sequences are independent, so the path shards by "
              "sequence with replicated weights); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.trace_summary:
        trace_summary(*args.trace_summary)
        return
    import focus_inputs as fi
    over = {} if args.keep_ratio is None else dict(keep_ratio=args.keep_ratio, budget_mode=1)
    if args.budget != "workload":
        over.update(budget_mode=2, alpha=1.5, constraints=3 if args.budget == "dynamic-constrained" else 0)
    wl = fi.workload(args.workload, **over)
    if args.pmc_summary:
        pmc_summary(args.pmc_summary[0], args.pmc_summary[1], wl.name, wl.keep_ratio)
        return
    if args.mfma_summary:
        mfma_summary(args.mfma_summary, wl.name, wl.keep_ratio)
        return

    import torch
    import paper_2601_23278_amd as pk
    from paper_2601_23278_amd import runner

    B, n = wl.block_size, wl.batch
    budget_text = {0: "top-k %d" % wl.topk, 1: "keep ratio %.3f" % wl.keep_ratio,
                   2: "dynamic budget alpha %.2f, constraints %d" % (wl.alpha, wl.constraints),
                   3: "per-sequence budgets U{0..%d}" % B}[wl.budget_mode]
    R = Runner(wl, pk, runner, torch, args.constant_weights)
    head = R.measure(args.steps, args.warmup, budget_text)
    classes = head["classes"]
    gemm_ms, flops = classes["gemm"]["ms"], head["gemm"]["flops_per_step"]
    achieved = head["gemm"]["TFLOPs"]
    traffic = None
    ratio0 = wl.keep_ratio if wl.budget_mode == 1 else -1.0
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic_%s_keep%03d.json" % (wl.name, int(round(1000 * max(ratio0, 0)))))
    if wl.budget_mode == 1 and os.path.exists(tpath):
        rec = json.load(open(tpath))
        t = rec.get("gemm_hbm_bytes_per_step")
        # only a figure measured on this workload and ratio, and one that the chip could have moved in the measured time
        if rec.get("workload") == wl.name and abs(rec.get("keep_ratio", -1) - ratio0) < 1e-6 and t and t <= PEAK_HBM_GBS * 1e9 * gemm_ms * 1e-3:
            traffic = t
    mfma_busy = None
    mpath = os.path.join(ROOT, "profiles", "pmc_mfma_%s_keep%03d.json" % (wl.name, int(round(1000 * max(ratio0, 0)))))
    if wl.budget_mode == 1 and os.path.exists(mpath):
        rec = json.load(open(mpath))
        if rec.get("workload") == wl.name and abs(rec.get("keep_ratio", -1) - ratio0) < 1e-6:
            mfma_busy = dict(projections_pct=rec.get("gemm_mfma_busy_pct"), attention_pct=rec.get("attention_mfma_busy_pct"),
                             note="hardware counter (share of actual cycles with the matrix cores busy), from profiles/, not measured by this run")
    roofline = dict(bound="mfma", kernel="gemm (all dense projections of a step)", achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS,
                    unit="TFLOP/s", frac=round(achieved / PEAK_BF16_TFLOPS, 4), traffic=traffic, mfma_busy_counter=mfma_busy,
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

    if args.pmc_calibrate:
        a_ = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        b_ = torch.empty_like(a_)
        a_.fill_(1)
        torch.cuda.synchronize()
        b_.copy_(a_)
        torch.cuda.synchronize()
        del a_, b_

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
    # the two shapes on which the library's own kernels are the lowest: the O and the down projection of 2048 rows (plain
    # products with a bf16 result, without the residual read-add-write that the step's kernels carry)
    qd = wl.n_q_heads * wl.head_dim
    go = torch.randn(2048, qd, device="cuda:0").to(torch.bfloat16)
    wo = (torch.randn(wl.hidden, qd, device="cuda:0") * 0.02).to(torch.bfloat16)
    gd = torch.randn(2048, wl.ffn, device="cuda:0").to(torch.bfloat16)
    wd = (torch.randn(wl.hidden, wl.ffn, device="cuda:0") * 0.02).to(torch.bfloat16)
    o_ms = timed_ms(lambda: torch.matmul(go, wo.t()), 20)
    d_ms = timed_ms(lambda: torch.matmul(gd, wd.t()), 20)
    ceilings = dict(hbm_copy_GBs=round(2.0 * (1 << 30) / (copy_ms * 1e-3) / 1e9, 1),
                    library_gemm_TFLOPs=round(2.0 * 2048 * 2 * wl.ffn * wl.hidden / (mm_ms * 1e-3) / 1e12, 1),
                    library_gemm_o_proj_TFLOPs=round(2.0 * 2048 * wl.hidden * qd / (o_ms * 1e-3) / 1e12, 1),
                    library_gemm_down_proj_TFLOPs=round(2.0 * 2048 * wl.hidden * wl.ffn / (d_ms * 1e-3) / 1e12, 1),
                    note="1 GiB device-to-device copy (read + write bytes); torch.matmul bf16 with random operands, back to back with warm caches: "
                         "2048 x %d x %d (gate/up shape), 2048 x %d x %d (O), 2048 x %d x %d (down)" % (2 * wl.ffn, wl.hidden, wl.hidden, qd, wl.hidden, wl.ffn))
    del src, dst, ga, gw, go, wo, gd, wd

    def brief(r):
        return {k: r[k] for k in ("label", "ms_per_step", "decoded_tokens_per_s", "rows_full", "rows_packed", "steps", "row_hint", "gemm", "phases")}

    sweep = method = others = None
    extras = not args.no_extras and args.workload == "c4_batch256" and wl.budget_mode == 1 and not args.constant_weights
    if extras:
        es = max(2, min(args.steps, 6))
        sweep = [brief(head)] + [brief(R.measure(es, 1, "keep ratio %.3f" % r, keep_ratio=r)) for r in (1.0, 0.5, 0.125) if abs(r - ratio0) > 1e-9]
        # the method's own budget rule (Eq. 4-5, alpha 1.5), without and with the structural constraints of Sec. 4.2
        method = [brief(R.measure(es, 1, "dynamic budget alpha 1.5, constraints %d" % c, budget_mode=2, alpha=1.5, constraints=c)) for c in (0, 3)]

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, min(args.cpu_seqs, wl.batch), min(args.cpu_layers, wl.n_layers))

    setup_s = R.setup_s
    R.sess.focus.focus_free()
    if extras:
        others = []
        for name in ("c3_llada36", "c5_ragged"):
            del R
            torch.cuda.empty_cache()
            w2 = fi.workload(name)
            R = Runner(w2, pk, runner, torch)
            r = R.measure(min(args.steps, w2.steps if w2.steps > 1 else 4), 1, "keep ratio %.3f" % w2.keep_ratio if w2.budget_mode == 1 else "per-sequence budgets U{0..%d}" % w2.block_size)
            r = brief(r)
            r["workload"] = workload_text(w2, r["label"])
            others.append(r)
            R.sess.focus.focus_free()

    line = {
        "metric": "decoded tokens/s at batch %d (%s, bf16, 1 GPU)" % (n, "8B-shaped" if not wl.n_experts else "mixture-of-experts, 16B total / 1.4B active shape"), "value": head["decoded_tokens_per_s"],
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic" if not args.constant_weights else "synthetic, every weight overwritten with 0.01 (diagnostic run)",
        "config": {"workload": workload_text(wl, budget_text),
                   "rows_full": n * B, "rows_packed": head["rows_packed"], "decoded_per_step": head["decoded_per_step"], "row_hint": head["row_hint"],
                   "experts": None if not wl.n_experts else "%d experts x %d, %d per token, shared %d, dense below layer %d"
                              % (wl.n_experts, wl.expert_ffn, wl.experts_per_token, wl.shared_ffn, wl.first_moe_layer)},
        "roofline": roofline, "dense_gemm": dense_gemm, "attention_hbm": dict(bound="hbm", achieved=head["phases"]["attention"]["GBs"], peak=PEAK_HBM_GBS, unit="GB/s",
                                                                              frac=head["phases"]["attention"]["frac_of_hbm_peak"], kv_bytes_per_step=head["phases"]["attention"]["bytes_per_step"]),
        "phases": head["phases"], "kernel_classes_ms": classes, "ceilings": ceilings, "cpu_baseline": cpu,
        "sweep": sweep, "method_budget": method, "other_workloads": others, "setup_s": round(setup_s, 1),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
