#!/usr/bin/env python3
"""Benchmark of the Tempo hot path on one MI355X.

A step is one pass of the whole hot path of one encoder layer over one batch of synthetic
input: GELU fwd+bwd, two LayerNorms fwd+bwd, attention softmax-dropout fwd+bwd, all through
the C ABI.  Inputs are resident in HBM before the timed region; buffer sets are rotated so
that nothing is served from the 256 MB Infinity Cache.  One JSON line is printed.

    python bench.py [--steps K] [--warmup W] [--config 4 --batch 64 --dtype f32] [--no-cpu-baseline]

With no arguments the headline workload is configuration 4 (RoBERTa-large-shaped full-layer
sweep) at its largest batch, 64, in float32 (the paper accounts activations at 32 bits), and
the per-kernel tables of the same batch in bfloat16 and of configurations 1-3 are measured in
the same run and reported under "other_workloads".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor peak
ROTATE_BYTES = 2048 << 20      # distinct bytes a kernel must touch before it sees a buffer again
METRIC = "fwd+bwd HBM GB/s (% of peak) per layer; activation bytes saved/token"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults long enough for the clocks to settle: short runs read 3-4 % low
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--config", type=int, default=None,
                    help="workload configuration index (0-4); default: 4 at batch 64 in f32, "
                         "followed by the other workloads' per-kernel tables")
    ap.add_argument("--batch", type=int, default=None, help="batch override (config 4 sweep)")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default=None)
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default run only: skip the per-kernel tables of the other workloads")
    ap.add_argument("--seq", type=int, default=None, help="sequence length override (shape sweeps)")
    ap.add_argument("--hidden", type=int, default=None, help="hidden size override; heads = hidden/64")
    ap.add_argument("--kernel-iters", type=int, default=60, help="launches per kernel timing burst")
    ap.add_argument("--kernel-bursts", type=int, default=5, help="timed bursts per kernel")
    ap.add_argument("--kernel-warm-ms", type=float, default=30.0,
                    help="untimed replays of a kernel's burst before it is timed")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every kernel from Python instead of replaying HIP graphs")
    ap.add_argument("--only", default=None, help="time only this kernel (for profiling)")
    return ap.parse_args()


def unmasked_fraction(cfg, key_len=None):
    """Share of the score entries the attention forward has to read: masked entries (padding
    beyond key_len[b], or above the causal diagonal) are never needed."""
    if cfg.mask == "causal":
        return (cfg.seq + 1) / (2 * cfg.seq)
    if cfg.mask == "padding" and key_len is not None:
        return float(sum(min(max(int(k), 0), cfg.seq) for k in key_len)) / (len(key_len) * cfg.seq)
    return 1.0


def algorithmic_bytes(cfg, key_len=None):
    """Bytes each kernel must move per launch (reads of inputs + writes of outputs).  The
    attention forward counts only the unmasked score reads (all writes: dense consumers expect
    the zeros); "attn_fwd_dense" is the same with every score counted as read."""
    e = cfg.elem_bytes
    n_g = cfg.tokens * cfg.ffn
    N, M = cfg.tokens, cfg.hidden
    n_a = cfg.batch * cfg.heads * cfg.seq * cfg.seq
    return {
        "gelu_fwd": n_g * 2 * e + n_g / 8,
        "gelu_bwd": n_g * 3 * e + n_g / 8,
        "layernorm_fwd": N * M * 2 * e + 4 * N + 8 * M,
        "layernorm_bwd": N * M * 3 * e + 4 * N + 16 * M,
        "attn_fwd": n_a * (2 + unmasked_fraction(cfg, key_len)) * e + n_a / 8,
        "attn_fwd_dense": n_a * 3 * e + n_a / 8,
        "attn_bwd": n_a * 4 * e + n_a / 8,
        # variant outside the step: backward that draws the keep bits again, no mask read
        "attn_bwd_regen": n_a * 4 * e,
        # and the backward that reads the paper's mask layout, one byte per element
        "attn_bwd_bytemask": n_a * 4 * e + n_a,
        # the activation kernels on SiLU tables (same traffic as GELU)
        "silu_fwd": n_g * 2 * e + n_g / 8,
        "silu_bwd": n_g * 3 * e + n_g / 8,
    }


def activation_bytes_saved(cfg):
    """Bytes per token and layer that need not be kept for backward, by tensor inventory."""
    e, H, A, S = cfg.elem_bytes, cfg.hidden, cfg.heads, cfg.seq
    kept_base = {"gelu": 4 * H * e, "layernorm": 2 * (H * e + 8), "attention": 3 * A * S * e + A * S}
    kept_here = {"gelu": (4 * H) // 8, "layernorm": 2 * 4, "attention": A * S * e + (A * S) // 8}
    return {k: kept_base[k] - kept_here[k] for k in kept_base}


class Buffers:
    """R rotating sets of device buffers for one kernel family."""

    def __init__(self, make, footprint, min_sets=4):
        self.n = max(min_sets, min(16, -(-ROTATE_BYTES // max(footprint, 1))))
        self.sets = [make(i) for i in range(self.n)]
        self.i = 0

    def next(self):
        s = self.sets[self.i]
        self.i = (self.i + 1) % self.n
        return s


DEFAULT_WORKLOAD = dict(index=4, batch=64, dtype="f32")
# measured beside the headline in a default run: per-kernel tables only
OTHER_WORKLOADS = (dict(index=4, batch=64, dtype="bf16"), dict(index=1), dict(index=2), dict(index=3))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2210_10246_amd import binding as B
    from paper_2210_10246_amd import workloads as W

    B.load()
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    default_run = args.config is None
    if default_run:
        d = DEFAULT_WORKLOAD
        cfg = W.config(d["index"], batch=args.batch or d["batch"], dtype=args.dtype or d["dtype"])
    else:
        cfg = W.config(args.config, batch=args.batch, dtype=args.dtype)
    if args.seq is not None or args.hidden is not None:
        from dataclasses import replace
        hidden = args.hidden or cfg.hidden
        seq = args.seq or cfg.seq
        lo, hi = (seq // 2, seq) if cfg.mask == "padding" else (0, 0)
        cfg = replace(cfg, seq=seq, hidden=hidden, heads=hidden // 64, len_lo=lo, len_hi=hi,
                      name=f"{cfg.name}-s{seq}-h{hidden}")
    import gc
    line = measure(cfg, args, headline=True)
    if default_run and not args.no_other_workloads and args.only is None and not args.no_kernel_timing:
        others = {}
        for o in OTHER_WORKLOADS:
            ocfg = W.config(o["index"], batch=o.get("batch"), dtype=o.get("dtype"))
            gc.collect()             # the previous workload's buffers and graphs
            torch.cuda.empty_cache()
            r = measure(ocfg, args, headline=False)
            others[r["config"]["workload"]] = {
                "dtype": r["dtype"], "value": r["value"], "ms_per_step": r["ms_per_step"],
                "frac_of_hbm_peak": r["frac_of_hbm_peak"], "worst_kernel": r["worst_kernel"],
                "kernels": {k: {f: v[f] for f in ("us", "GB/s", "frac_of_peak", "bytes",
                                                  "frac_of_pattern_copy") if f in v}
                            for k, v in r["kernels"].items()}}
        line["other_workloads"] = others
    print(json.dumps(line))


def measure(cfg, args, headline):
    """One workload: the whole step timed over args.steps steps (a fifth of that for the
    workloads measured beside the headline), then every kernel on its own."""
    import numpy as np
    import torch
    from paper_2210_10246_amd import binding as B
    from paper_2210_10246_amd import workloads as W

    dev = torch.device("cuda:0")
    steps = args.steps if headline else max(8, args.steps // 5)
    warmup = args.warmup if headline else max(4, args.warmup // 5)
    dt = cfg.dtype
    tdt = W.torch_dtype(dt)
    e = cfg.elem_bytes
    N, M = cfg.tokens, cfg.hidden
    shape_a = (cfg.batch, cfg.heads, cfg.seq, cfg.seq)
    n_g, n_a = N * cfg.ffn, int(np.prod(shape_a))
    # ---- seeded inputs, generated once on the host and copied into every rotating set
    g_in = W.gelu_inputs(cfg)
    l_in = W.layernorm_inputs(cfg)
    a_in = W.attention_inputs(cfg)
    algo = algorithmic_bytes(cfg, None if a_in["key_len"] is None else a_in["key_len"].tolist())
    key_len = None if a_in["key_len"] is None else a_in["key_len"].to(dev)
    gamma, beta = l_in["gamma"].to(dev), l_in["beta"].to(dev)
    gx0, gdy0 = g_in["x"].to(dev), g_in["dy"].to(dev)
    lx0, ldy0 = l_in["x"].to(dev), l_in["dy"].to(dev)
    as0, ado0 = a_in["scores"].to(dev), a_in["dout"].to(dev)
    ws_bytes = B.tempo_layernorm_bwd_workspace_bytes(N, M)

    def gelu_set(_):
        return dict(x=gx0.clone(), dy=gdy0.clone(), y=torch.empty_like(gx0), dx=torch.empty_like(gx0),
                    m=torch.empty(B.mask_words(n_g), dtype=torch.int32, device=dev))

    def ln_set(_):
        return dict(x=lx0.clone(), dy=ldy0.clone(), y=torch.empty_like(lx0), dx=torch.empty_like(lx0),
                    rstd=torch.empty(N, dtype=torch.float32, device=dev),
                    dg=torch.empty(M, dtype=torch.float32, device=dev),
                    db=torch.empty(M, dtype=torch.float32, device=dev),
                    ws=torch.empty(ws_bytes, dtype=torch.uint8, device=dev))

    def attn_set(_):
        return dict(s=as0.clone(), do=ado0.clone(), P=torch.empty_like(as0), out=torch.empty_like(as0),
                    dS=torch.empty_like(as0), out_re=torch.empty_like(as0),
                    k=torch.empty(B.mask_words(n_a), dtype=torch.int32, device=dev))

    gelu_b = Buffers(gelu_set, 4 * n_g * e)
    ln_b = Buffers(ln_set, 4 * N * M * e, min_sets=8)   # a step runs two LayerNorms
    attn_b = Buffers(attn_set, 6 * n_a * e)
    seed, p, kind, eps = cfg.dropout_seed, cfg.p, cfg.gelu_kind, cfg.eps
    causal = a_in["causal"]

    def k_gelu_fwd(s): B.tempo_gelu_fwd(s["x"], s["y"], s["m"], kind)
    def k_gelu_bwd(s): B.tempo_gelu_bwd(s["dy"], s["y"], s["m"], s["dx"], kind)
    def k_ln_fwd(s): B.tempo_layernorm_fwd(s["x"], gamma, beta, s["y"], s["rstd"], None, eps)
    def k_ln_bwd(s): B.tempo_layernorm_bwd(s["dy"], s["y"], gamma, beta, s["rstd"], s["dx"], s["dg"], s["db"], s["ws"])
    def k_attn_fwd(s): B.tempo_attn_softmax_dropout_fwd(s["s"], key_len, causal, s["P"], s["out"], s["k"], p, seed, 0)
    def k_attn_bwd(s): B.tempo_attn_softmax_dropout_bwd(s["do"], s["P"], s["k"], s["dS"], s["out_re"], p)

    def k_attn_bwd_regen(s): B.tempo_attn_softmax_dropout_bwd_regen(s["do"], s["P"], s["dS"], s["out_re"], p, seed, 0)

    def k_attn_bwd_bytemask(s):
        if "kb" not in s:      # the byte mask of this set, made once from its bit mask
            s["kb"] = torch.empty(n_a, dtype=torch.uint8, device=dev)
            B.tempo_mask_bits_to_bytes(s["k"], s["kb"], n_a)
        B.tempo_attn_softmax_dropout_bwd_bytemask(s["do"], s["P"], s["kb"], s["dS"], s["out_re"], p)

    kernels = {
        "gelu_fwd": (k_gelu_fwd, gelu_b), "gelu_bwd": (k_gelu_bwd, gelu_b),
        "layernorm_fwd": (k_ln_fwd, ln_b), "layernorm_bwd": (k_ln_bwd, ln_b),
        "attn_fwd": (k_attn_fwd, attn_b), "attn_bwd": (k_attn_bwd, attn_b),
    }
    def k_silu_fwd(s): B.tempo_silu_fwd(s["x"], s["y"], s["m"])
    def k_silu_bwd(s): B.tempo_silu_bwd(s["dy"], s["y"], s["m"], s["dx"])

    # timed, not part of the step
    variants = {"attn_bwd_regen": (k_attn_bwd_regen, attn_b),
                "attn_bwd_bytemask": (k_attn_bwd_bytemask, attn_b),
                "silu_fwd": (k_silu_fwd, gelu_b), "silu_bwd": (k_silu_bwd, gelu_b)}

    # every set gets a valid forward state once (backward kernels read y / P / masks)
    for s in gelu_b.sets: k_gelu_fwd(s)
    for s in ln_b.sets: k_ln_fwd(s)
    for s in attn_b.sets: k_attn_fwd(s)
    torch.cuda.synchronize()

    PHASES = 4   # a step of phase ph touches buffer sets that no other phase touches

    def step(ph):
        g, a = gelu_b.sets[ph], attn_b.sets[ph]
        l1, l2 = ln_b.sets[2 * ph], ln_b.sets[2 * ph + 1]
        # forward order of an encoder layer, then backward in reverse
        k_attn_fwd(a); k_ln_fwd(l1); k_gelu_fwd(g); k_ln_fwd(l2)
        k_ln_bwd(l2); k_gelu_bwd(g); k_ln_bwd(l1); k_attn_bwd(a)

    assert ln_b.n >= 2 * PHASES and gelu_b.n >= PHASES and attn_b.n >= PHASES
    step_bytes = (algo["gelu_fwd"] + algo["gelu_bwd"] + 2 * (algo["layernorm_fwd"] + algo["layernorm_bwd"])
                  + algo["attn_fwd"] + algo["attn_bwd"])

    def capture(fn):
        """Record fn's launches into a HIP graph (the kernels are launch-bound from Python:
        a LayerNorm launch lasts ~10 us, a ctypes call about as long)."""
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    use_graph = not args.no_graph
    ms_per_step = float("nan")
    if args.only is None:
        for i in range(PHASES):
            step(i)
        torch.cuda.synchronize()
        if use_graph:
            # one graph per step, and one holding PHASES consecutive steps: the timed loop
            # replays the long one steps // PHASES times and single steps for the remainder
            graphs = [capture(lambda ph=ph: step(ph)) for ph in range(PHASES)]
            def all_phases():
                for ph in range(PHASES):
                    step(ph)
            cycle = capture(all_phases)
            for gph in graphs + [cycle]:
                gph.replay()
            def run_steps(k):
                for _ in range(k // PHASES):
                    cycle.replay()
                for i in range(k % PHASES):
                    graphs[i].replay()
        else:
            def run_steps(k):
                for i in range(k):
                    step(i % PHASES)
        run_steps(warmup)   # the untimed warm-up steps, launched the same way as the timed ones
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(steps)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # ---- per-kernel launch durations: events on the stream the kernels are launched on,
    # around a replayed graph of kernel_iters back-to-back launches over rotating buffers
    def time_launches(fn, bufs):
        """Average duration of one launch of fn: events on the launch stream around
        kernel_bursts replays of a graph of kernel_iters back-to-back launches over the
        rotating buffer sets, after the clocks have settled."""
        for _ in range(max(3, bufs.n)):
            fn(bufs.next())
        torch.cuda.synchronize()

        def burst():
            for _ in range(args.kernel_iters):
                fn(bufs.next())
        body = capture(burst).replay if use_graph else burst
        t_warm = time.perf_counter()
        while True:
            body()
            torch.cuda.synchronize()
            if time.perf_counter() - t_warm > args.kernel_warm_ms * 1e-3:
                break
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(args.kernel_bursts):
            body()
        ev1.record()
        ev1.synchronize()
        return ev0.elapsed_time(ev1) * 1e3 / (args.kernel_iters * args.kernel_bursts)

    per_kernel = {}
    if not args.no_kernel_timing:
        for name, (fn, bufs) in {**kernels, **variants}.items():
            if args.only is not None and name != args.only:
                continue
            us = time_launches(fn, bufs)
            gbs = algo[name] / us * 1e-3
            per_kernel[name] = {"us": round(us, 2), "GB/s": round(gbs, 1),
                                "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4),
                                "bytes": int(algo[name]), "buffer_sets": bufs.n}
            if name + "_dense" in algo:   # every input element counted as read
                per_kernel[name]["dense_bytes"] = int(algo[name + "_dense"])
                per_kernel[name]["dense_GB/s"] = round(algo[name + "_dense"] / us * 1e-3, 1)

    # ---- the plain streaming kernel with each kernel's own mix of read and write tensors, on
    # that kernel's own buffers (run after every kernel has been timed: it overwrites outputs).
    # What the memory system delivers depends on the mix, so this is the ceiling to hold a
    # kernel against; the mask's 1/8 byte per element is left out of the pattern.
    pattern = {
        "gelu_fwd": (lambda s: ([s["x"]], [s["y"]]), gelu_b),
        "gelu_bwd": (lambda s: ([s["dy"], s["y"]], [s["dx"]]), gelu_b),
        "layernorm_fwd": (lambda s: ([s["x"]], [s["y"]]), ln_b),
        "layernorm_bwd": (lambda s: ([s["dy"], s["y"]], [s["dx"]]), ln_b),
        "attn_fwd": (lambda s: ([s["s"]], [s["P"], s["out"]]), attn_b),
        "attn_bwd": (lambda s: ([s["do"], s["P"]], [s["dS"], s["out_re"]]), attn_b),
    }
    if not args.no_kernel_timing:
        for name, (pick, bufs) in pattern.items():
            if name not in per_kernel:
                continue
            r0, w0 = pick(bufs.sets[0])
            us = time_launches(lambda s, pick=pick: B.tempo_copy_streams(*pick(s)), bufs)
            nb = (len(r0) + len(w0)) * r0[0].numel() * r0[0].element_size()
            gbs = nb / us * 1e-3
            k = per_kernel[name]
            k["pattern_copy"] = {"reads": len(r0), "writes": len(w0), "bytes": nb,
                                 "us": round(us, 2), "GB/s": round(gbs, 1)}
            k["frac_of_pattern_copy"] = round(k["GB/s"] / gbs, 4)

    # ---- what a plain 16-byte copy reaches on this GPU (read + write bytes per second): at
    # 256 MiB, and moving as many bytes as the slowest kernel of the step moves per launch
    def time_copy(nb):
        srcs = [torch.empty(nb, dtype=torch.uint8, device=dev).fill_(i) for i in range(3)]
        dsts = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(3)]

        def copies():
            for i in range(30):
                B.tempo_copy(srcs[i % 3], dsts[i % 3], blocks_per_cu=65536)   # one access per lane
        copies()
        torch.cuda.synchronize()
        body = capture(copies).replay if use_graph else copies
        t_warm = time.perf_counter()
        while True:
            body()
            torch.cuda.synchronize()
            if time.perf_counter() - t_warm > args.kernel_warm_ms * 1e-3:
                break
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        body()
        ev1.record()
        ev1.synchronize()
        us = ev0.elapsed_time(ev1) * 1e3 / 30
        return us, 2 * nb / us * 1e-3

    copy_gbs = None
    copy_same = None
    if not args.no_kernel_timing and args.only in (None, "copy"):
        copy_gbs = round(time_copy(256 << 20)[1], 1)
        in_step = {k: v for k, v in per_kernel.items() if k in kernels}
        if in_step:
            dom = max(in_step, key=lambda k: in_step[k]["us"])
            nb = int(in_step[dom]["bytes"] // 2) // 16 * 16
            us, gbs = time_copy(nb)
            copy_same = {"as_many_bytes_as": dom, "bytes": 2 * nb, "us": round(us, 2),
                         "GB/s": round(gbs, 1)}

    if copy_gbs:
        for v in per_kernel.values():
            v["frac_of_copy_kernel"] = round(v["GB/s"] / copy_gbs, 4)

    value = step_bytes / (ms_per_step * 1e-3) * 1e-9 if ms_per_step == ms_per_step else None
    roofline = None
    if per_kernel:
        weight = {k: v["us"] * (2 if k.startswith("layernorm") else 1) for k, v in per_kernel.items()
                  if k in kernels} or {k: v["us"] for k, v in per_kernel.items()}
        dom = max(weight, key=weight.get)
        k = per_kernel[dom]
        traffic, traffic_source = recorded_traffic(cfg, dom)
        roofline = {"kernel": dom, "bound": "hbm", "achieved": k["GB/s"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": k["frac_of_peak"], "traffic": traffic,
                    # not measured by this process: counters need a rocprofv3 run of their own
                    "traffic_source": traffic_source,
                    "us_per_launch": k["us"], "algorithmic_bytes": k["bytes"],
                    # the plain streaming kernel with this kernel's mix of read and write tensors
                    "pattern_copy": k.get("pattern_copy"),
                    "frac_of_pattern_copy": k.get("frac_of_pattern_copy")}
    # the kernel of the step furthest below the roofline
    worst = None
    in_step = {k: v for k, v in per_kernel.items() if k in kernels}
    if in_step:
        w = min(in_step, key=lambda k: in_step[k]["frac_of_peak"])
        worst = {"kernel": w, "frac": in_step[w]["frac_of_peak"], "GB/s": in_step[w]["GB/s"],
                 "us_per_launch": in_step[w]["us"],
                 "frac_of_pattern_copy": in_step[w].get("frac_of_pattern_copy")}

    cpu = None
    if headline and not args.no_cpu_baseline and args.only is None:
        cpu = cpu_baseline(cfg, algo)

    saved = activation_bytes_saved(cfg)
    # the same from the buffers this run actually used: what a standard layer keeps for backward
    # (its input, and for attention scores, P, Out and a byte mask) against what these kernels
    # keep (mask bits, rstd, P and mask bits); the outputs y are kept by both
    nbytes = lambda t: t.numel() * t.element_size()
    g0, l0, a0 = gelu_b.sets[0], ln_b.sets[0], attn_b.sets[0]
    measured = {
        "gelu": (nbytes(g0["x"]) - nbytes(g0["m"])) // N,
        "layernorm": 2 * (nbytes(l0["x"]) + nbytes(l0["rstd"])) // N,   # x and mean, twice
        "attention": (nbytes(a0["s"]) + nbytes(a0["out"]) + n_a - nbytes(a0["k"])) // N,
    }
    device = {"name": torch.cuda.get_device_name(0),
              "compute_units": torch.cuda.get_device_properties(0).multi_processor_count,
              "clocks": device_clocks()}
    line = {
        "metric": METRIC, "value": None if value is None else round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": None if value is None else round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dt,
        "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}, batch {cfg.batch}, {dt}", "batch": cfg.batch, "seq_len": cfg.seq,
                   "hidden": cfg.hidden, "heads": cfg.heads, "ffn": cfg.ffn, "mask": cfg.mask,
                   "dropout_p": cfg.p, "gelu": cfg.gelu_kind,
                   "step": "attn fwd, LN fwd, GELU fwd, LN fwd, LN bwd, GELU bwd, LN bwd, attn bwd",
                   "launch": "eager" if args.no_graph else "HIP graph replay (one graph of four steps, each on its own buffer sets)",
                   "algorithmic_bytes_per_step": int(step_bytes)},
        "frac_of_hbm_peak": None if value is None else round(value / HBM_PEAK_GBS, 4),
        # the same step with every score of the attention forward counted as read
        "value_dense_count": None if value is None else round(
            (step_bytes - algo["attn_fwd"] + algo["attn_fwd_dense"]) / (ms_per_step * 1e-3) * 1e-9, 1),
        "copy_kernel_GB/s": copy_gbs,
        "copy_kernel_same_bytes": copy_same,
        "roofline": roofline,
        "worst_kernel": worst,
        "cpu_baseline": cpu,
        "kernels": per_kernel,
        "activation_bytes_saved_per_token": {**saved, "total": sum(saved.values()),
                                             "from_buffers": measured},
        "device": device,
    }
    return line


def device_clocks():
    """Clock and power state as the driver's sysfs files report it (nothing is pinned by this
    benchmark).  Plain file reads: no child process is started from a process that uses the GPU."""
    import glob
    out = {}
    for card in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        for name in ("pp_dpm_sclk", "pp_dpm_mclk", "power_dpm_force_performance_level"):
            try:
                with open(f"{card}/{name}") as f:
                    text = f.read().strip()
            except OSError:
                continue
            lines = text.splitlines()
            active = [l.strip() for l in lines if l.rstrip().endswith("*")]
            out[name] = (active or lines)[:2]
        if out:
            break
    return out or None


def profile_tag(cfg):
    """Name of the committed rocprofv3 summaries of a workload: the configuration index, plus
    batch and dtype where they differ from the configuration's own."""
    from paper_2210_10246_amd import workloads as W
    base = W.config(cfg.index)
    tag = f"config{cfg.index}"
    if (cfg.batch, cfg.dtype) != (base.batch, base.dtype):
        tag += f"_b{cfg.batch}_{cfg.dtype}"
    return tag


def recorded_traffic(cfg, kernel):
    """HBM bytes per launch of `kernel` as recorded in the committed rocprofv3 FETCH_SIZE /
    WRITE_SIZE summary of this workload (counter values scaled by the copy-kernel calibration),
    and where that figure comes from; (None, None) if no summary is kept for the workload."""
    from paper_2210_10246_amd import workloads as W
    rel = os.path.join("profiles", f"hbm_traffic_{profile_tag(cfg)}.json")
    if cfg != W.config(cfg.index, batch=cfg.batch, dtype=cfg.dtype):
        return None, None    # a shape override: the recorded counters do not apply
    try:
        with open(os.path.join(ROOT, rel)) as f:
            rec = json.load(f)["kernels"][kernel]
    except (OSError, KeyError, ValueError):
        return None, None
    return int(rec["fetch_bytes"] + rec["write_bytes"]), f"recorded: {rel}"


def cpu_baseline(cfg, algo):
    """The float64 oracle, as it stands, on a leading fraction of the rows of the same
    workload, sized for roughly 10-30 s of single-threaded numpy work."""
    import numpy as np
    from oracle import tempo_oracle as O
    from paper_2210_10246_amd import workloads as W

    # leading 1/frac of the rows: 10-30 s of numpy work (rounding to bfloat16 costs the oracle
    # about twice what rounding to float32 does)
    total = (algo["gelu_fwd"] + algo["gelu_bwd"] + 2 * (algo["layernorm_fwd"] + algo["layernorm_bwd"])
             + algo["attn_fwd"] + algo["attn_bwd"]) / cfg.elem_bytes
    frac = 1
    while total / frac > (100e6 if cfg.dtype == "f32" else 50e6) and frac < cfg.batch:
        frac *= 2
    dt = cfg.dtype
    rows = max(1, cfg.tokens // frac)
    ab = max(1, cfg.batch // frac) if cfg.batch >= frac else 1
    a_frac = cfg.batch / ab
    g = W.gelu_inputs(cfg, rows=rows)
    l = W.layernorm_inputs(cfg, rows=rows)
    a = W.attention_inputs(cfg, batch=ab)
    gx, gdy = W.as_f64(g["x"]), W.as_f64(g["dy"])
    lx, ldy = W.as_f64(l["x"]), W.as_f64(l["dy"])
    gam, bet = W.as_f64(l["gamma"]), W.as_f64(l["beta"])
    sc, do = W.as_f64(a["scores"]), W.as_f64(a["dout"])
    kl = None if a["key_len"] is None else a["key_len"].numpy()
    t0 = time.perf_counter()
    y, m = O.gelu_fwd(gx, cfg.gelu_kind, dt)
    O.gelu_bwd(gdy, y, m, cfg.gelu_kind, dt)
    for _ in range(2):
        ly, rstd, _ = O.layernorm_fwd(lx, gam, bet, cfg.eps, dt)
        O.layernorm_bwd(ldy, ly, gam, bet, rstd, dt)
    P, _, K = O.attn_softmax_dropout_fwd(sc, kl, a["causal"], cfg.p, cfg.dropout_seed, 0, dt)
    O.attn_softmax_dropout_bwd(do, P, K, cfg.p, dt)
    sec = time.perf_counter() - t0
    row_frac = rows / cfg.tokens
    sample_bytes = ((algo["gelu_fwd"] + algo["gelu_bwd"]) * row_frac
                    + 2 * (algo["layernorm_fwd"] + algo["layernorm_bwd"]) * row_frac
                    + (algo["attn_fwd"] + algo["attn_bwd"]) / a_frac)
    return {"value": round(sample_bytes / sec * 1e-9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "seconds": round(sec, 2), "host_cores_available": os.cpu_count(),
            "sample": f"first {rows} of {cfg.tokens} rows for GELU and LayerNorm, first {ab} of "
                      f"{cfg.batch} sequences for attention; numpy float64, single thread"}


if __name__ == "__main__":
    main()
