#!/usr/bin/env python3
"""Benchmark of the fused FP8-state AdamW step on one MI355X.

A "step" is one pass of the whole hot path (dequantize + inverse expansion, moment and weight
update, group statistics, exponent and scale, expansion + requantization) over one flat
parameter buffer with every input resident in HBM.  The default workload is the full
Llama-2-7B-sized parameter set (6.74e9 fp32 master weights, bf16 gradients, E4M3 moments with
group size 128).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--group-size 128]

The default run times the 7B set (the headline: `value`, `roofline`, `cpu_baseline`) and then the
other configurations of the report -- cfg1, cfg2, cfg4 at G = 32 / 128 / 512, cfg5 -- each at its
stated length, the sub-millisecond ones also at steady clocks, each beside the copy control (the
step's bytes in the step's access pattern without its arithmetic); they land in `configs` of the
same JSON line.  `--only` times the chosen workload alone.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def bytes_per_param(G: int) -> float:
    """Algorithmic HBM bytes per parameter per step: read w 4 + g 2 + m_q 1 + v_q 1 and write
    w 4 + m_q 1 + v_q 1, plus 4 fp32 metadata words per group read and written."""
    return 14.0 + 32.0 / G


def read_profile_traffic(workload: str, G: int):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "coat_fp8_adamw_step_%s_G%d_pmc.txt" % (workload, G))
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
    return float(m.group(1)) if m else None


def cpu_baseline(G: int, sample_params: int, steps: int):
    """The CPU oracle, as it stands, timed on this host on a bounded sample of the workload."""
    import numpy as np
    import synth_inputs as S
    from oracle import coat_ref as R
    n = sample_params
    w = S.weights(n, seed=0)
    st = S.zero_state(n, G)
    # step 1 starts from the all-zero state (cheaper: nothing to dequantize); it is not timed
    R.fp8_adamw_step(w, S.grads_normal(n, 0, 1, G=G, outlier_frac=0.01), st["m_q"], st["m_scale"], st["m_k"],
                     st["v_q"], st["v_scale"], st["v_k"], R.make_hparams(step=1, group_size=G, **HP))
    dt = 0.0
    for t in range(2, steps + 2):
        g = S.grads_normal(n, 0, t, G=G, outlier_frac=0.01)        # drawn outside the timed region
        t0 = time.perf_counter()
        R.fp8_adamw_step(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"],
                         R.make_hparams(step=t, group_size=G, **HP))
        dt += time.perf_counter() - t0
    assert np.all(np.isfinite(w))
    return dict(value=n * steps / dt, unit="params/s", cores=R.num_threads(), kind="oracle",
                sample="first %d parameters of the workload, %d steps after one untimed step, %.1f s" % (n, steps, dt))


def bench_half(args, C, S, torch, dev, gen, n, G):
    """coat_quant_group / coat_dequant_group alone: 5 + 8/G algorithmic bytes per element each
    (fp32 in + code and metadata out, or the reverse)."""
    x = S.torch_weights(n, dev, gen, sigma=1e-3)
    out = (torch.empty(n, dtype=torch.uint8, device=dev), torch.empty(n // G, dtype=torch.float32, device=dev),
           torch.empty(n // G, dtype=torch.float32, device=dev))
    C.coat_quant_group(x, G, out=out)
    y = torch.empty_like(x)

    def run():
        if args.op == "quant":
            C.coat_quant_group(x, G, out=out)
        else:
            C.coat_dequant_group(out[0], out[1], out[2], G, out=y)

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    avg_s = e0.elapsed_time(e1) / args.steps / 1e3
    algo = (5.0 + 8.0 / G) * n
    print(json.dumps({
        "metric": "elements/sec, coat_%s_group (E4M3, per-group scale + dynamic range expansion)" % args.op,
        "value": n * args.steps / wall, "unit": "elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d elements, G=%d" % (args.workload, n, G)},
        "roofline": {"bound": "hbm", "achieved": algo / avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": algo / avg_s / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "%s_kernel<%d>" % (args.op, G)}}))


def bench_act(args, C, S, torch, dev, gen):
    """The activation quantizers of Sec. 5.2 on a [tokens, hidden] bf16 tensor.  Several distinct
    input / output buffer sets are cycled so that the working set (far) exceeds the 256 MB of
    last-level cache and the figure is an HBM figure.  Algorithmic bytes per element:
      act_group        2 in + 1 out + 4/G scales                              = 3 + 4/G
      act_tensor       stage 1: 2 in + 4/G out (the reduction rides along); then 2 in + 1 out = 5 + 4/G
      act_tensor_pre   (group maxima supplied) 4/G in + 2 in + 1 out           = 3 + 4/G"""
    G = args.act_group_size
    hidden = 4096
    n = args.act_tokens * hidden
    ng = n // G
    sets = []
    for _ in range(args.act_buffers):
        x = S.torch_activations(n, dev, gen, hidden=hidden)
        sets.append(dict(x=x, q=torch.empty(n, dtype=torch.uint8, device=dev),
                         pg=torch.empty(ng, dtype=torch.float32, device=dev),
                         ts=torch.empty(1, dtype=torch.float32, device=dev),
                         ta=torch.empty(1, dtype=torch.float32, device=dev)))
    ws = C.act_workspace(dev)
    for b in sets:
        C.coat_act_quant_tensor(b["x"], G, out=(b["q"], b["ts"], b["pg"], b["ta"]), workspace=ws)   # group maxima for _pre

    def run(i):
        b = sets[i % len(sets)]
        if args.op == "act_group":
            C.coat_act_quant_group(b["x"], G, out=(b["q"], b["pg"]))
        elif args.op == "act_tensor":
            C.coat_act_quant_tensor(b["x"], G, out=(b["q"], b["ts"], b["pg"], b["ta"]), workspace=ws)
        else:
            C.coat_act_quant_tensor_from_group_amax(b["x"], b["pg"], G, out=(b["q"], b["ts"], b["ta"]), workspace=ws)

    for i in range(args.warmup):
        run(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        run(i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    avg_s = e0.elapsed_time(e1) / args.steps / 1e3
    per = {"act_group": 3.0 + 4.0 / G, "act_tensor": 5.0 + 4.0 / G, "act_tensor_pre": 3.0 + 4.0 / G}[args.op]
    algo = per * n
    print(json.dumps({
        "metric": "elements/sec, %s (bf16 -> E4M3, Sec. 5.2)" % args.op,
        "value": n * args.steps / wall, "unit": "elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "activations %d x %d, G=%d, %d buffer sets cycled" % (args.act_tokens, hidden, G, len(sets))},
        "roofline": {"bound": "hbm", "achieved": algo / avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": algo / avg_s / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "avg_call_us": avg_s * 1e6, "algorithmic_bytes_per_call": algo}}))


WORKLOAD_TEXT = {"cfg1": "one 1024x1024 weight", "cfg2": "one Llama-2-7B decoder layer",
                 "cfg3": "full Llama-2-7B-sized parameter set", "cfg4": "one Llama-2-7B decoder layer",
                 "cfg5": "full Llama-2-13B-sized parameter set"}


def run_step_config(C, S, torch, dev, workload, G, grads_kind, warmup, steps, steady_steps=0, copy_control=True,
                    flags=None, emit_bf16=False, multi=False, multi_small=0):
    """Allocate one workload, run `warmup` untimed and `steps` timed steps (HIP events around every
    launch, on the launch stream), optionally `steady_steps` more as one back-to-back block, then the
    copy control on the same buffers.  Returns the figures of one row of the report."""
    import time
    flags = flags or {}
    shapes_of = "cfg2" if workload == "cfg4" else workload
    n = S.workload_numel(shapes_of)
    assert n % G == 0
    gen = S.torch_generator(dev, 0)
    w = S.torch_weights(n, dev, gen)
    st = S.torch_zero_state(n, G, dev)
    if flags.get("bf16_scale"):
        st["m_scale"], st["v_scale"] = st["m_scale"].to(torch.bfloat16), st["v_scale"].to(torch.bfloat16)
    if flags.get("bf16_k"):
        st["m_k"], st["v_k"] = st["m_k"].to(torch.bfloat16), st["v_k"].to(torch.bfloat16)
    # two gradient buffers, alternated, so that consecutive steps do not see identical input
    if grads_kind == "normal":
        mask = S.torch_outlier_group_mask(n // G, dev, gen, 0.01 if workload != "cfg1" else 0.0)
        grads = [S.torch_grads_normal(n, dev, gen, G=G, outlier_mask=mask) for _ in range(2)]
        del mask
    else:
        grads = [S.torch_grads_lognormal(n, dev, gen) for _ in range(2)]
    w_bf16 = torch.empty(n, dtype=torch.bfloat16, device=dev) if emit_bf16 else None
    torch.cuda.synchronize()

    plans = None
    if multi:
        # the same flat buffers seen as the workload's separate tensors (the model's weight matrices, plus
        # multi_small extra 4096-element vectors standing in for norm weights), one plan per gradient buffer
        sizes = [r * c for r, c in S.workload_shapes(shapes_of)]
        for _ in range(multi_small):
            big = max(range(len(sizes)), key=lambda i: sizes[i])
            sizes[big] -= 4096
            sizes.append(4096)
        assert sum(sizes) == n and all(x % G == 0 for x in sizes)
        plans = []
        for gbuf in grads:
            tens, off = [], 0
            for x in sizes:
                d = dict(w=w[off:off + x], grad=gbuf[off:off + x], weight_decay=HP["weight_decay"])
                for k in ("m_q", "v_q"):
                    d[k] = st[k][off:off + x]
                for k in ("m_scale", "m_k", "v_scale", "v_k"):
                    d[k] = st[k][off // G:(off + x) // G]
                if emit_bf16:
                    d["w_bf16"] = w_bf16[off:off + x]
                tens.append(d)
                off += x
            plans.append(C.MultiPlan(tens, G))

    def step(t):
        hp = C.make_hparams(step=t, group_size=G, **flags, **HP)
        if plans is not None:
            C.coat_fp8_adamw_step_multi(plans[t & 1], hp)
        elif emit_bf16:
            C.coat_fp8_adamw_step_bf16w(w, w_bf16, grads[t & 1], st["m_q"], st["m_scale"], st["m_k"],
                                        st["v_q"], st["v_scale"], st["v_k"], hp)
        else:
            C.coat_fp8_adamw_step(w, grads[t & 1], st["m_q"], st["m_scale"], st["m_k"],
                                  st["v_q"], st["v_scale"], st["v_k"], hp)

    t = 0
    for _ in range(warmup):
        t += 1
        step(t)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        t += 1
        ev[i][0].record()
        step(t)
        ev[i][1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    launch_ms = [a.elapsed_time(b) for a, b in ev]
    avg_launch_s = sum(launch_ms) / len(launch_ms) / 1e3
    per_param = (bytes_per_param(G) + (2.0 if emit_bf16 else 0.0) - (8.0 / G if flags.get("bf16_scale") else 0.0)
                 - (8.0 / G if flags.get("bf16_k") else 0.0))
    algo_bytes = per_param * n
    row = dict(workload=workload, params=n, group_size=G, grads=grads_kind, steps=steps, warmup=warmup,
               ms_per_step=wall / steps * 1e3, avg_launch_ms=avg_launch_s * 1e3, params_per_s=n * steps / wall,
               hbm_gbs=algo_bytes / avg_launch_s / 1e9, algorithmic_bytes_per_launch=algo_bytes)
    row["frac_of_peak"] = row["hbm_gbs"] / HBM_PEAK_GBS
    if steady_steps:
        # a sub-millisecond kernel needs tens of milliseconds of back-to-back launches before the part
        # reaches its steady clocks: the same step, `steady_steps` launches timed as one block
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steady_steps):
            t += 1
            step(t)
        e1.record()
        torch.cuda.synchronize()
        s_ms = e0.elapsed_time(e1) / steady_steps
        row["steady"] = dict(steps=steady_steps, ms_per_step=s_ms, hbm_gbs=algo_bytes / s_ms / 1e6,
                             frac_of_peak=algo_bytes / s_ms / 1e6 / HBM_PEAK_GBS)
    finite = bool(torch.isfinite(w[:: max(1, n // (1 << 20))]).all().item())
    if not finite:
        sys.exit("bench.py: non-finite weights after the timed steps (%s)" % workload)
    if copy_control and not (emit_bf16 or flags.get("bf16_scale") or flags.get("bf16_k")):
        # the copy control: the same bytes in the same access pattern without the arithmetic (destroys the state)
        reps = max(steps, 5) + steady_steps
        for i in range(2):
            C.coat_bench_copy_control(w, grads[i & 1], st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], G)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            C.coat_bench_copy_control(w, grads[i & 1], st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], G)
        e1.record()
        torch.cuda.synchronize()
        c_gbs = algo_bytes / (e0.elapsed_time(e1) / reps) / 1e6
        best = row["steady"]["hbm_gbs"] if steady_steps else row["hbm_gbs"]
        row["copy_control_gbs"] = c_gbs
        row["frac_of_copy_control"] = best / c_gbs
    row["tensors"] = len(plans[0].tensors) if plans else 1
    del w, st, grads, plans, w_bf16
    torch.cuda.empty_cache()
    return row


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="cfg4 = the cfg2 shapes under log-normal gradients (use with --group-size 32/128/512)")
    ap.add_argument("--group-size", type=int, default=128)
    ap.add_argument("--grads", default=None, choices=["normal", "lognormal"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", action="store_true",
                    help="time the chosen workload alone (no report on the other configurations, no copy control)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27)
    ap.add_argument("--cpu-steps", type=int, default=24)
    ap.add_argument("--op", default="step",
                    choices=["step", "quant", "dequant", "act_group", "act_tensor", "act_tensor_pre", "copy_control"],
                    help="step: the fused optimizer step (the metric); quant / dequant: its two halves alone; "
                         "act_*: the activation quantizers (per group, per tensor with Group Scaling, the same "
                         "with the group maxima supplied); copy_control: the step's traffic without its arithmetic")
    ap.add_argument("--act-tokens", type=int, default=8192, help="rows of the activation tensor (hidden = 4096)")
    ap.add_argument("--act-group-size", type=int, default=16)
    ap.add_argument("--act-buffers", type=int, default=8)
    ap.add_argument("--m-e5m2", action="store_true", help="first moment in E5M2 (a cell of the paper's Table 1)")
    ap.add_argument("--v-e5m2", action="store_true", help="second moment in E5M2")
    ap.add_argument("--m-plain", action="store_true", help="first moment without dynamic range expansion")
    ap.add_argument("--v-plain", action="store_true", help="second moment without dynamic range expansion")
    ap.add_argument("--bf16-scale", action="store_true", help="per-group scales stored as bf16 (14 + 24/G B/param)")
    ap.add_argument("--precise-dq", action="store_true", help="the more accurate inverse expansion (COAT_FLAG_PRECISE_DQ)")
    ap.add_argument("--bf16-k", action="store_true", help="per-group exponents stored as bf16 (with --bf16-scale: 14 + 16/G B/param)")
    ap.add_argument("--emit-bf16", action="store_true", help="also write the bf16 copy of the new weights (+2 B/param)")
    ap.add_argument("--multi", action="store_true",
                    help="step the workload as its separate tensors through ONE multi-tensor launch")
    ap.add_argument("--multi-small", type=int, default=0, help="with --multi: also split off this many 4096-element tensors")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain device copy of known size instead (scales the rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the step needs no communication; a sharded run is "
                 "the same kernel on n/P elements per GPU). Use --gpus 1.")

    import torch
    import paper_2410_19313_amd as C
    import synth_inputs as S

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU path to time")
    C.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        # 4 GiB read + 4 GiB written per launch by torch's elementwise copy kernel
        src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "launches": args.steps,
                          "bytes_read_per_launch": src.numel() * 4, "bytes_written_per_launch": src.numel() * 4}))
        return
    G = args.group_size
    grads_kind = args.grads or ("lognormal" if args.workload == "cfg4" else "normal")
    n = S.workload_numel("cfg2" if args.workload == "cfg4" else args.workload)
    assert n % G == 0

    gen = S.torch_generator(dev, 0)
    if args.op.startswith("act_"):
        bench_act(args, C, S, torch, dev, gen)
        return
    if args.op in ("quant", "dequant"):
        bench_half(args, C, S, torch, dev, gen, n, G)
        return
    if args.op == "copy_control":
        # the control alone, under the step's report format (for profiles)
        w = S.torch_weights(n, dev, gen)
        st = S.torch_zero_state(n, G, dev)
        g = S.torch_grads_normal(n, dev, gen, G=G)
        for _ in range(args.warmup):
            C.coat_bench_copy_control(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], G)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            C.coat_bench_copy_control(w, g, st["m_q"], st["m_scale"], st["m_k"], st["v_q"], st["v_scale"], st["v_k"], G)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        print(json.dumps({"op": "copy_control", "workload": args.workload, "params": n, "group_size": G, "ms_per_launch": ms,
                          "hbm_gbs": bytes_per_param(G) * n / ms / 1e6, "frac_of_peak": bytes_per_param(G) * n / ms / 1e6 / HBM_PEAK_GBS}))
        return

    flags = dict(m_e5m2=args.m_e5m2, v_e5m2=args.v_e5m2, m_plain=args.m_plain, v_plain=args.v_plain, bf16_scale=args.bf16_scale,
                 bf16_k=args.bf16_k, precise_dq=args.precise_dq)
    generic = any(flags.values())
    head = run_step_config(C, S, torch, dev, args.workload, G, grads_kind, args.warmup, args.steps,
                           copy_control=not args.only, flags=flags, emit_bf16=args.emit_bf16, multi=args.multi,
                           multi_small=args.multi_small)
    achieved = head["hbm_gbs"]
    out = {
        "metric": "params updated/sec, FP8-state AdamW (E4M3 m/v, per-group scale + dynamic range expansion)",
        "value": head["params_per_s"],
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %s, %d params, G=%d, grads %s" % (args.workload, WORKLOAD_TEXT[args.workload], n, G, grads_kind) + (
                    ", m %s%s, v %s%s" % ("E5M2" if args.m_e5m2 else "E4M3", "" if args.m_plain else "+expand",
                                            "E5M2" if args.v_e5m2 else "E4M3", "" if args.v_plain else "+expand")
                    if generic else "") + (", bf16 weight copy" if args.emit_bf16 else "") + (", bf16 scales" if args.bf16_scale else "") + (", bf16 exponents" if args.bf16_k else "") + (", precise dequantization" if args.precise_dq else "") + (
                        ", %d tensors in one multi-tensor launch" % head["tensors"] if args.multi else ""),
            "params": n, "group_size": G, "hbm_gbs": achieved, "hbm_frac_of_peak": achieved / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": (read_profile_traffic(args.workload, G)
                                 if not (generic or args.emit_bf16 or args.multi) else None),   # the counters were read for the default kernel
                     "algorithmic_bytes_per_launch": head["algorithmic_bytes_per_launch"], "avg_launch_ms": head["avg_launch_ms"],
                     "traffic_gbs": None,            # counter bytes over this run's launch time, filled in below
                     "copy_control_gbs": head.get("copy_control_gbs"), "frac_of_copy_control": head.get("frac_of_copy_control"),
                     "kernel": "adamw_step%s_kernel<%d, %s>" % ("_multi" if args.multi else "", G, "generic" if generic else "default")},
    }
    if out["roofline"]["traffic"]:
        out["roofline"]["traffic_gbs"] = out["roofline"]["traffic"] / (head["avg_launch_ms"] * 1e-3) / 1e9
    if not args.only and args.workload == "cfg3" and not (generic or args.emit_bf16 or args.multi):
        # the other configurations of the report, each at its stated length and, for the sub-millisecond
        # ones, once more at steady clocks; one row per configuration (cfg4: one per group size)
        rows = [run_step_config(C, S, torch, dev, "cfg1", 128, "normal", 3, 10, steady_steps=2000),
                run_step_config(C, S, torch, dev, "cfg2", 128, "normal", 3, 10, steady_steps=300)]
        for g4 in (32, 128, 512):
            rows.append(run_step_config(C, S, torch, dev, "cfg4", g4, "lognormal", 3, 10, steady_steps=300))
        free, _ = torch.cuda.mem_get_info()
        n5 = S.workload_numel("cfg5")
        if free > n5 * 10.2 + (4 << 30):
            rows.append(run_step_config(C, S, torch, dev, "cfg5", 128, "normal", 3, 5))
        else:
            rows.append(dict(workload="cfg5", skipped="needs %.0f GB of device memory, %.0f GB free" % (n5 * 10.2 / 1e9, free / 1e9)))
        head_row = {k: head[k] for k in ("workload", "params", "group_size", "grads", "steps", "warmup", "ms_per_step",
                                         "avg_launch_ms", "params_per_s", "hbm_gbs", "frac_of_peak") if k in head}
        head_row.update(copy_control_gbs=head.get("copy_control_gbs"), frac_of_copy_control=head.get("frac_of_copy_control"))
        out["configs"] = rows[:2] + [head_row] + rows[2:]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(G, min(args.cpu_sample, n), args.cpu_steps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
