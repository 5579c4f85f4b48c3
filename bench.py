#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X.

A step is one pass of the whole per-stage schedule (all m micro-batches: F, B, W of every one, plus the offloads
and reloads its memory budget needs, in the schedule's order) over synthetic tensors already resident in HBM.

Headline workload: the largest one a single GPU holds, the grouped-query bf16 stage (5 layers, hidden 8192,
64 query / 8 kv heads x 128, SwiGLU 28672, seq 4096; stage 3 of p = 16, m = 32) under its 120 GB activation budget,
with the dense-fill split B/W list the library's generator builds for that budget (offloads chosen item by item).
The other single-GPU workloads run as short named legs in the same process: the Llama bf16 stage without a budget,
the same shapes under 40 % of its activation peak (one transfer channel and two), the long-sequence stage under
64 GB.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBPS = 8000.0
HEADLINE = "cfg4_gqa_bf16"
KERNEL_NAMES = {"gemm_nt_store": "gemm_bf16_direct_kernel<NT, store>", "gemm_nt_resid": "gemm_bf16_direct_kernel<NT, residual>",
                "gemm_nt_qkv": "gemm_bf16_direct_kernel<NT, rotary epilogue>", "gemm_nt_gu": "gemm_bf16_direct_kernel<NT, SwiGLU epilogue>",
                "gemm_tn_accum": "gemm_bf16_direct_grouped_kernel<TN, fp32 accumulate>", "attn_fwd": "attn_fwd_mfma",
                "attn_bwd": "attn_bwd_dq_mfma + attn_bwd_dkv_mfma"}

PINNED = {}     # the process's pinned offload pool
CHUNKS = 1      # --chunks: model chunks on the stage (interleaved 1F1B instead of the configuration's schedule)
RECOMPUTE = 0   # --recompute: the memory-table variant in which F keeps no norm outputs and no MLP activation output


def schedule_flops(cfg):
    """Algorithmic flops of F + B + W for one micro-batch: 2*tokens*N*K per GEMM in each of F, B, W;
    causal attention 2*s^2*n_q*d forward, 5*s^2*n_q*d backward; elementwise work not counted."""
    s, h, f = cfg.seq * cfg.micro_batch, cfg.hidden, cfg.ffn
    gemm = 2 * s * (cfg.qkv_width * h + h * cfg.n_q_heads * cfg.head_dim + cfg.up_width * h + h * f)
    att = cfg.micro_batch * cfg.seq * cfg.seq * cfg.n_q_heads * cfg.head_dim
    return cfg.n_layers * (3 * gemm + 7 * att)


def class_algorithmic_bytes(cfg, name):
    """Mean algorithmic HBM bytes of one launch of a GEMM kernel class: every operand read once, the result written
    once (and read once where the epilogue adds to it), averaged over the launches of the class in one layer."""
    t, h, f = cfg.seq * cfg.micro_batch, cfg.hidden, cfg.ffn
    hq = cfg.n_q_heads * cfg.head_dim
    es = 2 if cfg.dtype == 1 else 4
    if name == "gemm_nt_store":       # the four dX products of B
        shapes = [(t, f, h), (t, h, cfg.up_width), (t, hq, h), (t, h, cfg.qkv_width)]
        return sum((m * k + n * k + m * n) * es for m, n, k in shapes) / len(shapes)
    if name == "gemm_nt_qkv":
        return (t * h + cfg.qkv_width * h + t * cfg.qkv_width) * es
    if name == "gemm_nt_gu":          # reads n2 and the weight, writes gate / up and (fused) the activation output
        return (t * h + cfg.up_width * h + t * cfg.up_width + t * f) * es
    if name == "gemm_nt_resid":       # output and down projections with the residual added
        shapes = [(t, h, hq), (t, h, f)]
        return sum((m * k + n * k + 2 * m * n) * es for m, n, k in shapes) / len(shapes)
    if name == "gemm_tn_accum":       # grouped launches over the 4 L weight-gradient products of a W op (class mean)
        shapes = [(h, f, t), (cfg.up_width, h, t), (h, hq, t), (cfg.qkv_width, h, t)]
        launches = -(-4 * cfg.n_layers // 16)                          # 16 products per grouped launch
        return cfg.n_layers * sum((m * k + n * k) * es + 2 * m * n * 4 for m, n, k in shapes) / launches
    return None


def measured_traffic(cfg, kernel_class):
    """HBM bytes per launch of a kernel class from the committed rocprofv3 --pmc summary of this same command
    (FETCH_SIZE and WRITE_SIZE scaled by what a plain copy of known size reads), and the digest of the kernel source
    the summary was taken with; None when there is no summary for this workload and class, or when the kernel
    source has changed since (the figure would describe another kernel)."""
    path = os.path.join(ROOT, "profiles", f"bench_{cfg.name.split('_')[0]}_hbm_traffic.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(rf"^traffic_bytes_per_launch\[{kernel_class}\]:\s*(\d+)", text, re.M)
    d = re.search(r"^kernel_source_sha256\[(\S+)\]:\s*([0-9a-f]+)", text, re.M)
    if not m or not d:
        return None
    src = os.path.join(ROOT, "paper_2510_05186_amd", "csrc", d.group(1))
    if hashlib.sha256(open(src, "rb").read()).hexdigest()[:16] != d.group(2)[:16]:
        return None
    return int(m.group(1))


def workload_budget(cfg):
    from paper_2510_05186_amd import binding as B
    from stage_inputs import configs as CFG
    from stage_inputs import schedules as G
    if cfg.budget_bytes:
        return cfg.budget_bytes
    if cfg.budget_frac_of_peak:
        base = G.split_bw_greedy(CFG.CFG2.n_stages, CFG.CFG2.n_microbatches)[CFG.CFG2.stage_index]
        return int(cfg.budget_frac_of_peak * B.plan(CFG.CFG2, base)[2])
    return 0


def build_lists(cfg, budget, duplex=False, t_op=None, link_gbps=55.0, reload_gbps=None):
    """The lists of all p stages (each shaped like this one) and what the generator decided."""
    from paper_2510_05186_amd import scheduler as SC
    from stage_inputs import schedules as G
    p, m = cfg.n_stages, cfg.n_microbatches
    if CHUNKS > 1:
        if budget:
            raise RuntimeError("--chunks runs the interleaved list without a budget")
        return [G.interleaved_one_f_one_b(p, m, i, CHUNKS) for i in range(p)], {"schedule": "interleaved 1F1B", "chunks": CHUNKS}
    if cfg.schedule == "1f1b":
        return [G.one_f_one_b(p, m, i) for i in range(p)], {"schedule": "1F1B"}
    lists, info = SC.workload_lists(cfg, budget, t_op=t_op, link_gbps=link_gbps, reload_gbps=reload_gbps, duplex=duplex,
                                    recompute=RECOMPUTE)
    i = cfg.stage_index
    knobs = {"generator": "split B/W greedy fill" + (", per-item offload under the budget, fill level by modelled makespan" if budget else ""),
             "in_flight_cap": info["caps"][i], "extra_fill": info["extra_fill"],
             "offload": info["offloaded_bytes"][i] > 0, "offloaded_bytes_per_step": info["offloaded_bytes"][i]}
    if "makespan_model" in info:
        knobs["model_makespan_ms"] = info["makespan_model"]
        knobs["candidates"] = [(c["extra_fill"], round(c["makespan_model"], 1)) for c in info["candidates"]]
    return lists, knobs


def make_stage(cfg, events, budget, duplex=False):
    from paper_2510_05186_amd import binding as B
    from paper_2510_05186_amd.stage import Stage
    from stage_inputs import tensors as T
    _, _, peak, _ = B.plan(cfg, events, budget=0, recompute=RECOMPUTE, n_chunks=CHUNKS)
    kb = B.query_sizes(cfg)[2]
    moved = sum(kb[k] for e in events if e[0] == "O" for k in e[3])
    # a budgeted handle is sized for ANY list under its budget (the generator is asked again once op times are
    # measured): arena from the budget, pinned pool for half as much again as the first list moves
    arena = int((min(peak, budget) if budget else peak) * 1.15) + (256 << 20)
    pool = None
    if moved:
        # one pinned block for the whole process, handed to every stage that offloads (the first one is the largest)
        import torch
        need = moved + moved // 2 + (256 << 20)
        if PINNED.get("pool") is None or PINNED["pool"].numel() < need:
            PINNED["pool"] = None
            PINNED["pool"] = torch.empty(need, dtype=torch.uint8, pin_memory=True)
        pool = PINNED["pool"]
    st = Stage(cfg, budget=budget, arena_bytes=arena, host_pool=pool,
               duplex=duplex, recompute=bool(RECOMPUTE), n_chunks=CHUNKS, grad_overwrite=True)
    st.set_weights_device(T.device_weights(cfg))
    for c in range(CHUNKS):
        for j in range(cfg.n_microbatches):
            x, dy = T.device_io(cfg, c * cfg.n_microbatches + j)
            st.bind(j, x, dy, chunk=c)
    return st, peak


def time_steps(st, events, steps, warmup, torch, kernel_timing=True):
    """W untimed steps, then K timed ones bracketed by device synchronisation.  The gradient accumulators are not
    cleared between steps: the first B / W of a step overwrite them (grad_overwrite)."""
    from paper_2510_05186_amd import binding as B
    arr = B.make_events(events)
    n = len(events)

    def one_step():
        st.reset()
        st.run_raw(arr, n)
        st.synchronize()

    for _ in range(warmup):
        one_step()
    B.check(st.lib.optstage_set_kernel_timing(st.h, 1 if kernel_timing else 0))
    torch.cuda.synchronize()
    agg = None
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step()
        s = st.stats()
        cur = {"ms_ops": list(s.ms_ops), "k_ms": list(s.kernel_ms), "k_work": list(s.kernel_work),
               "k_n": list(s.kernel_launches), "stall": list(s.stall_ms)}
        if agg is None:
            agg = cur
        else:
            for k in cur:
                agg[k] = [a + b for a, b in zip(agg[k], cur[k])]
        agg.update(peak=s.peak_bytes, off=s.bytes_offloaded, rel=s.bytes_reloaded, min_live=s.min_live_bytes,
                   avg_live=s.avg_live_bytes)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    B.check(st.lib.optstage_set_kernel_timing(st.h, 0))
    return wall, agg


def leg_record(cfg, events, budget, steps, wall, agg, knobs):
    """Throughput, op times, memory and transfer figures of one measured list."""
    flops = schedule_flops(cfg) * cfg.n_microbatches
    ms = wall / steps * 1e3
    n_f = cfg.n_microbatches * CHUNKS
    busy = sum(agg["ms_ops"][:3]) / steps
    rec = {"workload": cfg.name, "value": flops * steps / wall / 1e12, "unit": "TFLOP/s", "ms_per_step": ms, "steps": steps,
           "frac_of_bf16_peak": flops * steps / wall / 1e12 / (PEAK_BF16_TFLOPS if cfg.dtype == 1 else PEAK_FP32_TFLOPS),
           "mean_op_ms": {c: agg["ms_ops"][k] / steps / n_f for k, c in enumerate("FBW")},
           "stage_busy_frac": busy / ms, "hbm_budget_bytes": budget or None, "peak_hbm_bytes": agg["peak"],
           "avg_live_bytes": agg["avg_live"], "min_live_bytes_in_flight": agg["min_live"],
           "events": len(events), "events_sha256": hashlib.sha256(repr(list(map(tuple, events))).encode()).hexdigest()[:16],
           "schedule_knobs": knobs}
    if agg["off"]:
        rec["offload"] = {"bytes_offloaded_per_step": agg["off"], "bytes_reloaded_per_step": agg["rel"],
                          "d2h_GBps": agg["off"] * steps / (agg["ms_ops"][3] * 1e-3) / 1e9,
                          "h2d_GBps": agg["rel"] * steps / (agg["ms_ops"][5] * 1e-3) / 1e9,
                          "compute_stall_ms_per_step": {"at_owait": agg["stall"][0] / steps, "before_b": agg["stall"][1] / steps},
                          "stall_frac_of_step": (agg["stall"][0] + agg["stall"][1]) / steps / ms}
    return rec


def kernel_table(agg, steps, ms_per_step):
    from paper_2510_05186_amd import binding as B
    out = {}
    for i, name in enumerate(B.KERNEL_CLASSES):
        if agg["k_n"][i]:
            ms = agg["k_ms"][i]
            flop_class = i < 5 or i >= 10
            out[name] = {"launches_per_step": agg["k_n"][i] // steps, "avg_ms": ms / agg["k_n"][i],
                         "achieved": agg["k_work"][i] / (ms * 1e-3) / (1e12 if flop_class else 1e9),
                         "unit": "TFLOP/s" if flop_class else "GB/s", "share_of_step": ms / steps / ms_per_step}
    return out


def run_leg(cfg, duplex, steps, warmup, torch, kernel_timing=False, calibrate=True):
    """Builds the workload's lists, runs this stage's list, returns (record, kernels, context for the pipeline model)."""
    budget = workload_budget(cfg)
    lists, knobs = build_lists(cfg, budget, duplex)
    events = lists[cfg.stage_index]
    st, _ = make_stage(cfg, events, budget, duplex)
    if budget and calibrate and CHUNKS == 1:
        # one untimed step with the list built from nominal op times, then the generator again with the op times and
        # the host-link rate this box shows: the same handle takes the new list (a list may change every iteration)
        _, a0 = time_steps(st, events, 1, 0, torch, kernel_timing=False)
        n_f = cfg.n_microbatches
        t_op = {c: a0["ms_ops"][k] / n_f for k, c in enumerate("FBW")}
        link = a0["off"] / (a0["ms_ops"][3] * 1e-3) / 1e9 if a0["off"] and a0["ms_ops"][3] > 0 else 55.0
        back = a0["rel"] / (a0["ms_ops"][5] * 1e-3) / 1e9 if a0["rel"] and a0["ms_ops"][5] > 0 else link
        lists2, knobs2 = build_lists(cfg, budget, duplex, t_op=t_op, link_gbps=link, reload_gbps=back)
        knobs2["calibrated_with"] = {"t_op_ms": t_op, "d2h_GBps": link, "h2d_GBps": back}
        ev2 = lists2[cfg.stage_index]
        from paper_2510_05186_amd import binding as B
        kb = B.query_sizes(cfg)[2]
        moved = lambda ev: sum(kb[k] for e in ev if e[0] == "O" for k in e[3])
        if moved(ev2) == 0 or (st.host_pool is not None and moved(ev2) + (64 << 20) <= st.host_pool.numel()):
            lists, knobs, events = lists2, knobs2, ev2       # fits the pinned pool this stage was created with
        else:
            knobs["calibrated_list_not_taken"] = "needs a larger pinned pool or arena than this handle has"
    wall, agg = time_steps(st, events, steps, warmup, torch, kernel_timing=kernel_timing)
    rec = leg_record(cfg, events, budget, steps, wall, agg, knobs)
    rec["transfer_channels"] = 2 if duplex else 1
    kernels = kernel_table(agg, steps, rec["ms_per_step"]) if kernel_timing else None
    n_x = sum(1 for e in events if e[0] in ("O", "R"))
    ctx = {"cfg": cfg, "lists": lists, "events": events, "duplex": duplex, "budget": budget, "peak": agg["peak"],
           "t_op": [rec["mean_op_ms"][c] for c in "FBW"],
           "ms_per_byte": ((agg["ms_ops"][3] + agg["ms_ops"][5]) / steps / (agg["off"] + agg["rel"])) if n_x and agg["off"] else 0.0}
    st.close()
    del st
    torch.cuda.empty_cache()
    return rec, kernels, ctx


def compute_only_ms(cfg, events, torch):
    """The same compute order with no transfer and no budget: what the step would take if copies cost nothing."""
    comp = [e for e in events if e[0] in ("F", "B", "W")]
    st, _ = make_stage(cfg, comp, 0)
    wall, _ = time_steps(st, comp, 1, 1, torch, kernel_timing=False)
    st.close()
    del st
    torch.cuda.empty_cache()
    return wall * 1e3


def cpu_baseline(cfg):
    """The fp64 oracle, as it stands, timed on this machine's host cores on a bounded sample of the headline workload:
    ONE layer, one micro-batch, F + B + W at full shape."""
    import numpy as np
    from dataclasses import replace

    from oracle import stage_fp64 as O
    from stage_inputs import tensors as T
    one = replace(cfg, n_layers=1)
    sh = O.StageShape(one.family, 1, one.hidden, one.n_q_heads, one.n_kv_heads, one.head_dim, one.ffn, one.seq,
                      one.norm_eps, one.rope_base)
    ws = [{k: v.astype(np.float64) for k, v in T.layer_weights(one, 0).items()}]
    x = T.stage_input(one, 0).astype(np.float64)
    dy = T.output_grad(one, 0).astype(np.float64)
    t0 = time.perf_counter()
    O.stage_fbw(sh, ws, x, dy, attn_chunk=1024)
    dt = time.perf_counter() - t0
    fl = sum(O.flops_per_microbatch(sh).values())
    try:
        import threadpoolctl
        threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        threads = os.cpu_count()
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"1 of {cfg.n_layers} layers, 1 of {cfg.n_microbatches} micro-batches of {cfg.name}, F+B+W at full shape "
                      f"({fl / 1e12:.2f} TFLOP fp64 in {dt:.1f} s)", "host_cpus": os.cpu_count()}


def pipeline_model(ctx):
    """The oracle's simulator over all p stages' lists (every stage shaped like this one), fed with this stage's
    measured mean op times and its measured transfer time per byte: the stage's bubble fraction under the budget and
    the peak of the oracle's list-order accounting, which must equal what the library's allocator recorded."""
    from oracle import schedule as S
    cfg = ctx["cfg"]
    p, i = cfg.n_stages, cfg.stage_index
    t = S.memory_table(cfg.family, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn,
                       cfg.seq * cfg.micro_batch, cfg.elem_size)
    t_op = [dict(zip("FBW", ctx["t_op"]))] * p
    copy = lambda st, ev: ctx["ms_per_byte"] * sum(t[k] for k in ev[3])
    kw = dict(t_copy=copy, duplex=ctx["duplex"], n_chunks=CHUNKS, layers_per_chunk=cfg.n_layers // CHUNKS)
    tm = S.simulate(ctx["lists"], t_op, t_comm=0.0, **kw)
    # second run with the neighbour exchange priced: one [tokens, hidden] tensor over a 153 GB/s point-to-point link
    t_comm = cfg.seq * cfg.micro_batch * cfg.hidden * cfg.elem_size / 153e9 * 1e3
    tc = S.simulate(ctx["lists"], t_op, t_comm=t_comm, **kw)
    peak, _ = S.account_memory(ctx["events"], cfg.n_layers, t, limit=ctx["budget"] or None, recompute=bool(RECOMPUTE), n_chunks=CHUNKS)
    return {"stage_bubble_frac": tm.bubble[i], "makespan_ms": tm.makespan_global, "simulator_peak_bytes": peak,
            "allocator_peak_bytes": ctx["peak"], "peaks_equal": peak == ctx["peak"],
            "assumption": "p identical stages with this stage's measured mean T_F / T_B / T_W and transfer time per byte, "
                          "every device under the same byte budget, T_comm = 0",
            "with_t_comm": {"t_comm_ms": t_comm, "stage_bubble_frac": tc.bubble[i], "makespan_ms": tc.makespan_global}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default=HEADLINE)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle legs (cpu_baseline, pipeline models)")
    ap.add_argument("--no-legs", action="store_true", help="run the headline workload only")
    ap.add_argument("--duplex", action="store_true",
                    help="reloads on a stream of their own instead of the single transfer channel (headline workload)")
    ap.add_argument("--chunks", type=int, default=1,
                    help="model chunks on the stage: runs interleaved 1F1B over them (layers split evenly)")
    ap.add_argument("--recompute", action="store_true",
                    help="memory-table variant: F keeps no norm outputs and no MLP activation output, B rebuilds them")
    ap.add_argument("--microbatches", type=int, default=0,
                    help="run the workload with this many micro-batches instead of its own count (a shorter run for "
                         "counter profiles: the per-dispatch figures of a kernel do not depend on it); implies --no-legs")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a kernel of known traffic "
                         "that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(no collectives or sharding exist on this path)", file=sys.stderr)
        sys.exit(2)

    import torch

    from stage_inputs import configs as CFG
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the stage has no CPU path", file=sys.stderr)
        sys.exit(3)
    cfg = CFG.CONFIGS[args.config]
    if args.microbatches:
        from dataclasses import replace
        cfg = replace(cfg, n_microbatches=args.microbatches)
        args.no_legs = True
    global RECOMPUTE, CHUNKS
    RECOMPUTE = int(args.recompute)
    CHUNKS = max(1, args.chunks)
    if args.calibration_copy_mib:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    rec, kernels, ctx = run_leg(cfg, args.duplex, args.steps, args.warmup, torch, kernel_timing=True)
    peak_tf = PEAK_BF16_TFLOPS if cfg.dtype == 1 else PEAK_FP32_TFLOPS
    # the dominant kernel: the class with the largest share of the step
    dom_name = max(kernels, key=lambda k: kernels[k]["share_of_step"])
    dom = kernels[dom_name]
    flop_class = dom["unit"] == "TFLOP/s"
    peak = peak_tf if flop_class else PEAK_HBM_GBPS
    roofline = {"bound": "mfma" if flop_class else "hbm", "kernel": KERNEL_NAMES.get(dom_name, dom_name), "kernel_class": dom_name,
                "achieved": dom["achieved"], "peak": peak, "unit": dom["unit"], "frac": dom["achieved"] / peak,
                "avg_launch_ms": dom["avg_ms"], "launches_per_step": dom["launches_per_step"], "share_of_step": dom["share_of_step"],
                "algorithmic_bytes": class_algorithmic_bytes(cfg, dom_name), "traffic": measured_traffic(cfg, dom_name)}
    out = {
        "metric": "stage TFLOP/s (F+B+W) + bubble % under HBM budget; MFMA util vs bf16 peak",
        "value": rec["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "layers": cfg.n_layers, "hidden": cfg.hidden, "heads": cfg.n_q_heads,
                   "kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim, "ffn": cfg.ffn, "seq": cfg.seq,
                   "micro_batch": cfg.micro_batch, "stage": cfg.stage_index, "p": cfg.n_stages,
                   "m": cfg.n_microbatches, "schedule": cfg.schedule, "schedule_knobs": rec["schedule_knobs"],
                   "events": rec["events"], "events_sha256": rec["events_sha256"], "transfer_channels": rec["transfer_channels"],
                   "memory_table": "recompute n1, n2, a in B" if RECOMPUTE else "store all"},
        "frac_of_bf16_peak": rec["frac_of_bf16_peak"], "stage_busy_frac": rec["stage_busy_frac"],
        "mean_op_ms": rec["mean_op_ms"], "hbm_budget_bytes": rec["hbm_budget_bytes"], "peak_hbm_bytes": rec["peak_hbm_bytes"],
        "avg_live_bytes": rec["avg_live_bytes"], "min_live_bytes_in_flight": rec["min_live_bytes_in_flight"],
        "roofline": roofline, "kernels": kernels,
    }
    if "offload" in rec:
        out["offload"] = rec["offload"]
        out["offload"]["ms_same_order_without_copies"] = compute_only_ms(cfg, ctx["events"], torch)
        out["offload"]["overlap_cost"] = rec["ms_per_step"] / out["offload"]["ms_same_order_without_copies"]
    models = [("headline", ctx)]

    legs = {}
    if not args.no_legs and cfg.name == HEADLINE and CHUNKS == 1 and not RECOMPUTE:
        r2, k2, c2 = run_leg(CFG.CFG2, False, 3, 1, torch, kernel_timing=True)
        r2["kernels"] = k2
        legs["cfg2_llama_bf16"] = r2
        models.append(("cfg2_llama_bf16", c2))
        base3 = None
        for duplex in (False, True):
            r3, _, c3 = run_leg(CFG.CFG3, duplex, 2, 1, torch)
            if base3 is None:
                base3 = compute_only_ms(CFG.CFG3, c3["events"], torch)
            r3["ms_same_order_without_copies"] = base3
            r3["overlap_cost"] = r3["ms_per_step"] / base3
            name = "cfg3_llama_bf16_offload" + ("_duplex" if duplex else "")
            legs[name] = r3
            models.append((name, c3))
        r5, _, c5 = run_leg(CFG.CFG5, False, 2, 1, torch)
        r5["ms_same_order_without_copies"] = compute_only_ms(CFG.CFG5, c5["events"], torch)
        r5["overlap_cost"] = r5["ms_per_step"] / r5["ms_same_order_without_copies"]
        legs["cfg5_longseq_bf16"] = r5
        models.append(("cfg5_longseq_bf16", c5))
        out["legs"] = legs

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
        for name, c in models:
            pm = pipeline_model(c)
            if name == "headline":
                out["pipeline_model"] = pm
                out["bubble_frac_under_budget"] = pm["stage_bubble_frac"]
            else:
                legs[name]["pipeline_model"] = pm
    print(json.dumps(out))


if __name__ == "__main__":
    main()
