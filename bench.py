#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X.

A step is one pass of the whole per-stage schedule (all m micro-batches: F, B, W of every one, in the
schedule's order) over synthetic tensors already resident in HBM.  Default workload: the Llama-style
bf16 stage (4 layers, hidden 4096, 32 heads x 128, SwiGLU 11008, seq 4096; stage 1 of p = 8, m = 16,
split B/W schedule, no offload).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3


def schedule_flops(cfg):
    """Algorithmic flops of F + B + W for one micro-batch: 2*tokens*N*K per GEMM in each of F, B, W;
    causal attention 2*s^2*n_q*d forward, 5*s^2*n_q*d backward; elementwise work not counted."""
    s, h, f = cfg.seq * cfg.micro_batch, cfg.hidden, cfg.ffn
    gemm = 2 * s * (cfg.qkv_width * h + h * cfg.n_q_heads * cfg.head_dim + cfg.up_width * h + h * f)
    att = cfg.micro_batch * cfg.seq * cfg.seq * cfg.n_q_heads * cfg.head_dim
    return cfg.n_layers * (3 * gemm + 7 * att)


def nt_store_algorithmic_bytes(cfg):
    """Mean algorithmic HBM bytes of one launch of the dominant kernel class (C = A B^T, plain store): each
    operand read once and the result written once, (M K + N K + M N) * elem_size, averaged over the six such
    GEMMs a layer runs per micro-batch (QKV and gate/up projections in F; the four dX GEMMs of B)."""
    t, h, f = cfg.seq * cfg.micro_batch, cfg.hidden, cfg.ffn
    hq = cfg.n_q_heads * cfg.head_dim
    shapes = [(t, cfg.qkv_width, h), (t, cfg.up_width, h), (t, f, h), (t, h, cfg.up_width), (t, hq, h), (t, h, cfg.qkv_width)]
    es = 2 if cfg.dtype == 1 else 4
    return sum((m * k + n * k + m * n) * es for m, n, k in shapes) / len(shapes)


def measured_traffic(cfg):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of this same
    command (FETCH_SIZE and WRITE_SIZE, scaled by what a plain copy of known size reads); None when no
    summary exists for this workload."""
    import re
    path = os.path.join(ROOT, "profiles", f"bench_{cfg.name.split('_')[0]}_hbm_traffic.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", open(path).read(), re.M)
    except OSError:
        return None
    return int(m.group(1)) if m else None


CHUNKS = 1      # --chunks: model chunks on the stage (interleaved 1F1B instead of the configuration's schedule)
RECOMPUTE = 0   # --recompute: the memory-table variant in which F keeps no norm outputs and no MLP activation output


def adaoffload_instance(cfg, budget, tflops=900.0, link_gbps=56.0):
    """The paper's abstract instance for this workload (all p stages alike): op times from the flop counts at a
    nominal rate, transfer time from the offloadable bytes at the measured host-link rate, Eq. 7's parameters
    from the library's memory table."""
    from paper_2510_05186_amd import binding as B
    from paper_2510_05186_amd import scheduler as SC
    s, h, f = cfg.seq * cfg.micro_batch, cfg.hidden, cfg.ffn
    gemm = 2 * s * (cfg.qkv_width * h + h * cfg.n_q_heads * cfg.head_dim + cfg.up_width * h + h * f)
    att = cfg.micro_batch * cfg.seq * cfg.seq * cfg.n_q_heads * cfg.head_dim
    ms = lambda fl: cfg.n_layers * fl / (tflops * 1e9)
    t_op = {"F": ms(gemm + 2 * att), "B": ms(gemm + 5 * att), "W": ms(gemm)}
    _, act_per_mb, kb = B.query_sizes(cfg, recompute=RECOMPUTE)
    gamma = sum(kb[k] for k in cfg.offload_kinds) * cfg.n_layers
    slack = 2 * (kb["DY"] + kb["DX_MID"])                 # what B holds beyond the forward activations
    rebuilt = RECOMPUTE * cfg.n_layers * (kb["N1"] + kb["N2"] + kb["A"])    # B makes them, W releases them
    p = cfg.n_stages
    return SC.Instance(p=p, m=cfg.n_microbatches, t_op=[t_op] * p, t_comm=0.0, t_off=[gamma / (link_gbps * 1e6)] * p,
                       delta=[{"F": act_per_mb, "B": rebuilt, "W": -act_per_mb - rebuilt}] * p, gamma=[gamma] * p,
                       limit=[max(budget - slack, act_per_mb)] * p, offload_stages=tuple(range(p)),
                       item=(0, tuple(cfg.offload_kinds)))


def build_schedule(cfg, budget=0, generator="greedy"):
    """Event list of this stage for the configuration's schedule family; with a budget the generator's
    knobs (in-flight cap, which micro-batches to offload, how long copies may overlap) are searched with the
    library's own planner until the list fits.  generator "adaoffload": the dense-fill list of the paper's
    Alg. 1 for the whole pipeline, this stage's part, repaired against the planner if it does not fit as is."""
    from paper_2510_05186_amd import binding as B
    from stage_inputs import schedules as G
    p, m, i = cfg.n_stages, cfg.n_microbatches, cfg.stage_index
    if CHUNKS > 1:
        if budget:
            raise RuntimeError("--chunks runs the interleaved list without a budget search")
        return G.interleaved_one_f_one_b(p, m, i, CHUNKS), {"schedule": "interleaved 1F1B", "chunks": CHUNKS}
    if budget and generator == "adaoffload":
        from paper_2510_05186_amd import scheduler as SC
        inst = adaoffload_instance(cfg, budget)
        sol = SC.adaoffload(inst, tolerance=0.5 * inst.t_op[0]["F"])
        ev = SC.expand_items(sol.lists[i], cfg.n_layers, cfg.offload_kinds)
        fits = lambda e: (lambda r: (r[0] == B.OK, r[1]))(B.plan(cfg, e, budget=budget, recompute=RECOMPUTE))
        knobs = {"generator": "adaoffload", "offload": any(e[0] == "O" for e in ev), "placement": "as generated"}
        build_schedule.all_stages = [SC.expand_items(l, cfg.n_layers, cfg.offload_kinds) for l in sol.lists]
        if not fits(ev)[0]:
            ev = G.repair_to_fit(ev, fits)
            knobs["placement"] = "repaired"
        if ev is not None:
            return ev, knobs
    if cfg.schedule == "1f1b":
        return G.one_f_one_b(p, m, i), {}
    if not budget:
        return G.split_bw_greedy(p, m)[i], {}
    for cap in range(p - i, 0, -1):
        comp = G.split_bw_greedy(p, m, cap_of_stage=lambda s, c=cap: c)[i]
        if B.plan(cfg, comp, budget=budget, recompute=RECOMPUTE)[0] == B.OK:
            return comp, {"in_flight_cap": cap, "offload": False}
        def fits(ev):
            st, bad, _, _ = B.plan(cfg, ev, budget=budget, recompute=RECOMPUTE)
            return st == B.OK, bad
        for lead in (2, 1):
            # optimistic placement (copies overlap neighbouring ops), then repaired against the planner
            ev = G.add_offload(comp, cfg.n_layers, cfg.offload_kinds, min_gap=1, lead=lead, wait_delay=2)
            if not any(e[0] == "O" for e in ev):
                continue
            ev = G.repair_to_fit(ev, fits)
            if ev is not None:
                return ev, {"in_flight_cap": cap, "offload": True, "lead": lead, "placement": "repaired"}
    raise RuntimeError("no schedule fits the budget")


def make_stage(cfg, events, budget, torch, duplex=False):
    from paper_2510_05186_amd import binding as B
    from stage_inputs import tensors as T
    from paper_2510_05186_amd.stage import Stage
    _, _, peak, _ = B.plan(cfg, events, budget=0, recompute=RECOMPUTE, n_chunks=CHUNKS)
    n_off = sum(1 for e in events if e[0] == "O")
    pool = 0
    if n_off:
        kb = B.query_sizes(cfg)[2]
        per_mb = sum(kb[k] for k in cfg.offload_kinds) * cfg.n_layers
        pool = per_mb * cfg.n_microbatches
    st = Stage(cfg, budget=budget, arena_bytes=int(peak * 1.15) + (256 << 20), host_pool_bytes=pool, duplex=duplex,
               recompute=bool(RECOMPUTE), n_chunks=CHUNKS)
    st.set_weights_device(T.device_weights(cfg))
    for c in range(CHUNKS):
        for j in range(cfg.n_microbatches):
            x, dy = T.device_io(cfg, c * cfg.n_microbatches + j)
            st.bind(j, x, dy, chunk=c)
    return st, peak


def time_steps(st, events, steps, warmup, torch, kernel_timing=True):
    from paper_2510_05186_amd import binding as B
    arr = B.make_events(events)
    n = len(events)

    def one_step():
        st.reset()
        with torch.cuda.stream(st.compute_stream):
            st.zero_grads_async()
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
               "k_n": list(s.kernel_launches), "peak": s.peak_bytes, "off": s.bytes_offloaded, "rel": s.bytes_reloaded}
        if agg is None:
            agg = cur
        else:
            for k in ("ms_ops", "k_ms", "k_work", "k_n"):
                agg[k] = [a + b for a, b in zip(agg[k], cur[k])]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    B.check(st.lib.optstage_set_kernel_timing(st.h, 0))
    return wall, agg


def oracle_leg(cfg, t_op_ms, events_all_stages, copy_ms_per_event, duplex=False, n_chunks=1):
    """CPU baseline: the fp64 oracle, as it stands, timed on this machine's host cores on a bounded sample
    (ONE layer of the workload's stage, one micro-batch, F + B + W at full shape), and the oracle's
    pipeline simulator fed with the measured op times (all p stages assumed identical to this one)."""
    import numpy as np

    from oracle import schedule as S
    from oracle import stage_fp64 as O
    from stage_inputs import tensors as T
    from dataclasses import replace
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
    base = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"1 of {cfg.n_layers} layers, 1 of {cfg.n_microbatches} micro-batches, F+B+W at full shape "
                      f"({fl / 1e12:.2f} TFLOP fp64 in {dt:.1f} s)", "host_cpus": os.cpu_count()}
    p = cfg.n_stages
    t_op = [{"F": t_op_ms[0], "B": t_op_ms[1], "W": t_op_ms[2]}] * p
    tm = S.simulate(events_all_stages, t_op, t_comm=0.0, t_copy=lambda i, ev: copy_ms_per_event, duplex=duplex,
                    n_chunks=n_chunks, layers_per_chunk=cfg.n_layers // n_chunks)
    # second run with the neighbour exchange priced: one [tokens, hidden] tensor over a 153 GB/s point-to-point link
    t_comm_ms = cfg.seq * cfg.micro_batch * cfg.hidden * cfg.elem_size / 153e9 * 1e3
    tc = S.simulate(events_all_stages, t_op, t_comm=t_comm_ms, t_copy=lambda i, ev: copy_ms_per_event, duplex=duplex,
                    n_chunks=n_chunks, layers_per_chunk=cfg.n_layers // n_chunks)
    model = {"stage_bubble_frac": tm.bubble[cfg.stage_index], "makespan_ms": tm.makespan_global,
             "assumption": "p identical stages with this stage's measured mean T_F/T_B/T_W, T_comm = 0",
             "with_t_comm": {"t_comm_ms": t_comm_ms, "stage_bubble_frac": tc.bubble[cfg.stage_index],
                             "makespan_ms": tc.makespan_global}}
    return base, model


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg2_llama_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-offload-leg", action="store_true")
    ap.add_argument("--generator", default="greedy", choices=("greedy", "adaoffload"),
                    help="how the event list of a budgeted workload is produced")
    ap.add_argument("--duplex", action="store_true",
                    help="reloads on a stream of their own instead of the single transfer channel (offload workloads)")
    ap.add_argument("--chunks", type=int, default=1,
                    help="model chunks on the stage: runs interleaved 1F1B over them (layers split evenly)")
    ap.add_argument("--recompute", action="store_true",
                    help="memory-table variant: F keeps no norm outputs and no MLP activation output, B rebuilds them")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a kernel of known traffic "
                         "that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(no collectives or sharding exist on this path)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2510_05186_amd import binding as B
    from stage_inputs import configs as CFG
    from stage_inputs import schedules as G
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the stage has no CPU path", file=sys.stderr)
        sys.exit(3)
    cfg = CFG.CONFIGS[args.config]
    global RECOMPUTE, CHUNKS
    RECOMPUTE = int(args.recompute)
    CHUNKS = max(1, args.chunks)
    budget = 0
    if cfg.budget_bytes:
        budget = cfg.budget_bytes
    elif cfg.budget_frac_of_peak:
        base_ev, _ = build_schedule(CFG.CFG2)
        budget = int(cfg.budget_frac_of_peak * B.plan(CFG.CFG2, base_ev)[2])
    events, knobs = build_schedule(cfg, budget, args.generator)
    if args.calibration_copy_mib:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    st, peak_plan = make_stage(cfg, events, budget, torch, args.duplex)
    wall, agg = time_steps(st, events, args.steps, args.warmup, torch)
    flops = schedule_flops(cfg) * cfg.n_microbatches
    ms_per_step = wall / args.steps * 1e3
    value = flops * args.steps / wall / 1e12
    peak_tf = PEAK_BF16_TFLOPS if cfg.dtype == 1 else PEAK_FP32_TFLOPS

    kernels = {}
    for i, name in enumerate(B.KERNEL_CLASSES):
        if agg["k_n"][i]:
            ms = agg["k_ms"][i]
            unit = "TFLOP/s" if i < 5 else "GB/s"
            rate = agg["k_work"][i] / (ms * 1e-3) / (1e12 if i < 5 else 1e9)
            kernels[name] = {"launches_per_step": agg["k_n"][i] // args.steps, "avg_ms": ms / agg["k_n"][i],
                             "achieved": rate, "unit": unit, "share_of_step": ms / args.steps / ms_per_step}
    dom = kernels.get("gemm_nt_store", {"achieved": 0.0})
    roofline = {"bound": "mfma", "kernel": "gemm_bf16_direct_kernel<NT,store>" if cfg.dtype == 1 else "gemm_f32_kernel",
                "achieved": dom["achieved"], "peak": peak_tf, "unit": "TFLOP/s", "frac": dom["achieved"] / peak_tf,
                "avg_launch_ms": dom.get("avg_ms"), "launches_per_step": dom.get("launches_per_step"),
                "algorithmic_bytes": nt_store_algorithmic_bytes(cfg), "traffic": measured_traffic(cfg)}
    busy_ms = sum(agg["ms_ops"][:3]) / args.steps
    n_f = cfg.n_microbatches * CHUNKS
    t_op_ms = [agg["ms_ops"][k] / args.steps / n_f for k in range(3)]
    out = {
        "metric": "stage TFLOP/s (F+B+W) + bubble % under HBM budget; MFMA util vs bf16 peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "layers": cfg.n_layers, "hidden": cfg.hidden, "heads": cfg.n_q_heads,
                   "kv_heads": cfg.n_kv_heads, "head_dim": cfg.head_dim, "ffn": cfg.ffn, "seq": cfg.seq,
                   "micro_batch": cfg.micro_batch, "stage": cfg.stage_index, "p": cfg.n_stages,
                   "m": cfg.n_microbatches, "schedule": cfg.schedule, "schedule_knobs": knobs,
                   "events": len(events), "events_sha256": hashlib.sha256(repr(list(map(tuple, events))).encode()).hexdigest()[:16],
                   "memory_table": "recompute n1, n2, a in B" if RECOMPUTE else "store all"},
        "frac_of_bf16_peak": value / peak_tf,
        "stage_busy_frac": busy_ms / ms_per_step,
        "stage_idle_frac": 1.0 - busy_ms / ms_per_step,
        "mean_op_ms": {"F": t_op_ms[0], "B": t_op_ms[1], "W": t_op_ms[2]},
        "peak_hbm_bytes": agg["peak"], "hbm_budget_bytes": budget or None,
        "roofline": roofline, "kernels": kernels,
    }
    if agg["off"]:
        out["offload"] = {"duplex": bool(args.duplex), "bytes_per_step": agg["off"], "d2h_GBps": agg["off"] * args.steps / (agg["ms_ops"][3] * 1e-3) / 1e9,
                          "h2d_GBps": agg["rel"] * args.steps / (agg["ms_ops"][5] * 1e-3) / 1e9}
    st.close()
    del st
    torch.cuda.empty_cache()

    if not args.no_offload_leg and cfg.name == "cfg2_llama_bf16" and CHUNKS == 1:
        # same shapes under 40 % of this run's activation peak, with offload of (attention input, QKV, MLP input):
        # on the single transfer channel of the paper's model and with reloads on a stream of their own
        c3 = CFG.CFG3
        b3 = int(c3.budget_frac_of_peak * peak_plan)
        ev3, knobs3 = build_schedule(c3, b3, args.generator)
        comp_only = [e for e in ev3 if e[0] in ("F", "B", "W")]
        st3b, _ = make_stage(c3, comp_only, 0, torch)
        w3b, _ = time_steps(st3b, comp_only, 1, 1, torch, kernel_timing=False)
        st3b.close()
        del st3b
        torch.cuda.empty_cache()
        legs = {}
        for duplex in (False, True):
            st3, _ = make_stage(c3, ev3, b3, torch, duplex)
            w3, a3 = time_steps(st3, ev3, 1, 1, torch, kernel_timing=False)
            st3.close()
            del st3
            torch.cuda.empty_cache()
            legs[duplex] = {
                "value": flops / w3 / 1e12, "unit": "TFLOP/s", "ms_per_step": w3 * 1e3, "overlap_cost": w3 / w3b,
                "d2h_GBps": a3["off"] / (a3["ms_ops"][3] * 1e-3) / 1e9 if a3["ms_ops"][3] else None,
                "h2d_GBps": a3["rel"] / (a3["ms_ops"][5] * 1e-3) / 1e9 if a3["ms_ops"][5] else None}
            peak3, off3, rel3 = a3["peak"], a3["off"], a3["rel"]
        out["offload_leg"] = {
            "workload": c3.name, "hbm_budget_bytes": b3, "peak_hbm_bytes": peak3, "schedule_knobs": knobs3,
            "ms_same_order_without_copies": w3b * 1e3, "bytes_offloaded": off3, "bytes_reloaded": rel3,
            "single_channel": legs[False], "duplex": legs[True]}

    if not args.no_cpu_baseline:
        lists = G.split_bw_greedy(cfg.n_stages, cfg.n_microbatches) if cfg.schedule != "1f1b" else \
            [G.one_f_one_b(cfg.n_stages, cfg.n_microbatches, i) for i in range(cfg.n_stages)]
        if CHUNKS > 1:
            lists = [G.interleaved_one_f_one_b(cfg.n_stages, cfg.n_microbatches, i, CHUNKS) for i in range(cfg.n_stages)]
        copy_ms = 0.0
        if args.generator == "adaoffload" and getattr(build_schedule, "all_stages", None) and budget:
            # the generator's lists for every stage, transfers included, with this stage's measured mean copy time
            lists = build_schedule.all_stages
            n_x = agg["k_n"] and sum(1 for e in events if e[0] in ("O", "R"))
            copy_ms = (agg["ms_ops"][3] + agg["ms_ops"][5]) / args.steps / n_x if n_x else 0.0
        base, model = oracle_leg(cfg, t_op_ms, lists, copy_ms, args.duplex, CHUNKS)
        model["lists"] = "adaoffload, all stages, transfers included" if copy_ms else "compute ops only"
        out["cpu_baseline"] = base
        out["pipeline_model"] = model
    print(json.dumps(out))


if __name__ == "__main__":
    main()
