"""Every benchmark workload in its own regime at full shape, through the C-ABI.

* the Llama bf16 stage (4 layers, hidden 4096, seq 4096): two micro-batches through all four layers against the
  fp64 oracle: outputs, input gradients, and the weight gradients accumulated over both;
* the same shapes under 40 % of the no-offload activation peak, the larger grouped-query stage under 120 GB with a
  dense fill, and the long-sequence stage under 64 GB: the lists the benchmark runs (per-item offload chosen by the
  library's generator) with the oracle's order rules and accounting event by event, a checksum of every offloaded
  buffer before its offload = in pinned memory = after its reload, and outputs and gradients bit for bit those of
  the same compute order without any transfer, single channel and duplex.
"""
import functools
import os
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import schedule as S
from oracle import stage_fp64 as O
from paper_2510_05186_amd import binding as B
from paper_2510_05186_amd import scheduler as SC
from paper_2510_05186_amd.stage import Stage
from stage_inputs import configs as CFG
from stage_inputs import schedules as G
from stage_inputs import tensors as T
from gpu_util import TOL, close, host, oracle_shape, rel_err, report, rms_err

pytestmark = pytest.mark.gpu
BF16 = 1
_KEEP = {}


def oracle_table(cfg):
    return S.memory_table(cfg.family, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn,
                          cfg.seq * cfg.micro_batch, cfg.elem_size)


# ------------------------------------------------------------------ cfg 2: all four layers against the oracle

def _cfg2_gpu():
    """Two micro-batches through the whole 4-layer stage (split B/W order); results kept on the host."""
    if "cfg2" not in _KEEP:
        cfg = replace(CFG.CFG2, name="cfg2_m2", n_microbatches=2)
        ws = T.device_weights(cfg)
        st = Stage(cfg)
        st.set_weights_device(ws)
        io = [T.device_io(cfg, j) for j in range(2)]
        for j in range(2):
            st.bind(j, *io[j])
        st.run([("F", 0), ("F", 1), ("B", 0), ("B", 1), ("W", 0), ("W", 1)])
        st.synchronize()
        assert st.stats().live_bytes == 0
        _KEEP["cfg2"] = {
            "cfg": cfg,
            "w": [{k: host(v) for k, v in w.items()} for w in ws],
            "x": [host(io[j][0]) for j in range(2)], "dy": [host(io[j][1]) for j in range(2)],
            "y": [host(st.y[j]) for j in range(2)], "dx": [host(st.dx[j]) for j in range(2)],
            "g": [{k: host(v) for k, v in g.items()} for g in st.grads]}
        st.close()
        del st, ws, io
        torch.cuda.empty_cache()
    return _KEEP["cfg2"]


@functools.lru_cache(maxsize=None)
def _cfg2_oracle(j, stored):
    """stored=False: the exact float64 chain.  stored=True: the same chain with every op's output held in bf16 (the
    workload's storage type), float64 inside the ops."""
    r = _cfg2_gpu()
    print(f"fp64 oracle ({'bf16 storage' if stored else 'exact chain'}): micro-batch {j} through 4 layers at full shape "
          "(about 22 TFLOP on the host)", flush=True)
    return O.stage_fbw(oracle_shape(r["cfg"]), r["w"], r["x"][j], r["dy"][j], attn_chunk=1024,
                       store=O.round_bf16 if stored else None)


# Four layers deep, storage rounding alone puts ANY executor that keeps its tensors in bf16 1-2e-2 away from the exact
# chain (the gradient reacts to a 1e-3 change of a forward tensor with a 5e-3 change of its own), and two executors
# that round at the same places still end up as far from each other as from the exact chain: a rounding that falls
# the other way in one element moves everything downstream, so after a few ops the two are independent draws of the
# same noise.  What can be asked of the HIP path at this depth is that it is no further from the exact chain than
# the storage type alone puts an executor with exact arithmetic, measured here by the oracle itself: by every
# measure at most a quarter more.  (Single kernels and single layers are held to the exact chain directly.)
def _against_both(got, exact, stored, label):
    from gpu_util import block_rms_err
    gpu = (rel_err(got, exact), rms_err(got, exact), block_rms_err(got, exact))
    ideal = (rel_err(stored, exact), rms_err(stored, exact), block_rms_err(stored, exact))
    print(f"  {label} vs the exact chain: max-rel {gpu[0]:.2e} rms-rel {gpu[1]:.2e} worst block {gpu[2]:.2e}; "
          f"exact arithmetic on bf16 storage: {ideal[0]:.2e} / {ideal[1]:.2e} / {ideal[2]:.2e}", flush=True)
    assert np.all(np.isfinite(got))
    for g, i in zip(gpu, ideal):
        assert g <= 1.25 * i + 1e-3, (label, gpu, ideal)
    return gpu[0]


def test_cfg2_four_layers_one_microbatch_against_oracle():
    r = _cfg2_gpu()
    y, dx, _, _ = _cfg2_oracle(0, False)
    ys, dxs, _, _ = _cfg2_oracle(0, True)
    assert _against_both(r["y"][0], y, ys, "cfg2 y[0] after 4 layers") < TOL[BF16]     # outputs: the stated tolerance holds
    _against_both(r["dx"][0], dx, dxs, "cfg2 dx[0] after 4 layers")
    report()


def test_cfg2_weight_gradients_accumulated_over_two_microbatches_against_oracle():
    r = _cfg2_gpu()
    ex = [_cfg2_oracle(j, False) for j in range(2)]
    st = [_cfg2_oracle(j, True) for j in range(2)]
    assert _against_both(r["y"][1], ex[1][0], st[1][0], "cfg2 y[1]") < TOL[BF16]
    _against_both(r["dx"][1], ex[1][1], st[1][1], "cfg2 dx[1]")
    for l in range(r["cfg"].n_layers):
        for name in ("wqkv", "wo", "wgu", "wd"):
            _against_both(r["g"][l][name], ex[0][2][l][name] + ex[1][2][l][name], st[0][2][l][name] + st[1][2][l][name],
                          f"cfg2 dW layer {l} {name}, 2 micro-batches")
        for name in ex[0][3][l]:
            _against_both(r["g"][l][name], ex[0][3][l][name] + ex[1][3][l][name], st[0][3][l][name] + st[1][3][l][name],
                          f"cfg2 d{name} layer {l}, 2 micro-batches")
    report()
    _KEEP.pop("cfg2", None)
    _cfg2_oracle.cache_clear()


@pytest.mark.skipif(os.environ.get("OPTSTAGE_DEEP_TESTS") != "1",
                    reason="150 TFLOP of fp64 on the host (about four minutes); set OPTSTAGE_DEEP_TESTS=1 to run it")
def test_cfg4_five_layers_forward_and_input_gradient_against_oracle():
    """The grouped-query stage (hidden 8192, 64 / 8 heads, ffn 28672) through all five layers at full shape, one
    micro-batch: stage output and input gradient against the oracle's exact chain and its bf16-storage chain (F and
    B only: about 75 TFLOP of fp64 per chain on the host).  At this width and depth storage rounding alone puts even the
    output 2.7e-2 RMS from the exact chain (one layer: 1.15e-2), so the only bar is the one of the deep comparisons:
    no further from the exact chain than exact arithmetic on bf16 storage, plus a quarter."""
    cfg = replace(CFG.CFG4, name="cfg4_m1", n_microbatches=1)
    ws = T.device_weights(cfg)
    st = Stage(cfg)
    st.set_weights_device(ws)
    x, dy = T.device_io(cfg, 0)
    st.bind(0, x, dy)
    st.run([("F", 0), ("B", 0), ("W", 0)])
    st.synchronize()
    assert st.stats().live_bytes == 0
    got_y, got_dx = host(st.y[0]), host(st.dx[0])
    w = [{k: host(v) for k, v in layer.items()} for layer in ws]
    xh, dyh = host(x), host(dy)
    st.close()
    del st, ws, x, dy
    torch.cuda.empty_cache()
    sh = oracle_shape(cfg)
    out = {}
    for stored in (False, True):
        print(f"fp64 oracle ({'bf16 storage' if stored else 'exact chain'}): F and B through 5 layers at full shape", flush=True)
        store = O.round_bf16 if stored else None
        y, saved = O.stage_forward(sh, w, xh, attn_chunk=1024, store=store)
        dx, _, _ = O.stage_backward_input(sh, w, saved, dyh, attn_chunk=1024, store=store)
        del saved
        out[stored] = (y, dx)
    _against_both(got_y, out[False][0], out[True][0], "cfg4 y after 5 layers")
    _against_both(got_dx, out[False][1], out[True][1], "cfg4 dx after 5 layers")


# ------------------------------------------------------------------ budgeted workloads at full shape

def _setup(cfg, events, budget, pool, duplex, weights, io, arena=None):
    st = Stage(cfg, budget=budget, host_pool_bytes=pool, arena_bytes=arena, duplex=duplex, grad_overwrite=True)
    st.set_weights_device(weights)
    for j in range(cfg.n_microbatches):
        st.bind(j, *io[j])
    code, bad = st.validate(events)
    assert code == B.OK, (code, bad, B.lib().optstage_last_error())
    return st


def _results(st, cfg):
    return ([st.y[j].clone() for j in range(cfg.n_microbatches)], [st.dx[j].clone() for j in range(cfg.n_microbatches)],
            {(l, n): v.clone() for l in range(cfg.n_layers) for n, v in st.grads[l].items()})


def _same_bits(a, b):
    for j in range(len(a[0])):
        assert torch.equal(a[0][j], b[0][j]) and torch.equal(a[1][j], b[1][j]), j
    for key in a[2]:
        assert torch.equal(a[2][key], b[2][key]), key


def regime_check(cfg, budget, events, label):
    """events: this stage's list (with transfers) for cfg.n_microbatches micro-batches under `budget`."""
    m, L = cfg.n_microbatches, cfg.n_layers
    t = oracle_table(cfg)
    assert any(e[0] == "O" for e in events), "the budget must bind: this list offloads nothing"
    S.check_order(events, m, L)
    peak, trace = S.account_memory(events, L, t, limit=budget)
    assert peak <= budget and trace[-1] == 0
    moved = sum(t[k] for e in events if e[0] == "O" for k in e[3])
    comp = [e for e in events if e[0] in ("F", "B", "W")]
    peak_free, _ = S.account_memory(comp, L, t)
    assert peak_free > budget, "without offload the same order must overrun the budget"
    print(f"{label}: m={m} budget {budget / 1e9:.2f} GB, peak {peak / 1e9:.2f} GB (same order without transfers "
          f"{peak_free / 1e9:.2f} GB), {moved / 1e9:.2f} GB offloaded in {sum(1 for e in events if e[0] == 'O')} events", flush=True)
    weights = T.device_weights(cfg)
    io = [T.device_io(cfg, j) for j in range(m)]

    # (1) the same compute order with no transfer and no budget: the reference bits
    st = _setup(cfg, comp, 0, 0, False, weights, io, arena=int(peak_free * 1.1) + (256 << 20))
    st.run(comp)
    st.synchronize()
    assert st.stats().peak_bytes == peak_free
    ref = _results(st, cfg)
    assert all(torch.isfinite(y.float()).all() for y in ref[0])
    st.close()
    del st
    torch.cuda.empty_cache()

    pool = moved + (64 << 20)                                       # more than can ever be away at one time
    # (2) event by event, with checksums around every offload and reload
    st = _setup(cfg, events, budget, pool, False, weights, io)
    sums = {}
    for ev in events:
        if ev[0] == "O":
            for k in ev[3]:
                sums[(ev[1], ev[2], k)] = st.checksum(ev[1], ev[2], k, where=0)
        st.run([ev])
        if ev[0] == "O":
            for k in ev[3]:
                assert st.checksum(ev[1], ev[2], k, where=1) == sums[(ev[1], ev[2], k)], ("pinned copy", ev)
        if ev[0] == "R":
            for k in ev[3]:
                assert st.checksum(ev[1], ev[2], k, where=0) == sums[(ev[1], ev[2], k)], ("after reload", ev)
    st.synchronize()
    s = st.stats()
    assert s.peak_bytes == peak and s.live_bytes == 0 and s.bytes_offloaded == s.bytes_reloaded == sum(
        st.kind_bytes[k] for e in events if e[0] == "O" for k in e[3])
    assert [e[4] for e in st.trace()] == trace                     # live bytes after every event = the oracle's
    _same_bits(_results(st, cfg), ref)
    st.close()
    del st
    torch.cuda.empty_cache()

    # (3) the whole list enqueued at once (copies overlap compute), one transfer channel and two
    for duplex in (False, True):
        st = _setup(cfg, events, budget, pool, duplex, weights, io)
        for it in range(2):                                        # a second iteration on the same handle
            st.reset()
            st.run(events)
            st.synchronize()
            s = st.stats()
            assert s.peak_bytes == peak and s.live_bytes == 0 and s.min_live_bytes > 0
            tr = st.trace()
            assert [e[4] for e in tr] == trace and len(tr) == s.n_trace == len(events)
            _same_bits(_results(st, cfg), ref)
        busy = sum(s.ms_ops[:3])
        print(f"  {'duplex' if duplex else 'single channel'}: compute {busy:.1f} ms, stall at OWAIT {s.stall_ms[0]:.1f} ms, "
              f"before B {s.stall_ms[1]:.1f} ms, d2h {s.bytes_offloaded / max(s.ms_ops[3], 1e-9) / 1e6:.1f} GB/s, "
              f"h2d {s.bytes_reloaded / max(s.ms_ops[5], 1e-9) / 1e6:.1f} GB/s", flush=True)
        st.close()
        del st
        torch.cuda.empty_cache()


def test_cfg3_full_shape_offload_under_40_percent_of_the_peak():
    cfg2_list = G.split_bw_greedy(CFG.CFG2.n_stages, CFG.CFG2.n_microbatches)[CFG.CFG2.stage_index]
    budget = int(CFG.CFG3.budget_frac_of_peak * S.account_memory(cfg2_list, CFG.CFG2.n_layers, oracle_table(CFG.CFG2))[0])
    m = CFG.CFG3.n_microbatches                     # the whole list the benchmark runs: all 16 micro-batches
    cfg = CFG.CFG3
    lists, info = SC.workload_lists(CFG.CFG3, budget, m=m)
    regime_check(cfg, budget, lists[cfg.stage_index], "cfg3")


def test_cfg4_dense_fill_offloads_under_120_gb():
    m = CFG.CFG4.n_microbatches                     # the whole list the benchmark runs: all 32 micro-batches
    cfg = CFG.CFG4
    lists, info = SC.workload_lists(CFG.CFG4, CFG.CFG4.budget_bytes, m=m)
    assert info["caps"][cfg.stage_index] > cfg.n_stages - cfg.stage_index          # denser than p - i in flight
    regime_check(cfg, CFG.CFG4.budget_bytes, lists[cfg.stage_index], "cfg4")


def test_cfg5_long_sequence_stage_under_64_gb():
    cfg = CFG.CFG5
    lists, info = SC.workload_lists(cfg, cfg.budget_bytes)
    regime_check(cfg, cfg.budget_bytes, lists[cfg.stage_index], "cfg5")
