"""CPU-only checks of the boundary: the library loads, exports every symbol the headers declare, and its
pure-host planner (ordering rules + list-order memory accounting) agrees bit for bit with the oracle."""
import ctypes
from dataclasses import replace
import os
import random
import re

import pytest

from oracle import schedule as S
from paper_2510_05186_amd import binding as B
from stage_inputs import configs as CFG
from stage_inputs import schedules as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for hdr in ("optstage.h", "optstage_ops.h"):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(optstage_[a-z_0-9]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 30
    L = ctypes.CDLL(B.LIB_PATH)
    for n in sorted(names):
        assert hasattr(L, n), n
    assert names == set(B.EXPORTS)


def oracle_table(cfg):
    return S.memory_table(cfg.family, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn,
                          cfg.seq * cfg.micro_batch, cfg.elem_size)


@pytest.mark.parametrize("cfg", [CFG.CFG1, CFG.CFG2, CFG.CFG4, CFG.CFG5, CFG.CFG6], ids=lambda c: c.name)
def test_memory_table_matches_oracle(cfg):
    ws, act, kinds = B.query_sizes(cfg)
    t = oracle_table(cfg)
    assert kinds == t
    assert act == S.op_delta("F", cfg.n_layers, t)
    assert ws > 0


@pytest.mark.parametrize("cfg", [CFG.CFG1, CFG.CFG2, CFG.CFG4], ids=lambda c: c.name)
def test_recompute_memory_table_matches_oracle(cfg):
    _, act, kinds = B.query_sizes(cfg, recompute=1)
    t = oracle_table(cfg)
    assert kinds == t
    assert act == S.op_delta("F", cfg.n_layers, t, recompute=True) < S.op_delta("F", cfg.n_layers, t)


def test_recompute_plan_matches_oracle_accounting():
    cfg = small_cfg()
    t = oracle_table(cfg)
    p, m, L = 4, cfg.n_microbatches, cfg.n_layers
    lists = [G.one_f_one_b(p, m, i) for i in range(p)] + G.split_bw_greedy(p, m)
    more = [G.add_offload(base, L, ("X_IN", "QKV", "X_MID", "GU"), min_gap=gap, lead=1) for base in lists for gap in (1, 3)]
    for ev in lists + more:
        S.check_order(ev, m, L, recompute=True)
        peak, trace = S.account_memory(ev, L, t, recompute=True)
        st, bad, lib_peak, live = B.plan(cfg, ev, recompute=1)
        assert st == B.OK, B.lib().optstage_last_error()
        assert lib_peak == peak and live == trace
        assert peak < S.account_memory(ev, L, t)[0]
        st, bad, _, _ = B.plan(cfg, ev, budget=peak - 1, recompute=1)
        assert st == B.E_BUDGET
        with pytest.raises(S.ScheduleError) as ei:
            S.account_memory(ev, L, t, limit=peak - 1, recompute=True)
        assert ei.value.index == bad
    # a kind F does not keep cannot be offloaded: same event rejected on both sides
    ev = G.add_offload(lists[0], L, ("N2",), min_gap=1)
    with pytest.raises(S.ScheduleError) as ei:
        S.check_order(ev, m, L, recompute=True)
    st, bad, _, _ = B.plan(cfg, ev, recompute=1)
    assert st == B.E_ORDER and bad == ei.value.index


def test_plan_with_model_chunks_matches_oracle():
    """A stage that holds two model chunks: the planner's order rules and accounting are the oracle's."""
    cfg = small_cfg(m=4, L=4)
    t = oracle_table(cfg)
    m, L, v = cfg.n_microbatches, cfg.n_layers, 2
    for i in range(2):
        base = G.interleaved_one_f_one_b(2, m, i, v)
        for ev in (base, G.add_offload(base, L, ("X_IN", "QKV", "GU"), min_gap=2, lead=1)):
            S.check_order(ev, m, L, n_chunks=v)
            peak, trace = S.account_memory(ev, L, t, n_chunks=v)
            st, bad, lib_peak, live = B.plan(cfg, ev, n_chunks=v)
            assert st == B.OK, B.lib().optstage_last_error()
            assert lib_peak == peak and live == trace
            st, bad, _, _ = B.plan(cfg, ev, budget=peak - 1, n_chunks=v)
            assert st == B.E_BUDGET
            with pytest.raises(S.ScheduleError) as ei:
                S.account_memory(ev, L, t, limit=peak - 1, n_chunks=v)
            assert ei.value.index == bad
    kinds = ("QKV",)
    bad_lists = [
        [("F", 0, 0), ("B", 0, 1)],                                            # B of a chunk before its F
        [("F", 1, 1)],                                                         # chunk 1 starts at micro-batch 0
        [("F", 0, 0), ("F", 0, 1), ("O", 0, 3, kinds), ("OWAIT", 0, 3, kinds), ("B", 0, 1)],   # not reloaded
        [("F", 0, 0), ("O", 0, 2, kinds)],                                     # layer 2 belongs to chunk 1
    ]
    for ev in bad_lists:
        with pytest.raises(S.ScheduleError) as ei:
            S.check_order(ev, m, L, n_chunks=v)
        st, bad, _, _ = B.plan(cfg, ev, n_chunks=v)
        assert st == B.E_ORDER and bad == ei.value.index, (ev, st, bad, ei.value.index)
    assert B.plan(cfg, [("F", 0, 2)], n_chunks=v)[0] == B.E_ARG               # no such chunk
    d = B.make_desc(cfg, n_chunks=3)                                           # 4 layers do not split in three
    assert B.lib().optstage_query_sizes(d, None, None, None) == B.E_ARG


def small_cfg(m=6, L=3):
    return CFG.shrunken(CFG.CFG4, hidden=256, n_q=4, n_kv=2, ffn=384, seq=192, n_layers=L, n_microbatches=m)


def test_plan_matches_oracle_accounting_on_generated_schedules():
    cfg = small_cfg()
    t = oracle_table(cfg)
    p, m, L = 4, cfg.n_microbatches, cfg.n_layers
    lists = [G.one_f_one_b(p, m, i) for i in range(p)] + G.split_bw_greedy(p, m)
    more = []
    for base in lists:
        for gap in (1, 2, 4):
            for lead in (1, 2):
                more.append(G.add_offload(base, L, ("X_IN", "QKV", "X_MID"), min_gap=gap, lead=lead))
        more.append(G.add_offload(base, L, ("N1", "GU", "A", "LSE", "STATS", "O", "N2"), min_gap=1))
    for ev in lists + more:
        S.check_order(ev, m, L)
        peak, trace = S.account_memory(ev, L, t)
        st, bad, lib_peak, live = B.plan(cfg, ev)
        assert st == B.OK, B.lib().optstage_last_error()
        assert lib_peak == peak and live == trace
        # budget exactly at the peak passes, one byte less fails at the same event as the oracle
        assert B.plan(cfg, ev, budget=peak)[0] == B.OK
        st, bad, _, _ = B.plan(cfg, ev, budget=peak - 1)
        assert st == B.E_BUDGET
        with pytest.raises(S.ScheduleError) as ei:
            S.account_memory(ev, L, t, limit=peak - 1)
        assert ei.value.index == bad


def test_plan_rejects_what_the_oracle_rejects():
    cfg = small_cfg(m=2, L=2)
    q = ("QKV",)
    bad_lists = [
        [("B", 0), ("F", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("W", 0), ("B", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 1), ("F", 0), ("B", 0), ("W", 0), ("B", 1), ("W", 1)],
        [("F", 0), ("F", 0), ("B", 0), ("W", 0)],
        [("F", 0), ("B", 0), ("W", 0)],
        [("O", 0, 0, q), ("F", 0), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("O", 0, 0, q), ("OWAIT", 0, 0, q), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("O", 0, 0, q), ("R", 0, 0, q), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("O", 0, 0, q), ("O", 0, 0, q), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("OWAIT", 0, 0, q), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("B", 0), ("O", 0, 0, q), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
    ]
    for ev in bad_lists:
        with pytest.raises(S.ScheduleError) as ei:
            S.check_order(ev, 2, 2)
        st, bad, _, _ = B.plan(cfg, ev)
        assert st == B.E_ORDER, ev
        assert bad == ei.value.index, (ev, bad, ei.value.index)
    # argument errors: bad layer, non-offloadable kind, micro-batch out of range
    assert B.plan(cfg, [("F", 0), ("O", 0, 5, q)])[0] == B.E_ARG
    assert B.plan(cfg, [("F", 0), ("O", 0, 0, ("DY",))])[0] == B.E_ARG
    assert B.plan(cfg, [("F", 7)])[0] == B.E_ARG


def test_plan_random_valid_interleavings():
    rng = random.Random(7)
    cfg = small_cfg(m=4, L=2)
    t = oracle_table(cfg)
    m, L = 4, 2
    for _ in range(200):
        # random valid compute order
        nxt = {"F": 0, "B": 0, "W": 0}
        ev = []
        while nxt["W"] < m:
            cands = []
            if nxt["F"] < m:
                cands.append("F")
            if nxt["B"] < nxt["F"]:
                cands.append("B")
            if nxt["W"] < nxt["B"]:
                cands.append("W")
            c = rng.choice(cands)
            ev.append((c, nxt[c]))
            nxt[c] += 1
        ev = G.add_offload(ev, L, tuple(rng.sample(S.F_KINDS, rng.randint(1, 4))), min_gap=rng.randint(0, 3), lead=rng.randint(1, 3))
        S.check_order(ev, m, L)
        peak, trace = S.account_memory(ev, L, t)
        st, _, lib_peak, live = B.plan(cfg, ev)
        assert st == B.OK and lib_peak == peak and live == trace


@pytest.mark.parametrize("recompute", [False, True])
def test_planner_equals_oracle_accounting_on_random_valid_lists(recompute):
    """Property over the schedule grammar, host only: for random valid lists (compute order, offloaded items and
    transfer positions all drawn) the library's planner reports the oracle's live bytes after every event and the
    oracle's peak, accepts a budget equal to that peak and refuses one allocation granule less."""
    import numpy as np
    from stage_inputs import schedules as G
    cfg = replace(CFG.shrunken(CFG.CFG2, hidden=256, n_q=2, n_kv=2, ffn=512, seq=256, n_layers=3, n_microbatches=5), name="plan_random")
    t = S.memory_table(cfg.family, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn, cfg.seq * cfg.micro_batch, cfg.elem_size)
    kinds = ("X_IN", "QKV", "X_MID", "O", "GU", "LSE") if recompute else ("X_IN", "N1", "QKV", "X_MID", "O", "GU", "A", "STATS")
    for seed in range(40):
        rng = np.random.default_rng(seed)
        ev = G.random_valid_list(rng, cfg.n_microbatches, cfg.n_layers, kinds, p_offload=0.5)
        S.check_order(ev, cfg.n_microbatches, cfg.n_layers, recompute=recompute)
        peak, trace = S.account_memory(ev, cfg.n_layers, t, recompute=recompute)
        code, bad, ppeak, live = B.plan(cfg, ev, budget=peak, recompute=int(recompute))
        assert code == B.OK and ppeak == peak and list(live[:len(ev)]) == trace, (seed, code, bad)
        assert B.plan(cfg, ev, budget=peak - S.ALIGN, recompute=int(recompute))[0] == B.E_BUDGET, seed
