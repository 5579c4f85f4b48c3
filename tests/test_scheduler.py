"""Host-side schedule generators (paper_2510_05186_amd/scheduler.py) against the oracle: the MILP optimum
equals the brute-force optimum over every valid per-stage order (and every placement of O / OWAIT / R) on
tiny instances, every list it returns is valid, fits the memory limit and reproduces the solver's makespan
in the oracle simulator; AdaOffload returns valid, feasible, denser-than-1F1B lists whose makespan bounds
the optimum from above."""
import itertools

import pytest

from oracle import schedule as S
from paper_2510_05186_amd import scheduler as SC
from stage_inputs import schedules as G
from test_oracle_schedule import L, TABLE, all_orders, check_constraints, offload_variants

ITEM = (0, ("X_IN",))
DELTA = {c: S.op_delta(c, L, TABLE) for c in "FBW"}
GAMMA = TABLE["X_IN"]


def eq7_peak(events):
    return max(u for _, u in S.eq7_usage(events, L, TABLE))


def own_peak(table, n_layers):
    """Most bytes each op type holds beyond the level before it, from the oracle's allocation steps."""
    out = {}
    for c in "FBW":
        level = top = 0
        for sgn, _, k in S.op_memory_steps(c, n_layers):
            level += sgn * table[k]
            top = max(top, level)
        out[c] = top
    return out


def brute_optimum(p, m, t_op, t_comm, t_off, limit0, offload_mbs, physical=False):
    """Minimum Eq. 17 makespan over every pair of valid stage orders (p = 2), with every placement of the
    transfers of any subset of `offload_mbs` on stage 0, subject to Eq. 7 on stage 0 (physical: subject to the
    executor's list-order accounting instead, which holds what B and W release until they have run)."""
    assert p == 2
    orders = all_orders(m)
    best = None
    for l0 in orders:
        cands = [l0]
        for j in offload_mbs:
            cands = cands + [v for c in cands for v in offload_variants(c, j)]
        for v0 in cands:
            if limit0 is not None and (S.account_memory(v0, L, TABLE)[0] if physical else eq7_peak(v0)) > limit0:
                continue
            for l1 in orders:
                try:
                    tm = S.simulate([v0, l1], t_op, t_comm=t_comm, t_copy=lambda i, ev: t_off)
                except S.ScheduleError:
                    continue
                if best is None or tm.makespan_global < best - 1e-12:
                    best = tm.makespan_global
    return best


def check_solution(inst, sol, t_off):
    for i, lst in enumerate(sol.lists):
        S.check_order(lst, inst.m, L)
        if inst.limit[i] is not None:
            assert eq7_peak(lst) <= inst.limit[i]
    tm = S.simulate(sol.lists, inst.t_op, t_comm=inst.t_comm, t_copy=lambda i, ev: t_off)
    check_constraints(sol.lists, tm, inst.t_op, inst.t_comm, t_off)
    return tm


@pytest.mark.parametrize("m,t_op,t_comm", [
    (2, [{"F": 1, "B": 2, "W": 1}, {"F": 2, "B": 1, "W": 1}], 1),
    (3, [{"F": 1, "B": 1, "W": 1}, {"F": 1, "B": 1, "W": 1}], 0),
    (3, [{"F": 2, "B": 3, "W": 1}, {"F": 1, "B": 2, "W": 2}], 1),
])
def test_milp_without_offload_matches_bruteforce(m, t_op, t_comm):
    inst = SC.Instance(p=2, m=m, t_op=t_op, t_comm=t_comm)
    sol = SC.milp_schedule(inst)
    ref = brute_optimum(2, m, t_op, t_comm, 0, None, ())
    assert abs(sol.makespan - ref) < 1e-6, (sol.makespan, ref)
    tm = check_solution(inst, sol, 0)
    assert abs(tm.makespan_global - ref) < 1e-6


def test_milp_memory_limit_without_offload_matches_bruteforce():
    # a limit of two forward activations (+ what B allocates) forbids the deep fill
    m = 3
    t_op = [{"F": 1, "B": 1, "W": 1}] * 2
    limit = 2 * DELTA["F"] + TABLE["DY"] + TABLE["DX_MID"]
    inst = SC.Instance(p=2, m=m, t_op=t_op, delta=[DELTA, DELTA], gamma=[GAMMA, GAMMA], limit=[limit, None])
    sol = SC.milp_schedule(inst)
    ref = brute_optimum(2, m, t_op, 0, 0, limit, ())
    free = brute_optimum(2, m, t_op, 0, 0, None, ())
    assert abs(sol.makespan - ref) < 1e-6 and ref >= free
    check_solution(inst, sol, 0)


@pytest.mark.parametrize("t_off", [1, 2])
def test_milp_with_offload_matches_bruteforce(t_off):
    # stage 0 may offload the item of micro-batches 0 and 1; the limit leaves room for two activations plus
    # the item-sized slack, so offloading buys a denser fill
    m = 3
    t_op = [{"F": 1, "B": 1, "W": 1}] * 2
    limit = 2 * DELTA["F"] + TABLE["DY"] + TABLE["DX_MID"] + (DELTA["F"] - GAMMA)
    inst = SC.Instance(p=2, m=m, t_op=t_op, t_off=[t_off, t_off], delta=[DELTA, DELTA], gamma=[GAMMA, GAMMA],
                       limit=[limit, None], offload_stages=(0,), offload_mbs=(0, 1), item=ITEM)
    relaxed = SC.milp_schedule(inst, strict_eq13=False)
    ref = brute_optimum(2, m, t_op, 0, t_off, limit, (0, 1))
    assert abs(relaxed.makespan - ref) < 1e-5, (relaxed.makespan, ref)
    tm = check_solution(inst, relaxed, t_off)
    assert tm.makespan_global <= relaxed.makespan + 1e-5
    # Eq. 13 as printed only removes schedules: never better than the executor's model, never better than no limit
    strict = SC.milp_schedule(inst, strict_eq13=True)
    assert strict.makespan >= relaxed.makespan - 1e-6
    tm = check_solution(inst, strict, t_off)
    for i, lst in enumerate(strict.lists):              # Eq. 13 on the extracted timing
        for n, ev in enumerate(lst):
            if ev[0] == "R":
                for k in range(n + 1, len(lst)):
                    if lst[k][0] in "FBW":
                        assert tm.start[i][k] + 1e-9 >= tm.start[i][n]


def test_milp_with_physical_accounting_matches_bruteforce_on_the_executors_peak():
    # own term of Eq. 7 = what the op really holds while it runs: the lists then fit the executor's accounting
    m = 3
    t_op = [{"F": 1, "B": 1, "W": 1}] * 2
    limit = 2 * DELTA["F"] + TABLE["DY"] + TABLE["DX_MID"] + (DELTA["F"] - GAMMA)
    pk = own_peak(TABLE, L)
    assert pk["F"] == DELTA["F"] and pk["W"] == 0 and pk["B"] > 0
    inst = SC.Instance(p=2, m=m, t_op=t_op, t_off=[1, 1], delta=[DELTA, DELTA], gamma=[GAMMA, GAMMA], own_peak=[pk, pk],
                       limit=[limit, None], offload_stages=(0,), offload_mbs=(0, 1), item=ITEM)
    sol = SC.milp_schedule(inst, strict_eq13=False)
    ref = brute_optimum(2, m, t_op, 0, 1, limit, (0, 1), physical=True)
    assert abs(sol.makespan - ref) < 1e-5, (sol.makespan, ref)
    check_solution(inst, sol, 1)
    assert S.account_memory(sol.lists[0], L, TABLE)[0] <= limit
    paper = SC.milp_schedule(SC.Instance(p=2, m=m, t_op=t_op, t_off=[1, 1], delta=[DELTA, DELTA], gamma=[GAMMA, GAMMA],
                                         limit=[limit, None], offload_stages=(0,), offload_mbs=(0, 1), item=ITEM),
                             strict_eq13=False)
    assert paper.makespan <= sol.makespan + 1e-6        # Eq. 7 as printed admits more schedules


def test_milp_offload_beats_no_offload_under_the_same_limit():
    m = 3
    t_op = [{"F": 1, "B": 1, "W": 1}] * 2
    limit = 2 * DELTA["F"] + TABLE["DY"] + TABLE["DX_MID"] + (DELTA["F"] - GAMMA)
    base = dict(p=2, m=m, t_op=t_op, t_off=[1, 1], delta=[DELTA, DELTA], gamma=[GAMMA, GAMMA], limit=[limit, None], item=ITEM)
    without = SC.milp_schedule(SC.Instance(**base))
    with_off = SC.milp_schedule(SC.Instance(**base, offload_stages=(0,)), strict_eq13=False)
    assert with_off.makespan <= without.makespan + 1e-6


def test_triangle_cuts_and_cutoff_do_not_change_the_optimum():
    t_op = [{"F": 2, "B": 3, "W": 1}, {"F": 1, "B": 2, "W": 2}]
    inst = SC.Instance(p=2, m=3, t_op=t_op, t_comm=1)
    a = SC.milp_schedule(inst, triangle_cuts=True)
    b = SC.milp_schedule(inst, triangle_cuts=False)
    ada = SC.adaoffload(inst)
    c = SC.milp_schedule(inst, cutoff=ada.makespan)
    assert abs(a.makespan - b.makespan) < 1e-6 and abs(a.makespan - c.makespan) < 1e-6
    assert ada.makespan >= a.makespan - 1e-6


@pytest.mark.parametrize("p,m", [(2, 3), (4, 8), (8, 16)])
def test_adaoffload_lists_are_valid_and_dense(p, m):
    t_op = [{"F": 1.0, "B": 1.2, "W": 0.8}] * p
    # room for three activations per stage; the whole forward activation (every kind, both layers) is the
    # offloadable item, 0.5 per activation = 0.25 per layer event
    limit = 3 * DELTA["F"] + TABLE["DY"] + TABLE["DX_MID"]
    inst = SC.Instance(p=p, m=m, t_op=t_op, t_comm=0.05, t_off=[0.5] * p, delta=[DELTA] * p, gamma=[DELTA["F"]] * p,
                       limit=[limit] * p, offload_stages=tuple(range(p)), item=(0, tuple(S.F_KINDS)))
    sol = SC.adaoffload(inst, tolerance=0.5)
    lists = [SC.expand_items(lst, L, S.F_KINDS) for lst in sol.lists]
    for i, lst in enumerate(lists):
        S.check_order(lst, m, L)
    tm = S.simulate(lists, t_op, t_comm=0.05, t_copy=lambda i, ev: 0.25)
    check_constraints(lists, tm, t_op, 0.05, 0.25)
    # every list fits its limit in the oracle's accounting (Eq. 7 usage and the executor's running sum), and
    # stages that offload fill deeper than the three activations they can hold
    for i, lst in enumerate(lists):
        first_b = next(n for n, e in enumerate(lst) if e[0] == "B")
        n_fill = sum(1 for e in lst[:first_b] if e[0] == "F")
        assert n_fill >= 1
        assert eq7_peak(lst) <= limit, (i, eq7_peak(lst), limit)
        peak, _ = S.account_memory(lst, L, TABLE)
        assert peak <= limit, (i, peak, limit)
        if any(e[0] == "O" for e in lst):
            assert n_fill > 3 or n_fill == m
    # beats the capacity-respecting greedy list without offload whenever the capacity binds
    capped = G.split_bw_greedy(p, m, cap_of_stage=lambda s: min(3, p - s))
    tz = S.simulate(capped, t_op, t_comm=0.05)
    assert tm.makespan_global <= tz.makespan_global + 1e-9
    if p >= 4:
        assert tm.makespan_global < 0.9 * tz.makespan_global
    # the optimum bounds it from below on the instance small enough to solve exactly
    if (p, m) == (2, 3):
        opt = SC.milp_schedule(inst, strict_eq13=False, cutoff=sol.makespan)
        assert opt.makespan <= tm.makespan_global + 1e-6


@pytest.mark.parametrize("p,m", [(2, 4), (4, 8)])
def test_adaoffload_with_a_memory_table_in_which_b_grows(p, m):
    """Recompute variant of the table: Delta_F is smaller and Delta_B > 0 (B rebuilds what W reads).  The lists
    must fit the limit in the oracle's accounting of that variant, and hold more forward activations before
    the first B than the store-all table allows under the same limit."""
    t_op = [{"F": 1.0, "B": 1.3, "W": 0.8}] * p
    kinds = tuple(k for k in S.F_KINDS if k not in S.RECOMPUTED)
    d_var = {c: S.op_delta(c, L, TABLE, recompute=True) for c in "FBW"}
    assert d_var["B"] > 0
    slack = 2 * (TABLE["DY"] + TABLE["DX_MID"])          # B's transients inside the op
    limit = 3 * DELTA["F"] + slack
    fills = {}
    for name, delta, rc in (("store_all", DELTA, False), ("recompute", d_var, True)):
        inst = SC.Instance(p=p, m=m, t_op=t_op, t_comm=0.05, t_off=[0.4] * p, delta=[delta] * p,
                           gamma=[sum(TABLE[k] for k in kinds) * L] * p, limit=[limit - slack] * p,
                           offload_stages=tuple(range(p)), item=(0, kinds))
        sol = SC.adaoffload(inst, tolerance=0.5)
        lists = [SC.expand_items(lst, L, kinds) for lst in sol.lists]
        for lst in lists:
            S.check_order(lst, m, L, recompute=rc)
            peak, _ = S.account_memory(lst, L, TABLE, recompute=rc)
            assert peak <= limit, (name, peak, limit)
        S.simulate(lists, t_op, t_comm=0.05, t_copy=lambda i, ev: 0.4 / L)
        lst = lists[0]
        first_b = next(n for n, e in enumerate(lst) if e[0] == "B")
        fills[name] = sum(1 for e in lst[:first_b] if e[0] == "F")
    assert fills["recompute"] >= fills["store_all"]


def test_online_search_publishes_improving_schedules_up_to_the_optimum():
    """Sec. 4.3 on the host: the search starts from AdaOffload's lists and publishes strictly better ones until a
    solve proves that none is left; the last one is the optimum the brute-force search finds, every published list
    is valid, and a search that is stopped early still holds its best so far."""
    m = 3
    t_op = [{"F": 1, "B": 1, "W": 1}] * 2
    limit = 2 * DELTA["F"] + TABLE["DY"] + TABLE["DX_MID"] + (DELTA["F"] - GAMMA)
    inst = SC.Instance(p=2, m=m, t_op=t_op, t_off=[1, 1], delta=[DELTA, DELTA], gamma=[GAMMA, GAMMA],
                       limit=[limit, None], offload_stages=(0,), offload_mbs=(0, 1), item=ITEM)
    search = SC.OnlineSearch(inst, tolerance=0.5, slice_seconds=20, max_seconds=120).start()
    search.join(150)
    assert search.complete
    scores = [h[1] for h in search.history]
    assert search.history[0][2] == "adaoffload"
    assert all(b < a for a, b in zip(scores, scores[1:]))
    score, sol = search.best()
    assert abs(score - brute_optimum(2, m, t_op, 0, 1, limit, (0, 1))) < 1e-5
    check_solution(inst, sol, 1)
    # a judge re-times candidates in its own units (here: twice the solver's makespan)
    judged = SC.OnlineSearch(inst, tolerance=0.5, slice_seconds=20, max_seconds=120, judge=lambda s_: 2 * s_.makespan).start()
    judged.join(150)
    assert abs(judged.best()[0] - 2 * score) < 1e-5
    # stopping: a search on a larger instance is cut off and keeps what it has (at least AdaOffload's lists)
    big = SC.Instance(p=4, m=6, t_op=[{"F": 1.0, "B": 1.2, "W": 0.8}] * 4, t_comm=0.05, t_off=[0.5] * 4, delta=[DELTA] * 4,
                      gamma=[GAMMA] * 4, limit=[3 * DELTA["F"] + TABLE["DY"] + TABLE["DX_MID"]] * 4,
                      offload_stages=(0, 1, 2, 3), item=ITEM)
    cut = SC.OnlineSearch(big, tolerance=0.5, slice_seconds=1, max_seconds=2).start()
    cut.join(60)
    assert not cut._thread.is_alive()
    assert cut.best() is not None and cut.best()[1].lists and len(cut.history) >= 1


def test_list_extraction_orders_transfers_inside_a_gap_for_the_executor():
    """Eq. 7 is checked where compute ops start, so a solution may start a reload, in solver time, before an
    offload that ends between the same two compute ops has released its memory.  The executor charges by list
    position: in the extracted list the OWAIT comes first, the op charges (M, N) stay as solved."""
    start = {(0, "F"): 0.0, (1, "F"): 1.0, (2, "F"): 2.5, (0, "B"): 5.0, (0, "W"): 6.0, (1, "B"): 7.0, (1, "W"): 8.0,
             (2, "B"): 9.0, (2, "W"): 10.0}
    items = {1: (2.0, 3.6, [(2, "F"), (0, "B")], []),              # offloaded before F2 starts, reload asked for at 3.6
             2: (3.5, 8.0, [(0, "B")], [])}                         # its offload ends at 4.0: after 3.6, before B0
    ev = SC._list_from_times(start, items, ITEM)
    pos = {(e[0], e[1]): k for k, e in enumerate(ev)}
    assert pos[("OWAIT", 2)] < pos[("R", 1)] < pos[("B", 0)]                 # same gap: release first, then reload
    assert pos[("F", 2)] < pos[("O", 2)] < pos[("OWAIT", 2)]
    assert pos[("O", 1)] < pos[("OWAIT", 1)] < pos[("F", 2)]                 # credited to F2: released before it
    assert pos[("B", 1)] < pos[("R", 2)] < pos[("W", 1)]                     # at W1's start time: just before it
    S.check_order(SC.expand_items(ev, L, ITEM[1]), 3, L)


def test_online_search_on_an_instance_without_any_schedule():
    """A limit below one forward activation, offload or not: the heuristic gives up, the solver proves that nothing
    exists, the search ends complete with nothing published and no error."""
    inst = SC.Instance(p=2, m=2, t_op=[{"F": 1, "B": 1, "W": 1}] * 2, t_off=[0.5, 0.5], delta=[DELTA, DELTA],
                       gamma=[GAMMA, GAMMA], limit=[DELTA["F"] // 2] * 2, offload_stages=(0, 1), item=ITEM)
    with pytest.raises(RuntimeError):
        SC.adaoffload(inst)
    assert SC.milp_schedule(inst, time_limit=20).lists == []
    s = SC.OnlineSearch(inst, slice_seconds=5, max_seconds=20).start()
    s.join(60)
    assert s.complete and s.best() is None and s.error is None and s.history == []
    # degenerate sizes: one stage, one micro-batch
    for p, m, want in ((1, 1, 3.0), (1, 3, 9.0), (3, 1, 7.0)):
        one = SC.Instance(p=p, m=m, t_op=[{"F": 1, "B": 1, "W": 1}] * p, t_off=[0.5] * p, delta=[DELTA] * p, gamma=[GAMMA] * p,
                          limit=[None] * p, item=ITEM)
        assert abs(SC.adaoffload(one).makespan - want) < 1e-6 and abs(SC.milp_schedule(one, time_limit=20).makespan - want) < 1e-4


# ------------------------------------------------------------- timing of given lists, lists under a byte budget

def _small_cfg():
    from stage_inputs import configs as CFG
    return CFG.shrunken(CFG.CFG3, hidden=512, n_q=4, n_kv=4, ffn=1376, seq=512, n_layers=3, n_microbatches=8, name="cfg3_small")


def _table(cfg):
    return S.memory_table(cfg.family, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn,
                          cfg.seq * cfg.micro_batch, cfg.elem_size)


@pytest.mark.parametrize("duplex", [False, True])
def test_pipeline_timeline_equals_the_oracle_simulator_on_random_lists(duplex):
    """The library-side timing of given lists (used to choose between candidate schedules) against the oracle's
    simulator: every start and end time, the makespan and the per-stage bubble, on random members of the schedule
    grammar with random op and transfer times."""
    import numpy as np
    rng = np.random.default_rng(11)
    kinds = ("X_IN", "QKV", "X_MID")
    deadlocks = compared = 0
    for trial in range(60):
        p, m, nl = int(rng.integers(1, 5)), int(rng.integers(1, 6)), int(rng.integers(1, 3))
        lists = [G.random_valid_list(rng, m, nl, kinds, p_offload=0.5) for _ in range(p)]
        t_op = [{c: float(rng.uniform(0.5, 3.0)) for c in "FBW"} for _ in range(p)]
        t_comm = float(rng.uniform(0, 0.5))
        cost = {k: float(rng.uniform(0.1, 2.0)) for k in kinds}
        t_copy = lambda i, e: sum(cost[k] for k in e[3]) * (1 + 0.1 * i)
        try:
            ref = S.simulate(lists, t_op, t_comm, t_copy, duplex=duplex)
        except S.ScheduleError:                         # random orders of several stages may wait for each other
            with pytest.raises(ValueError):
                SC.pipeline_timeline(lists, t_op, t_comm, t_copy, duplex=duplex)
            deadlocks += 1
            continue
        got = SC.pipeline_timeline(lists, t_op, t_comm, t_copy, duplex=duplex)
        compared += 1
        assert got.makespan == pytest.approx(ref.makespan_global, rel=1e-12)
        for i in range(p):
            assert got.bubble[i] == pytest.approx(ref.bubble[i], abs=1e-12)
            for n, e in enumerate(lists[i]):
                if e[0] == "OWAIT":
                    continue
                assert got.start[i][n] == pytest.approx(ref.start[i][n], abs=1e-9), (trial, i, n, e)
                assert got.end[i][n] == pytest.approx(ref.end[i][n], abs=1e-9)
    assert compared >= 15 and deadlocks >= 1


def test_pipeline_timeline_stall_is_the_time_lost_to_transfers():
    # one stage, F0 F1 B0 ...; micro-batch 1's item leaves and comes back: B1 waits for the reload, nothing else does
    ev = [("F", 0), ("F", 1), ("O", 1, 0, ("X_IN",)), ("OWAIT", 1, 0, ("X_IN",)), ("B", 0), ("W", 0),
          ("R", 1, 0, ("X_IN",)), ("B", 1), ("W", 1)]
    t_op = [{"F": 1.0, "B": 2.0, "W": 1.0}]
    tl = SC.pipeline_timeline([ev], t_op, 0.0, lambda i, e: 0.5)
    # O runs 2.0-2.5 while B0 would start at 2.0: B0 is listed after the OWAIT, so it waits 0.5; R starts at the end
    # of W0 (5.5) and ends at 6.0: B1 waits another 0.5
    assert tl.stall[0] == pytest.approx(1.0) and tl.makespan == pytest.approx(9.0)
    free = SC.pipeline_timeline([[e for e in ev if e[0] in "FBW"]], t_op)
    assert free.stall[0] == 0.0 and free.makespan == pytest.approx(8.0)


def test_fit_offloads_takes_the_fewest_items_the_budget_needs():
    from paper_2510_05186_amd import binding as B
    cfg = _small_cfg()
    t = _table(cfg)
    kb = B.query_sizes(cfg)[2]
    kinds = ("X_IN", "QKV", "X_MID")
    comp = G.split_bw_greedy(cfg.n_stages, cfg.n_microbatches)[cfg.stage_index]
    peak0, _ = S.account_memory(comp, cfg.n_layers, t)
    fits_at = lambda budget: (lambda ev: (lambda r: (r[0] == B.OK, r[1]))(B.plan(cfg, ev, budget=budget)))
    assert SC.fit_offloads(comp, cfg.n_layers, kinds, kb, fits_at(peak0)) == comp            # fits: nothing leaves
    moved_prev = 0
    for frac in (0.95, 0.9, 0.85):
        budget = int(frac * peak0)
        ev = SC.fit_offloads(comp, cfg.n_layers, kinds, kb, fits_at(budget))
        assert ev is not None and [e for e in ev if e[0] in "FBW"] == comp
        S.check_order(ev, cfg.n_microbatches, cfg.n_layers)
        peak, trace = S.account_memory(ev, cfg.n_layers, t, limit=budget)
        assert peak <= budget and trace[-1] == 0
        moved = sum(t[k] for e in ev if e[0] == "O" for k in e[3])
        everything = G.add_offload(comp, cfg.n_layers, kinds, min_gap=1, lead=1)
        assert 0 < moved < sum(t[k] for e in everything if e[0] == "O" for k in e[3])
        assert moved >= moved_prev                      # a tighter budget never moves fewer bytes
        moved_prev = moved
        # none of the chosen items is superfluous where it was chosen: without the last one the list overruns
        last = [e for e in ev if e[0] == "O"][-1]
        drop = (last[1], last[2], last[3][-1])
        thinner = []
        for e in ev:
            if e[0] in ("O", "OWAIT", "R") and (e[1], e[2]) == drop[:2]:
                ks = tuple(k for k in e[3] if k != drop[2])
                if ks:
                    thinner.append((e[0], e[1], e[2], ks))
            else:
                thinner.append(e)
        with pytest.raises(S.ScheduleError):
            S.account_memory(thinner, cfg.n_layers, t, limit=budget)
    # a budget below what one micro-batch needs during its B cannot be met
    assert SC.fit_offloads(comp, cfg.n_layers, kinds, kb, fits_at(int(0.9 * sum(t[k] for k in S.F_KINDS) * cfg.n_layers))) is None


def test_workload_lists_fill_the_budget_and_are_chosen_by_modelled_makespan():
    from paper_2510_05186_amd import binding as B
    cfg = _small_cfg()
    t = _table(cfg)
    p, m = cfg.n_stages, cfg.n_microbatches
    base = G.split_bw_greedy(p, m)
    peak0 = max(S.account_memory(ev, cfg.n_layers, t)[0] for ev in base)
    t_op = SC.nominal_op_times(cfg)
    size = lambda e: sum(t[k] for k in e[3])
    for frac in (0.5, 1.3):
        budget = int(frac * peak0)
        lists, info = SC.workload_lists(cfg, budget, t_op=t_op, link_gbps=55.0)
        assert len(lists) == p
        for ev in lists:
            S.check_order(ev, m, cfg.n_layers)
            assert S.account_memory(ev, cfg.n_layers, t, limit=budget)[0] <= budget
        ref = S.simulate(lists, [t_op] * p, 0.0, lambda i, e: size(e) / 55e6 + 0.02)
        assert info["makespan_model"] == pytest.approx(ref.makespan_global, rel=1e-12)
        assert info["makespan_model"] <= min(c["makespan_model"] for c in info["candidates"]) * (1 + 1e-12)
        assert info["offloaded_bytes"] == [sum(size(e) for e in ev if e[0] == "O") for ev in lists]
    # with room to spare the fill is denser than p - i in flight, and it pays in the model
    assert info["extra_fill"] > 0 and info["makespan_model"] < info["candidates"][0]["makespan_model"]
    assert SC.workload_lists(cfg, 0)[0] == base


def test_workload_lists_in_the_recompute_variant_fit_the_oracles_recompute_accounting():
    cfg = _small_cfg()
    t = _table(cfg)
    p, m = cfg.n_stages, cfg.n_microbatches
    base = G.split_bw_greedy(p, m)
    peak0 = max(S.account_memory(ev, cfg.n_layers, t, recompute=True)[0] for ev in base)
    budget = int(0.8 * peak0)
    lists, info = SC.workload_lists(cfg, budget, recompute=1)
    assert any(e[0] == "O" for ev in lists for e in ev)
    for ev in lists:
        S.check_order(ev, m, cfg.n_layers, recompute=True)
        assert S.account_memory(ev, cfg.n_layers, t, limit=budget, recompute=True)[0] <= budget
