"""Pins for oracle/schedule.py: closed forms, an independent time-stepped checker,
brute-force enumeration of tiny schedules, a direct check of the paper's
constraints on every simulated timing, and live-set memory accounting."""
import itertools

import pytest

from oracle import schedule as S
from stage_inputs import schedules as G

TABLE = S.memory_table(S.LLAMA, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=96, tokens=32, elem_size=2)
L = 2


# ------------------------------------------------------------------ independent re-implementations
def tick_sim(lists, t_op, t_comm, t_copy, duplex=False):
    """Integer time-stepped polling simulator (nothing shared with S.simulate).  duplex: offloads and
    reloads are polled as two independent serial queues instead of one."""
    p = len(lists)
    fin = [dict() for _ in range(p)]          # event index -> finish tick
    begun = [dict() for _ in range(p)]
    busy_c = [0] * p
    busy_x = [[0, 0] for _ in range(p)]
    t = 0
    total = sum(len(l) for l in lists)

    def finished(i, n, t):
        return n in fin[i] and fin[i][n] <= t

    def find(i, op, j):
        for n, ev in enumerate(lists[i]):
            if ev[0] == op and ev[1] == j:
                return n
        return None

    while sum(len(f) for f in fin) < total:
        for i in range(p):
            for n, ev in enumerate(lists[i]):               # OWAIT events complete when their copy did
                if ev[0] == "OWAIT" and n not in fin[i]:
                    o = [k for k, e in enumerate(lists[i]) if e[0] == "O" and e[1:] == ev[1:]][0]
                    if finished(i, o, t) and all(m in begun[i] or lists[i][m][0] == "OWAIT" and m in fin[i] or lists[i][m][0] in ("O", "R") for m in range(n)):
                        fin[i][n] = fin[i][o]
            comp = [n for n, ev in enumerate(lists[i]) if ev[0] in "FBW" and n not in begun[i]]
            if comp and busy_c[i] <= t:
                n = comp[0]
                op, j = lists[i][n][0], lists[i][n][1]
                ok = True
                for m in range(n):
                    e = lists[i][m]
                    if e[0] == "OWAIT":
                        o = [k for k, e2 in enumerate(lists[i]) if e2[0] == "O" and e2[1:] == e[1:]][0]
                        ok &= finished(i, o, t)
                    if e[0] in "FBW":
                        ok &= finished(i, m, t)
                if op == "F" and i > 0:
                    u = find(i - 1, "F", j)
                    ok &= u in fin[i - 1] and fin[i - 1][u] + t_comm <= t
                if op == "B":
                    if i < p - 1:
                        u = find(i + 1, "B", j)
                        ok &= u in fin[i + 1] and fin[i + 1][u] + t_comm <= t
                    for m, e in enumerate(lists[i]):
                        if e[0] == "R" and e[1] == j:
                            ok &= finished(i, m, t)
                if ok:
                    begun[i][n] = t
                    fin[i][n] = t + t_op[i][op]
                    busy_c[i] = fin[i][n]
            for kinds, lane in ((("O",), 0), (("R",), 1)) if duplex else ((("O", "R"), 0),):
              xfer = [n for n, ev in enumerate(lists[i]) if ev[0] in kinds and n not in begun[i]]
              if xfer and busy_x[i][lane] <= t:
                n = xfer[0]
                ev = lists[i][n]
                ok = True
                if ev[0] == "O":
                    ok &= finished(i, find(i, "F", ev[1]), t)
                else:
                    for m in range(n):
                        if lists[i][m][0] in "FBW":
                            ok &= finished(i, m, t)
                    o = [k for k, e2 in enumerate(lists[i]) if e2[0] == "O" and e2[1:] == ev[1:]][0]
                    ok &= finished(i, o, t)
                if ok:
                    begun[i][n] = t
                    fin[i][n] = t + t_copy
                    busy_x[i][lane] = fin[i][n]
        t += 1
        assert t < 400, "tick simulator stuck"
    comp_ends = [fin[i][n] for i in range(p) for n, ev in enumerate(lists[i]) if ev[0] in "FBW"]
    comp_starts = [begun[i][n] for i in range(p) for n, ev in enumerate(lists[i]) if ev[0] in "FBW"]
    return max(comp_ends) - min(comp_starts), begun, fin


def liveset_peak(events, n_layers, table):
    """Peak bytes by tracking the set of live buffers (not a running sum of deltas)."""
    live = set()
    peak = 0

    def total():
        return sum(table[k] for (_, _, k) in live)

    for ev in events:
        op, j = ev[0], ev[1]
        if op == "F":
            for l in range(n_layers):
                for k in S.F_KINDS:
                    live.add((j, l, k))
            peak = max(peak, total())
        elif op == "B":
            live.add((j, n_layers - 1, "DY"))
            peak = max(peak, total())
            for l in reversed(range(n_layers)):
                live.add((j, l, "DX_MID"))
                peak = max(peak, total())
                live -= {(j, l, "X_MID"), (j, l, "LSE")}
                if l > 0:
                    live.add((j, l - 1, "DY"))
                    peak = max(peak, total())
                live -= {(j, l, "X_IN"), (j, l, "STATS")}
        elif op == "W":
            live = {b for b in live if b[0] != j}
        elif op == "OWAIT":
            live -= {(j, ev[2], k) for k in ev[3]}
        elif op == "R":
            live |= {(j, ev[2], k) for k in ev[3]}
            peak = max(peak, total())
    assert not live
    return peak


def check_constraints(lists, tm, t_op, t_comm, t_copy, duplex=False):
    """Every paper constraint, checked directly on a timed schedule (duplex: Eq. 8-11 per direction)."""
    eps = 1e-9
    p = len(lists)
    for i in range(p):
        ev = lists[i]
        st, en = tm.start[i], tm.end[i]
        comp = [n for n, e in enumerate(ev) if e[0] in "FBW"]
        xfer = [n for n, e in enumerate(ev) if e[0] in ("O", "R")]
        for a, b in itertools.combinations(comp, 2):                 # Eq. 5: no overlap
            assert en[a] <= st[b] + eps or en[b] <= st[a] + eps
        for a, b in itertools.combinations(xfer, 2):                 # Eq. 8-11: one transfer at a time
            if duplex and ev[a][0] != ev[b][0]:
                continue
            assert en[a] <= st[b] + eps or en[b] <= st[a] + eps
        idx = {(e[0], e[1]): n for n, e in enumerate(ev) if e[0] in "FBW"}
        for (op, j), n in idx.items():
            assert abs(en[n] - st[n] - t_op[i][op]) < eps
            if op == "F":
                assert en[idx[("F", j)]] <= st[idx[("B", j)]] + eps  # Eq. 6
                assert en[idx[("B", j)]] <= st[idx[("W", j)]] + eps
                if i > 0:                                            # Eq. 3
                    up = [k for k, e in enumerate(lists[i - 1]) if e[:2] == ("F", j)][0]
                    assert st[n] + eps >= tm.end[i - 1][up] + t_comm
            if op == "B" and i < p - 1:                              # Eq. 4
                dn = [k for k, e in enumerate(lists[i + 1]) if e[:2] == ("B", j)][0]
                assert st[n] + eps >= tm.end[i + 1][dn] + t_comm
            if op != "F" and j > 0:                                  # fixed micro-batch order
                assert en[idx[(op, j - 1)]] <= st[n] + eps
        for n, e in enumerate(ev):
            if e[0] == "O":
                assert st[n] + eps >= en[idx[("F", e[1])]]           # offload after its F
            if e[0] == "R":
                o = [k for k, e2 in enumerate(ev) if e2[0] == "O" and e2[1:] == e[1:]][0]
                assert st[n] + eps >= en[o]
                assert en[n] <= st[idx[("B", e[1])]] + eps           # reload completes before its consumer
                for m in comp:
                    if m < n:
                        assert st[n] + eps >= en[m]                  # Eq. 14
            if e[0] == "OWAIT":
                o = [k for k, e2 in enumerate(ev) if e2[0] == "O" and e2[1:] == e[1:]][0]
                for m in comp:
                    if m > n:
                        assert st[m] + eps >= en[o]                  # Eq. 12


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("p,m", [(4, 4), (8, 16), (2, 3), (3, 7)])
def test_1f1b_bubble_closed_form(p, m):
    lists = [G.one_f_one_b(p, m, i) for i in range(p)]
    for i in range(p):
        S.check_order(lists[i], m, L)
    t_op = [{"F": 1.0, "B": 2.0, "W": 0.0}] * p          # B and W fused, identical stages, T_comm = 0
    tm = S.simulate(lists, t_op)
    assert abs(tm.makespan_global - (m + p - 1) * 3.0) < 1e-12
    for i in range(p):
        assert abs(tm.bubble[i] - (p - 1) / (m + p - 1)) < 1e-12
    if (p, m) == (4, 4):
        assert abs(tm.bubble[0] - 3 / 7) < 1e-12
    if (p, m) == (8, 16):
        assert abs(tm.bubble[1] - 7 / 23) < 1e-12
    check_constraints(lists, tm, t_op, 0.0, 0.0)
    # in-flight micro-batches: Eq. 7 usage peaks at min(p - i, m) * Delta_F
    dF = S.op_delta("F", L, TABLE)
    for i in range(p):
        use = max(u for _, u in S.eq7_usage(lists[i], L, TABLE))
        assert use == min(p - i, m) * dF


def test_single_microbatch_closed_form():
    p = 5
    lists = [[("F", 0), ("B", 0), ("W", 0)] for _ in range(p)]
    t_op = [{"F": 1.0 + 0.1 * i, "B": 2.0 + 0.2 * i, "W": 0.7 + 0.05 * i} for i in range(p)]
    tc = 0.3
    tm = S.simulate(lists, t_op, t_comm=tc)
    want = sum(t["F"] for t in t_op) + sum(t["B"] for t in t_op) + t_op[0]["W"] + 2 * (p - 1) * tc
    assert abs(tm.makespan_global - want) < 1e-12
    check_constraints(lists, tm, t_op, tc, 0.0)


def test_memory_signs_and_conservation():
    dF, dB, dW = (S.op_delta(c, L, TABLE) for c in "FBW")
    assert dF > 0 and dB < 0 and dW < 0 and dF + dB + dW == 0
    assert all(v % 256 == 0 for v in TABLE.values())
    ev = G.one_f_one_b(4, 6, 1)
    peak, trace = S.account_memory(ev, L, TABLE)
    assert trace[-1] == 0 and peak >= dF
    assert peak == liveset_peak(ev, L, TABLE)
    # the fine-grained peak exceeds Eq. 7's op-level figure by at most B's two transient buffers
    eq7 = max(u for _, u in S.eq7_usage(ev, L, TABLE))
    assert eq7 <= peak <= eq7 + TABLE["DY"] + TABLE["DX_MID"]


def test_memory_table_values():
    # llama-style layer at hidden 4096, 32 heads x 128, ffn 11008, 4096 tokens, bf16: 514.5 MiB
    t = S.memory_table(S.LLAMA, 4096, 32, 32, 128, 11008, 4096, 2)
    assert sum(t[k] for k in S.F_KINDS) == int(514.5 * 2**20) + 32 * 1024
    assert t["QKV"] == 96 * 2**20 and t["GU"] == 172 * 2**20 and t["LSE"] == 2**19
    # rounding to 256 bytes
    t = S.memory_table(S.GPT, 3, 1, 1, 5, 7, 3, 4)
    assert t["X_IN"] == 256 and t["STATS"] == 256 and t["GU"] == 256


def test_recompute_variant_of_the_memory_table():
    """F keeps no norm outputs and no MLP activation output; B rebuilds them for W.  The figures are worked out
    by hand from the shapes, not through the table code."""
    # llama 7B layer, per token in bf16: kept by F in the store-all table 16 h + 6 f + 4 n_q + 8 bytes
    # (x_in, n1, x_mid, n2, o: 2 h each; qkv 6 h; gu 4 f; a 2 f; lse 4 n_q; rstd x2 8); the variant drops 4 h + 2 f
    h, f, nq, tok = 4096, 11008, 32, 8192
    t = S.memory_table(S.LLAMA, h, nq, nq, 128, f, tok, 2)
    full, var = S.op_delta("F", 1, t), S.op_delta("F", 1, t, recompute=True)
    assert full == tok * (16 * h + 6 * f + 4 * nq + 8)
    assert full - var == tok * (4 * h + 2 * f)
    assert abs((full - var) / full - 0.2915) < 1e-4
    for Ln in (1, 3):
        d0 = [S.op_delta(c, Ln, TABLE) for c in "FBW"]
        d1 = [S.op_delta(c, Ln, TABLE, recompute=True) for c in "FBW"]
        moved = Ln * (TABLE["N1"] + TABLE["N2"] + TABLE["A"])
        assert d1 == [d0[0] - moved, d0[1] + moved, d0[2]] and sum(d1) == 0
    # one layer, one micro-batch, by hand: B holds dy, then a, n2, dx_mid on top of what F kept, drops x_mid and
    # lse, adds n1, drops x_in and stats
    T1 = TABLE
    kept = sum(T1[k] for k in S.F_KINDS if k not in ("N1", "N2", "A"))
    ev = [("F", 0), ("B", 0), ("W", 0)]
    peak, trace = S.account_memory(ev, 1, T1, recompute=True)
    in_b = kept + T1["DY"] + T1["A"] + T1["N2"] + T1["DX_MID"]
    assert trace[0] == kept and peak == max(in_b, in_b - T1["X_MID"] - T1["LSE"] + T1["N1"])
    assert trace[1] == in_b - T1["X_MID"] - T1["LSE"] + T1["N1"] - T1["X_IN"] - T1["STATS"] and trace[2] == 0
    # same list, store-all: after B the two variants hold the same bytes (W's operands)
    assert S.account_memory(ev, 1, T1)[1][1] == trace[1]
    # every F ahead of every B: the peak falls inside B 0, where the variant holds a subset of the store-all
    # buffers of micro-batch 0 and none of the three kinds for the m - 1 micro-batches still waiting for B
    m = 5
    ev = [("F", j) for j in range(m)] + [(c, j) for j in range(m) for c in "BW"]
    p0, _ = S.account_memory(ev, L, TABLE)
    p1, _ = S.account_memory(ev, L, TABLE, recompute=True)
    moved = L * (TABLE["N1"] + TABLE["N2"] + TABLE["A"])
    assert (m - 1) * moved <= p0 - p1 <= m * moved
    # the kinds F does not keep cannot be offloaded
    bad = [("F", 0), ("O", 0, 0, ("N1",)), ("OWAIT", 0, 0, ("N1",)), ("R", 0, 0, ("N1",)), ("B", 0), ("W", 0)]
    S.check_order(bad, 1, 1)
    with pytest.raises(S.ScheduleError) as ei:
        S.check_order(bad, 1, 1, recompute=True)
    assert ei.value.index == 1


# ------------------------------------------------------------------ several model chunks per stage
def tick_sim_chunks(lists, t_op, t_comm, before_of):
    """Integer time-stepped simulator for compute-only lists with model chunks.  before_of(i, c) names the
    (stage, chunk) holding the previous piece of the model, or None for the first piece; it is written out by
    the caller, not computed from the oracle's placement code."""
    p = len(lists)
    pieces = {(i, e[2] if len(e) > 2 else 0) for i in range(p) for e in lists[i]}
    after_of = {before_of(i, c): (i, c) for (i, c) in pieces if before_of(i, c) is not None}
    fin = [dict() for _ in range(p)]
    begun = [dict() for _ in range(p)]
    busy = [0] * p

    def end_of(i, op, j, c):
        for n, e in enumerate(lists[i]):
            if e[0] == op and e[1] == j and (e[2] if len(e) > 2 else 0) == c:
                return fin[i].get(n)
        raise AssertionError("missing op")

    t = 0
    while sum(len(f) for f in fin) < sum(len(l) for l in lists):
        for i in range(p):
            todo = [n for n in range(len(lists[i])) if n not in begun[i]]
            if not todo or busy[i] > t:
                continue
            n = todo[0]
            e = lists[i][n]
            op, j, c = e[0], e[1], (e[2] if len(e) > 2 else 0)
            ok = True
            if op == "F" and before_of(i, c) is not None:
                i2, c2 = before_of(i, c)
                u = end_of(i2, "F", j, c2)
                ok = u is not None and u + (t_comm if i2 != i else 0) <= t
            if op == "B" and (i, c) in after_of:
                i2, c2 = after_of[(i, c)]
                u = end_of(i2, "B", j, c2)
                ok = u is not None and u + (t_comm if i2 != i else 0) <= t
            if ok:
                begun[i][n] = t
                fin[i][n] = t + t_op[i][op]
                busy[i] = fin[i][n]
        t += 1
        assert t < 2000, "tick simulator stuck"
    return max(max(f.values()) for f in fin) - min(min(b.values()) for b in begun), begun, fin


@pytest.mark.parametrize("p,m,v", [(2, 2, 2), (4, 8, 2), (4, 4, 3), (8, 16, 2)])
def test_interleaved_1f1b_bubble_closed_form(p, m, v):
    """1F1B with v model chunks per stage idles (p - 1) / (v m + p - 1) of the time when a chunk's backward
    costs twice its forward and transfers between stages are free: the warm-up and cool-down ramps are those
    of plain 1F1B on pieces v times shorter."""
    lists = [G.interleaved_one_f_one_b(p, m, i, v) for i in range(p)]
    for lst in lists:
        S.check_order(lst, m, v, n_chunks=v)
    t_op = [{"F": 1.0, "B": 2.0, "W": 0.0}] * p
    tm = S.simulate(lists, t_op, n_chunks=v)
    assert abs(tm.makespan_global - (3.0 * m * v + 3.0 * (p - 1))) < 1e-12
    assert all(abs(b - (p - 1) / (v * m + p - 1)) < 1e-12 for b in tm.bubble)
    # one chunk per stage: the makespan of plain 1F1B (its warm-up is twice as deep, which costs memory, not time)
    one = S.simulate([G.interleaved_one_f_one_b(p, m, i, 1) for i in range(p)], t_op)
    assert abs(one.makespan_global - S.simulate([G.one_f_one_b(p, m, i) for i in range(p)], t_op).makespan_global) < 1e-12
    # integer tick simulator with the placement written out by hand: chunk c of stage i follows chunk c of stage
    # i - 1, and chunk c of stage 0 follows chunk c - 1 of the last stage
    before = lambda i, c: (i - 1, c) if i > 0 else ((p - 1, c - 1) if c > 0 else None)
    ti = [{"F": 1, "B": 2, "W": 1}] * p
    span, begun, fin = tick_sim_chunks(lists, ti, 1, before)
    tm = S.simulate(lists, ti, t_comm=1, n_chunks=v)
    assert span == tm.makespan_global
    for i in range(p):
        for n in range(len(lists[i])):
            assert begun[i][n] == tm.start[i][n] and fin[i][n] == tm.end[i][n]


def test_v_shaped_placement_by_hand():
    """Two stages, two chunks, V shape: the model runs stage 0 chunk 0, stage 1 chunk 0, stage 1 chunk 1, stage 0
    chunk 1.  One micro-batch is a serial chain; times worked out by hand with T_F = 1, T_B = 2, T_W = 1 and a
    transfer of 0.5 between stages (none where consecutive pieces share a stage)."""
    s0 = [("F", 0, 0), ("F", 0, 1), ("B", 0, 1), ("W", 0, 1), ("B", 0, 0), ("W", 0, 0)]
    s1 = [("F", 0, 0), ("F", 0, 1), ("B", 0, 1), ("B", 0, 0), ("W", 0, 1), ("W", 0, 0)]
    t_op = [{"F": 1.0, "B": 2.0, "W": 1.0}] * 2
    tm = S.simulate([s0, s1], t_op, t_comm=0.5, n_chunks=2, placement="v")
    # stage 0: F c0 0..1; stage 1: F c0 1.5..2.5, F c1 2.5..3.5; stage 0: F c1 4..5, B c1 5..7, W c1 7..8;
    # stage 1: B c1 7.5..9.5, B c0 9.5..11.5, W 11.5..12.5, W 12.5..13.5; stage 0: B c0 12..14, W c0 14..15
    assert tm.start[0] == [0.0, 4.0, 5.0, 7.0, 12.0, 14.0]
    assert tm.start[1] == [1.5, 2.5, 7.5, 9.5, 11.5, 12.5]
    assert tm.makespan_global == 15.0
    assert [S.virtual_stage(i, c, 2, "v") for i, c in ((0, 0), (1, 0), (1, 1), (0, 1))] == [0, 1, 2, 3]
    # the same lists read as interleaved (stage 0 chunk 1 would follow stage 1 chunk 0... and stage 1 chunk 1 stage
    # 0 chunk 1) deadlock on stage 1, which lists F of chunk 1 before stage 0 has run it
    span, begun, fin = tick_sim_chunks([s0, s1], [{"F": 2, "B": 4, "W": 2}] * 2, 1,
                                       lambda i, c: {(0, 0): None, (1, 0): (0, 0), (1, 1): (1, 0), (0, 1): (1, 1)}[(i, c)])
    tm2 = S.simulate([s0, s1], [{"F": 2, "B": 4, "W": 2}] * 2, t_comm=1, n_chunks=2, placement="v")
    assert span == tm2.makespan_global == 30


@pytest.mark.parametrize("p,m,placement", [(2, 4, "v"), (4, 8, "v"), (4, 8, "interleaved"), (8, 16, "v")])
def test_split_bw_lists_with_chunks(p, m, placement):
    """Zero-bubble style lists over two chunks per stage: valid per chunk, consistent across stages (the simulator
    finds no deadlock and agrees with the integer tick simulator whose placement is written out by hand), every
    stage within its in-flight cap, and no slower than interleaved 1F1B, which has no freedom to move W."""
    v = 2
    lists = G.split_bw_greedy_chunks(p, m, v, placement)
    for lst in lists:
        S.check_order(lst, m, v, n_chunks=v)
    t_op = [{"F": 1, "B": 1, "W": 1}] * p
    tm = S.simulate(lists, t_op, t_comm=0, n_chunks=v, placement=placement)
    if placement == "v":       # chunk 0 runs down the stages, chunk 1 back up; the turn is on the last stage
        before = lambda i, c: ((i - 1, 0) if i > 0 else None) if c == 0 else ((i + 1, 1) if i < p - 1 else (p - 1, 0))
    else:
        before = lambda i, c: (i - 1, c) if i > 0 else ((p - 1, c - 1) if c > 0 else None)
    span, begun, fin = tick_sim_chunks(lists, t_op, 0, before)
    assert span == tm.makespan_global
    ref = S.simulate([G.interleaved_one_f_one_b(p, m, i, v) for i in range(p)], t_op, n_chunks=v)
    assert tm.makespan_global <= ref.makespan_global
    dF = S.op_delta("F", 1, TABLE)
    slack = TABLE["DY"] + TABLE["DX_MID"]
    peaks = [S.account_memory(lst, v, TABLE, n_chunks=v)[0] for lst in lists]
    assert all(pk <= 2 * p * dF + slack for pk in peaks)
    if placement == "v":       # what the V shape is for: every stage holds the same (up to B's transients)
        assert max(peaks) - min(peaks) <= slack
    # a smaller cap is honoured too
    tight = G.split_bw_greedy_chunks(p, m, v, placement, cap_of_stage=lambda i: p + 1)
    for lst in tight:
        S.check_order(lst, m, v, n_chunks=v)
        assert S.account_memory(lst, v, TABLE, n_chunks=v)[0] <= (p + 1) * dF + slack
    S.simulate(tight, t_op, n_chunks=v, placement=placement)


def test_chunked_lists_order_rules_and_accounting():
    Lc, v, m = 2, 2, 4
    lst = G.interleaved_one_f_one_b(2, m, 0, v)
    S.check_order(lst, m, Lc * v, n_chunks=v)
    # per chunk: B needs that chunk's F, W that chunk's B, micro-batches in order per chunk
    bad = [("F", 0, 0), ("B", 0, 1)]
    with pytest.raises(S.ScheduleError) as ei:
        S.check_order(bad + [("W", 0, 1)], 1, 2, n_chunks=2)
    assert ei.value.index == 1
    with pytest.raises(S.ScheduleError):
        S.check_order([("F", 0, 0), ("F", 1, 1)], 2, 2, n_chunks=2)          # chunk 1 starts at micro-batch 0
    with pytest.raises(S.ScheduleError):
        S.check_order([("F", 0, 2)], 1, 2, n_chunks=2)                        # no such chunk
    S.check_order([("F", 0, 1), ("F", 0, 0), ("B", 0, 0), ("B", 0, 1), ("W", 0, 1), ("W", 0, 0)], 1, 2, n_chunks=2)
    # a chunk op moves the bytes of the chunk's layers only: the same totals as a one-chunk stage with
    # n_layers / n_chunks layers on which every (chunk, micro-batch) pair is a micro-batch of its own
    relabelled = [(e[0], e[2] * m + e[1]) for e in lst]
    pk, tr = S.account_memory(lst, Lc * v, TABLE, n_chunks=v)
    pk1, tr1 = S.account_memory(relabelled, Lc, TABLE)
    assert pk == pk1 and tr == tr1 and tr[-1] == 0
    # stage 0 of p = 2: 2 (p - 1) + (v - 1) p = 4 warm-up forward chunk-ops and the first steady-state one
    # precede its first backward
    dF = S.op_delta("F", Lc, TABLE)
    first_b = next(n for n, e in enumerate(lst) if e[0] == "B")
    assert tr[first_b - 1] == 5 * dF
    # transfers name the layer on the stage; B of a chunk needs the reloads of that chunk's layers only
    kinds = ("QKV",)
    ev = [("F", 0, 0), ("O", 0, 1, kinds), ("F", 0, 1), ("OWAIT", 0, 1, kinds), ("B", 0, 1), ("W", 0, 1),
          ("R", 0, 1, kinds), ("B", 0, 0), ("W", 0, 0)]
    S.check_order(ev, 1, 4, n_chunks=2)
    with pytest.raises(S.ScheduleError) as ei:
        S.check_order([("F", 0, 0), ("F", 0, 1), ("O", 0, 3, kinds), ("OWAIT", 0, 3, kinds), ("B", 0, 1)], 1, 4, n_chunks=2)
    assert ei.value.index == 4
    tm = S.simulate([ev], [{"F": 1.0, "B": 2.0, "W": 1.0}], t_copy=lambda i, e: 0.5, n_chunks=2, layers_per_chunk=2)
    # F c0 0..1, F c1 1..2, B c1 2..4, W c1 4..5: the offload starts when F of chunk 0 ends, the reload when W of
    # chunk 1 ends, and B of chunk 0 when the reload (0.5) is in
    assert tm.start[0][1] == 1.0 and tm.start[0][6] == 5.0 and tm.start[0][7] == 5.5


# ------------------------------------------------------------------ brute force
def all_orders(m):
    ops = [(c, j) for j in range(m) for c in "FBW"]

    def rec(prefix, remaining):
        if not remaining:
            yield list(prefix)
            return
        for o in sorted(remaining):
            c, j = o
            if c == "B" and ("F", j) in remaining:
                continue
            if c == "W" and ("B", j) in remaining:
                continue
            if j > 0 and (c, j - 1) in remaining:
                continue
            yield from rec(prefix + [o], remaining - {o})
    return list(rec([], set(ops)))


@pytest.mark.parametrize("m", [1, 2, 3])
def test_bruteforce_makespan_agrees(m):
    orders = all_orders(m)
    t_op = [{"F": 1, "B": 2, "W": 1}, {"F": 2, "B": 1, "W": 1}]
    best_a = best_b = None
    n_checked = 0
    stride = 1
    for l0 in orders[::stride]:
        for l1 in orders[::stride]:
            try:
                tm = S.simulate([l0, l1], t_op, t_comm=1)
            except S.ScheduleError:
                # stage 1 cannot run B j before stage 0's F j etc. -> the tick simulator must also stall
                with pytest.raises(AssertionError):
                    tick_sim([l0, l1], t_op, 1, 0)
                continue
            span, begun, fin = tick_sim([l0, l1], t_op, 1, 0)
            assert span == tm.makespan_global
            for i, lst in enumerate((l0, l1)):
                for n in range(len(lst)):
                    assert begun[i][n] == tm.start[i][n] and fin[i][n] == tm.end[i][n]
            check_constraints([l0, l1], tm, t_op, 1, 0)
            best_a = span if best_a is None else min(best_a, span)
            best_b = tm.makespan_global if best_b is None else min(best_b, tm.makespan_global)
            n_checked += 1
    assert best_a == best_b and n_checked > 0


def offload_variants(order, j, kinds=("X_IN",), layer=0):
    """Every placement of O / OWAIT / R for micro-batch j's item in a compute order."""
    nF = order.index(("F", j))
    nB = order.index(("B", j))
    out = []
    n = len(order)
    for a in range(nF + 1, nB + 1):
        for b in range(a, nB + 1):
            for c in range(b, nB + 1):
                lst = list(order)
                for pos, ev in sorted([(c, ("R", j, layer, kinds)), (b, ("OWAIT", j, layer, kinds)),
                                       (a, ("O", j, layer, kinds))], key=lambda x: -x[0]):
                    lst.insert(pos, ev)
                # inserting at equal positions in reverse keeps O, OWAIT, R in order
                i_o, i_w, i_r = (lst.index(e) for e in (("O", j, layer, kinds), ("OWAIT", j, layer, kinds), ("R", j, layer, kinds)))
                if i_o < i_w < i_r:
                    out.append(lst)
    assert n and out
    return out


def test_bruteforce_with_offload_equal_times_capacity_three():
    # toy setting of the paper's illustration: all processing times equal, memory holds three
    # activations; the best makespan must be found identically by both simulators, and every
    # schedule's peak identically by running-sum and live-set accounting
    m = 3
    dF = S.op_delta("F", L, TABLE)
    limit = 3 * dF + TABLE["DY"] + TABLE["DX_MID"]
    t_op = [{"F": 1, "B": 1, "W": 1}] * 2
    best = {}
    count = 0
    for l0 in all_orders(m):
        for v0 in offload_variants(l0, 0):
            S.check_order(v0, m, L)
            pk, _ = S.account_memory(v0, L, TABLE)
            assert pk == liveset_peak(v0, L, TABLE)
            l1 = G.one_f_one_b(2, m, 1)
            try:
                tm = S.simulate([v0, l1], t_op, t_comm=0, t_copy=lambda i, ev: 1)
            except S.ScheduleError:
                continue
            span, begun, fin = tick_sim([v0, l1], t_op, 0, 1)
            assert span == tm.makespan_global, (v0, span, tm.makespan_global)
            for n, ev in enumerate(v0):
                if ev[0] != "OWAIT":
                    assert begun[0][n] == tm.start[0][n], (v0, n)
            check_constraints([v0, l1], tm, t_op, 0, 1)
            if pk <= limit:
                best["a"] = min(best.get("a", 10**9), span)
                best["b"] = min(best.get("b", 10**9), tm.makespan_global)
            count += 1
    assert count > 20 and best["a"] == best["b"]


def two_item_variants(order, m):
    """Offload micro-batch 0 and micro-batch 1 (layer 0, X_IN): every placement in which a reload of one may
    be listed while the offload of the other is still in flight."""
    out = []
    for v0 in offload_variants(order, 0):
        for v1 in offload_variants(v0, 1):
            out.append(v1)
    return out


def test_bruteforce_duplex_channels():
    # two offloaded items, copy time longer than an op: with one channel the second item's offload can delay
    # the first item's reload; with two channels it cannot.  Both simulators must agree in both modes, every
    # timing must satisfy the constraints (Eq. 8-11 per direction in duplex mode), duplex is never slower,
    # and it is strictly faster for at least one enumerated schedule.
    m = 3
    t_op = [{"F": 1, "B": 1, "W": 1}] * 2
    l1 = G.one_f_one_b(2, m, 1)
    faster = 0
    count = 0
    for l0 in all_orders(m)[::7]:
        for v in two_item_variants(l0, m)[::5]:
            try:
                S.check_order(v, m, L)
                one = S.simulate([v, l1], t_op, t_comm=0, t_copy=lambda i, ev: 2)
                two = S.simulate([v, l1], t_op, t_comm=0, t_copy=lambda i, ev: 2, duplex=True)
            except S.ScheduleError:
                continue
            for tm, dup in ((one, False), (two, True)):
                span, begun, fin = tick_sim([v, l1], t_op, 0, 2, duplex=dup)
                assert span == tm.makespan_global, (v, dup, span, tm.makespan_global)
                for n, ev in enumerate(v):
                    if ev[0] != "OWAIT":
                        assert begun[0][n] == tm.start[0][n], (v, dup, n)
                check_constraints([v, l1], tm, t_op, 0, 2, duplex=dup)
            assert two.makespan_global <= one.makespan_global
            faster += two.makespan_global < one.makespan_global
            count += 1
    assert count > 30 and faster > 0, (count, faster)


def test_offload_lowers_peak_monotonically():
    m, p, i = 6, 4, 0
    base = G.split_bw_greedy(p, m)[i]
    S.check_order(base, m, L)
    pk0, _ = S.account_memory(base, L, TABLE)
    prev = pk0
    for min_gap in (6, 4, 2):
        ev = G.add_offload(base, L, ("X_IN", "QKV", "X_MID"), min_gap=min_gap)
        S.check_order(ev, m, L)
        pk, tr = S.account_memory(ev, L, TABLE)
        assert tr[-1] == 0 and pk <= prev and pk == liveset_peak(ev, L, TABLE)
        prev = pk
    assert prev < pk0
    with pytest.raises(S.ScheduleError):
        S.account_memory(base, L, TABLE, limit=pk0 - 1)
    S.account_memory(base, L, TABLE, limit=pk0)


def test_order_violations_are_caught():
    good = G.one_f_one_b(2, 2, 0)
    S.check_order(good, 2, L)
    bad_lists = [
        [("B", 0), ("F", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("W", 0), ("B", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 1), ("F", 0), ("B", 0), ("W", 0), ("B", 1), ("W", 1)],
        [("F", 0), ("F", 0), ("B", 0), ("W", 0)],
        [("F", 0), ("B", 0), ("W", 0)],
        [("O", 0, 0, ("QKV",)), ("F", 0), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("O", 0, 0, ("QKV",)), ("OWAIT", 0, 0, ("QKV",)), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("O", 0, 0, ("QKV",)), ("R", 0, 0, ("QKV",)), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("O", 0, 0, ("DY",)), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
        [("F", 0), ("O", 0, 5, ("QKV",)), ("B", 0), ("W", 0), ("F", 1), ("B", 1), ("W", 1)],
    ]
    for b in bad_lists:
        with pytest.raises(S.ScheduleError):
            S.check_order(b, 2, L)


def test_split_bw_generator_is_valid_and_beats_1f1b():
    p, m = 4, 8
    lists = G.split_bw_greedy(p, m)
    for i in range(p):
        S.check_order(lists[i], m, L)
    t_op = [{"F": 1.0, "B": 1.0, "W": 1.0}] * p
    tm = S.simulate(lists, t_op)
    check_constraints(lists, tm, t_op, 0.0, 0.0)
    ref = S.simulate([G.one_f_one_b(p, m, i) for i in range(p)], t_op)
    assert tm.makespan_global <= ref.makespan_global
    # in-flight cap p - i holds
    dF = S.op_delta("F", L, TABLE)
    for i in range(p):
        assert max(u for _, u in S.eq7_usage(lists[i], L, TABLE)) <= (p - i) * dF


def test_repair_to_fit_with_the_oracle_as_planner():
    m, p, i = 8, 6, 1
    comp = G.split_bw_greedy(p, m, cap_of_stage=lambda s: 3)[i]
    S.check_order(comp, m, L)
    pk0, _ = S.account_memory(comp, L, TABLE)
    kinds = ("X_IN", "QKV", "X_MID", "GU")
    opt = G.add_offload(comp, L, kinds, min_gap=1, lead=2, wait_delay=2)
    pk_opt, _ = S.account_memory(opt, L, TABLE)

    def planner(limit):
        def fits(ev):
            try:
                S.check_order(ev, m, L)
                S.account_memory(ev, L, TABLE, limit=limit)
                return True, len(ev)
            except S.ScheduleError as e:
                return False, e.index
        return fits
    # a budget between what the tightest placement needs and what the optimistic one needs
    tight = G.add_offload(comp, L, kinds, min_gap=1, lead=0, wait_delay=0)
    pk_tight, _ = S.account_memory(tight, L, TABLE)
    assert pk_tight < pk_opt <= pk0
    limit = (pk_tight + pk_opt) // 2
    fixed = G.repair_to_fit(opt, planner(limit))
    assert fixed is not None
    S.check_order(fixed, m, L)
    pk, tr = S.account_memory(fixed, L, TABLE, limit=limit)
    assert pk <= limit and tr[-1] == 0
    assert sorted(map(str, fixed)) == sorted(map(str, opt))          # same events, only moved
    assert [e for e in fixed if e[0] in "FBW"] == comp                # compute order untouched
    # an impossible budget is reported, not looped on
    assert G.repair_to_fit(opt, planner(S.op_delta("F", L, TABLE) - 1)) is None


def test_gpt_workload_has_the_shapes_the_paper_prints():
    """Appendix "Configuration": the GPT-family workload (cfg 6) is the 1.5B / 3.6B column of the model table at the
    paper's sequence length, one stage of a p = 16 pipeline holding its equal share of the layers."""
    import os
    from stage_inputs import configs as CFG
    table = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "model_configuration.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, small, large = line.split()
                assert small == large                      # the two usable columns print the same shapes
                table[name] = int(small)
    c = CFG.CFG6
    assert c.hidden == table["hidden-size"] and c.ffn == table["ffn-hidden-size"]
    assert c.n_q_heads == table["num-attention-heads"] and c.n_kv_heads == table["num-query-groups"]
    assert c.n_q_heads * c.head_dim == c.hidden
    assert c.seq == table["sequence-length"]
    assert c.n_layers * c.n_stages == table["num-layers"] and c.n_stages == 16
    assert c.family == CFG.GPT


def test_backward_memory_steps_by_hand_and_chunk_offset():
    """The order in which a B op of two layers takes and frees buffers, written out from the layer's data flow: the
    incoming dY, then per layer (last first) the gradient at the mid residual, the mid residual and the softmax
    statistics freed once attention is differentiated, the next dY made before this layer's input is freed.  A
    model chunk that starts at layer 3 tags the same steps with layers 3 and 4."""
    want = [(+1, 1, "DY"),
            (+1, 1, "DX_MID"), (-1, 1, "X_MID"), (-1, 1, "LSE"), (+1, 0, "DY"), (-1, 1, "X_IN"), (-1, 1, "STATS"),
            (+1, 0, "DX_MID"), (-1, 0, "X_MID"), (-1, 0, "LSE"), (-1, 0, "X_IN"), (-1, 0, "STATS")]
    assert S.op_memory_steps("B", 2) == want
    assert S.op_memory_steps("B", 2, first_layer=3) == [(s, l + 3, k) for s, l, k in want]
    assert [l for _, l, _ in S.op_memory_steps("F", 2, first_layer=3)] == [3] * len(S.F_KINDS) + [4] * len(S.F_KINDS)


def test_index_bounds_are_exclusive():
    """Micro-batch m and layer L do not exist (indices run from 0)."""
    ok = [("F", 0), ("O", 0, L - 1, ("QKV",)), ("OWAIT", 0, L - 1, ("QKV",)), ("R", 0, L - 1, ("QKV",)), ("B", 0), ("W", 0)]
    S.check_order(ok, 1, L)
    with pytest.raises(S.ScheduleError):
        S.check_order(G.one_f_one_b(1, 2, 0), 1, L)         # a valid list of two micro-batches, checked for one
    with pytest.raises(S.ScheduleError):
        S.check_order([("F", 0), ("O", 0, L, ("QKV",)), ("OWAIT", 0, L, ("QKV",)), ("R", 0, L, ("QKV",)), ("B", 0), ("W", 0)], 1, L)


def test_eq7_usage_with_an_offloaded_item_by_hand():
    """Eq. 7 as printed: an op is charged its own Delta, the Delta of every op before it, minus Gamma of every
    offload completed before it, plus Gamma of every reload started before it."""
    d = {c: S.op_delta(c, L, TABLE) for c in "FBW"}
    item = ("QKV", "X_MID")
    g = TABLE["QKV"] + TABLE["X_MID"]
    ev = [("F", 0), ("O", 0, 1, item), ("OWAIT", 0, 1, item), ("F", 1), ("R", 0, 1, item), ("B", 0), ("W", 0), ("B", 1), ("W", 1)]
    use = dict(S.eq7_usage(ev, L, TABLE))
    assert use[0] == d["F"]
    assert use[3] == 2 * d["F"] - g                      # F1: the offload of micro-batch 0 has completed
    assert use[5] == 2 * d["F"] - g + g + d["B"]         # B0: and its reload has started
    assert use[6] == 2 * d["F"] + d["B"] + d["W"]
    assert use[8] == 2 * (d["F"] + d["B"] + d["W"]) == 0


def test_makespan_per_stage_is_the_longest_span_of_a_stage():
    """Eq. 16 against Eq. 17 on 1F1B with unit times: stage 0 runs from the first F to the last W, so its span is the
    whole makespan; the last stage starts p - 1 steps late and ends earlier, and must not set the figure."""
    p, m = 3, 4
    lists = [G.one_f_one_b(p, m, i) for i in range(p)]
    t = S.simulate(lists, [{"F": 1.0, "B": 1.0, "W": 1.0}] * p)
    spans = [max(e for e in t.end[i] if e is not None) - min(s for s in t.start[i] if s is not None) for i in range(p)]
    assert t.makespan_per_stage == max(spans) == spans[0] == t.makespan_global
    assert spans[p - 1] < spans[0]


def test_sizes_round_up_to_the_allocation_grain():
    """Buffer sizes are whole multiples of the allocator's grain, the smallest that holds the bytes."""
    a = S.ALIGN
    assert [S._round_up(n) for n in (1, a - 1, a, a + 1, 2 * a, 2 * a + 1)] == [a, a, a, 2 * a, 2 * a, 3 * a]


def test_v_shaped_placement_with_four_chunks():
    """Four chunks per stage in the V-shaped placement make a W: even chunks run down the stages, odd ones back
    up, so on p = 3 stages the 12 pieces sit on stages 0 1 2 2 1 0 0 1 2 2 1 0."""
    p, v = 3, 4
    where = {S.virtual_stage(i, c, p, "v"): i for i in range(p) for c in range(v)}
    assert [where[n] for n in range(p * v)] == [0, 1, 2, 2, 1, 0, 0, 1, 2, 2, 1, 0]
    assert [S._holder(n, p, "v") for n in range(p * v)] == [(where[n], n // p) for n in range(p * v)]
    where = {S.virtual_stage(i, c, p, "interleaved"): i for i in range(p) for c in range(v)}
    assert [where[n] for n in range(p * v)] == [0, 1, 2] * v
