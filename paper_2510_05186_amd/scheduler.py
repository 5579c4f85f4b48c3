"""Host-side schedule generation for the stage executor.

Two generators of per-stage event lists (the input of optstage_run):

* ``adaoffload``  the dense-fill initial schedule of the paper's appendix "AdaOffload" (Alg. 1): as many
  forward ops before the first backward op of a stage as its start estimate, a tolerance and the memory
  capacity allow, every forward activation offloaded, the rest of the list by PipeOffload-style rules
  (backward as soon as it can run, weight gradients in the gaps, reloads one op ahead of their consumer).
* ``milp_schedule``  the mixed-integer program of the paper's appendix "Mathematical Models" (Eq. 2-17) for
  small instances, solved with HiGHS through scipy.optimize.milp, with the fixed micro-batch order, the
  one-direction precedence variables and the triangle cuts of Sec. 4.1.

Both work on the paper's abstract instance (p stages, m identical micro-batches, one offloadable item per
forward op) and return lists in the executor's vocabulary: ("F"|"B"|"W", j) and ("O"|"OWAIT"|"R", j, layer,
kinds).  List order carries the paper's precedence binaries: an op listed after OWAIT(x) is credited x's
memory (M = 1, Eq. 12), an op listed after R(x) is charged it (N = 1, Eq. 13) and R(x) starts after the ops
listed before it (N = 0, Eq. 14).

Readings where the appendix is silent or inconsistent (the same ones the executor follows): Eq. 5 holds for
every pair of distinct ops of a stage; Eq. 12 bounds the start of the credited op (E - T, not E - T_comm); an
offload starts after its forward op ended, its reload after the offload ended, and the backward op of the
same micro-batch after the reload ended; only forward activations are offloaded; offloads, like reloads,
run in micro-batch order (identical micro-batches, forward and backward ops already in that order), so K and
L are constants and only H is decided.
"""
from __future__ import annotations

import bisect
import itertools
from dataclasses import dataclass, field

import numpy as np

OPS = ("F", "B", "W")


@dataclass
class Instance:
    """The paper's parameters for one pipeline (identical micro-batches)."""
    p: int                       # stages
    m: int                       # micro-batches
    t_op: list                   # per stage {"F": T_F, "B": T_B, "W": T_W}
    t_comm: float = 0.0
    t_off: list | None = None    # per stage: duration of one offload (= one reload), T_offload
    delta: list | None = None    # per stage {"F": Delta_F, "B": Delta_B, "W": Delta_W} (Eq. 7)
    gamma: list | None = None    # per stage: bytes of the offloadable item, Gamma
    own_peak: list | None = None  # per stage {"F","B","W"}: most bytes an op holds beyond the level before it
                                  # while it runs.  None = Eq. 7 as printed: the op's own term is its net Delta,
                                  # which credits the release of a B or W op before it has run; a device holds
                                  # those bytes until the op ends (own term 0 for W, B's transient peak for B)
    limit: list | None = None    # per stage: M_limit (None entry = unlimited)
    offload_stages: tuple = ()   # stages that may offload
    offload_mbs: tuple | None = None   # micro-batches that may offload (None = all)
    item: tuple = (0, ("X_IN",))  # (layer, kinds) the O / OWAIT / R events name

    def __post_init__(self):
        self.t_off = self.t_off or [0.0] * self.p
        self.delta = self.delta or [{"F": 0, "B": 0, "W": 0}] * self.p
        self.gamma = self.gamma or [0] * self.p
        self.limit = self.limit or [None] * self.p


@dataclass
class Solution:
    lists: list                  # per stage event list
    makespan: float              # Eq. 17
    start: dict = field(default_factory=dict)    # (i, j, c) -> start time
    offloaded: dict = field(default_factory=dict)  # (i, j) -> bool
    status: str = ""


# ----------------------------------------------------------------------------------------------- MILP

def _fixed_precedence(u, v):
    """Order of two ops of one stage fixed by the model (Eq. 6, fixed micro-batch order and what follows
    from them by transitivity): +1 u before v, -1 v before u, 0 free."""
    (ju, cu), (jv, cv) = u, v
    ru, rv = OPS.index(cu), OPS.index(cv)
    if ju <= jv and ru <= rv:
        return 1
    if jv <= ju and rv <= ru:
        return -1
    return 0


def milp_schedule(inst: Instance, time_limit: float = 60.0, cutoff: float | None = None,
                  triangle_cuts: bool = True, strict_eq13: bool = True) -> Solution:
    """Solves Eq. 2-17 to optimality (small instances).  cutoff: a known makespan (e.g. AdaOffload's), added
    as C <= cutoff; scipy's interface takes no starting point, so this is how an initial solution helps.
    strict_eq13: Eq. 13 as printed makes an op that is charged a reload's memory start no earlier than that
    reload; the stage executor charges by list position and lets the compute stream run on while the reload
    waits for the transfer channel, which is the model without Eq. 13 (False).  A tiny secondary cost keeps N
    at 0 wherever Eq. 14 does not force it, so that the extracted list charges no op needlessly."""
    from scipy.optimize import Bounds, LinearConstraint, milp
    from scipy.sparse import lil_matrix

    p, m = inst.p, inst.m
    ops = [(j, c) for j in range(m) for c in OPS]
    names = []
    lo, hi, integ = [], [], []

    def var(name, lb, ub, integer):
        names.append(name)
        lo.append(lb)
        hi.append(ub)
        integ.append(1 if integer else 0)
        return len(names) - 1

    big = sum(sum(inst.t_op[i].values()) for i in range(p)) * m + (2 * p) * inst.t_comm + \
        2 * m * sum(inst.t_off[i] for i in range(p)) + 1.0
    C = var("C", 0, big, False)
    E = {(i, u): var(f"E{i}{u}", 0, big, False) for i in range(p) for u in ops}
    P = {}
    for i in range(p):
        for u, v in itertools.combinations(ops, 2):
            if _fixed_precedence(u, v) == 0:
                P[(i, u, v)] = var(f"P{i}{u}{v}", 0, 1, True)
    off = [i for i in range(p) if i in inst.offload_stages and inst.gamma[i] > 0]
    Wv, Ov, Rv, Hv, Mv, Nv = {}, {}, {}, {}, {}, {}
    for i in off:
        for j in range(m):
            may = inst.offload_mbs is None or j in inst.offload_mbs
            Wv[(i, j)] = var(f"w{i},{j}", 0, 1 if may else 0, True)
            Ov[(i, j)] = var(f"O{i},{j}", 0, big, False)
            Rv[(i, j)] = var(f"R{i},{j}", 0, big, False)
            for v in ops:
                Mv[(i, j, v)] = var(f"M{i},{j}{v}", 0, 1, True)
                Nv[(i, j, v)] = var(f"N{i},{j}{v}", 0, 1, True)
        for j, j2 in itertools.permutations(range(m), 2):
            Hv[(i, j, j2)] = var(f"H{i},{j},{j2}", 0, 1, True)      # offload j starts before reload j2

    rows = []           # (coefficients {var: a}, lb, ub)

    def ge(coef, rhs):
        rows.append((coef, rhs, np.inf))

    def le(coef, rhs):
        rows.append((coef, -np.inf, rhs))

    def before(i, u, v):
        """Linear expression (coefficients, constant) of the 0/1 value 'u before v'."""
        f = _fixed_precedence(u, v)
        if f:
            return {}, 1.0 if f > 0 else 0.0
        if (i, u, v) in P:
            return {P[(i, u, v)]: 1.0}, 0.0
        return {P[(i, v, u)]: -1.0}, 1.0

    for i in range(p):
        T = inst.t_op[i]
        for u in ops:
            ge({E[(i, u)]: 1.0}, T[u[1]])                                   # starts at or after 0
        ge({E[(0, (0, "F"))]: -1.0}, -inst.t_op[0]["F"])                    # first op starts at 0
        for j in range(m):
            if i > 0:                                                        # Eq. 3
                ge({E[(i, (j, "F"))]: 1.0, E[(i - 1, (j, "F"))]: -1.0}, inst.t_comm + T["F"])
            if i < p - 1:                                                    # Eq. 4
                ge({E[(i, (j, "B"))]: 1.0, E[(i + 1, (j, "B"))]: -1.0}, inst.t_comm + T["B"])
            ge({C: 1.0, E[(i, (j, "W"))]: -1.0}, 0.0)                        # Eq. 17 with the first start at 0
        for u, v in itertools.combinations(ops, 2):                          # Eq. 5 for every pair
            coef, const = before(i, u, v)
            # u before v: E_v >= E_u + T_v - big (1 - b)
            c1 = {E[(i, v)]: 1.0, E[(i, u)]: -1.0}
            for k, a in coef.items():
                c1[k] = c1.get(k, 0.0) - big * a
            ge(c1, T[v[1]] - big + big * const)
            # v before u: E_u >= E_v + T_u - big b
            c2 = {E[(i, u)]: 1.0, E[(i, v)]: -1.0}
            for k, a in coef.items():
                c2[k] = c2.get(k, 0.0) + big * a
            ge(c2, T[u[1]] - big * const)
        if triangle_cuts:                                                     # Sec. 4.1, triangle inequality cuts
            for a, b, c in itertools.permutations(ops, 3):
                ca, ka = before(i, a, b)
                cb, kb = before(i, b, c)
                cc, kc = before(i, a, c)
                if not (ca or cb or cc):
                    continue
                coef = dict(cc)
                for k, x in ca.items():
                    coef[k] = coef.get(k, 0.0) - x
                for k, x in cb.items():
                    coef[k] = coef.get(k, 0.0) - x
                ge(coef, ka + kb - 1.0 - kc)
        # Eq. 7 for every op of the stage
        if inst.limit[i] is not None:
            D, G = inst.delta[i], inst.gamma[i]
            for v in ops:
                coef, const = {}, float(D[v[1]] if inst.own_peak is None else inst.own_peak[i][v[1]])
                for u in ops:
                    if u == v:
                        continue
                    cu, ku = before(i, u, v)
                    const += D[u[1]] * ku
                    for k, a in cu.items():
                        coef[k] = coef.get(k, 0.0) + D[u[1]] * a
                if i in off:
                    for j in range(m):
                        coef[Mv[(i, j, v)]] = coef.get(Mv[(i, j, v)], 0.0) - G
                        coef[Nv[(i, j, v)]] = coef.get(Nv[(i, j, v)], 0.0) + G
                le(coef, inst.limit[i] - const)
    for i in off:
        T, to = inst.t_op[i], inst.t_off[i]
        for j in range(m):
            w, o, r = Wv[(i, j)], Ov[(i, j)], Rv[(i, j)]
            ge({o: 1.0, E[(i, (j, "F"))]: -1.0, w: -big}, -big)               # offload after its forward op
            ge({r: 1.0, o: -1.0, w: -big}, to - big)                          # reload after its offload
            ge({E[(i, (j, "B"))]: 1.0, r: -1.0, w: -big}, T["B"] + to - big)  # consumer after the reload
            for j2 in range(j + 1, m):                                        # Eq. 8, 9 with K, L in micro-batch order
                w2 = Wv[(i, j2)]
                ge({Ov[(i, j2)]: 1.0, o: -1.0, w: -big, w2: -big}, to - 2 * big)
                ge({Rv[(i, j2)]: 1.0, r: -1.0, w: -big, w2: -big}, to - 2 * big)
            for j2 in range(m):
                if j2 == j:
                    continue
                h, w2 = Hv[(i, j, j2)], Wv[(i, j2)]
                ge({Rv[(i, j2)]: 1.0, o: -1.0, h: -big, w: -big, w2: -big}, to - 3 * big)   # Eq. 10
                ge({o: 1.0, Rv[(i, j2)]: -1.0, h: big, w: -big, w2: -big}, to - 2 * big)    # Eq. 11
            for v in ops:
                M_, N_ = Mv[(i, j, v)], Nv[(i, j, v)]
                le({M_: 1.0, w: -1.0}, 0.0)                                   # Eq. 15
                le({N_: 1.0, w: -1.0}, 0.0)
                st = {E[(i, v)]: 1.0}
                ge({**st, o: -1.0, M_: -big}, T[v[1]] + to - big)             # Eq. 12 (start of v)
                if strict_eq13:
                    ge({**st, r: -1.0, N_: -big}, T[v[1]] - big)              # Eq. 13
                ge({r: 1.0, E[(i, v)]: -1.0, N_: big, w: -big}, -big)         # Eq. 14
    if cutoff is not None:
        le({C: 1.0}, cutoff + 1e-6)

    A = lil_matrix((len(rows), len(names)))
    lb = np.empty(len(rows))
    ub = np.empty(len(rows))
    for r, (coef, a, b) in enumerate(rows):
        for k, x in coef.items():
            A[r, k] = x
        lb[r], ub[r] = a, b
    cost = np.zeros(len(names))
    cost[C] = 1.0
    for k in Nv.values():
        cost[k] = 1e-7
    res = milp(cost, constraints=LinearConstraint(A.tocsr(), lb, ub), integrality=np.array(integ),
               bounds=Bounds(np.array(lo, dtype=float), np.array(hi, dtype=float)),
               options={"time_limit": time_limit, "mip_rel_gap": 0.0})
    if res.x is None:
        return Solution(lists=[], makespan=float("inf"), status=res.message)
    x = res.x
    sol = Solution(lists=[], makespan=float(x[C]), status=res.message)
    for i in range(p):
        for u in ops:
            sol.start[(i, u[0], u[1])] = float(x[E[(i, u)]] - inst.t_op[i][u[1]])
        for j in range(m):
            sol.offloaded[(i, j)] = bool(i in off and x[Wv[(i, j)]] > 0.5)
    for i in range(p):
        st = {u: float(x[E[(i, u)]] - inst.t_op[i][u[1]]) for u in ops}
        items = {}
        for j in range(m):
            if sol.offloaded[(i, j)]:
                items[j] = (float(x[Ov[(i, j)]]), float(x[Rv[(i, j)]]),
                            [u for u in ops if x[Mv[(i, j, u)]] > 0.5], [u for u in ops if x[Nv[(i, j, u)]] > 0.5])
        sol.lists.append(_list_from_times(st, items, inst.item))
    sol.makespan = float(x[C])
    return sol


def _list_from_times(start, items, item):
    """Event list of one stage from the solver's values.  Compute ops by start time; O at its start time
    (hence after its forward op); OWAIT just before the first op credited with the memory (M = 1); R at its
    start time but never after an op charged with it (N = 1), never before its OWAIT.  Eq. 7 looks at memory
    only where a compute op starts, so the solver leaves the order of an OWAIT and an R that fall between the
    same two compute ops open; the executor charges by list position, so within such a gap every OWAIT goes
    before every R (both moved to the start of the op that ends the gap, which changes no op's charge)."""
    layer, kinds = item
    kinds = tuple(kinds)
    rank = {"OWAIT": 0, "R": 1, "F": 2, "B": 2, "W": 2, "O": 3}
    ev = [(t, rank[u[1]], OPS.index(u[1]), u[0], (u[1], u[0])) for u, t in start.items()]
    op_starts = sorted(round(t, 9) for t in start.values())

    def gap_end(t):
        k = bisect.bisect_left(op_starts, round(t, 9))
        return op_starts[k] if k < len(op_starts) else float("inf")

    for j, (o_t, r_t, cred, chg) in items.items():
        ev.append((o_t, rank["O"], 0, j, ("O", j, layer, kinds)))
        r_key = min([r_t] + [start[u] for u in chg])
        w_key = min([r_key] + [start[u] for u in cred])
        ev.append((gap_end(w_key), rank["OWAIT"], 0, j, ("OWAIT", j, layer, kinds)))
        ev.append((gap_end(r_key), rank["R"], 0, j, ("R", j, layer, kinds)))
    ev.sort(key=lambda e: (round(e[0], 9), e[1], e[2], e[3]))
    return [e[4] for e in ev]


# ----------------------------------------------------------------------------------------- AdaOffload

def est_start_first_backward(inst: Instance):
    """EstStart(B_{s,0}) of Alg. 1, step 1 (the algorithm only names it): the time the first micro-batch
    needs to run forward through every stage and backward down to stage s, with nothing else in its way."""
    p = inst.p
    t = 0.0
    for s in range(p):
        t += inst.t_op[s]["F"] + (inst.t_comm if s < p - 1 else 0.0)
    est = [0.0] * p
    for s in reversed(range(p)):
        est[s] = t
        t += inst.t_op[s]["B"] + inst.t_comm
    return est


def adaoffload(inst: Instance, tolerance: float = 0.0, lead: int = 1) -> Solution:
    """Alg. 1, in bytes: a forward activation costs Delta_F while on the device and Delta_F - Gamma once its
    offload has ended (Gamma < Delta_F when only some tensor kinds are offloaded); a stage without a limit
    holds everything.  Where Delta_B > 0 (a memory table in which B rebuilds tensors that F did not keep) a
    micro-batch between its B and its W costs Delta_F + Delta_B, and room for the next B's growth is kept free
    the way Gamma is kept free for the next reload.
      Step 1  EstStart(B_{s,0}) per stage (est_start_first_backward).
      Step 2  forward ops are placed back to back, each followed by its offload, until the next one would end
              after EstStart + tolerance or would not fit even with the offloads that have completed by then.
              That count is the stage's fill; when the same fill fits without offloading, nothing is offloaded.
      Step 3  PipeOffload-style rules for the rest, built by list scheduling over all stages: a backward op
              runs as soon as its inputs are there, else a forward op if it fits (Gamma is kept free for the
              reload of the next backward op), else a weight-gradient op; a weight-gradient op that ends before
              anything else could start goes first.  Reloads are listed `lead` compute ops ahead of their
              consumer, the credit of an offload (OWAIT) as late as possible: right before the op that needs
              the bytes.
    Returns the lists and this construction's own makespan estimate (it ignores the reloads' share of the
    transfer channel; time the lists with a simulator)."""
    p, m = inst.p, inst.m
    est = est_start_first_backward(inst)
    layer, kinds = inst.item
    kinds = tuple(kinds)
    dF = [inst.delta[s]["F"] for s in range(p)]
    dB = [max(0, inst.delta[s]["B"]) for s in range(p)]
    can_off = [s in inst.offload_stages and inst.gamma[s] > 0 and inst.limit[s] is not None for s in range(p)]

    def held(s, n_on_device, n_away, n_after_b):
        return n_on_device * dF[s] + n_away * (dF[s] - inst.gamma[s]) + n_after_b * dB[s]

    def fits(s, n_on_device, n_away, offloading, n_after_b=0):
        if inst.limit[s] is None:
            return True
        reserve = (inst.gamma[s] if offloading else 0) + dB[s]
        return held(s, n_on_device, n_away, n_after_b) + dF[s] + reserve <= inst.limit[s]

    def fill_of(s, offloading):
        T, to = inst.t_op[s], inst.t_off[s]
        t = sum(inst.t_op[k]["F"] + inst.t_comm for k in range(s))      # arrival of micro-batch 0
        n, chan, freed_at = 0, 0.0, []
        while n < m:
            if n >= 1 and t + T["F"] > est[s] + tolerance:
                break
            away = sum(1 for f in freed_at if f <= t) if offloading else 0
            if not fits(s, n - away, away, offloading):
                break
            t += T["F"]
            n += 1
            if offloading:
                chan = max(chan, t) + to
                freed_at.append(chan)
        return max(1, n)

    fill, offloading = [], []
    for s in range(p):
        plain = fill_of(s, False)
        dense = fill_of(s, True) if can_off[s] else plain
        offloading.append(dense > plain)
        fill.append(max(plain, dense))

    # ---- compute order of every stage by list scheduling (times are this construction's own estimate)
    end = {}
    t_free = [0.0] * p
    chan = [0.0] * p
    nf, nb, nw = [0] * p, [0] * p, [0] * p
    o_end = [dict() for _ in range(p)]
    order = [[] for _ in range(p)]

    def room_at(s, t):
        """Earliest time >= t at which one more forward activation fits on stage s (None: not before another
        op of the stage finishes): an offloaded activation shrinks when its offload ends, except the item of
        the next backward op, which is kept or already reloaded."""
        live = list(range(nw[s], nf[s]))
        after_b = nb[s] - nw[s]
        if not offloading[s]:
            return t if fits(s, len(live), 0, False, after_b) else None
        stay = sum(1 for j in live if j <= nb[s])
        away = sorted(o_end[s][j] for j in live if j > nb[s])
        for k in range(len(away) + 1):                                # k offloads have ended
            if fits(s, stay + len(away) - k, k, True, after_b):
                return t if k == 0 else max(t, away[k - 1])
        return None

    remaining = 3 * p * m
    while remaining:
        best = None
        for s in range(p):
            T = inst.t_op[s]
            cands = []
            jb, jf = nb[s], nf[s]
            if jb < m and jb < nf[s]:
                dep = end.get((s + 1, jb, "B")) if s < p - 1 else end.get((s, jb, "F"))
                if dep is not None:
                    ready = dep + (inst.t_comm if s < p - 1 else 0.0)
                    if offloading[s] and jb in o_end[s]:
                        ready = max(ready, o_end[s][jb] + inst.t_off[s])      # offload ended, reload done
                    # B's own growth must fit; if it does not, a pending weight-gradient op releases memory first
                    n_live = nf[s] - nw[s]
                    grows = dB[s] and inst.limit[s] is not None
                    if not grows or nw[s] == nb[s] or held(s, n_live, 0, nb[s] - nw[s]) + dB[s] <= inst.limit[s]:
                        cands.append((max(t_free[s], ready), 0, "B", jb))
            if jf < m:
                dep = end.get((s - 1, jf, "F")) if s > 0 else 0.0
                if dep is not None:
                    ready = max(t_free[s], dep + (inst.t_comm if s > 0 else 0.0))
                    # before the first backward op only `fill` forward ops; afterwards memory alone decides
                    when = room_at(s, ready)
                    if (nb[s] > 0 or nf[s] < fill[s]) and when is not None:
                        cands.append((when, 1, "F", jf))
            if nw[s] < nb[s]:
                cands.append((max(t_free[s], end[(s, nw[s], "B")]), 2, "W", nw[s]))
            if not cands:
                continue
            # the op that can start first; among those that start together backward > forward > weight gradient.
            # A weight-gradient op that ends before the earliest other candidate starts goes first.
            cands.sort()
            pick = cands[0]
            for c in cands:
                if c[2] == "W" and c[0] + T["W"] <= pick[0] + 1e-12:
                    pick = c
                    break
            if best is None or (pick[0], s) < (best[1][0], best[0]):
                best = (s, pick)
        if best is None:
            raise RuntimeError("AdaOffload construction stalled: the limit holds no forward activation")
        s, (st, _, c, j) = best
        en = st + inst.t_op[s][c]
        end[(s, j, c)] = en
        t_free[s] = en
        order[s].append((c, j))
        if c == "F":
            nf[s] += 1
            if offloading[s]:
                chan[s] = max(chan[s], en) + inst.t_off[s]
                o_end[s][j] = chan[s]
        elif c == "B":
            nb[s] += 1
        else:
            nw[s] += 1
        remaining -= 1

    lists = [_with_transfers(order[s], offloading[s], inst.limit[s], dF[s], inst.gamma[s], lead, layer, kinds, dB[s])
             for s in range(p)]
    return Solution(lists=lists, makespan=max(end[(s, m - 1, "W")] for s in range(p)),
                    start={k: v - inst.t_op[k[0]][k[2]] for k, v in end.items()},
                    offloaded={(s, j): bool(offloading[s]) for s in range(p) for j in range(m)}, status="adaoffload")


def _with_transfers(order, offloading, limit, d_f, gamma, lead, layer, kinds, d_b=0):
    """Inserts O / OWAIT / R into one stage's compute order: O right after every forward op; R `lead` compute ops
    ahead of its backward op (never before its own forward op); OWAIT as late as possible, i.e. right before the
    forward op or reload that would not fit otherwise (oldest offload first), or right before its own reload."""
    if not offloading:
        return list(order)
    pos = {op: n for n, op in enumerate(order)}
    r_before = {}                               # compute index -> micro-batches whose reload goes before it
    for (c, j), n in pos.items():
        if c == "B":
            r_before.setdefault(max(n - lead, pos[("F", j)] + 1), []).append(j)
    out, used, pending, credited = [], 0, [], set()

    def make_room(need):
        nonlocal used
        while used + need > limit and pending:
            jj = pending.pop(0)
            out.append(("OWAIT", jj, layer, kinds))
            credited.add(jj)
            used -= gamma

    for n, (c, j) in enumerate(order):
        for jj in sorted(r_before.get(n, [])):
            if jj not in credited:
                pending.remove(jj)
                out.append(("OWAIT", jj, layer, kinds))
                credited.add(jj)
                used -= gamma
            make_room(gamma)
            out.append(("R", jj, layer, kinds))
            used += gamma
        if c == "F":
            make_room(d_f)
            used += d_f
        elif c == "B" and d_b:
            make_room(d_b)
            used += d_b
        elif c == "W":
            used -= d_f + d_b
        out.append((c, j))
        if c == "F":
            out.append(("O", j, layer, kinds))
            pending.append(j)
    return out


def expand_items(events, n_layers, kinds):
    """Whole-activation offload of the paper (one item per forward op) written out for the executor's finer
    granularity: the item's O / OWAIT / R become one event per layer over the given kinds, in layer order."""
    out = []
    for e in events:
        if e[0] in ("O", "OWAIT", "R"):
            out.extend((e[0], e[1], l, tuple(kinds)) for l in range(n_layers))
        else:
            out.append(e)
    return out


# ------------------------------------------------------------------- timing of given lists (Eq. 3-6, 8-14)

@dataclass
class Timeline:
    start: list                  # per stage, aligned with the list (None for OWAIT)
    end: list
    makespan: float              # Eq. 17: last end - first start over all stages' compute ops
    busy: list                   # per stage: summed compute time
    bubble: list                 # per stage: 1 - busy / makespan
    stall: list                  # per stage: time compute ops spent waiting for an offload (Eq. 12) or a reload


def pipeline_timeline(lists, t_op, t_comm=0.0, t_copy=None, duplex=False) -> Timeline:
    """Earliest start times of every event of p per-stage lists (one model chunk per stage), as the executor and
    the paper's constraints order them: compute ops of a stage one after the other in list order (Eq. 5), F of
    stage i after F of stage i - 1 plus T_comm (Eq. 3), B after B of stage i + 1 plus T_comm (Eq. 4), transfers of
    a stage one at a time in list order (Eq. 8-11; per direction when `duplex`), an offload after its F, a compute
    op listed after OWAIT(x) after offload x ended (Eq. 12), a reload after the compute ops listed before it
    (Eq. 14) and after its item's offload, B j after every reload of micro-batch j.
    t_op[i] = {"F", "B", "W"} durations; t_copy(i, event) = duration of that O or R event.
    Built as a longest-path pass over the precedence graph (a cycle = lists that deadlock each other)."""
    p = len(lists)
    t_copy = t_copy or (lambda i, ev: 0.0)
    node = {}                                   # (stage, index) -> id
    dur, preds = [], []

    def add(i, n, d):
        node[(i, n)] = len(dur)
        dur.append(d)
        preds.append([])
        return len(dur) - 1

    where_f = [dict() for _ in range(p)]        # j -> node of F j on stage i
    where_b = [dict() for _ in range(p)]
    for i, ev in enumerate(lists):
        for n, e in enumerate(ev):
            if e[0] in OPS:
                v = add(i, n, t_op[i][e[0]])
                if e[0] == "F":
                    where_f[i][e[1]] = v
                elif e[0] == "B":
                    where_b[i][e[1]] = v
            elif e[0] in ("O", "R"):
                add(i, n, t_copy(i, e))
    lag = {}                                    # (pred, succ) -> extra delay on that edge
    for i, ev in enumerate(lists):
        last_compute = None
        last_copy = [None, None]                # last transfer per channel (offload, reload)
        gate = []                               # offloads whose OWAIT has been passed
        off_node, rel_nodes = {}, {}
        for n, e in enumerate(ev):
            if e[0] in OPS:
                v = node[(i, n)]
                if last_compute is not None:
                    preds[v].append(last_compute)
                preds[v].extend(gate)
                j = e[1]
                if e[0] == "F" and i > 0:
                    u = where_f[i - 1].get(j)
                    if u is None:
                        raise ValueError(f"stage {i - 1} never runs F {j}")
                    preds[v].append(u)
                    lag[(u, v)] = t_comm
                if e[0] == "B":
                    if i < p - 1:
                        u = where_b[i + 1].get(j)
                        if u is None:
                            raise ValueError(f"stage {i + 1} never runs B {j}")
                        preds[v].append(u)
                        lag[(u, v)] = t_comm
                    preds[v].extend(rel_nodes.get(j, []))
                last_compute = v
            elif e[0] == "O":
                v = node[(i, n)]
                preds[v].append(where_f[i][e[1]])
                if last_copy[0] is not None:
                    preds[v].append(last_copy[0])
                last_copy[0] = v
                for k in e[3]:
                    off_node[(e[1], e[2], k)] = v
            elif e[0] == "OWAIT":
                gate = gate + [off_node[(e[1], e[2], k)] for k in e[3]]
            elif e[0] == "R":
                v = node[(i, n)]
                ch = 1 if duplex else 0
                if last_copy[ch] is not None:
                    preds[v].append(last_copy[ch])
                if last_compute is not None:
                    preds[v].append(last_compute)
                preds[v].extend(off_node[(e[1], e[2], k)] for k in e[3])
                last_copy[ch] = v
                rel_nodes.setdefault(e[1], []).append(v)
    n_nodes = len(dur)
    succs = [[] for _ in range(n_nodes)]
    indeg = [0] * n_nodes
    for v in range(n_nodes):
        preds[v] = list(dict.fromkeys(preds[v]))
        indeg[v] = len(preds[v])
        for u in preds[v]:
            succs[u].append(v)
    t_start = [0.0] * n_nodes
    ready = [v for v in range(n_nodes) if indeg[v] == 0]
    seen = 0
    while ready:
        u = ready.pop()
        seen += 1
        end_u = t_start[u] + dur[u]
        for v in succs[u]:
            t = end_u + lag.get((u, v), 0.0)
            if t > t_start[v]:
                t_start[v] = t
            indeg[v] -= 1
            if indeg[v] == 0:
                ready.append(v)
    if seen != n_nodes:
        raise ValueError("the lists deadlock each other")
    start = [[None] * len(ev) for ev in lists]
    end = [[None] * len(ev) for ev in lists]
    first, last = float("inf"), 0.0
    busy, stall = [0.0] * p, [0.0] * p
    is_compute = [False] * n_nodes
    for i, ev in enumerate(lists):
        for n, e in enumerate(ev):
            if e[0] in OPS:
                is_compute[node[(i, n)]] = True
    for i, ev in enumerate(lists):
        for n, e in enumerate(ev):
            if e[0] == "OWAIT":
                continue
            v = node[(i, n)]
            start[i][n], end[i][n] = t_start[v], t_start[v] + dur[v]
            if e[0] in OPS:
                first, last = min(first, start[i][n]), max(last, end[i][n])
                busy[i] += dur[v]
                # waiting that only a transfer explains: the op could have started once its compute predecessors
                # (the op before it on this stage, the neighbour's op) were done
                free = max([t_start[u] + dur[u] + lag.get((u, v), 0.0) for u in preds[v] if is_compute[u]] + [0.0])
                stall[i] += max(0.0, t_start[v] - free)
    makespan = last - first if last > first else 0.0
    return Timeline(start=start, end=end, makespan=makespan, busy=busy,
                    bubble=[1.0 - b / makespan if makespan > 0 else 0.0 for b in busy], stall=stall)


# --------------------------------------------------- lists under a byte budget with per-item offload (Sec. 3, Eq. 7)

def fit_offloads(comp, n_layers, kinds, kind_bytes, fits, lead=1):
    """Adds to a compute order the fewest offloads that make it fit: the decision variable of Sec. 3 is per
    item, and Eq. 7 only asks that the bytes in use stay within the limit.

    `fits(events) -> (ok, index of the first failing event)` is the consumer's planner (ordering rules and
    list-order accounting against the budget); no accounting happens here.  While the list fails at an
    allocating event, one more item (micro-batch, layer, kind) that is on the device at that point and not
    needed there is offloaded: the micro-batch whose B is furthest away first, within it the layer B reaches
    last, the smallest kind first.  Its O follows its F directly (the copy has the longest time to run under
    compute), its OWAIT sits right before the event that needed the bytes (the credit as late as possible), its R
    `lead` compute ops ahead of its B.  A reload that itself does not fit where it is listed first makes other
    items leave, then moves down to right before its B.  Returns None when nothing more can leave."""
    comp = [e for e in comp if e[0] in OPS]
    pos_f = {e[1]: n for n, e in enumerate(comp) if e[0] == "F"}
    pos_b = {e[1]: n for n, e in enumerate(comp) if e[0] == "B"}
    kinds = sorted(kinds, key=lambda k: (kind_bytes[k], k))
    chosen = {}                                  # (j, layer, kind) -> [owait slot, reload slot]

    def assemble():
        slots = {}
        for (j, l, k), (w, r) in chosen.items():
            slots.setdefault(("O", pos_f[j] + 1, j, l), []).append(k)
            slots.setdefault(("OWAIT", w, j, l), []).append(k)
            slots.setdefault(("R", r, j, l), []).append(k)
        before = {}
        for (op, at, j, l), ks in slots.items():
            before.setdefault(at, []).append((op, j, l, tuple(ks)))
        out, owner = [], []                      # owner[n] = compute slot of event n
        for n in range(len(comp) + 1):
            # at one slot: credits of earlier offloads, then the offloads that start here, then the credits of
            # those (an offload nothing overlaps), then reloads (the layer B reaches first is reloaded first)
            def rank(e):
                if e[0] == "O":
                    return 1
                if e[0] == "R":
                    return 3
                return 2 if pos_f[e[1]] + 1 == n else 0
            for e in sorted(before.get(n, []), key=lambda e: (rank(e), e[1], -e[2] if e[0] == "R" else e[2])):
                out.append(e)
                owner.append(n)
            if n < len(comp):
                out.append(comp[n])
                owner.append(n)
        return out, owner

    for _ in range(3 * len(pos_f) * n_layers * max(1, len(kinds)) + 8):
        ev, owner = assemble()
        ok, bad = fits(ev)
        if ok:
            return ev
        if bad >= len(ev):
            return None
        n = owner[bad]
        failing = ev[bad]
        cands = [(j, l, k) for j in pos_f for l in range(n_layers) for k in kinds
                 if (j, l, k) not in chosen and pos_f[j] < n and max(n, pos_b[j] - lead) > n
                 and not (failing[0] in OPS and failing[1] == j)]
        if failing[0] == "R":
            cands = [c for c in cands if c[0] != failing[1]]
        if cands:
            j, l, k = min(cands, key=lambda c: (-pos_b[c[0]], c[1], kind_bytes[c[2]], c[2]))
            chosen[(j, l, k)] = [n, max(n, pos_b[j] - lead)]
            continue
        if failing[0] == "R":
            moved = False
            for k in failing[3]:
                key = (failing[1], failing[2], k)
                if chosen[key][1] < pos_b[failing[1]]:
                    chosen[key][1] = pos_b[failing[1]]
                    moved = True
            if moved:
                continue
        return None
    return None


def budgeted_lists(p, m, n_layers, kinds, kind_bytes, fits, base_lists, t_op, t_copy_of_event, duplex=False,
                   t_comm=0.0, max_extra=None, leads=(1, 2)):
    """Per-stage lists for a pipeline in which every device has the same byte budget, chosen by modelled makespan.

    base_lists(cap_of_stage) -> p compute orders (split B/W) in which stage i holds at most cap_of_stage(i)
    micro-batches between F and W; `fits` as in fit_offloads (all stages have the same shape).  For every fill
    level e = 0 .. max_extra the caps are p - i + e (a denser fill than p - i in flight shortens the bubble and
    costs memory); a stage whose list cannot be made to fit even with offloads gets its cap lowered until it can.
    Every candidate is timed with pipeline_timeline from the given op times and t_copy_of_event(event) -> ms; the
    fastest is returned as (lists, info).  A stage that has to offload gets, of the reload leads in `leads`, the one
    whose list the timeline of that stage alone finishes first (how far ahead of its B a reload is listed decides
    whether it runs under compute or holds B up, and how early the offload before it must be credited).  Fill levels
    tried: 0 to 3, then every fourth, and the densest."""
    max_extra = p - 1 if max_extra is None else max_extra
    size = lambda e: sum(kind_bytes[k] for k in e[3])
    memo = {}
    best = None
    tried = []
    seen = set()
    for extra in sorted({e for e in range(max_extra + 1) if e < 4 or e % 4 == 0 or e == max_extra}):
        caps = [min(m, p - i + extra) for i in range(p)]
        lists = None
        while True:
            comp = base_lists(lambda i, c=tuple(caps): c[i])
            out, lowered = [], False
            for i in range(p):
                ev = comp[i]
                if not fits(ev)[0]:
                    key = (tuple(sorted(t_op[i].items())), tuple(comp[i]))
                    if key not in memo:                  # many fill levels give a stage the same compute order
                        pick, t_pick = None, None
                        for ld in leads:
                            cand = fit_offloads(comp[i], n_layers, kinds, kind_bytes, fits, lead=ld)
                            if cand is None:
                                continue
                            t = pipeline_timeline([cand], [t_op[i]], t_copy=lambda s_, e: t_copy_of_event(e),
                                                  duplex=duplex).makespan
                            if t_pick is None or t < t_pick * (1 - 1e-9):
                                pick, t_pick = cand, t
                        memo[key] = pick
                    ev = memo[key]
                if ev is None:
                    if caps[i] == 1:
                        raise RuntimeError("one micro-batch does not fit the budget")
                    caps[i] -= 1
                    lowered = True
                    break
                out.append(ev)
            if not lowered:
                lists = out
                break
        key = tuple(caps)
        if key in seen:
            continue
        seen.add(key)
        tl = pipeline_timeline(lists, t_op, t_comm=t_comm, t_copy=lambda i, e: t_copy_of_event(e), duplex=duplex)
        info = {"extra_fill": extra, "caps": list(caps), "makespan_model": tl.makespan, "bubble_model": list(tl.bubble),
                "stall_model": list(tl.stall),
                "offloaded_bytes": [sum(size(e) for e in ev if e[0] == "O") for ev in lists]}
        tried.append({k: info[k] for k in ("extra_fill", "caps", "makespan_model")})
        if best is None or tl.makespan < best[1]["makespan_model"] * (1 - 1e-9):
            best = (lists, info)
    best[1]["candidates"] = tried
    return best


def nominal_op_times(cfg, tflops=1100.0):
    """T_F, T_B, T_W in ms of one micro-batch on one stage from the algorithmic flop counts (2 tokens N K per GEMM in
    each of F, B, W; causal attention 2 s^2 n_q d forward, 5 s^2 n_q d backward) at a nominal rate: the stand-in for
    measured op times where none exist yet."""
    s, h, f = cfg.seq * cfg.micro_batch, cfg.hidden, cfg.ffn
    gemm = 2 * s * (cfg.qkv_width * h + h * cfg.n_q_heads * cfg.head_dim + cfg.up_width * h + h * f)
    att = cfg.micro_batch * cfg.seq * cfg.seq * cfg.n_q_heads * cfg.head_dim
    ms = lambda fl: cfg.n_layers * fl / (tflops * 1e9)
    return {"F": ms(gemm + 2 * att), "B": ms(gemm + 5 * att), "W": ms(gemm)}


def workload_lists(cfg, budget, t_op=None, link_gbps=55.0, copy_latency_ms=0.02, duplex=False, m=None, max_extra=None,
                   recompute=0, reload_gbps=None):
    """The lists of all p stages for a benchmark workload with a split B/W schedule under `budget` bytes of
    activations per device (0 = no budget: the plain split B/W lists with p - i micro-batches in flight), every stage
    shaped like cfg.  The library's planner decides what fits; offloads are chosen item by item (fit_offloads), the
    fill level by modelled makespan (budgeted_lists) from t_op (default: nominal_op_times) and the host-link rate
    (reload_gbps: the rate of reloads where it differs from that of offloads, as it does when both run at once).
    m overrides the micro-batch count (tests run fewer).  -> (lists, info)"""
    from stage_inputs import schedules as G
    from . import binding as B
    p = cfg.n_stages
    m = cfg.n_microbatches if m is None else m
    if not budget:
        return G.split_bw_greedy(p, m), {"extra_fill": 0, "caps": [min(m, p - i) for i in range(p)], "offloaded_bytes": [0] * p}
    import dataclasses
    c = dataclasses.replace(cfg, n_microbatches=m)
    kb = B.query_sizes(c, recompute=recompute)[2]
    t_op = t_op or nominal_op_times(cfg)

    def fits(ev):
        st, bad, _, _ = B.plan(c, ev, budget=budget, recompute=recompute)
        return st == B.OK, bad

    rate = {"O": link_gbps, "R": reload_gbps or link_gbps}
    return budgeted_lists(p, m, cfg.n_layers, tuple(cfg.offload_kinds), kb, fits,
                          lambda cap: G.split_bw_greedy(p, m, cap_of_stage=cap), [dict(t_op)] * p,
                          lambda e: sum(kb[k] for k in e[3]) / (rate[e[0]] * 1e6) + copy_latency_ms, duplex=duplex,
                          max_extra=max_extra)


# ------------------------------------------------------------------------------- online scheduling (Sec. 4.3)

class OnlineSearch:
    """The solver working beside training: a host thread that starts from AdaOffload's lists and keeps asking
    the MILP for something strictly better, publishing every improvement; the training loop reads `best()` between
    iterations and hands the new lists to the stage (which takes a different list every iteration).

    The paper's solver reports incumbents through a callback.  scipy's interface has none, so the same stream of
    improving schedules is produced by a sequence of solves, each bounded by `slice_seconds` and by C <= (best so
    far) - min_gain: a solve either returns a better schedule (published), proves there is none (search complete),
    or runs out of time (the next solve gets a longer slice).  `strict_eq13` and the instance's `own_peak` are
    passed through, so that what is published fits the executor's accounting.

    judge(solution) -> float may re-time a candidate (e.g. with a simulator fed with measured op times); by default
    the solver's own makespan is used.  Improvements are compared in the judge's units."""

    def __init__(self, inst: Instance, tolerance: float = 0.0, slice_seconds: float = 5.0, max_seconds: float = 120.0,
                 min_gain: float = 1e-6, strict_eq13: bool = False, judge=None):
        import threading
        self.inst, self.tolerance = inst, tolerance
        self.slice_seconds, self.max_seconds, self.min_gain = slice_seconds, max_seconds, min_gain
        self.strict_eq13, self.judge = strict_eq13, judge
        self._lock = threading.Lock()
        self._stop = threading.Event()
        self._best = None                     # (score, Solution)
        self.history = []                     # (seconds since start, score, status) of every publication
        self.complete = False                 # True once a solve proved that nothing better exists (with best()
                                              # still None: that no schedule exists under the limits)
        self.error = None                     # exception that ended the search thread, if any
        self._thread = threading.Thread(target=self._run, name="optstage-online-search", daemon=True)

    def start(self):
        self._thread.start()
        return self

    def stop(self, wait: bool = True):
        self._stop.set()
        if wait and self._thread.is_alive():
            self._thread.join()

    def join(self, timeout=None):
        self._thread.join(timeout)

    def best(self):
        """(score, Solution) of the best schedule published so far, or None before the first."""
        with self._lock:
            return self._best

    def _publish(self, sol: Solution, t0: float):
        import time
        score = float(self.judge(sol)) if self.judge else float(sol.makespan)
        with self._lock:
            if self._best is None or score < self._best[0] - self.min_gain:
                self._best = (score, sol)
                self.history.append((time.monotonic() - t0, score, sol.status))
                return True
        return False

    def _run(self):
        try:
            self._search()
        except Exception as e:                         # the thread must not die silently: the loop reads `error`
            self.error = e

    def _search(self):
        import time
        t0 = time.monotonic()
        inst = self.inst
        bound, bound_proven = None, False             # C <= bound for the next solve; proven = it is a solver's own makespan
        try:
            sol = adaoffload(inst, tolerance=self.tolerance)
            # the construction's own makespan ignores the reloads' share of the channel: time its lists under the
            # model the solver uses before publishing them or bounding a solve by them
            sol.makespan = pipeline_timeline(sol.lists, inst.t_op, inst.t_comm, lambda i, e: inst.t_off[i]).makespan
            self._publish(sol, t0)
            bound = sol.makespan - self.min_gain
        except RuntimeError:                           # the heuristic found no list (limit too tight for it):
            pass                                       # the solver starts without a bound
        slice_s = self.slice_seconds
        while not self._stop.is_set() and time.monotonic() - t0 < self.max_seconds:
            sol = milp_schedule(inst, time_limit=slice_s, cutoff=bound, strict_eq13=self.strict_eq13)
            if sol.lists:
                self._publish(sol, t0)
                # the next solve must beat this one in the solver's own units, whatever the judge made of it:
                # otherwise a candidate the judge rejects would come back from every solve
                bound, bound_proven = sol.makespan - self.min_gain, True
                if "ptimal" in sol.status:            # proven optimal under the bound: nothing better exists
                    self.complete = True
                    return
            elif "nfeasible" in sol.status:
                if bound is not None and not bound_proven:
                    bound = None                       # a heuristic list's timing is no proof: ask again without it
                    continue
                self.complete = True                   # no schedule beats the incumbent (or none exists at all)
                return
            else:                                      # out of time without an incumbent: look longer
                slice_s *= 2
