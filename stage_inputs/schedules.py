"""Deterministic per-stage schedule generators (inputs of the build, not part of the
method: the paper obtains its schedules from a MILP solver, here they are given).

They only arrange events; whether a list fits a memory budget is decided by
whoever consumes it (the library's validator, or the oracle's accounting), so
the offload generator exposes its policy knobs and the caller searches them.

Event tuples: ("F", j) ("B", j) ("W", j) ("O", j, layer, kinds) ("OWAIT", j, layer, kinds)
("R", j, layer, kinds).
"""
from __future__ import annotations


def one_f_one_b(p: int, m: int, i: int) -> list:
    """Plain 1F1B for stage i of p: min(p-i-1, m) warm-up forwards, then alternate one
    forward / one backward; the weight pass W j runs right after B j (fused backward)."""
    warm = min(p - i - 1, m)
    ev = [("F", j) for j in range(warm)]
    f, b = warm, 0
    while b < m:
        if f < m:
            ev.append(("F", f))
            f += 1
        ev += [("B", b), ("W", b)]
        b += 1
    return ev


def split_bw_greedy(p: int, m: int, cap_of_stage=None) -> list:
    """Zero-bubble style lists for all p stages: a unit-time lock-step sweep where each
    stage, whenever idle, runs the first ready op by priority B > F > W; F j is held
    back while `cap_of_stage(i)` micro-batches are in flight (F done, W not done).
    W is therefore pushed into slots where neither B nor F is ready."""
    cap_of_stage = cap_of_stage or (lambda i: p - i)
    lists = [[] for _ in range(p)]
    nf, nb, nw = [0] * p, [0] * p, [0] * p
    done_f = [dict() for _ in range(p)]     # j -> finish tick
    done_b = [dict() for _ in range(p)]
    t = 0
    while any(nw[i] < m for i in range(p)):
        chosen = []
        for i in range(p):
            pick = None
            j = nb[i]
            if j < m and j < nf[i] and done_f[i].get(j, t + 1) <= t and \
                    (i == p - 1 or done_b[i + 1].get(j, t + 1) <= t):
                pick = ("B", j)
            if pick is None:
                j = nf[i]
                if j < m and (nf[i] - nw[i]) < cap_of_stage(i) and \
                        (i == 0 or done_f[i - 1].get(j, t + 1) <= t):
                    pick = ("F", j)
            if pick is None:
                j = nw[i]
                if j < m and j < nb[i] and done_b[i].get(j, t + 1) <= t:
                    pick = ("W", j)
            chosen.append(pick)
        for i, pick in enumerate(chosen):
            if pick is None:
                continue
            lists[i].append(pick)
            op, j = pick
            if op == "F":
                nf[i] += 1
                done_f[i][j] = t + 1
            elif op == "B":
                nb[i] += 1
                done_b[i][j] = t + 1
            else:
                nw[i] += 1
        t += 1
        if t > 10 * (3 * m + 2 * p) + 100:
            raise RuntimeError("generator did not terminate")
    return lists


def add_offload(compute_list: list, n_layers: int, kinds: tuple, min_gap: int = 2, lead: int = 1) -> list:
    """Insert O / OWAIT / R events into a compute order.

    A micro-batch j is offloaded when at least `min_gap` compute ops lie between F j and
    B j.  Its O events (one per layer, all `kinds`) follow F j directly; the matching
    OWAITs sit just before the next compute op that follows F j's successor (so the
    copy overlaps one compute op); the R events sit `lead` compute ops ahead of B j so
    the reload overlaps them."""
    comp = [e for e in compute_list]
    pos_f = {e[1]: n for n, e in enumerate(comp) if e[0] == "F"}
    pos_b = {e[1]: n for n, e in enumerate(comp) if e[0] == "B"}
    before = {n: [] for n in range(len(comp) + 1)}      # events to emit before compute op n
    for j in sorted(pos_f):
        gap = pos_b[j] - pos_f[j] - 1
        if gap < max(1, min_gap):
            continue
        o_at = pos_f[j] + 1
        wait_at = min(pos_f[j] + 2, pos_b[j])
        r_at = max(wait_at, pos_b[j] - lead)
        for l in range(n_layers):
            before[o_at].append((0, ("O", j, l, tuple(kinds))))
        for l in range(n_layers):
            before[wait_at].append((1, ("OWAIT", j, l, tuple(kinds))))
        for l in reversed(range(n_layers)):             # B consumes the last layer first
            before[r_at].append((2, ("R", j, l, tuple(kinds))))
    out = []
    for n in range(len(comp) + 1):
        # at one position: waits first (free memory), then reloads, then new offloads
        for _, ev in sorted(before[n], key=lambda x: {1: 0, 2: 1, 0: 2}[x[0]]):
            out.append(ev)
        if n < len(comp):
            out.append(comp[n])
    return out
