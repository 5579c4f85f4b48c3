"""Deterministic per-stage schedule generators (inputs of the build, not part of the
method: the paper obtains its schedules from a MILP solver, here they are given).

They only arrange events; whether a list fits a memory budget is decided by
whoever consumes it (the library's validator, or the oracle's accounting), so
the offload generator exposes its policy knobs and the caller searches them.

Event tuples: ("F", j) ("B", j) ("W", j) ("O", j, layer, kinds) ("OWAIT", j, layer, kinds)
("R", j, layer, kinds); compute events of model chunk c on a stage that holds several: (op, j, c).
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


def interleaved_one_f_one_b(p: int, m: int, i: int, n_chunks: int) -> list:
    """1F1B with n_chunks model chunks per stage (chunk c of stage i is piece c p + i of the model), for stage
    i of p; m must be a multiple of p.  Forward chunk-ops come in rounds of p micro-batches per chunk; the k-th
    forward op is chunk (k mod p n_chunks) div p of micro-batch (k div p n_chunks) p + k mod p, the k-th
    backward op the same with the chunks in reverse.  Warm-up: 2 (p - i - 1) + (n_chunks - 1) p forward ops,
    then one forward / one backward, then the remaining backward ops; W runs right after its B.
    Compute events of chunk c are written (op, j, c)."""
    if m % p:
        raise ValueError("interleaved 1F1B needs the micro-batch count to be a multiple of the stage count")
    total = m * n_chunks

    def fwd(k):
        return ("F", (k // (p * n_chunks)) * p + k % p, (k % (p * n_chunks)) // p)

    def bwd(k):
        return ((k // (p * n_chunks)) * p + k % p, n_chunks - 1 - (k % (p * n_chunks)) // p)

    warm = min(2 * (p - i - 1) + (n_chunks - 1) * p, total)
    ev = [fwd(k) for k in range(warm)]
    f, b = warm, 0
    while b < total:
        if f < total:
            ev.append(fwd(f))
            f += 1
        j, c = bwd(b)
        ev += [("B", j, c), ("W", j, c)]
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


def _piece(i: int, c: int, p: int, placement: str) -> int:
    """Position in the model of chunk c of stage i: "interleaved" chunk c covers pieces c p .. c p + p - 1 in stage
    order; "v" runs odd chunks through the stages in reverse (stage 0 holds the first and the last piece)."""
    return c * p + (i if (placement == "interleaved" or c % 2 == 0) else p - 1 - i)


def split_bw_greedy_chunks(p: int, m: int, n_chunks: int, placement: str = "v", cap_of_stage=None) -> list:
    """Zero-bubble style lists for stages that hold n_chunks model chunks each (V-shaped or interleaved placement):
    the unit-time lock-step sweep of split_bw_greedy over the p n_chunks pieces of the model.  An idle stage runs,
    in this order of preference: a ready B (the piece nearest the loss first), a ready F (the deepest piece first,
    so that micro-batches already under way finish before new ones start), where a new micro-batch is admitted
    only while the chunk activations of the admitted ones (held, F done and W not done, or still to come) stay within
    `cap_of_stage(i)` (default 2 p, every stage alike: what the V shape is for; at least n_chunks),
    a ready W (oldest first).  Compute events are written (op, j, chunk)."""
    cap_of_stage = cap_of_stage or (lambda i: 2 * p)
    n_pieces = p * n_chunks
    holder = {}
    for i in range(p):
        for c in range(n_chunks):
            holder[_piece(i, c, p, placement)] = (i, c)
    lists = [[] for _ in range(p)]
    nf = {k: 0 for k in holder.values()}
    nb = dict(nf)
    nw = dict(nf)
    done_f, done_b = {}, {}                     # (piece, j) -> finish tick
    t = 0
    total = 3 * m * n_pieces
    placed = 0
    while placed < total:
        chosen = []
        for i in range(p):
            chunks = sorted(range(n_chunks), key=lambda c: -_piece(i, c, p, placement))    # deepest piece first
            pick = None
            for c in chunks:                                                             # B
                v, j = _piece(i, c, p, placement), nb[(i, c)]
                if j < m and j < nf[(i, c)] and done_f.get((v, j), t + 1) <= t and \
                        (v == n_pieces - 1 or done_b.get((v + 1, j), t + 1) <= t):
                    pick = ("B", j, c)
                    break
            if pick is None:                                                             # F
                first = chunks[-1]                      # the chunk a micro-batch visits first on this stage
                # a micro-batch admitted on its first chunk will need room for all its chunks here: the cap
                # counts those to come as well, or the later chunks could find the stage full for good
                committed = n_chunks * nf[(i, first)] - sum(nw[(i, c)] for c in range(n_chunks))
                for c in chunks:
                    v, j = _piece(i, c, p, placement), nf[(i, c)]
                    if c == first and committed + n_chunks > cap_of_stage(i):
                        continue
                    if j < m and (v == 0 or done_f.get((v - 1, j), t + 1) <= t):
                        pick = ("F", j, c)
                        break
            if pick is None:                                                             # W
                cands = [(done_b[(_piece(i, c, p, placement), nw[(i, c)])], c) for c in range(n_chunks)
                         if nw[(i, c)] < nb[(i, c)] and done_b[(_piece(i, c, p, placement), nw[(i, c)])] <= t]
                if cands:
                    c = min(cands)[1]
                    pick = ("W", nw[(i, c)], c)
            chosen.append(pick)
        for i, pick in enumerate(chosen):
            if pick is None:
                continue
            lists[i].append(pick)
            op, j, c = pick
            v = _piece(i, c, p, placement)
            if op == "F":
                nf[(i, c)] += 1
                done_f[(v, j)] = t + 1
            elif op == "B":
                nb[(i, c)] += 1
                done_b[(v, j)] = t + 1
            else:
                nw[(i, c)] += 1
            placed += 1
        t += 1
        if t > 10 * (3 * m * n_chunks + 2 * n_pieces) + 100:
            raise RuntimeError("generator did not terminate (in-flight cap too small for this shape?)")
    return lists


def add_offload(compute_list: list, n_layers: int, kinds: tuple, min_gap: int = 2, lead: int = 1,
                wait_delay: int = 1) -> list:
    """Insert O / OWAIT / R events into a compute order.

    A micro-batch j is offloaded when at least `min_gap` compute ops lie between F j and
    B j.  Its O events (one per layer, all `kinds`) follow F j directly; the matching
    OWAITs sit `wait_delay` compute ops later (the copy overlaps that many ops; 0 = the
    next op waits for the copy); the R events sit `lead` compute ops ahead of B j so the
    reload overlaps them (0 = B j waits for the whole reload)."""
    comp = [e for e in compute_list]
    chunk = lambda e: e[2] if len(e) > 2 else 0
    n_chunks = 1 + max(chunk(e) for e in comp)
    per_chunk = n_layers // n_chunks                    # n_layers counts the layers of all chunks of the stage
    pos_f = {(chunk(e), e[1]): n for n, e in enumerate(comp) if e[0] == "F"}
    pos_b = {(chunk(e), e[1]): n for n, e in enumerate(comp) if e[0] == "B"}
    before = {n: [] for n in range(len(comp) + 1)}      # events to emit before compute op n
    for key in sorted(pos_f, key=lambda k: pos_f[k]):
        c, j = key
        gap = pos_b[key] - pos_f[key] - 1
        if gap < max(1, min_gap):
            continue
        o_at = pos_f[key] + 1
        wait_at = min(pos_f[key] + 1 + wait_delay, pos_b[key])
        r_at = max(wait_at, pos_b[key] - lead)
        layers = range(c * per_chunk, (c + 1) * per_chunk)
        for l in layers:
            before[o_at].append((1, ("O", j, l, tuple(kinds))))
        for l in layers:
            before[wait_at].append((2 if wait_at == o_at else 0, ("OWAIT", j, l, tuple(kinds))))
        for l in reversed(layers):                      # B consumes the last layer first
            before[r_at].append((3, ("R", j, l, tuple(kinds))))
    out = []
    for n in range(len(comp) + 1):
        # at one position: completions of earlier offloads first (they free memory), then the offloads that
        # start here and (zero overlap) their own completions, then reloads
        for _, ev in sorted(before[n], key=lambda x: x[0]):
            out.append(ev)
        if n < len(comp):
            out.append(comp[n])
    return out


def repair_to_fit(events: list, fits, max_rounds: int = 2000) -> list | None:
    """Feedback-driven repair of an offloading list that overruns its budget.  `fits(events)` is the
    consumer's planner: it returns (ok, index of the first failing event).  While the list fails at an
    allocating event, the earliest offload still pending at that point has its OWAIT moved to just
    before the failing event (its memory is then credited there); if none is pending, the latest
    reload that was issued early is moved down to just before its consumer B.  Returns None when no
    move is left.  No accounting happens here: only the planner's verdicts steer the moves."""
    ev = list(events)
    for _ in range(max_rounds):
        ok, bad = fits(ev)
        if ok:
            return ev
        if bad >= len(ev):
            return None
        moved = False
        # (a) an offload issued before `bad` whose OWAIT comes after it
        seen_o = {}
        for n in range(bad):
            e = ev[n]
            if e[0] == "O":
                seen_o[e[1:]] = n
            elif e[0] == "OWAIT":
                seen_o.pop(e[1:], None)
        if seen_o:
            key = min(seen_o, key=lambda k: seen_o[k])
            w = next(n for n in range(bad, len(ev)) if ev[n][0] == "OWAIT" and ev[n][1:] == key)
            item = ev.pop(w)
            ev.insert(bad, item)
            moved = True
        else:
            # (b) the latest reload before `bad` whose B comes after `bad`: push it down to its B
            for n in range(bad - 1, -1, -1):
                e = ev[n]
                if e[0] == "R":
                    b = next(k for k in range(n, len(ev)) if ev[k][0] == "B" and ev[k][1] == e[1])
                    if b > bad:
                        item = ev.pop(n)
                        ev.insert(b - 1, item)
                        moved = True
                        break
        if not moved:
            return None
    return None


def random_valid_list(rng, m, n_layers, kinds, p_offload=0.6):
    """A random member of the schedule grammar: compute ops in a random order that keeps F j before B j before W j
    and every op type in increasing micro-batch order; a random subset of (micro-batch, layer, kind set) items
    offloaded, each with O somewhere after its F, OWAIT after the O, R after the OWAIT, all before its B."""
    nxt = {"F": 0, "B": 0, "W": 0}
    comp = []
    while len(comp) < 3 * m:
        can = [c for c in "FBW" if nxt[c] < m and (c == "F" or nxt[c] < nxt["FB"[("BW".index(c))]])]
        c = can[int(rng.integers(len(can)))]
        comp.append((c, nxt[c]))
        nxt[c] += 1
    ev = list(comp)
    for j in range(m):
        for l in range(n_layers):
            if rng.random() < p_offload:
                ks = tuple(k for k in kinds if rng.random() < 0.7) or (kinds[0],)
                f, b = ev.index(("F", j)), ev.index(("B", j))
                pos = sorted(int(x) for x in rng.integers(f + 1, b + 1, 3))       # insertion points, in list order
                for off, name in zip(pos, ("O", "OWAIT", "R")):
                    ev.insert(off + ("O", "OWAIT", "R").index(name), (name, j, l, ks))
    return ev
