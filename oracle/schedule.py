"""Schedule semantics oracle: event grammar, activation-memory table, list-order
memory accounting, and a discrete-event (as-soon-as-possible) timing simulator
for p pipeline stages.

TEST INFRASTRUCTURE ONLY (see oracle/stage_fp64.py); pure host Python with
integer byte arithmetic; shares no code with the HIP path.

Paper passages followed (Sec. 3 and the formulation in the appendix on the
mathematical model):
  * ops (i, j, c), c in {F, B, W}; transfers Offload (O) and Reload (R)
  * Eq. 3 / Eq. 4  pipeline data dependencies between neighbouring stages
  * Eq. 5          one compute op at a time per stage
  * Eq. 6          F before B before W for each micro-batch
  * fixed micro-batch order: same-type ops run in increasing micro-batch index
  * Eq. 7          memory in use at every op stays within M_limit: completed ops
                   contribute Delta, completed offloads subtract Gamma, started
                   reloads add Gamma
  * Eq. 8-11       one transfer at a time on the GPU<->CPU channel
  * Eq. 12-14      an op that counts an offload's freed memory starts after that
                   offload has ended; a reload occupies memory from its start; a
                   reload ordered after an op starts once that op has ended
  * Eq. 16 / 17    makespan: per-stage span (post-validation) or global span
Readings where the text is silent or inconsistent are listed in this
repository's design notes; the ones that matter here: Eq. 5 applies to every
pair of distinct ops on a stage; Eq. 12's left side is the op's start time;
an offload starts after the F that made the data ends; a reload starts after
the same item's offload ends and ends before B of its micro-batch starts.

A stage schedule is ONE ordered list of events
    ("F", j) ("B", j) ("W", j) ("O", j, layer, kinds) ("OWAIT", j, layer, kinds)
    ("R", j, layer, kinds)
where kinds is a tuple of activation kind names.  A stage that holds several
model chunks (the interleaved and V-shaped schedules of the comparison methods,
Sec. 5) writes its compute ops ("F", j, chunk); its n_layers layers are split
evenly over the chunks in order, transfers name the layer on the stage, and
every rule above applies per chunk (Eq. 6, the fixed micro-batch order), with
Eq. 3 / Eq. 4 following the chunk's position in the model (`virtual_stage`).  List order is the order
relation of the paper's precedence binaries: compute ops run in list order; the
copy channel serves O and R in list order; a compute op listed after OWAIT(x)
starts after offload x ended and x's bytes are credited from that position; an
R listed after compute op X starts after X ended, is charged from its list
position, and overlaps the compute ops listed after it.
"""
from __future__ import annotations

from dataclasses import dataclass, field

GPT = 0
LLAMA = 1

F_KINDS = ("X_IN", "N1", "QKV", "O", "LSE", "X_MID", "N2", "GU", "A", "STATS")
B_KINDS = ("DY", "DX_MID")
W_FREED = ("N1", "QKV", "O", "DX_MID", "N2", "GU", "A", "DY")
RECOMPUTED = ("N1", "N2", "A")     # cheap functions of X_IN, X_MID, GU: the recompute variant does not keep them in F
ALIGN = 256


def _round_up(n: int) -> int:
    return (n + ALIGN - 1) // ALIGN * ALIGN


def memory_table(family, hidden, n_q_heads, n_kv_heads, head_dim, ffn, tokens, elem_size):
    """Bytes of each activation kind for ONE layer of ONE micro-batch (store-all
    inventory), each buffer rounded up to 256 bytes.  Gamma of an item is its
    entry; Delta of F/B/W follow from `op_memory_steps`."""
    e = elem_size
    qkv_w = (n_q_heads + 2 * n_kv_heads) * head_dim
    up_w = 2 * ffn if family == LLAMA else ffn
    n_stats = 2 if family == LLAMA else 4          # rstd per norm (+ mean for LayerNorm), fp32
    raw = {
        "X_IN": tokens * hidden * e, "N1": tokens * hidden * e, "QKV": tokens * qkv_w * e,
        "O": tokens * n_q_heads * head_dim * e, "LSE": n_q_heads * tokens * 4,
        "X_MID": tokens * hidden * e, "N2": tokens * hidden * e, "GU": tokens * up_w * e,
        "A": tokens * ffn * e, "STATS": n_stats * tokens * 4,
        "DY": tokens * hidden * e, "DX_MID": tokens * hidden * e,
    }
    return {k: _round_up(v) for k, v in raw.items()}


def chunk_of(ev):
    """Model chunk of a compute event: ("F", j) is chunk 0, ("F", j, c) chunk c."""
    return ev[2] if len(ev) > 2 else 0


def virtual_stage(i, c, p, placement="interleaved"):
    """Position of chunk c of stage i in the model's order of p * n_chunks pieces.
    "interleaved": chunk c holds pieces c p .. c p + p - 1 in stage order (1F1B-I);
    "v": odd chunks run through the stages in reverse (ZB-V: stage 0 holds the first
    and the last piece)."""
    if placement == "interleaved" or c % 2 == 0:
        return c * p + i
    if placement == "v":
        return c * p + (p - 1 - i)
    raise ValueError(placement)


def _holder(v, p, placement):
    c = v // p
    i = v % p if (placement == "interleaved" or c % 2 == 0) else p - 1 - v % p
    return i, c


def op_memory_steps(op, n_layers, recompute=False, first_layer=0):
    """Ordered (+1/-1, layer, kind) steps a compute op performs on the activation
    arena.  F keeps everything it produces.  B walks layers last to first: it
    creates the layer's output-gradient buffer DY (kept for W) and DX_MID (kept
    for W), and releases X_MID, LSE, X_IN, STATS once their last reader is done.
    W releases everything still held.

    recompute: the memory-table variant in which F keeps no N1, N2, A and B
    rebuilds them for W (A and N2 before the MLP part of the layer is
    differentiated, N1 before the attention part's norm), so Delta_F shrinks and
    Delta_B grows by the same bytes while W is unchanged.

    first_layer: the op covers layers first_layer .. first_layer + n_layers - 1 of
    the stage (a model chunk)."""
    steps = []
    for sgn, l, k in _op_memory_steps(op, n_layers, recompute):
        steps.append((sgn, l + first_layer, k))
    return steps


def _op_memory_steps(op, n_layers, recompute):
    steps = []
    if op == "F":
        for l in range(n_layers):
            for k in F_KINDS:
                if not (recompute and k in RECOMPUTED):
                    steps.append((+1, l, k))
    elif op == "B":
        steps.append((+1, n_layers - 1, "DY"))
        for l in reversed(range(n_layers)):
            if recompute:
                steps.append((+1, l, "A"))
                steps.append((+1, l, "N2"))
            steps.append((+1, l, "DX_MID"))
            steps.append((-1, l, "X_MID"))
            steps.append((-1, l, "LSE"))
            if recompute:
                steps.append((+1, l, "N1"))
            if l > 0:
                steps.append((+1, l - 1, "DY"))
            steps.append((-1, l, "X_IN"))
            steps.append((-1, l, "STATS"))
    elif op == "W":
        for l in range(n_layers):
            for k in W_FREED:
                steps.append((-1, l, k))
    else:
        raise ValueError(op)
    return steps


def op_delta(op, n_layers, table, recompute=False):
    """Net memory change Delta of a compute op (the parameter of Eq. 7)."""
    return sum(sgn * table[k] for sgn, _, k in op_memory_steps(op, n_layers, recompute))


class ScheduleError(Exception):
    def __init__(self, index, msg):
        super().__init__(f"event {index}: {msg}")
        self.index = index


def check_order(events, n_microbatches, n_layers, recompute=False, n_chunks=1):
    """Validity of one stage's list (raises ScheduleError naming the first bad event).
    In the recompute variant the kinds F does not keep cannot be offloaded.  With
    several model chunks (n_layers counts all of them) the rules hold per chunk."""
    if n_layers % n_chunks:
        raise ValueError("n_layers must be a multiple of n_chunks")
    per_chunk = n_layers // n_chunks
    done = {"F": set(), "B": set(), "W": set()}     # (chunk, j)
    nxt = {(op, c): 0 for op in "FBW" for c in range(n_chunks)}
    state = {}                      # (j, layer, kind) -> "O" | "OWAIT" | "R"
    for idx, ev in enumerate(events):
        op, j = ev[0], ev[1]
        if not (0 <= j < n_microbatches):
            raise ScheduleError(idx, "micro-batch index out of range")
        if op in ("F", "B", "W"):
            c = chunk_of(ev)
            if not (0 <= c < n_chunks):
                raise ScheduleError(idx, "chunk out of range")
            if (c, j) in done[op]:
                raise ScheduleError(idx, f"{op} {j} listed twice")
            if j != nxt[(op, c)]:
                raise ScheduleError(idx, f"{op} ops must run in increasing micro-batch order")
            if op == "B" and (c, j) not in done["F"]:
                raise ScheduleError(idx, "B before F")
            if op == "W" and (c, j) not in done["B"]:
                raise ScheduleError(idx, "W before B")
            if op == "B":
                for key, st in state.items():
                    if key[0] == j and key[1] // per_chunk == c and st != "R":
                        raise ScheduleError(idx, f"B {j} while {key} is offloaded and not reloaded")
            done[op].add((c, j))
            nxt[(op, c)] += 1
        elif op in ("O", "OWAIT", "R"):
            layer, kinds = ev[2], ev[3]
            if not (0 <= layer < n_layers) or len(kinds) == 0:
                raise ScheduleError(idx, "bad layer or empty kind set")
            c = layer // per_chunk
            for k in kinds:
                if k not in F_KINDS or (recompute and k in RECOMPUTED):
                    raise ScheduleError(idx, f"kind {k} cannot be offloaded")
                key = (j, layer, k)
                st = state.get(key)
                if op == "O":
                    if (c, j) not in done["F"] or (c, j) in done["B"]:
                        raise ScheduleError(idx, "offload outside the F..B window of its micro-batch")
                    if st is not None:
                        raise ScheduleError(idx, f"{key} offloaded twice")
                    state[key] = "O"
                elif op == "OWAIT":
                    if st != "O":
                        raise ScheduleError(idx, f"OWAIT of {key} without a pending offload")
                    state[key] = "OWAIT"
                else:
                    if st != "OWAIT":
                        raise ScheduleError(idx, f"reload of {key} before its offload completed")
                    state[key] = "R"
        else:
            raise ScheduleError(idx, f"unknown op {op}")
    for op in ("F", "B", "W"):
        if len(done[op]) != n_microbatches * n_chunks:
            raise ScheduleError(len(events), f"missing {op} ops")
    for key, st in state.items():
        if st != "R":
            raise ScheduleError(len(events), f"{key} never reloaded")


def account_memory(events, n_layers, table, limit=None, recompute=False, n_chunks=1):
    """List-order logical accounting.  Returns (peak, trace) where trace[i] is the
    bytes in use after event i; raises ScheduleError at the first allocation
    that would exceed `limit` (checked before committing it)."""
    live = 0
    peak = 0
    trace = []
    for idx, ev in enumerate(events):
        op = ev[0]
        if op in ("F", "B", "W"):
            steps = [(sgn, table[k]) for sgn, _, k in op_memory_steps(op, n_layers // n_chunks, recompute)]
        elif op == "OWAIT":
            steps = [(-1, table[k]) for k in ev[3]]
        elif op == "R":
            steps = [(+1, table[k]) for k in ev[3]]
        else:
            steps = []
        for sgn, b in steps:
            if sgn > 0:
                if limit is not None and live + b > limit:
                    raise ScheduleError(idx, f"needs {live + b} bytes, limit {limit}")
                live += b
                peak = max(peak, live)
            else:
                live -= b
                if live < 0:
                    raise ScheduleError(idx, "negative live bytes")
        trace.append(live)
    return peak, trace


def eq7_usage(events, n_layers, table, recompute=False):
    """Memory in use during each compute op exactly as Eq. 7 counts it: the op's own
    Delta, plus Delta of every compute op ordered before it, minus Gamma of every
    offload completed before it, plus Gamma of every reload started before it."""
    out = []
    for idx, ev in enumerate(events):
        if ev[0] not in ("F", "B", "W"):
            continue
        use = op_delta(ev[0], n_layers, table, recompute)
        for prev in events[:idx]:
            if prev[0] in ("F", "B", "W"):
                use += op_delta(prev[0], n_layers, table, recompute)
            elif prev[0] == "OWAIT":
                use -= sum(table[k] for k in prev[3])
            elif prev[0] == "R":
                use += sum(table[k] for k in prev[3])
        out.append((idx, use))
    return out


@dataclass
class Timing:
    start: list = field(default_factory=list)   # per stage: list aligned with events (None for OWAIT)
    end: list = field(default_factory=list)
    makespan_global: float = 0.0                 # Eq. 17
    makespan_per_stage: float = 0.0              # Eq. 16
    busy: list = field(default_factory=list)     # per stage, sum of compute durations
    bubble: list = field(default_factory=list)   # per stage, 1 - busy / makespan_global


def simulate(schedules, t_op, t_comm=0.0, t_copy=None, duplex=False, n_chunks=1, placement="interleaved",
             layers_per_chunk=None):
    """ASAP timing of p stages.

    schedules[i]  event list of stage i
    t_op[i]       {"F": T_F, "B": T_B, "W": T_W} for stage i (of ONE chunk's op when the stage holds several)
    n_chunks, placement   model chunks per stage and where they sit in the model (`virtual_stage`): the F of a
                  chunk waits for the F of the piece before it (Eq. 3), the B for the B of the piece after
                  it (Eq. 4); t_comm applies when that piece is on another stage
    layers_per_chunk      needed with transfers on a multi-chunk stage: maps an event's layer to its chunk
    t_copy        callable (stage, event) -> duration of that O or R event
    duplex        False: one serial transfer channel per stage, as the paper models it (Eq. 8-11);
                  True: offloads and reloads each have their own serial channel (a full-duplex host
                  link), so Eq. 8-11 hold within a direction only
    """
    p = len(schedules)
    t_copy = t_copy or (lambda i, ev: 0.0)
    start = [[None] * len(s) for s in schedules]
    end = [[None] * len(s) for s in schedules]
    ptr = [0] * p
    compute_free = [0.0] * p        # end of the last compute op issued on stage i
    copy_free = [[0.0, 0.0] for _ in range(p)]   # end of the last transfer per channel: [offload, reload]
    ch_r = 1 if duplex else 0
    gate = [0.0] * p                # compute ops listed from here on start no earlier (OWAIT)
    end_F = [dict() for _ in range(p)]
    end_B = [dict() for _ in range(p)]
    end_O = [dict() for _ in range(p)]          # (j, layer, kind) -> end
    end_R = [dict() for _ in range(p)]          # (j, chunk) -> latest reload end
    n_virtual = p * n_chunks

    def chunk_of_layer(layer):
        if n_chunks == 1:
            return 0
        if layers_per_chunk is None:
            raise ValueError("layers_per_chunk is needed for transfers on a multi-chunk stage")
        return layer // layers_per_chunk

    progress = True
    while progress:
        progress = False
        for i in range(p):
            while ptr[i] < len(schedules[i]):
                ev = schedules[i][ptr[i]]
                op, j = ev[0], ev[1]
                if op in ("F", "B", "W"):
                    c = chunk_of(ev)
                    v = virtual_stage(i, c, p, placement)
                    ready = max(compute_free[i], gate[i])
                    if op == "F" and v > 0:
                        i2, c2 = _holder(v - 1, p, placement)
                        if (j, c2) not in end_F[i2]:
                            break
                        ready = max(ready, end_F[i2][(j, c2)] + (t_comm if i2 != i else 0.0))      # Eq. 3
                    if op == "B":
                        if v < n_virtual - 1:
                            i2, c2 = _holder(v + 1, p, placement)
                            if (j, c2) not in end_B[i2]:
                                break
                            ready = max(ready, end_B[i2][(j, c2)] + (t_comm if i2 != i else 0.0))  # Eq. 4
                        ready = max(ready, end_R[i].get((j, c), 0.0))          # reload completes first
                    s, e = ready, ready + t_op[i][op]
                    compute_free[i] = e
                    if op == "F":
                        end_F[i][(j, c)] = e
                    elif op == "B":
                        end_B[i][(j, c)] = e
                elif op == "O":
                    s = max(copy_free[i][0], end_F[i][(j, chunk_of_layer(ev[2]))])   # after its F ended
                    e = s + t_copy(i, ev)
                    copy_free[i][0] = e
                    for k in ev[3]:
                        end_O[i][(j, ev[2], k)] = e
                elif op == "OWAIT":
                    s = e = None
                    gate[i] = max([gate[i]] + [end_O[i][(j, ev[2], k)] for k in ev[3]])   # Eq. 12
                elif op == "R":
                    s = max([copy_free[i][ch_r], compute_free[i]] +            # Eq. 14; its channel is free
                            [end_O[i][(j, ev[2], k)] for k in ev[3]])
                    e = s + t_copy(i, ev)
                    copy_free[i][ch_r] = e
                    key = (j, chunk_of_layer(ev[2]))
                    end_R[i][key] = max(end_R[i].get(key, 0.0), e)
                else:
                    raise ValueError(op)
                start[i][ptr[i]], end[i][ptr[i]] = s, e
                ptr[i] += 1
                progress = True
    if any(ptr[i] < len(schedules[i]) for i in range(p)):
        raise ScheduleError(ptr[0], "cross-stage deadlock: schedules are mutually inconsistent")
    res = Timing(start=start, end=end)
    comp = [[(start[i][n], end[i][n]) for n, ev in enumerate(schedules[i]) if ev[0] in ("F", "B", "W")]
            for i in range(p)]
    first = min(c[0][0] for c in comp if c)
    last = max(c[-1][1] for c in comp if c)
    res.makespan_global = last - first
    res.makespan_per_stage = max(c[-1][1] - c[0][0] for c in comp if c)
    res.busy = [sum(e - s for s, e in c) for c in comp]
    res.bubble = [1.0 - b / res.makespan_global if res.makespan_global > 0 else 0.0 for b in res.busy]
    return res
