"""CPU oracle of the nano-operation pipeline model used by the auto-search
(paper Sec. 4.1.2 - 4.1.3).  TEST INFRASTRUCTURE ONLY: imported by tests, never by the
product, and sharing no code with the C++ planner.

The model, in the paper's terms: every operation of the layer is duplicated into one
nano-operation per nano-batch (a token range); two nano-operations are dependent iff their
parent operations are dependent and their ranges intersect; compute-bound nano-operations
(KQV, then O + Up/Gate + Down) run one at a time on the compute resource in launch order,
memory-bound ones (decode attention) one at a time on the memory resource; operations bound
by different resources may overlap.  A nano-operation's duration is D_best / P, where D_best
is its interference-free time and P its normalised performance: while a GEMM and an
attention kernel overlap, the GEMM runs at P = R_gemm and attention at P = P_attn(1 - R_gemm)
(the R -> P table, with the R of overlapping kernels summing to 1); a kernel that runs alone
runs at the stand-alone speed of the implementation the table row names.

Every nano-operation has its own resource share (Sec. 4.1.1: "R" belongs to the nano-operation),
so ``rows`` may name one table row per nano-batch - the row in force is that of the attention
nano-operation currently on the memory resource - and the nano-batches may be launched in any
``order`` whose dependencies can be met (Sec. 4.1.2: number, size and order of the
nano-operations are what the search decides).

The two resources are two streams of the device: a nano-operation that waits for one on the
other stream starts ``sync`` later than that one ends (a measured latency of the device; the
paper's model has no such term, and ``sync`` = 0 gives the paper's model).

Sec. 4.1.2 also lets every operation have its own number of nano-operations (Fig. 6: the
operations near a bubble are split further than the others).  ``makespan_parts`` models that:
one token partition per operation, the dependency rule above between the pieces, and the launch
order stated in ``launch_order``.

It is written as a fixed-step time integration - slow and plain - so that it can check the
event-driven C++ implementation.
"""
from __future__ import annotations

import itertools
from typing import List, Optional, Sequence


def interp_dense(table: Sequence[float], granule: int, m: int) -> float:
    """Interference-free time of a dense op on m tokens from times at granule, 2*granule, ..."""
    x = m / granule
    if x <= 1:
        return table[0]
    i = int(x) - 1
    if i + 1 >= len(table):
        return table[-1] * x / len(table)
    f = x - int(x)
    return table[i] + f * (table[i + 1] - table[i])


def makespan(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, bounds, overlap,
             row: Optional[dict], dt: float = 0.02, misc=None, layers: int = 1, rows: Optional[list] = None,
             order: Optional[list] = None, sync: float = 0.0) -> Optional[float]:
    """dense: dict op -> table of the best implementation; row: dict(p_gemm, p_attn,
    p_attn_solo[, p_gemm_solo][, dense]) or None.  A row that carries its own "dense" tables
    (the times of the GEMM implementation it was measured with) makes every GEMM of an
    overlapped pipeline run in that implementation: its table gives D, and the overlapped
    speed p_gemm (normalised to the best implementation) is re-expressed relative to it.
    misc: ((a, b), (a, b), (a, b)) fixed + per-token cost of the small kernels added to the KQV
    stage, the O/Up/Gate/Down stage and the attention stage.
    layers > 1: that many consecutive layers (the output of a layer is the next layer's input,
    Sec. 2.1), pipelined across the layer boundary: on the compute resource the KQV
    nano-operation of a range in layer l + 1 is launched right behind the O/Up/Gate/Down
    nano-operation of that range in layer l; the total time is returned.
    rows: one row per nano-batch (the row of the attention nano-operation that is running decides the
    speeds; all rows belong to one GEMM implementation, so rows[0] supplies the GEMM tables).
    order: order[k] = index of the nano-batch launched k-th; None (the function's result) when
    an attention nano-operation would be launched before a KQV nano-operation it needs.
    sync: a nano-operation that waits for one on the other resource starts that much later than
    the moment the last of them ends (the latency of a dependency across two streams)."""
    if rows is not None:
        row = rows[0]
    if overlap and row is not None and row.get("dense") is not None:
        dense = row["dense"]
        solo = row.get("p_gemm_solo", 1.0)
        row = dict(row, p_gemm=row["p_gemm"] / solo, p_gemm_solo=1.0)
        if rows is not None:
            rows = [dict(r, p_gemm=r["p_gemm"] / r.get("p_gemm_solo", 1.0), p_gemm_solo=1.0) for r in rows]
    n = len(bounds) - 1
    order = list(order) if order is not None else list(range(n))
    position = {i: k for k, i in enumerate(order)}
    kqv, att, rest = [], [], []
    for i in range(n):
        m = bounds[i + 1] - bounds[i]
        kqv.append(interp_dense(dense["KQV"], granule, m))
        rest.append(sum(interp_dense(dense[o], granule, m) for o in ("O", "UG", "D")))
        att.append(attn_fixed + attn_per_mb * (attn_mb_prefix[bounds[i + 1]] - attn_mb_prefix[bounds[i]]))
        if misc is not None:
            kqv[-1] += misc[0][0] + misc[0][1] * m
            rest[-1] += misc[1][0] + misc[1][1] * m
            att[-1] += misc[2][0] + misc[2][1] * m
    if not overlap:
        return (sum(kqv) + sum(att) + sum(rest)) * layers
    # launch order on the compute resource: all KQV nano-ops of the first layer, then per layer
    # O+UG+D of every nano-batch, each followed by the next layer's KQV of the same range
    compute = [("kqv", i, 0) for i in order]
    memory = []
    for l in range(layers):
        for i in order:
            compute.append(("rest", i, l))
            if l + 1 < layers:
                compute.append(("kqv", i, l + 1))
        memory += [("att", i, l) for i in order]
    for i in range(n):
        lo = req_start[bounds[i]]
        if any(bounds[j + 1] > lo and position[j] > position[i] for j in range(i + 1)):
            return None
    work = {}
    for l in range(layers):
        for i in range(n):
            work[("kqv", i, l)] = kqv[i]
            work[("att", i, l)] = att[i]
            work[("rest", i, l)] = rest[i]
    done = {}                               # nano-operation -> the time it ended

    def ready(op):
        kind, i, l = op
        if kind == "kqv":
            return True                     # the launch order already puts it behind its predecessor
        if kind == "rest":
            needs = [("att", i, l)]
        else:
            lo = req_start[bounds[i]]       # attention also reads K/V appended by earlier ranges
            needs = [("kqv", j, l) for j in range(i + 1) if bounds[j + 1] > lo]
        return all(p in done and t >= done[p] + sync - 1e-9 for p in needs)

    t = 0.0
    ci = mi = 0
    left = dict(work)
    while ci < len(compute) or mi < len(memory):
        c = compute[ci] if ci < len(compute) and ready(compute[ci]) else None
        m = memory[mi] if mi < len(memory) and ready(memory[mi]) else None
        if c is None and m is None:         # both resources wait out a synchronisation latency
            assert sync > 0, "deadlock"
            t += dt
            continue
        sc = sm = 1.0
        cur = row
        if rows is not None and mi < len(memory):
            cur = rows[memory[mi][1]]       # the attention nano-operation at the head of the memory resource
        if cur is not None:
            if c is not None and m is not None:
                sc, sm = cur["p_gemm"], cur["p_attn"]
            elif m is not None:
                sm = cur["p_attn_solo"]
            else:
                sc = cur.get("p_gemm_solo", 1.0)
        if c is not None:
            left[c] -= sc * dt
            if left[c] <= 0:
                done[c] = t + dt
                ci += 1
        if m is not None:
            left[m] -= sm * dt
            if left[m] <= 0:
                done[m] = t + dt
                mi += 1
        t += dt
    return t


def all_bounds(n_tokens: int, granule: int, n_nano: int) -> List[List[int]]:
    cuts = list(range(granule, n_tokens, granule))
    return [[0, *c, n_tokens] for c in itertools.combinations(cuts, n_nano - 1)]


def brute_force_ops(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, bounds, rows, dt: float = 0.02):
    """Minimum makespan of ONE structure over every assignment of table rows to its nano-batches
    and every launch order."""
    n = len(bounds) - 1
    best = None
    for assign in itertools.product(rows, repeat=n):
        for order in itertools.permutations(range(n)):
            t = makespan(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, bounds, True, None, dt,
                         rows=list(assign), order=list(order))
            if t is not None and (best is None or t < best[0]):
                best = (t, assign, order)
    return best


def brute_force(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, n_tokens, rows, max_nano,
                dt: float = 0.02, misc=None):
    """Minimum makespan over every structure and every table row, and the unsplit time."""
    unsplit = makespan(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, [0, n_tokens], False, None,
                       misc=misc)
    best = (unsplit, [0, n_tokens], None)
    for n in range(2, max_nano + 1):
        for b in all_bounds(n_tokens, granule, n):
            for r in (rows or [None]):
                t = makespan(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, b, True, r, dt, misc)
                if t < best[0]:
                    best = (t, b, r)
    return best, unsplit


KINDS = ("KQV", "ATTN", "O", "UG", "D")
FEEDS = {"ATTN": "KQV", "O": "ATTN", "UG": "O", "D": "UG"}      # child operation -> parent operation


def launch_order(parts: dict) -> list:
    """Order in which one layer's nano-operations are handed to the device when every operation
    has its own partition ``parts[kind]`` (boundaries from 0 to the number of tokens).
    KQV pieces go first, in token order, and an attention piece is launched as soon as the KQV
    piece holding its last token has been launched.  Then the O, Up/Gate and Down pieces: among
    the pieces whose input rows have all been launched, the one that ends at the smallest token
    goes next, and O goes before Up/Gate before Down when they end at the same token."""
    seq = []
    attn_left = list(range(len(parts["ATTN"]) - 1))
    for k in range(len(parts["KQV"]) - 1):
        seq.append(("KQV", k))
        while attn_left and parts["ATTN"][attn_left[0] + 1] <= parts["KQV"][k + 1]:
            seq.append(("ATTN", attn_left.pop(0)))
    waiting = {kind: list(range(len(parts[kind]) - 1)) for kind in ("O", "UG", "D")}
    launched_up_to = {"ATTN": parts["ATTN"][-1], "O": 0, "UG": 0, "D": 0}
    while any(waiting.values()):
        ready = []
        for rank, kind in enumerate(("O", "UG", "D")):
            if waiting[kind]:
                end = parts[kind][waiting[kind][0] + 1]
                if launched_up_to[FEEDS[kind]] >= end:
                    ready.append((end, rank, kind))
        end, _, kind = min(ready)
        seq.append((kind, waiting[kind].pop(0)))
        launched_up_to[kind] = end
    return seq


def makespan_parts(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, parts: dict, overlap,
                   rows: Optional[list] = None, dt: float = 0.02, misc=None, layers: int = 1,
                   sync: float = 0.0) -> float:
    """``makespan`` with a partition per operation.  rows: one table row per attention piece (the
    row of the attention piece at the head of the memory resource decides the speeds; all rows
    belong to one GEMM implementation) or None for no interference.  The small kernels of ``misc``
    are charged to the KQV pieces, to the Up/Gate pieces (the norm in front of them) and to the
    attention pieces.  layers > 1: the KQV piece of the next layer is launched right behind the
    Down piece of this layer that completes its tokens."""
    if rows is not None and overlap and rows[0].get("dense") is not None:
        dense = rows[0]["dense"]
        rows = [dict(r, p_gemm=r["p_gemm"] / r.get("p_gemm_solo", 1.0), p_gemm_solo=1.0) for r in rows]
    table = {"KQV": "KQV", "O": "O", "UG": "UG", "D": "D"}
    extra = {"KQV": 0, "UG": 1, "ATTN": 2}
    work, span = {}, {}
    for kind in KINDS:
        for j in range(len(parts[kind]) - 1):
            lo, hi = parts[kind][j], parts[kind][j + 1]
            span[(kind, j)] = (lo, hi)
            if kind == "ATTN":
                w = attn_fixed + attn_per_mb * (attn_mb_prefix[hi] - attn_mb_prefix[lo])
            else:
                w = interp_dense(dense[table[kind]], granule, hi - lo)
            if misc is not None and kind in extra:
                w += misc[extra[kind]][0] + misc[extra[kind]][1] * (hi - lo)
            work[(kind, j)] = w
    seq = launch_order(parts)
    if not overlap:
        return sum(work[p] for p in seq) * layers
    compute, memory = [(kind, j, 0) for kind, j in seq if kind == "KQV"], []
    for l in range(layers):
        next_layer_kqv = [(kind, j) for kind, j in seq if kind == "KQV"]
        for kind, j in seq:
            if kind in ("O", "UG", "D"):
                compute.append((kind, j, l))
            if kind == "D" and l + 1 < layers:
                while next_layer_kqv and span[next_layer_kqv[0]][1] <= span[(kind, j)][1]:
                    compute.append((*next_layer_kqv.pop(0), l + 1))
        memory += [(kind, j, l) for kind, j in seq if kind == "ATTN"]
    done = {}                                 # piece -> the time it ended

    def ready(op):
        kind, j, l = op
        if kind == "KQV":
            return True                       # queued behind the Down pieces that complete its rows
        lo, hi = span[(kind, j)]
        if kind == "ATTN":
            lo = req_start[lo]                # it also reads K/V appended by the request's earlier tokens
        parent = FEEDS[kind]
        # a piece on the other resource must have ended `sync` ago (attention after KQV, O after
        # attention); pieces of the same resource follow each other without it
        wait = sync if kind in ("ATTN", "O") else 0.0
        return all((parent, i, l) in done and t >= done[(parent, i, l)] + wait - 1e-9
                   for i in range(len(parts[parent]) - 1)
                   if max(lo, parts[parent][i]) < min(hi, parts[parent][i + 1]))

    left = {(kind, j, l): work[(kind, j)] for (kind, j) in work for l in range(layers)}
    t = 0.0
    ci = mi = 0
    while ci < len(compute) or mi < len(memory):
        c = compute[ci] if ci < len(compute) and ready(compute[ci]) else None
        m = memory[mi] if mi < len(memory) and ready(memory[mi]) else None
        if c is None and m is None:
            assert sync > 0, "deadlock"
            t += dt
            continue
        sc = sm = 1.0
        if rows is not None:
            cur = rows[memory[mi][1]] if mi < len(memory) else rows[-1]
            if c is not None and m is not None:
                sc, sm = cur["p_gemm"], cur["p_attn"]
            elif m is not None:
                sm = cur["p_attn_solo"]
            else:
                sc = cur.get("p_gemm_solo", 1.0)
        if c is not None:
            left[c] -= sc * dt
            if left[c] <= 0:
                done[c] = t + dt
                ci += 1
        if m is not None:
            left[m] -= sm * dt
            if left[m] <= 0:
                done[m] = t + dt
                mi += 1
        t += dt
    return t


def all_partitions(n_tokens: int, granule: int, max_pieces: int) -> List[List[int]]:
    out = []
    for n in range(1, max_pieces + 1):
        out += all_bounds(n_tokens, granule, n) if n > 1 else [[0, n_tokens]]
    return out


def brute_force_parts(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, n_tokens, rows, max_pieces,
                      dt: float = 0.05, misc=None):
    """Minimum makespan over every choice of a partition per operation (at most max_pieces pieces
    each) and of a table row per attention piece."""
    options = all_partitions(n_tokens, granule, max_pieces)
    best = None
    for combo in itertools.product(options, repeat=len(KINDS)):
        parts = dict(zip(KINDS, combo))
        n_attn = len(parts["ATTN"]) - 1
        for assign in (itertools.product(rows, repeat=n_attn) if rows else [None]):
            t = makespan_parts(dense, granule, attn_fixed, attn_per_mb, attn_mb_prefix, req_start, parts, True,
                               list(assign) if assign is not None else None, dt, misc)
            if best is None or t < best[0]:
                best = (t, parts, assign)
    return best
