"""Plain statement of the placement-repair rule (test infrastructure only).

The paper (Sec. 3.5, Sec. 5.1) fixes WHAT a repaired placement must satisfy --
every logical expert on a live rank -- and the three sources a slot's weights
can come from (already local, a surviving peer copy, the DRAM backup).  It does
not give the balancer's algorithm, so this file spells out the greedy rule the
library documents, with Python lists and loops only, written separately from the
C++ version.  Pins: Fig. 5 (middle panel), coverage invariants, source-kind
definitions, feasibility by pigeonhole.  PARITY UNPINNED by the paper: the
tie-breaking order of the greedy rule itself.
"""
NONE, LOCAL, PEER, DRAM = -1, 0, 1, 2


def plan_repair(cur, active, R, S, S_prim, E, load=None):
    P = R * S
    cur = [int(v) for v in cur]
    load = [1.0] * E if load is None else [float(v) for v in load]
    live = [bool(active[p // S]) for p in range(P)]
    now = list(cur)
    kind = [LOCAL if live[p] and cur[p] >= 0 else NONE for p in range(P)]
    src = [-1] * P

    def copies(e):                       # live copies in the placement under construction
        return sum(1 for p in range(P) if live[p] and now[p] == e)

    def rank_load(r):
        return sum(load[now[p]] / copies(now[p]) for p in range(r * S, r * S + S) if now[p] >= 0)

    def free_slot_for(e):
        cands = [p for p in range(P) if live[p] and now[p] == -1
                 and e not in now[(p // S) * S:(p // S) * S + S]]
        return min(cands, key=lambda p: (rank_load(p // S), p)) if cands else -1

    had = [sum(1 for p in range(P) if cur[p] == e) for e in range(E)]
    live_before = [sum(1 for p in range(P) if live[p] and cur[p] == e) for e in range(E)]
    unplaced = 0
    # A. coverage
    missing = sorted((e for e in range(E) if live_before[e] == 0), key=lambda e: (-load[e], e))
    for e in missing:
        p = free_slot_for(e)
        if p < 0:
            victims = [q for q in range(P) if live[q] and now[q] >= 0 and copies(now[q]) >= 2]
            if victims:
                p = min(victims, key=lambda q: ((q % S) < S_prim, load[now[q]] / copies(now[q]), q))
        if p < 0:
            unplaced += 1
            continue
        now[p], kind[p] = e, DRAM
    # B. re-create lost replicas from surviving peers
    while True:
        cands = []
        for e in range(E):
            c = copies(e)
            if live_before[e] == 0 or c == 0 or c >= had[e]:
                continue
            p = free_slot_for(e)
            if p >= 0:
                cands.append((-(load[e] / c), e, p))
        if not cands:
            break
        _, e, p = min(cands)
        peers = sorted((q for q in range(P) if live[q] and cur[q] == e),
                       key=lambda q: ((q % S) >= S_prim, q))
        now[p], kind[p], src[p] = e, PEER, peers[0]
    return dict(p2l=now, kind=kind, src_slot=src, local=kind.count(LOCAL), peer=kind.count(PEER),
                dram=kind.count(DRAM), unplaced=unplaced)


def plan_transition(cur, target, active, writable, R, S, S_prim):
    """Sources for moving from placement `cur` to a given `target` placement -- the
    step "resume preferred placement" of the reintegration sequence (Sec. 3.6,
    Fig. 5 right panel), classified with Sec. 3.5's hierarchy.  active[r]: rank r
    holds usable copies (a possible source); writable[r]: rank r's slots may be
    filled (active ranks plus a relaunched rank that is loading its experts before
    it reports join-ready).  A source is a slot on an active rank that holds the
    expert now and receives no new weights in this batch; among several, primary
    slots first, then the lowest slot id.  Slots of non-writable ranks keep `cur`.
    """
    P = R * S
    cur, target = [int(v) for v in cur], [int(v) for v in target]
    new = [target[p] if writable[p // S] else cur[p] for p in range(P)]
    rewritten = [bool(writable[p // S]) and new[p] >= 0 and new[p] != cur[p] for p in range(P)]
    kind, src = [NONE] * P, [-1] * P
    for p in range(P):
        if not writable[p // S] or new[p] < 0:
            continue
        if not rewritten[p]:
            kind[p] = LOCAL
            continue
        holders = [q for q in range(P) if active[q // S] and cur[q] == new[p] and not rewritten[q]]
        if holders:
            kind[p] = PEER
            src[p] = min(holders, key=lambda q: ((q % S) >= S_prim, q))
        else:
            kind[p] = DRAM
    return dict(p2l=new, kind=kind, src_slot=src, local=kind.count(LOCAL), peer=kind.count(PEER),
                dram=kind.count(DRAM), unplaced=0)


# outcome per slot of carry_out_repair
UNTOUCHED, FROM_PEER, FROM_DRAM, FROM_DRAM_FALLBACK = 0, 1, 2, 3


def carry_out_repair(weights, backup, new_p2l, kind, src_slot, active_now, S):
    """Weight movement that satisfies a planned placement (Sec. 3.5's source
    hierarchy; Sec. 5.1: the active mask is looked up when a transfer is issued,
    and an expert whose planned source rank has gone inactive since the plan was
    made is filled from the DRAM backup instead).  Only the SOURCE rank is looked
    up: a destination may be a rank that is not active yet (Sec. 3.6: a relaunched
    rank loads its experts before it is join-ready).

    weights: list of P byte strings (what each slot holds now); backup: list of E
    byte strings.  Slots planned as already-local or empty are not touched.  Every
    transfer reads the state before the batch (a source is never also a
    destination).  Returns (new weights, outcome per slot).
    """
    P = len(weights)
    after = list(weights)
    outcome = [UNTOUCHED] * P
    for p in range(P):
        if kind[p] != PEER and kind[p] != DRAM:
            continue
        if kind[p] == PEER and active_now[src_slot[p] // S]:
            after[p] = weights[src_slot[p]]
            outcome[p] = FROM_PEER
        else:
            after[p] = backup[new_p2l[p]]
            outcome[p] = FROM_DRAM if kind[p] == DRAM else FROM_DRAM_FALLBACK
    return after, outcome
