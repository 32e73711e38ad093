"""CPU oracle of the padded equal-split layout and of the micro-op scheduling policy --
test infrastructure only.

Padded layout (the equal-split all-to-all of training; Sec. 6.2 contrasts it with the
unequal split used in inference): every expert owns C slots; the assignment with rank p
among those that chose expert e (flat token-major order) sits in slot e*C + p when p < C
and is dropped otherwise.  Written out as the definition, with plain loops.

Scheduling policy (Sec. 4.2 "Tensor partitioning", "Pipelining micro-ops"; Sec. 6.1
"Communication scheduler"): operations are cut into micro-ops; one link carries one
micro-op after the other; a ready all-to-all micro-op always goes before allreduce
micro-ops, and an allreduce micro-op is launched only while no all-to-all micro-op is ready
or on the link and no all-to-all has been announced.  `simulate` plays that policy on a
serial link in exact rational time.  Nothing in the product path imports this file, and it
shares no code with the HIP side.
"""
from __future__ import annotations

import dataclasses
from fractions import Fraction
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

ALL_TO_ALL, ALLREDUCE = 0, 1
ARRIVAL_ORDER, PRIORITY = 0, 1


# ---------------------------------------------------------------------------- padded layout
def padded_plan(expert_idx: np.ndarray, E: int, C: int):
    """expert_idx [T, k] -> counts [E], slot_of [T*k] (e*C + rank, -1 if dropped),
    src_of [E*C] (assignment held by each slot, -1 for an empty slot)."""
    flat = np.asarray(expert_idx, np.int64).reshape(-1)
    counts = np.zeros(E, np.int32)
    slot_of = np.full(flat.size, -1, np.int32)
    src_of = np.full(E * C, -1, np.int32)
    for i, e in enumerate(flat):              # flat index i = t*k + j, ascending: earlier wins
        p = counts[e]
        counts[e] += 1
        if p < C:
            slot_of[i] = e * C + p
            src_of[e * C + p] = i
    return counts, slot_of, src_of


def pack_padded(x: np.ndarray, src_of: np.ndarray, k: int) -> np.ndarray:
    """The send buffer of the first all-to-all: a kept slot holds its token's row, an empty
    slot zeros."""
    xs = np.zeros((src_of.size, x.shape[1]), x.dtype)
    held = src_of >= 0
    xs[held] = x[src_of[held] // k]
    return xs


def micro_ranges(C: int, n: int) -> List[Tuple[int, int]]:
    """Slot positions of micro-op m of n: the tensor is cut along the token dimension."""
    return [(m * C // n, (m + 1) * C // n) for m in range(n)]


def static_link_order(n: int) -> List[Tuple[int, int]]:
    """(all-to-all, micro-op) in the order in which a layer that owns its link sends them:
    the second all-to-all's micro-op m can only follow the FFN of m, so the first
    all-to-all stays one micro-op ahead (Sec. 4.2, pipelining of micro-ops)."""
    order = [(0, 0)]
    for m in range(n):
        if m + 1 < n:
            order.append((0, m + 1))
        order.append((1, m))
    return order


# ---------------------------------------------------------------------------- scheduling policy
@dataclasses.dataclass
class Micro:
    op: int
    micro: int
    kind: int
    posted: Fraction          # when the scheduler learns that it is ready to be launched
    data: Fraction            # when its data is there (>= posted: a launched micro-op waits on the link)
    duration: Fraction        # time on the link
    start: Optional[Fraction] = None
    end: Optional[Fraction] = None
    chosen: Optional[Fraction] = None


def simulate(micros: Sequence[Micro], policy: int, depth: int = 1,
             holds: Sequence[Tuple[Fraction, Fraction]] = ()) -> List[Micro]:
    """Plays the policy: returns the micro-ops in link order with chosen/start/end filled in.
    The scheduler keeps at most `depth` micro-ops on the (serial) link and takes a decision
    whenever a place is free and something may be launched.  Ties in `posted` keep the
    order of `micros`."""
    pending = sorted(range(len(micros)), key=lambda i: (micros[i].posted, i))
    ready: Dict[int, List[int]] = {0: [], 1: []}
    on_link: List[int] = []
    order: List[int] = []
    t = Fraction(0)
    link_free = Fraction(0)

    def held(at):
        return any(a <= at < b for a, b in holds)

    while pending or ready[0] or ready[1] or on_link:
        while pending and micros[pending[0]].posted <= t:
            i = pending.pop(0)
            q = micros[i].kind if policy == PRIORITY else 0
            ready[q].append(i)
        on_link = [i for i in on_link if micros[i].end > t]
        if not (pending or ready[0] or ready[1] or on_link):
            break
        launched = False
        if len(on_link) < depth:
            pick = None
            if ready[0]:
                pick = ready[0].pop(0)
            elif (policy == PRIORITY and ready[1] and not held(t)
                  and not any(micros[i].kind == ALL_TO_ALL for i in on_link)):
                pick = ready[1].pop(0)
            if pick is not None:
                m = micros[pick]
                m.chosen = t
                m.start = max(link_free, m.data, t)
                m.end = m.start + m.duration
                link_free = m.end
                on_link.append(pick)
                order.append(pick)
                launched = True
        if launched:
            continue
        # nothing can be launched now: advance to the next thing that changes the state
        nxt = []
        if pending:
            nxt.append(micros[pending[0]].posted)
        nxt += [micros[i].end for i in on_link]
        nxt += [b for a, b in holds if a <= t < b]
        nxt = [v for v in nxt if v > t]
        if not nxt:
            raise RuntimeError("the policy cannot make progress (a hold that never ends?)")
        t = min(nxt)
    return [micros[i] for i in order]


def completion(ops_micros: Sequence[Micro], op: int) -> Fraction:
    """An operation's completion time: from the moment its first micro-op's data is there to
    the end of its last micro-op."""
    mine = [m for m in ops_micros if m.op == op]
    return max(m.end for m in mine) - min(m.data for m in mine)


def check_log(records: Sequence[dict], policy: int) -> None:
    """What must hold for ANY run of the policy, read off the scheduler's own record of
    launches (op, micro, kind, ready_seq, issue_seq; kind 2 = a hold call with micro = on):
      * link order is the order of the records; within one operation the micro-ops that
        were posted in ascending order leave in ascending order;
      * arrival order: launches follow ready_seq;
      * priority: when an allreduce micro-op was chosen, no all-to-all micro-op was ready
        (none has ready_seq < that issue_seq and a later launch), and no hold was on."""
    launches = [r for r in records if r["kind"] in (ALL_TO_ALL, ALLREDUCE)]
    seqs = [r["issue_seq"] for r in records]
    assert seqs == sorted(seqs), "records are not in link order"
    per_op: Dict[int, List[Tuple[int, int]]] = {}
    for r in launches:
        per_op.setdefault(r["op"], []).append((r["ready_seq"], r["micro"]))
        assert r["ready_seq"] < r["issue_seq"], "launched before it was posted"
    for op, keys in per_op.items():
        assert keys == sorted(keys), f"operation {op}: micro-ops left out of order"
        assert len(set(m for _, m in keys)) == len(keys), f"operation {op}: a micro-op left twice"
    if policy == ARRIVAL_ORDER:
        rs = [r["ready_seq"] for r in launches]
        assert rs == sorted(rs), "arrival order violated"
        return
    hold_on = False
    for idx, r in enumerate(records):
        if r["kind"] == 2:
            hold_on = bool(r["micro"])
            continue
        if r["kind"] == ALLREDUCE:
            assert not hold_on, f"allreduce micro-op launched during a hold: {r}"
            for later in records[idx + 1:]:
                if later["kind"] == ALL_TO_ALL:
                    assert later["ready_seq"] > r["issue_seq"], (
                        f"allreduce micro-op {r} overtook a ready all-to-all micro-op {later}")
    a2a = [r for r in launches if r["kind"] == ALL_TO_ALL]
    rs = [r["ready_seq"] for r in a2a]
    assert rs == sorted(rs), "all-to-all micro-ops left out of their arrival order"
