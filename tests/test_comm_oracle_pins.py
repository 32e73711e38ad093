"""Pins of oracle/comm_oracle.py: the padded layout against the count-earlier definition,
the compact plan and closed forms; the scheduling policy against closed forms in exact
rational time (paper Sec. 4.2: an all-to-all never waits for more than the micro-ops already
on the link; allreduce uses every gap)."""
import itertools
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import comm_oracle as co
from oracle import moe_oracle as fo


# ----------------------------------------------------------------------------- padded layout
def brute_padded(idx, E, C):
    flat = idx.reshape(-1)
    slot = np.full(flat.size, -1, np.int32)
    for i in range(flat.size):
        pos = sum(1 for j in range(i) if flat[j] == flat[i])        # the definition, O(n^2)
        if pos < C:
            slot[i] = flat[i] * C + pos
    return slot


def test_padded_plan_is_the_count_earlier_definition_on_every_tiny_case():
    for T, E, k in ((4, 2, 1), (3, 3, 2), (5, 2, 2)):
        choices = [c for c in itertools.permutations(range(E), k)]
        for pick in itertools.product(range(len(choices)), repeat=T):
            idx = np.array([choices[p] for p in pick], np.int32)
            for C in range(1, T + 1):
                counts, slot_of, src_of = co.padded_plan(idx, E, C)
                assert np.array_equal(slot_of, brute_padded(idx, E, C))
                assert np.array_equal(counts, np.bincount(idx.reshape(-1), minlength=E))
                held = np.nonzero(src_of >= 0)[0]
                assert np.array_equal(slot_of[src_of[held]], held)          # inverse of each other
                assert held.size == np.minimum(counts, C).sum()


def test_padded_slots_are_the_compact_slots_shifted_per_expert():
    rng = np.random.Generator(np.random.PCG64(5))
    for T, E, k, C in ((300, 8, 2, 60), (257, 5, 1, 40), (64, 4, 3, 64)):
        idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
        counts, slot_p, src_p = co.padded_plan(idx, E, C)
        count_c, off, slot_c, src_c = fo.plan(idx, E, C)
        assert np.array_equal(counts, count_c)
        e = idx.reshape(-1)
        kept = slot_c >= 0
        assert np.array_equal(slot_p >= 0, kept)
        assert np.array_equal(slot_p[kept] - e[kept] * C, slot_c[kept] - off[e[kept]])
        for ee in range(E):                                                 # stability inside an expert
            mine = src_p[ee * C:(ee + 1) * C]
            n = min(counts[ee], C)
            assert (mine[:n] >= 0).all() and (np.diff(mine[:n]) > 0).all() and (mine[n:] == -1).all()


def test_padded_closed_forms():
    T, E, C = 40, 4, 7
    idx = (np.arange(T) % E).astype(np.int32).reshape(T, 1)                # round robin
    counts, slot_of, _ = co.padded_plan(idx, E, C)
    t = np.arange(T)
    want = np.where(t // E < C, (t % E) * C + t // E, -1)
    assert np.array_equal(slot_of, want) and (counts == T // E).all()
    idx = np.zeros((T, 1), np.int32)                                       # everyone picks expert 0
    counts, slot_of, src_of = co.padded_plan(idx, E, C)
    assert np.array_equal(slot_of, np.where(t < C, t, -1)) and counts[0] == T
    assert (src_of[C:] == -1).all()


def test_pack_padded_rows_and_zero_padding():
    rng = np.random.Generator(np.random.PCG64(9))
    T, E, k, C, d = 50, 4, 2, 20, 8
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    x = rng.standard_normal((T, d)).astype(np.float32)
    counts, slot_of, src_of = co.padded_plan(idx, E, C)
    xs = co.pack_padded(x, src_of, k)
    assert xs.shape == (E * C, d)
    for i, s in enumerate(slot_of):
        if s >= 0:
            assert np.array_equal(xs[s], x[i // k])
    empty = src_of < 0
    assert not xs[empty].any() and empty.sum() == E * C - np.minimum(counts, C).sum()


def test_micro_ranges_and_the_order_on_an_own_link():
    for C, n in ((640, 4), (10, 3), (7, 7), (1024, 8), (5, 1)):
        r = co.micro_ranges(C, n)
        assert r[0][0] == 0 and r[-1][1] == C
        assert all(a[1] == b[0] for a, b in zip(r, r[1:]))
        sizes = [b - a for a, b in r]
        assert max(sizes) - min(sizes) <= 1
    for n in (1, 2, 5):
        order = co.static_link_order(n)
        assert sorted(order) == [(a, m) for a in (0, 1) for m in range(n)]
        at = {v: i for i, v in enumerate(order)}
        for m in range(n):
            assert at[(0, m)] < at[(1, m)]                       # a micro-op returns after it went
            if m + 1 < n:
                assert at[(0, m + 1)] < at[(1, m)]               # the first all-to-all stays ahead
                assert at[(0, m)] < at[(0, m + 1)] and at[(1, m)] < at[(1, m + 1)]


# ----------------------------------------------------------------------------- scheduling policy
def cut(op, kind, posted, total, n, data=None):
    d = posted if data is None else data
    return [co.Micro(op, m, kind, F(posted), F(d), F(total, n)) for m in range(n)]


def test_an_operation_alone_takes_its_bytes_whatever_the_cut():
    for n in (1, 3, 8):
        for policy in (co.ARRIVAL_ORDER, co.PRIORITY):
            out = co.simulate(cut(1, co.ALLREDUCE, 2, 12, n), policy)
            assert [m.micro for m in out] == list(range(n))
            assert out[0].start == 2 and co.completion(out, 1) == 12


def test_arrival_order_makes_the_all_to_all_wait_for_the_whole_allreduce():
    L, S, t0 = 30, 4, 7
    ms = cut(1, co.ALLREDUCE, 0, L, 1) + cut(2, co.ALL_TO_ALL, t0, S, 2)
    out = co.simulate(ms, co.ARRIVAL_ORDER)
    assert co.completion(out, 2) == L + S - t0                  # blocked behind the allreduce


def test_priority_bounds_the_wait_by_the_micro_ops_on_the_link():
    L, S, n = 30, 4, 10                                          # allreduce micro-op: 3
    for depth in (1, 2, 3):
        for t0 in (F(1, 2), F(7), F(9), F(29)):
            ms = cut(1, co.ALLREDUCE, 0, L, n) + cut(2, co.ALL_TO_ALL, t0, S, 2)
            out = co.simulate(ms, co.PRIORITY, depth=depth)
            wait = min(m.start for m in out if m.op == 2) - t0
            assert 0 <= wait <= depth * F(L, n)
            if depth == 1:                                       # exactly to the end of the running one
                assert wait == -(-t0 // 3) * 3 - t0
            # the link never idles while something is ready: everything ends at L + S
            assert max(m.end for m in out) == L + S
            for a, b in zip(out, out[1:]):
                assert b.start >= a.end                          # one micro-op at a time
            # the allreduce is deferred by the all-to-all's time, not more (not at all when
            # its last micro-op was already on the link)
            assert max(m.end for m in out if m.op == 1) == (L + S if t0 <= 9 else L)


def test_priority_with_everything_ready_sends_the_all_to_alls_first():
    ms = (cut(1, co.ALLREDUCE, 0, 6, 6) + cut(2, co.ALL_TO_ALL, 0, 3, 3) + cut(3, co.ALLREDUCE, 0, 2, 2)
          + cut(4, co.ALL_TO_ALL, 0, 2, 2))
    out = co.simulate(ms, co.PRIORITY)
    assert [(m.op, m.micro) for m in out] == ([(2, 0), (2, 1), (2, 2), (4, 0), (4, 1)] +
                                              [(1, i) for i in range(6)] + [(3, 0), (3, 1)])
    out = co.simulate(ms, co.ARRIVAL_ORDER)
    assert [m.op for m in out] == [1] * 6 + [2] * 3 + [3] * 2 + [4] * 2


def test_allreduce_uses_the_gap_between_the_two_all_to_alls_but_not_a_hold():
    # first all-to-all at 0..4, expert computation until 10, second all-to-all posted at 10
    a2a = cut(2, co.ALL_TO_ALL, 0, 4, 1) + cut(3, co.ALL_TO_ALL, 10, 4, 1)
    ar = cut(1, co.ALLREDUCE, 0, 12, 6)                          # micro-ops of 2
    out = co.simulate(ar + a2a, co.PRIORITY)
    in_gap = [m for m in out if m.op == 1 and m.start >= 4 and m.end <= 10]
    assert len(in_gap) == 3                                      # 4..6, 6..8, 8..10
    assert min(m.start for m in out if m.op == 3) == 10          # and the second one starts on time
    # the caller announces the second all-to-all at 7: nothing new after that
    out = co.simulate(cut(1, co.ALLREDUCE, 0, 12, 6) + cut(2, co.ALL_TO_ALL, 0, 4, 1)
                      + cut(3, co.ALL_TO_ALL, 10, 4, 1), co.PRIORITY, holds=[(F(7), F(10))])
    assert not [m for m in out if m.op == 1 and 7 <= m.chosen < 10]
    assert len([m for m in out if m.op == 1 and m.end <= 10]) == 2


def test_a_posted_micro_op_whose_data_is_late_keeps_the_link():
    # posted at 0, data at 5: it is launched at once and the link waits with it
    ms = cut(2, co.ALL_TO_ALL, 0, 2, 1, data=5) + cut(1, co.ALLREDUCE, 0, 4, 2)
    out = co.simulate(ms, co.PRIORITY)
    assert [(m.op, m.start) for m in out] == [(2, 5), (1, 7), (1, 9)]
    assert co.completion(out, 2) == 2


def test_check_log_accepts_a_run_of_the_policy_and_catches_planted_mistakes():
    def rec(op, micro, kind, ready, issue):
        return dict(op=op, micro=micro, kind=kind, bytes=16, ready_seq=ready, issue_seq=issue)
    good = [rec(1, 0, 1, 0, 1), rec(2, 0, 0, 2, 3), rec(2, 1, 0, 2, 4), rec(1, 1, 1, 0, 5)]
    co.check_log(good, co.PRIORITY)
    overtaken = [rec(1, 0, 1, 0, 2), rec(1, 1, 1, 0, 3), rec(2, 0, 0, 1, 4)]   # a2a ready at 1, AR chosen at 3
    with pytest.raises(AssertionError):
        co.check_log(overtaken, co.PRIORITY)
    co.check_log(overtaken, co.ARRIVAL_ORDER)
    with pytest.raises(AssertionError):
        co.check_log(good, co.ARRIVAL_ORDER)
    held = [dict(op=-1, micro=1, kind=2, bytes=0, ready_seq=1, issue_seq=1), rec(1, 0, 1, 0, 2)]
    with pytest.raises(AssertionError):
        co.check_log(held, co.PRIORITY)
    twice = [rec(1, 0, 1, 0, 1), rec(1, 0, 1, 0, 2)]
    with pytest.raises(AssertionError):
        co.check_log(twice, co.PRIORITY)
