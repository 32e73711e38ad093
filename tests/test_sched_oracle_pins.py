"""Pins of the scheduling oracle (popularity estimate, Eq. (1), first-fit-decreasing,
two-phase check) against things other than itself: a hand-worked example, a textbook
packing instance, brute-force optimal packing, closed forms and invariants."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import sched_oracle as so
from workloads import paths

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "sched_hand_example.json")))


def test_hand_example_tables_and_estimate():
    g = GOLD
    sel = np.array(g["profile_sel"], np.int32)
    C = so.profile_counts(sel, g["l"], g["E"])
    assert len(C) == 1
    for j in range(g["E"] ** g["l"]):
        want = g["counts_rows"].get(str(j), [0, 0, 0])
        assert C[0][j].tolist() == want
    for j, (e, q) in g["row_top1"].items():
        assert so.row_topk(C[0][int(j)], 1) == ([e], [q])
    S, listed = so.estimate(C[0], np.array(g["batch_hist"], np.int32), g["k"], g["E"])
    assert S == g["S"] and listed == g["listed"]
    n_e = [so.devices_for_expert(s, 4, g["N"]) for s in S]
    np.testing.assert_allclose(n_e, g["n_e"], rtol=1e-12)


def test_hand_example_schedule_and_phase_two():
    g = GOLD
    C = so.profile_counts(np.array(g["profile_sel"], np.int32), g["l"], g["E"])
    r = so.two_phase(C[0], np.array(g["batch_hist"], np.int32), np.array(g["actual_next"], np.int32),
                     g["E"], g["k"], g["N"], g["max_pack"])
    replicas, hosted, used = r["plan1"]
    assert hosted == g["hosted"] and replicas == g["replicas"] and used == g["devices_used"]
    assert r["identical"] is g["identical"]
    replicas2, hosted2, _ = r["plan2"]
    assert hosted2 == g["hosted2"] and replicas2 == g["replicas2"]


def test_ffd_textbook_instance():
    # sizes 0.5 0.7 0.5 0.2 0.4 0.2 0.5 0.1 0.6 (sum 3.7): first-fit-decreasing fills
    # {0.7,0.2,0.1} {0.6,0.4} {0.5,0.5} {0.5,0.2}: four devices, which is optimal
    w = [5, 7, 5, 2, 4, 2, 5, 1, 6]
    replicas, hosted, used = so.schedule(w, 10, [True] * 9, N=6, max_pack=9)
    assert used == 4
    assert hosted[:4] == [[1, 3, 7], [8, 4], [0, 2], [6, 5]]
    assert hosted[4:] == [[], []] and replicas == [1] * 9


def optimal_bins(w, W):
    n = len(w)
    for b in range(1, n + 1):
        for assign in itertools.product(range(b), repeat=n):
            load = [0] * b
            for i, a in enumerate(assign):
                load[a] += w[i]
            if max(load) <= W:
                return b
    return n


def test_ffd_against_brute_force_optimum():
    rng = np.random.Generator(np.random.PCG64(3))
    for _ in range(40):
        n = int(rng.integers(1, 7))
        W = 1000
        w = [int(v) for v in rng.integers(1, W, size=n)]      # all below one device
        _, hosted, used = so.schedule(w, W, [True] * n, N=n, max_pack=n)
        opt = optimal_bins(w, W)
        assert opt <= used <= (11 * opt + 6) // 9 + (1 if (11 * opt + 6) % 9 else 0)
        for members in hosted:                                # no device over capacity
            assert sum(w[e] for e in members) <= W
        assert sorted(e for m in hosted for e in m) == list(range(n))


def test_replication_rounding_and_packing_limit():
    W = 1000
    # 2.5 devices -> 3, 2.499 -> 2, exactly one device -> a device of its own
    replicas, hosted, used = so.schedule([2500, 2499, 1000], W, [True] * 3, N=8, max_pack=4)
    assert replicas == [3, 2, 1] and used == 6
    assert hosted[:6] == [[0], [0], [0], [1], [1], [2]]
    # at most max_pack experts share a device even when their load would fit
    replicas, hosted, used = so.schedule([10] * 6, W, [True] * 6, N=4, max_pack=4)
    assert hosted[:2] == [[0, 1, 2, 3], [4, 5]] and used == 2


def test_experts_without_estimate():
    W = 100
    # two free devices: the three unestimated experts go round-robin onto them
    _, hosted, used = so.schedule([60, 0, 50, 0, 0], W, [True, False, True, False, False], N=4,
                                  max_pack=4)
    assert used == 2 and hosted == [[0], [2], [1, 4], [3]]
    # no free device: expert e goes to device e mod N
    _, hosted, used = so.schedule([60, 0, 50, 0, 0], W, [True, False, True, False, False], N=2,
                                  max_pack=4)
    assert used == 2 and hosted == [[0, 4], [2, 1, 3]]      # 1 -> 1, 3 -> 1, 4 -> 0


def test_oversubscription_wraps():
    W = 10
    replicas, hosted, used = so.schedule([25, 14, 6, 6], W, [True] * 4, N=3, max_pack=4)
    # 3 + 1 devices of their own, then {6} and {6} cannot share (12 > 10): 6 groups on 3 devices
    assert replicas == [3, 1, 1, 1] and used == 3
    assert hosted == [[0, 1], [0, 2], [0, 3]]


def test_replication_is_capped_at_the_device_count():
    """Sec. 5.2 replicates a popular expert on more devices; it cannot sit on more devices
    than exist.  Hand-worked: w = 25, W = 10 asks for round(2.5) = 3 devices, N = 2 gives 2."""
    replicas, hosted, used = so.schedule([25], 10, [True], N=2, max_pack=4)
    assert replicas == [2] and hosted == [[0], [0]] and used == 2
    # one device short: 3.4 -> 3 wanted, 3 exist -> 3; 3.5 -> 4 wanted, 3 exist -> 3
    assert so.schedule([34], 10, [True], N=3, max_pack=4)[0] == [3]
    assert so.schedule([35], 10, [True], N=3, max_pack=4)[0] == [3]
    # the cap is per expert: a second expert still gets its own (wrapped) device, and every
    # device hosts each expert at most once
    replicas, hosted, used = so.schedule([90, 10, 4], 10, [True] * 3, N=2, max_pack=4)
    assert replicas == [2, 1, 1] and used == 2
    assert hosted == [[0, 1], [0, 2]]
    # Eq. (1) side of the same case: all N_t tokens expect expert 0 with probability 1 on N = 2
    # devices -> n_0 = N = 2 exactly, never more
    assert so.devices_for_expert(5 << so.FIX, 5, 2) == 2.0


def test_top_lists():
    assert so.top_list([5, 9, 9, 1], 3) == [1, 2, 0]
    assert so.lists_identical([5, 9, 9, 1], [50, 90, 91, 10], 1) is False      # order matters
    assert so.lists_identical([5, 9, 8, 1], [50, 90, 80, 10], 1) is True
    assert so.lists_identical([3, 1], [7, 2], 2) is True                       # E < 2k


@pytest.mark.parametrize("kind,k", [("markov", 1), ("markov", 2), ("latent", 2)])
def test_table_invariants(kind, k):
    L, T, E, l = 6, 3000, 8, 2
    sel = paths.trace_generator(kind)(1, L, T, E, k)
    assert sel.shape == (L, T, k) and sel.min() >= 0 and sel.max() < E
    assert all(len(set(sel[i, t])) == k for i in range(L) for t in range(0, T, 97))
    C = so.profile_counts(sel, l, E)
    assert len(C) == L - l
    for a, Ci in enumerate(C):
        i = a + l - 1
        assert int(Ci.sum()) == T * k
        # a path's row total is k times the number of tokens on that path
        keys = sel[i - 1, :, 0] * E + sel[i, :, 0]
        assert np.array_equal(Ci.sum(1), k * np.bincount(keys, minlength=E ** l))
        for j in range(0, E ** l, 5):
            experts, probs = so.row_topk(Ci[j], k)
            tot = int(Ci[j].sum())
            assert len(experts) == min(k, int((Ci[j] > 0).sum()))
            for e, q in zip(experts, probs):
                assert q <= (int(Ci[j][e]) << 32) / tot < q + 1
            cs = [int(Ci[j][e]) for e in experts]
            assert cs == sorted(cs, reverse=True) and (not cs or cs[-1] >= max(
                [int(c) for e, c in enumerate(Ci[j]) if e not in experts] or [0]))
        S, listed = so.estimate(Ci, sel[i - l + 1:i + 1], k, E)
        assert sum(S) <= T << 32 and all(0 <= s <= T << 32 for s in S)
        assert all((s > 0) == f for s, f in zip(S, listed))


def test_deterministic_paths_are_estimated_exactly():
    # every token repeats its expert in every layer: each profiled path has a one-hot
    # next-layer distribution, the estimate equals the actual popularity, no fine-tuning
    rng = np.random.Generator(np.random.PCG64(8))
    E, L, l, T = 6, 5, 3, 500
    first = rng.integers(0, E, size=T).astype(np.int32)
    sel = np.repeat(first[None, :, None], L, axis=0)
    C = so.profile_counts(sel, l, E)
    r = so.two_phase(C[0], sel[0:l], sel[l], E, 1, N=E, max_pack=4)
    assert r["S"] == [int(c) << 32 for c in np.bincount(first, minlength=E)]
    assert r["identical"] and r["plan2"] is None
    # Eq. (1) closed form: n_e = N * count_e / N_t
    for e in range(E):
        assert so.devices_for_expert(r["S"][e], T, E) == pytest.approx(E * r["counts"][e] / T, rel=1e-12)
    # scheduling from the estimate and from the actual popularity agree
    assert so.schedule([E * s for s in r["S"]], T << 32, r["listed"], E, 4) == \
        so.schedule([E * c for c in r["counts"]], T, [c > 0 for c in r["counts"]], E, 4)


def test_path_length_carries_the_history():
    # A trace whose next expert is a function of the last TWO first choices,
    # e_{i+1} = (e_i + 2 e_{i-1} + 1) mod E: sample paths of length 2 have one-hot
    # distributions and estimate every batch exactly; paths of length 1 cannot.  (A path
    # index that dropped or swapped a layer of history fails the first half.)
    rng = np.random.Generator(np.random.PCG64(12))
    E, L, T = 7, 6, 4000
    sel = np.empty((L, T, 1), np.int32)
    sel[0, :, 0] = rng.integers(0, E, T)
    sel[1, :, 0] = rng.integers(0, E, T)
    for i in range(1, L - 1):
        sel[i + 1] = (sel[i] + 2 * sel[i - 1] + 1) % E
    prof, batch = sel[:, :3000], sel[:, 3000:]
    C2 = so.profile_counts(prof, 2, E)
    for a, Ci in enumerate(C2):
        i = a + 1
        assert ((Ci > 0).sum(1) <= 1).all()
        S, _ = so.estimate(Ci, batch[i - 1:i + 1], 1, E)
        counts = np.bincount(batch[i + 1].reshape(-1), minlength=E)
        assert S == [int(c) << 32 for c in counts]
        assert so.lists_identical(S, counts, 1)
    C1 = so.profile_counts(prof, 1, E)
    exact = []
    for a, Ci in enumerate(C1):
        S, _ = so.estimate(Ci, batch[a:a + 1], 1, E)
        counts = np.bincount(batch[a + 1].reshape(-1), minlength=E)
        exact.append(S == [int(c) << 32 for c in counts])
    assert not any(exact)
