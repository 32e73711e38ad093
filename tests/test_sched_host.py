"""The host-side scheduling functions of the library (Eq. (1), first-fit-decreasing
packing, top-2k list check, both phases for a layer) against the scheduling oracle.
They touch no GPU, so this runs everywhere the library loads."""
import json
import os

import numpy as np
import pytest

import paper_2210_17223_amd as moe
from oracle import sched_oracle as so

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "sched_hand_example.json")))


def as_lists(cnt, dev):
    return [list(map(int, dev[d, :cnt[d]])) for d in range(len(cnt))]


def check_schedule(N, E, w, W, has, max_pack):
    rep, cnt, dev, used = moe.moe_schedule_experts(N, E, w, W, has, max_pack)
    want_rep, want_hosted, want_used = so.schedule(list(map(int, w)), int(W), list(map(bool, has)), N,
                                                  max_pack)
    assert list(map(int, rep)) == want_rep
    assert as_lists(cnt, dev) == want_hosted
    assert used == want_used
    for d in range(N):
        assert (dev[d, cnt[d]:] == -1).all()


def test_hand_example():
    g = GOLD
    N, E, N_t = g["N"], g["E"], 4
    for s, want in zip(g["S"], g["n_e"]):
        assert moe.moe_devices_for_expert(s, N_t, N) == pytest.approx(want, rel=1e-12)
    w = [N * s for s in g["S"]]
    rep, cnt, dev, used = moe.moe_schedule_experts(N, E, w, N_t << 32, g["listed"], g["max_pack"])
    assert as_lists(cnt, dev) == g["hosted"] and list(rep) == g["replicas"] and used == g["devices_used"]
    counts = np.bincount(np.array(g["actual_next"]).reshape(-1), minlength=E)
    assert moe.moe_top_lists_identical(E, g["k"], g["S"], counts) is g["identical"]
    rep, cnt, dev, used, again = moe.moe_schedule_layer(N, E, g["k"], N_t, g["S"], counts, g["max_pack"])
    assert again and as_lists(cnt, dev) == g["hosted2"] and list(rep) == g["replicas2"]


def test_textbook_packing():
    rep, cnt, dev, used = moe.moe_schedule_experts(6, 9, [5, 7, 5, 2, 4, 2, 5, 1, 6], 10, [1] * 9, 9)
    assert used == 4 and as_lists(cnt, dev)[:4] == [[1, 3, 7], [8, 4], [0, 2], [6, 5]]


def test_random_schedules_match_the_oracle():
    rng = np.random.Generator(np.random.PCG64(21))
    for _ in range(300):
        E = int(rng.integers(1, 65))
        N = int(rng.integers(1, 40))
        W = int(rng.integers(1, 5000))
        style = rng.integers(0, 3)
        if style == 0:       # everything below one device
            w = rng.integers(0, W + 1, size=E)
        elif style == 1:     # a few heavy experts
            w = rng.integers(0, W // 4 + 2, size=E)
            heavy = rng.random(E) < 0.15
            w = np.where(heavy, rng.integers(W, (60 if rng.random() < 0.2 else 6) * W + 1, size=E), w)
        else:                # many ties
            w = rng.choice([0, W // 3, W // 2, W, 3 * W // 2], size=E)
        has = (rng.random(E) < 0.8) & (w > 0) if style != 2 else rng.random(E) < 0.7
        check_schedule(N, E, w.astype(np.uint64), W, has.astype(np.uint8), int(rng.integers(1, 6)))


def test_top_lists_and_layer_decision_match_the_oracle():
    rng = np.random.Generator(np.random.PCG64(22))
    for _ in range(300):
        E = int(rng.integers(1, 33))
        k = int(rng.integers(1, 4))
        N = int(rng.integers(1, 20))
        N_t = int(rng.integers(1, 3000))
        counts = rng.multinomial(N_t * k, rng.dirichlet(np.ones(E) * 0.5)).astype(np.int32)
        if rng.random() < 0.5:          # an estimate that ranks like the actual selection
            S = (counts.astype(np.uint64) << np.uint64(32)) // np.uint64(k)
            S = np.where(rng.random(E) < 0.1, np.uint64(0), S)
        else:
            S = (rng.integers(0, N_t + 1, size=E).astype(np.uint64) << np.uint64(32)) // np.uint64(E)
        same = so.lists_identical(list(map(int, S)), list(map(int, counts)), k)
        assert moe.moe_top_lists_identical(E, k, S, counts) is same
        rep, cnt, dev, used, again = moe.moe_schedule_layer(N, E, k, N_t, S, counts, 4)
        assert again is (not same)
        if same:
            want = so.schedule([N * int(s) for s in S], N_t << 32, [int(s) > 0 for s in S], N, 4)
        else:
            want = so.schedule([N * int(c) for c in counts], N_t * k, [int(c) > 0 for c in counts], N, 4)
        assert (list(map(int, rep)), as_lists(cnt, dev), used) == want


def test_refusals():
    with pytest.raises(moe.MoeError):
        moe.moe_schedule_experts(0, 4, [1, 1, 1, 1], 4, [1, 1, 1, 1], 4)       # no device
    with pytest.raises(moe.MoeError):
        moe.moe_schedule_experts(2, 4, [1, 1, 1, 1], 0, [1, 1, 1, 1], 4)       # W = 0
    with pytest.raises(moe.MoeError):
        moe.moe_schedule_layer(1 << 16, 4, 1, 1 << 16, [0] * 4, [0] * 4, 4)    # weights overflow
    s = moe.PathShape(4, 64, 1, 5)                                             # 64^5 paths
    assert moe.moe_path_count(s) == 0
    assert moe.moe_path_count(moe.PathShape(12, 16, 2, 3)) == 4096
