"""Parity of the scheduling kernels (sample-path tables, top-k rows, popularity estimate)
with the scheduling oracle: every output is an integer and must match bit for bit."""
import numpy as np
import pytest
import torch

import paper_2210_17223_amd as moe
from oracle import sched_oracle as so
from workloads import paths

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    # kind,    L,  T,     E,  k, l
    ("markov", 6,  20000, 8,  2, 3),
    ("latent", 12, 6000,  16, 1, 3),
    ("markov", 4,  5000,  64, 2, 2),
    ("latent", 5,  3000,  5,  3, 1),
    ("markov", 3,  1,     4,  1, 2),
]


def u64(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


@pytest.mark.parametrize("kind,L,T,E,k,l", CASES)
def test_tables_estimate_and_schedule(kind, L, T, E, k, l):
    sel = paths.trace_generator(kind)(3, L, T, E, k)
    if T > 100:                                    # some non-expert ids (padding tokens)
        sel[1, 5, 0] = -1
        sel[L - 1, 17, k - 1] = E
        sel[0, 40, 0] = E + 3
    s = moe.PathShape(L, E, k, l)
    P = moe.moe_path_count(s)
    assert P == E ** l
    tables = L - l
    counts = torch.zeros(tables * P * E, dtype=torch.int32, device=DEV)
    # profiling in two batches adds up
    cut = T // 3
    for lo, hi in ((0, cut), (cut, T)):
        if hi > lo:
            part = torch.from_numpy(np.ascontiguousarray(sel[:, lo:hi])).to(DEV)
            moe.moe_path_profile(s, part, hi - lo, counts)
    top_e = torch.empty(tables * P * k, dtype=torch.int32, device=DEV)
    top_q = torch.empty(tables * P * k, dtype=torch.int64, device=DEV)
    moe.moe_path_finalize(s, counts, top_e, top_q)
    torch.cuda.synchronize()

    C = so.profile_counts(sel, l, E)
    got_C = counts.cpu().numpy().view(np.uint32).reshape(tables, P, E)
    for a in range(tables):
        assert np.array_equal(got_C[a].astype(np.int64), C[a])
    got_e = top_e.cpu().numpy().reshape(tables, P, k)
    got_q = u64(top_q).reshape(tables, P, k)
    rows = range(P) if P <= 4096 else list(range(0, P, 7)) + [P - 1]
    for a in range(tables):
        for j in rows:
            experts, probs = so.row_topk(C[a][j], k)
            pad = k - len(experts)
            assert got_e[a, j].tolist() == experts + [-1] * pad
            assert got_q[a, j].tolist() == probs + [0] * pad

    # estimate for held-out batches of several sizes, then both scheduling phases
    S_dev = torch.empty(E, dtype=torch.int64, device=DEV)
    for b, N_t in enumerate([1, 63, 257, 1500]):
        batch = paths.trace_generator(kind)(50 + b, L, N_t, E, k)
        if N_t > 10:
            batch[0, 3, 0] = -1
        for a in range(tables):
            hist = np.ascontiguousarray(batch[a:a + l])
            moe.moe_popularity_estimate(s, torch.from_numpy(hist).to(DEV), N_t,
                                        top_e[a * P * k:(a + 1) * P * k],
                                        top_q[a * P * k:(a + 1) * P * k], S_dev)
            torch.cuda.synchronize()
            S = u64(S_dev)
            want_S, listed = so.estimate(C[a], hist, k, E)
            assert S.tolist() == want_S
            assert [int(v) > 0 for v in S] == listed
            nxt = batch[a + l]
            cnts = np.bincount(nxt[(nxt >= 0) & (nxt < E)].reshape(-1), minlength=E).astype(np.int32)
            N = E
            rep, cnt, dev, used, again = moe.moe_schedule_layer(N, E, k, N_t, S, cnts, 4)
            same = so.lists_identical(want_S, cnts.tolist(), k)
            assert again is (not same)
            if same:
                want = so.schedule([N * v for v in want_S], N_t << 32, listed, N, 4)
            else:
                want = so.schedule([N * int(c) for c in cnts], N_t * k, [c > 0 for c in cnts], N, 4)
            hosted = [list(map(int, dev[d, :cnt[d]])) for d in range(N)]
            assert (list(map(int, rep)), hosted, used) == want


def test_estimate_of_an_empty_batch_and_unprofiled_paths():
    s = moe.PathShape(4, 6, 2, 2)
    P = moe.moe_path_count(s)
    top_e = torch.full((P * 2,), -1, dtype=torch.int32, device=DEV)
    top_q = torch.zeros(P * 2, dtype=torch.int64, device=DEV)
    S = torch.full((6,), 77, dtype=torch.int64, device=DEV)
    hist = torch.zeros(2 * 10 * 2, dtype=torch.int32, device=DEV)
    moe.moe_popularity_estimate(s, hist, 0, top_e, top_q, S)          # no tokens: S is cleared
    torch.cuda.synchronize()
    assert not S.cpu().numpy().any()
    S.fill_(5)
    moe.moe_popularity_estimate(s, hist, 10, top_e, top_q, S)         # nothing profiled: all zero
    torch.cuda.synchronize()
    assert not S.cpu().numpy().any()
