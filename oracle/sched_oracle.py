"""CPU oracle of the popularity-based expert scheduling (paper Sec. 5.2): profiled
sample-path tables, the per-batch popularity estimate, Eq. (1), first-fit-decreasing
packing and the two-phase check.

TEST INFRASTRUCTURE ONLY: plain Python loops over exact integers, written from the
paper's description; nothing in the product path imports it.  It shares no code with
the HIP/C++ side.

Notation (paper's): L MoE layers, E experts, k experts per token, l the sample-path
length, N devices, N_t tokens in the batch.  sel[i][t][j] is the j-th choice of token t
in layer i (j = 0 the first choice).  Where the paper leaves a choice open the reading
taken is stated at the function; all of them are listed in the design notes.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

FIX = 32   # probabilities are held in 2^-32 fixed point so that batch sums are exact


def path_index(sel: np.ndarray, i: int, t: int, l: int, E: int) -> int:
    """Sample path of token t ending at layer i (Sec. 5.2, "Estimating expert popularity"):
    the first-choice experts of layers i-l+1 .. i, read as an l-digit number in base E,
    oldest layer first.  (Reading: with k > 1 the path follows the first choice only; the
    paper's inference runs use k = 1.)"""
    j = 0
    for m in range(i - l + 1, i + 1):
        e = int(sel[m][t][0])
        if not 0 <= e < E:
            return -1          # (reading: a token carrying a non-expert id, e.g. padding, is skipped)
        j = j * E + e
    return j


def profile_counts(sel: np.ndarray, l: int, E: int) -> List[np.ndarray]:
    """Profiling stage: for every layer i that has l layers of history and a successor
    (i = l-1 .. L-2), group the profiled tokens by their sample path j and count which
    experts they select in layer i+1 (all k choices count).  Returns C with
    C[i-(l-1)][j][e]; the distribution Psi_j^{i+1}(e) is C / sum_e C."""
    L, T, k = sel.shape
    out = []
    for i in range(l - 1, L - 1):
        C = np.zeros((E ** l, E), dtype=np.int64)
        for t in range(T):
            j = path_index(sel, i, t, l, E)
            if j < 0 or any(not 0 <= int(sel[i + 1][t][c]) < E for c in range(k)):
                continue
            for c in range(k):
                C[j][int(sel[i + 1][t][c])] += 1
        out.append(C)
    return out


def row_topk(row: Sequence[int], k: int) -> Tuple[List[int], List[int]]:
    """Top-k experts of one sample path's distribution and their probabilities
    {P_j^{i+1}(e)} in 2^-32 fixed point, floor(count * 2^32 / total).  Ties go to the lower
    expert index; experts the path never selected are not listed (a path that was never
    profiled lists nothing)."""
    tot = int(sum(int(c) for c in row))
    order = sorted(range(len(row)), key=lambda e: (-int(row[e]), e))
    experts, probs = [], []
    for e in order[:k]:
        if int(row[e]) > 0:
            experts.append(e)
            probs.append((int(row[e]) << FIX) // tot)
    return experts, probs


def estimate(C: np.ndarray, sel_hist: np.ndarray, k: int, E: int) -> Tuple[List[int], List[bool]]:
    """Popularity estimate for the layer after the history sel_hist[l][N_t][k] (the batch's
    selections in the last l layers): S(e) = sum over tokens t of P_{j(t)}(e) over the
    top-k experts of each token's path, in 2^-32 fixed point (the sum of Eq. (1) before
    the division by N_t); listed[e] tells whether e was in any token's top-k list."""
    l, T, _ = sel_hist.shape
    S = [0] * E
    listed = [False] * E
    for t in range(T):
        j = path_index(sel_hist, l - 1, t, l, E)
        if j < 0:
            continue
        experts, probs = row_topk(C[j], k)
        for e, q in zip(experts, probs):
            S[e] += q
            listed[e] = True
    return S, listed


def devices_for_expert(S_e: int, N_t: int, N: int) -> float:
    """Eq. (1): n_e = N * sum_t P(e) / N_t."""
    return N * (S_e / float(1 << FIX)) / N_t


def schedule(w: Sequence[int], W: int, has: Sequence[bool], N: int, max_pack: int):
    """Phase-1 resource scheduling from integer weights: n_e = w[e] / W devices for expert e
    (Eq. (1) with w = N * S and W = N_t * 2^32; or, with the actual popularity, w = N * count
    and W = N_t * k).

    Readings of what the paper leaves open:
    * an expert with n_e >= 1 is replicated on round-half-up(n_e) devices of its own (at
      most N);
    * experts with n_e < 1 are items of size n_e for first-fit-decreasing into devices of
      capacity 1 holding at most max_pack experts (Sec. 7.1: 4); order: size descending,
      then expert index;
    * experts without an estimate go evenly (round-robin in index order) onto the devices
      left free, or, if none is free, expert e goes to device e mod N (a deterministic
      stand-in for the paper's random choice);
    * if the estimate asks for more than N devices, device numbers wrap modulo N.
    Returns (replicas[e], hosted[d] = list of experts of device d, devices_used = devices
    that host estimated experts)."""
    E = len(w)
    replicas = [0] * E
    groups: List[List[int]] = []          # experts of each device, in device order
    small = []
    for e in range(E):
        if not has[e]:
            continue
        if w[e] >= W:
            r = min((2 * w[e] + W) // (2 * W), N)
            replicas[e] = r
            for _ in range(r):
                groups.append([e])
        else:
            small.append(e)
    small.sort(key=lambda e: (-w[e], e))
    bins: List[List[int]] = []
    load: List[int] = []
    for e in small:
        for b in range(len(bins)):
            if load[b] + w[e] <= W and len(bins[b]) < max_pack:
                bins[b].append(e)
                load[b] += w[e]
                break
        else:
            bins.append([e])
            load.append(w[e])
        replicas[e] = 1
    groups.extend(bins)
    used = len(groups)
    hosted: List[List[int]] = [[] for _ in range(N)]
    for g, members in enumerate(groups):
        for e in members:
            if e not in hosted[g % N]:
                hosted[g % N].append(e)
    rest = [e for e in range(E) if not has[e]]
    free = N - used
    for m, e in enumerate(rest):
        d = used + (m % free) if free > 0 else e % N
        hosted[d].append(e)
        replicas[e] = 1
    return replicas, hosted, min(used, N)


def top_list(scores: Sequence[int], m: int) -> List[int]:
    """The m most popular experts, most popular first, ties to the lower index."""
    return sorted(range(len(scores)), key=lambda e: (-int(scores[e]), e))[:m]


def lists_identical(S: Sequence[int], counts: Sequence[int], k: int) -> bool:
    """Phase-2 check: are the overall top-2k experts of the estimate and of the actual
    selection the same list (same experts, same order)?"""
    m = min(2 * k, len(S))
    return top_list(S, m) == top_list(counts, m)


def two_phase(C: np.ndarray, sel_hist: np.ndarray, sel_next: np.ndarray, E: int, k: int, N: int,
              max_pack: int):
    """One MoE layer of the inference scheduler: phase 1 schedules from the estimate; phase 2
    compares the top-2k lists once the gate has selected (sel_next[N_t][k]) and, if they
    differ, schedules again from the actual popularity.  Returns a dict of every
    intermediate so that tests can compare piece by piece."""
    N_t = sel_hist.shape[1]
    S, listed = estimate(C, sel_hist, k, E)
    w1 = [N * s for s in S]
    W1 = N_t << FIX
    plan1 = schedule(w1, W1, listed, N, max_pack)
    counts = [0] * E
    for t in range(N_t):
        for c in range(k):
            counts[int(sel_next[t][c])] += 1
    same = lists_identical(S, counts, k)
    plan2 = None
    if not same:
        w2 = [N * c for c in counts]
        plan2 = schedule(w2, N_t * k, [c > 0 for c in counts], N, max_pack)
    return dict(S=S, listed=listed, plan1=plan1, counts=counts, identical=same, plan2=plan2)
