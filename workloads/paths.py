"""Seeded synthetic expert-selection traces for the popularity estimator.

The paper profiles which experts real tokens select layer by layer (Sec. 5.2) on its
datasets; none of that is available, so two seeded generators stand in for it.  They
only draw selections sel[L][T][k] (a token's k distinct experts per layer, choice 0
being the first choice); nothing here computes the estimator.

* `markov_selections`: each choice slot keeps its previous-layer expert with probability
  `stay`, otherwise draws from a Zipf(alpha) law over a seeded permutation of the
  experts -- the pattern of configuration 5 (stay = 0.7, alpha = 1.0), vectorised.
* `latent_class_selections`: every token belongs to one of `classes` latent classes
  (its "part of speech"); in every layer a class has its own preferred experts, which a
  token of the class picks with probability `fidelity`, otherwise Zipf.  A longer path
  identifies the class better, as Sec. 7.3's path-length study reports for real data.
"""
from __future__ import annotations

import numpy as np


def _zipf(E: int, alpha: float) -> np.ndarray:
    p = (np.arange(E) + 1.0) ** (-alpha)
    return p / p.sum()


def _distinct_fill(rng: np.random.Generator, out_lt: np.ndarray, want: np.ndarray,
                   perm: np.ndarray, p: np.ndarray) -> None:
    """out_lt [T,k] <- want [T,k], redrawing (Zipf over perm) any choice that repeats an
    earlier choice of the same token until all k are distinct."""
    T, k = want.shape
    out_lt[:, 0] = want[:, 0]
    for j in range(1, k):
        col = want[:, j].copy()
        while True:
            clash = (out_lt[:, :j] == col[:, None]).any(1)
            n = int(clash.sum())
            if n == 0:
                break
            col[clash] = perm[rng.choice(len(p), size=n, p=p)]
        out_lt[:, j] = col


def markov_selections(seed: int, L: int, T: int, E: int, k: int, alpha: float = 1.0,
                      stay: float = 0.7) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 501])))
    perm = rng.permutation(E).astype(np.int32)
    p = _zipf(E, alpha)
    sel = np.empty((L, T, k), np.int32)
    for l in range(L):
        fresh = perm[rng.choice(E, size=(T, k), p=p)]
        if l == 0:
            want = fresh
        else:
            keep = rng.random((T, k)) < stay
            want = np.where(keep, sel[l - 1], fresh)
        _distinct_fill(rng, sel[l], want.astype(np.int32), perm, p)
    return sel


def latent_class_selections(seed: int, L: int, T: int, E: int, k: int, classes: int = 24,
                            fidelity: float = 0.8, alpha: float = 1.0,
                            class_skew: float = 1.0) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 502])))
    perm = rng.permutation(E).astype(np.int32)
    p = _zipf(E, alpha)
    # preferred experts of each class in each layer: [L][classes][k], distinct within a class
    pref = np.empty((L, classes, k), np.int32)
    for l in range(L):
        for c in range(classes):
            pref[l, c] = rng.choice(E, size=k, replace=False)
    cls = rng.choice(classes, size=T, p=_zipf(classes, class_skew))
    sel = np.empty((L, T, k), np.int32)
    for l in range(L):
        fresh = perm[rng.choice(E, size=(T, k), p=p)]
        follow = rng.random((T, k)) < fidelity
        want = np.where(follow, pref[l][cls], fresh)
        _distinct_fill(rng, sel[l], want.astype(np.int32), perm, p)
    return sel


def trace_generator(kind: str):
    return {"markov": markov_selections, "latent": latent_class_selections}[kind]
