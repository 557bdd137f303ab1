"""Seeded synthetic knowledge graph with power-law head/tail degrees.

Stands in for the public graphs the paper trains on: only the entity,
relation and edge counts and the heavy-tailed degree distribution are
reproduced, none of their content.
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class KG:
    N: int
    R: int
    head: np.ndarray      # [T] int32, triples sorted by (tail, head, rel)
    rel: np.ndarray       # [T] int32
    tail: np.ndarray      # [T] int32
    in_off: np.ndarray    # [N+1] int64, in-edge range of every entity
    keys: np.ndarray      # [T] int64 sorted packed (head, rel, tail) for membership

    @property
    def T(self) -> int:
        return int(self.head.shape[0])

    def pack(self, h, r, t):
        return (np.asarray(h, np.int64) * self.R + np.asarray(r, np.int64)) * self.N \
            + np.asarray(t, np.int64)

    def has_triple(self, h, r, t) -> bool:
        k = int(self.pack(h, r, t))
        i = int(np.searchsorted(self.keys, k))
        return i < self.keys.shape[0] and int(self.keys[i]) == k


def make_kg(N: int, R: int, T: int, alpha: float, seed: int) -> KG:
    """Draw T distinct directed triples without self loops.

    Entity weight w = u^(-1/(alpha-1)), u ~ U(0,1], capped at T/100.  Heads and
    tails are drawn proportionally to w through two different random
    permutations of the entity ids, so that out-hubs and in-hubs differ;
    relations are uniform.
    """
    rng = np.random.default_rng(seed)
    u = 1.0 - rng.random(N)
    w = np.minimum(u ** (-1.0 / (alpha - 1.0)), T / 100.0)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    perm_h = rng.permutation(N).astype(np.int64)
    perm_t = rng.permutation(N).astype(np.int64)

    have = np.empty(0, np.int64)
    rounds = 0
    while have.shape[0] < T:
        rounds += 1
        if rounds > 200:
            raise RuntimeError("could not draw enough distinct triples")
        m = int((T - have.shape[0]) * 1.25) + 16
        h = perm_h[np.minimum(np.searchsorted(cdf, rng.random(m)), N - 1)]
        t = perm_t[np.minimum(np.searchsorted(cdf, rng.random(m)), N - 1)]
        r = rng.integers(0, R, m, dtype=np.int64)
        ok = h != t
        k = (h[ok] * R + r[ok]) * N + t[ok]
        # keep first occurrences in draw order so that the result does not
        # depend on how the remainder is topped up
        k = k[np.sort(np.unique(k, return_index=True)[1])]
        if have.shape[0]:
            k = k[~np.isin(k, have, assume_unique=False)]
        have = np.concatenate([have, k[: T - have.shape[0]]])

    keys = np.sort(have)
    t = (keys % N).astype(np.int32)
    hr = keys // N
    r = (hr % R).astype(np.int32)
    h = (hr // R).astype(np.int32)
    order = np.lexsort((r, h, t))           # by tail, then head, then relation
    h, r, t = h[order], r[order], t[order]
    in_off = np.zeros(N + 1, np.int64)
    np.cumsum(np.bincount(t, minlength=N), out=in_off[1:])
    return KG(N=N, R=R, head=h, rel=r, tail=t, in_off=in_off, keys=keys)
