"""Synthetic knowledge graphs and embedding tables (inputs only; none of the method's arithmetic).

The paper's datasets (Table 3: FB15k, WN18, Freebase) are not available here, so the workloads are
stand-ins with the same entity / relation / triple counts and a power-law degree skew:

  * the rank rho in [1, n] of an endpoint is drawn with probability proportional to rho**(-s)
    (inverse CDF over a prefix table, binary search); heads and tails are independent;
  * the entity id is a fixed bijection of the rank, ``(rank * A + B) mod n``, so that frequently used rows
    are spread over the table instead of sitting next to each other;
  * relations are uniform, or drawn the same way with their own exponent;
  * self loops and repeated triples are allowed.

Embedding tables follow the initialisation the configurations state: uniform in
[-(gamma + 2) / dim, +(gamma + 2) / dim]; RotatE relation rows hold phases uniform in [-pi, pi).
"""
from __future__ import annotations

import math

import numpy as np

_SCRAMBLE_A = 2_654_435_761  # odd prime; coprime with every entity count used here (checked at run time)
_SCRAMBLE_B = 1_013_904_223


class ZipfTable:
    """P(rank = rho) proportional to rho**(-s) for rho = 1..n; ``sample`` maps uniforms to 0-based ranks."""

    def __init__(self, n: int, s: float):
        self.n, self.s = int(n), float(s)
        w = np.arange(1, self.n + 1, dtype=np.float64) ** (-self.s)
        self.cdf = np.cumsum(w)
        self.cdf /= self.cdf[-1]

    def sample(self, u: np.ndarray) -> np.ndarray:
        r = np.searchsorted(self.cdf, u, side="right")
        return np.minimum(r, self.n - 1).astype(np.int64)


def scramble(rank: np.ndarray, n: int) -> np.ndarray:
    """Bijection rank -> id on [0, n)."""
    if math.gcd(_SCRAMBLE_A, n) != 1:
        raise ValueError("scramble multiplier shares a factor with n")
    r = np.asarray(rank, dtype=np.uint64)
    return ((r * np.uint64(_SCRAMBLE_A) + np.uint64(_SCRAMBLE_B)) % np.uint64(n)).astype(np.int64)


class TripleSource:
    """Draws (h, r, t) triples of a synthetic graph with Zipf-distributed endpoints."""

    def __init__(self, n_entities: int, n_relations: int, s_entity: float, s_relation):
        self.n_entities, self.n_relations = int(n_entities), int(n_relations)
        self.ent = ZipfTable(n_entities, s_entity)
        self.rel = None if s_relation is None else ZipfTable(n_relations, s_relation)

    def draw(self, n: int, rng: np.random.Generator) -> np.ndarray:
        """[n, 3] int64 triples."""
        h = scramble(self.ent.sample(rng.random(n)), self.n_entities)
        t = scramble(self.ent.sample(rng.random(n)), self.n_entities)
        if self.rel is None:
            r = rng.integers(0, self.n_relations, size=n, dtype=np.int64)
        else:
            r = scramble(self.rel.sample(rng.random(n)), self.n_relations)
        return np.stack([h, r, t], axis=1)


def init_bound(gamma: float, ent_dim: int) -> float:
    return (gamma + 2.0) / float(ent_dim)


def init_tables_numpy(model: str, n_entities: int, n_relations: int, ent_dim: int, rel_dim: int, gamma: float,
                      seed: int):
    """float32 (E, R) on the host."""
    rng = np.random.default_rng(seed)
    a = init_bound(gamma, ent_dim)
    E = rng.uniform(-a, a, size=(n_entities, ent_dim)).astype(np.float32)
    if model == "rotate":
        R = rng.uniform(-math.pi, math.pi, size=(n_relations, rel_dim)).astype(np.float32)
    else:
        R = rng.uniform(-a, a, size=(n_relations, rel_dim)).astype(np.float32)
    return E, R


def init_tables_torch(model: str, n_entities: int, n_relations: int, ent_dim: int, rel_dim: int, gamma: float,
                      seed: int, device):
    """float32 (E, R) created directly in device memory (for tables too large for the host)."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    a = init_bound(gamma, ent_dim)
    E = torch.empty((n_entities, ent_dim), dtype=torch.float32, device=device)
    rows = max(1, (1 << 28) // ent_dim)  # fill in slices of about 1 GiB
    for s in range(0, n_entities, rows):
        E[s:s + rows].uniform_(-a, a, generator=g)
    R = torch.empty((n_relations, rel_dim), dtype=torch.float32, device=device)
    if model == "rotate":
        R.uniform_(-math.pi, math.pi, generator=g)
    else:
        R.uniform_(-a, a, generator=g)
    return E, R
