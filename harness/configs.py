"""The workload configurations and a batch stream built on the graph and index generators.

Inputs only: this module draws graphs, ids and initial tables; it evaluates nothing of the method.
Counts for ``small`` and ``freebase`` are the entity / relation counts of Table 3 of the paper (FB15k and
Freebase); the others are defined by this build's benchmark description.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

from . import graphs, sampler


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    model: str               # transe_l2 | transe_l1 | distmult | complex | rotate | rescal | transr
    n_entities: int
    n_relations: int
    n_triples: int           # size of the synthetic triple list (0: positives are drawn directly, not stored)
    s_entity: float          # Zipf exponent of the entity degrees
    s_relation: Optional[float]  # Zipf exponent of relation frequencies, None = uniform
    ent_dim: int             # floats per entity row
    rel_dim: int             # floats per relation row
    batch: int               # b
    chunk: int               # g
    neg_per_chunk: int       # k
    neg_mode: str            # uniform | degree
    side_mode: str           # tail | head | alternate
    gamma: float
    lr: float
    adv_temperature: float = 0.0
    bf16_inputs: bool = False
    loss: str = "logistic"   # logistic | ranking (the two losses of Sec. 2)
    steps: int = 20
    seed: int = 0

    @property
    def n_chunks(self) -> int:
        return self.batch // self.chunk

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


TINY = Workload("tiny", "transe_l2", 1_000, 20, 10_000, 1.1, None, 64, 64, 256, 32, 64, "uniform", "tail",
                12.0, 0.1, steps=20)
SMALL_DISTMULT = Workload("small-distmult", "distmult", 14_951, 1_345, 483_142, 1.0, 1.2, 400, 400, 1024, 128, 256,
                          "uniform", "alternate", 12.0, 0.1, steps=471)
SMALL_COMPLEX = SMALL_DISTMULT.scaled(name="small-complex", model="complex")
# RESCAL at the same graph and batch shape, rows of 200 floats: a relation row is a 200 x 200 matrix
SMALL_RESCAL = SMALL_DISTMULT.scaled(name="small-rescal", model="rescal", ent_dim=200, rel_dim=200 * 200)
# TransR at the same graph and batch shape, rows of 100 floats: a relation row is a translation and a 100 x 100 matrix
SMALL_TRANSR = SMALL_DISTMULT.scaled(name="small-transr", model="transr", ent_dim=100, rel_dim=100 + 100 * 100)
# Sec. 6.1.1 / Fig. 3 of the paper compares joint with independent negative sampling for TransE on FB15k: the same
# graph and batch with chunks of 128 positives sharing 256 corrupting entities, and with every positive drawing its
# own 256 (chunks of one positive)
SMALL_TRANSE_JOINT = SMALL_DISTMULT.scaled(name="small-transe_l2-joint", model="transe_l2")
SMALL_TRANSE_INDEPENDENT = SMALL_TRANSE_JOINT.scaled(name="small-transe_l2-independent", chunk=1)
MEDIUM = Workload("medium", "rotate", 2_500_000, 800, 16_000_000, 0.9, None, 400, 200, 1024, 128, 256, "degree",
                  "tail", 12.0, 0.1, adv_temperature=1.0, steps=1000)
LARGE = Workload("large", "transe_l2", 5_000_000, 800, 20_000_000, 0.9, None, 400, 400, 2048, 256, 1024, "uniform",
                 "tail", 12.0, 0.1, bf16_inputs=True, steps=9765)
FREEBASE_TRANSE = Workload("freebase-transe_l2", "transe_l2", 86_054_151, 14_824, 0, 1.0, 1.0, 400, 400, 1000, 1000,
                           200, "uniform", "tail", 12.0, 0.1, steps=100_000)
FREEBASE_COMPLEX = FREEBASE_TRANSE.scaled(name="freebase-complex", model="complex")

ALL = {w.name: w for w in (TINY, SMALL_DISTMULT, SMALL_COMPLEX, SMALL_RESCAL, SMALL_TRANSR, SMALL_TRANSE_JOINT,
                           SMALL_TRANSE_INDEPENDENT, MEDIUM, LARGE, FREEBASE_TRANSE,
                           FREEBASE_COMPLEX)}


class BatchStream:
    """Deterministic stream of (h, r, t, neg, side) for a workload.

    With a stored triple list (n_triples > 0 and ``materialise``), positives are positions drawn by the
    counter-based sampler; otherwise each step's positives are drawn directly from the graph's generating
    distribution with a generator seeded by (seed, step), which is what sampling with replacement from an
    i.i.d. triple list amounts to.
    """

    def __init__(self, w: Workload, materialise: bool = True):
        self.w = w
        self.source = graphs.TripleSource(w.n_entities, w.n_relations, w.s_entity, w.s_relation)
        self.triples = None
        if materialise and w.n_triples > 0:
            self.triples = self.source.draw(w.n_triples, np.random.default_rng([w.seed, 0xA11]))

    def step(self, s: int):
        w = self.w
        if self.triples is not None:
            pos = self.triples[sampler.batch_positions(w.seed, s, w.batch, self.triples.shape[0])]
        else:
            pos = self.source.draw(w.batch, np.random.default_rng([w.seed, 0xB22, s]))
        h = np.ascontiguousarray(pos[:, 0])
        r = np.ascontiguousarray(pos[:, 1])
        t = np.ascontiguousarray(pos[:, 2])
        side = sampler.side_of_step(w.side_mode, s)
        if w.neg_mode == "degree":
            neg = sampler.degree_negatives(w.seed, s, w.n_chunks, w.neg_per_chunk, h, t, side)
        else:
            neg = sampler.uniform_negatives(w.seed, s, w.n_chunks, w.neg_per_chunk, w.n_entities)
        return h, r, t, neg, side

    def steps(self, first: int, count: int):
        """Stacked ids of ``count`` consecutive steps: h, r, t [count, b], neg [count, C, k], side [count]."""
        out = [self.step(first + i) for i in range(count)]
        return (np.stack([o[0] for o in out]), np.stack([o[1] for o in out]), np.stack([o[2] for o in out]),
                np.stack([o[3] for o in out]), np.array([o[4] for o in out], dtype=np.int32))


def init_tables(w: Workload, device=None):
    """Initial (E, R): numpy float32 on the host when device is None, else torch tensors on that device."""
    if device is None:
        return graphs.init_tables_numpy(w.model, w.n_entities, w.n_relations, w.ent_dim, w.rel_dim, w.gamma,
                                        w.seed + 1)
    return graphs.init_tables_torch(w.model, w.n_entities, w.n_relations, w.ent_dim, w.rel_dim, w.gamma,
                                    w.seed + 1, device)
