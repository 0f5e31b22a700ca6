"""Seeded, stateless index generation for mini-batches (inputs only; none of the method's arithmetic).

Both the GPU library and the CPU oracle receive the ids produced here as plain arguments.  Every id is a
function of (seed, stream tag, step, chunk, slot) alone, so any step of any run can be regenerated without
replaying the ones before it.

Generator: ``key = mix(mix(mix(mix(seed + GOLDEN * tag) + step) + a) + j)`` with ``mix`` the 64-bit finaliser
below (xor-shift / multiply, three rounds), and ``id = floor(key * n / 2**64)``.

What is generated follows Sec. 3.3 of the paper:
  * positives: b triples drawn uniformly (with replacement) from the triple list;
  * joint negatives: the b positives form b/g consecutive groups of g and each group gets one shared list of k
    corrupting entities, drawn uniformly from all entities;
  * degree-proportional negatives: the corrupting heads (tails) are the heads (tails) of triples drawn
    uniformly from the same mini-batch, which samples entities in proportion to their degree in the batch.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
GOLDEN = np.uint64(0x9E3779B97F4A7C15)
TAG_POS, TAG_NEG_UNIFORM, TAG_NEG_DEGREE = 1, 2, 3


def mix64(z: np.ndarray) -> np.ndarray:
    """64-bit finaliser on uint64 arrays (wrap-around arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def keys(seed: int, tag: int, step: int, a, j) -> np.ndarray:
    """uint64 keys for (seed, tag, step, a, j); a and j broadcast against each other."""
    a = np.asarray(a, dtype=np.uint64)
    j = np.asarray(j, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + GOLDEN * np.uint64(tag))
        z = mix64(z + np.uint64(step))
        z = mix64(z + a)
        z = mix64(z + j)
    return z


def scale_to(key: np.ndarray, n: int) -> np.ndarray:
    """floor(key * n / 2**64) as int64, for 0 < n < 2**32."""
    assert 0 < n < (1 << 32)
    key = np.asarray(key, dtype=np.uint64)
    n64 = np.uint64(n)
    hi = key >> np.uint64(32)
    lo = key & np.uint64(0xFFFFFFFF)
    return ((hi * n64 + ((lo * n64) >> np.uint64(32))) >> np.uint64(32)).astype(np.int64)


def batch_positions(seed: int, step: int, b: int, n_triples: int) -> np.ndarray:
    """Positions in the triple list of the b positives of one step."""
    return scale_to(keys(seed, TAG_POS, step, 0, np.arange(b)), n_triples)


def uniform_negatives(seed: int, step: int, n_chunks: int, k: int, n_entities: int) -> np.ndarray:
    """[n_chunks, k] corrupting entity ids, uniform over all entities (joint negative sampling)."""
    c = np.arange(n_chunks)[:, None]
    j = np.arange(k)[None, :]
    return scale_to(keys(seed, TAG_NEG_UNIFORM, step, c, j), n_entities)


def degree_negatives(seed: int, step: int, n_chunks: int, k: int, batch_h: np.ndarray, batch_t: np.ndarray,
                     neg_side: int) -> np.ndarray:
    """[n_chunks, k] corrupting ids taken from the batch's own tails (neg_side 0) or heads (neg_side 1)."""
    b = batch_h.shape[0]
    c = np.arange(n_chunks)[:, None]
    j = np.arange(k)[None, :]
    pick = scale_to(keys(seed, TAG_NEG_DEGREE, step, c, j), b)
    pool = batch_h if neg_side == 1 else batch_t
    return np.ascontiguousarray(pool[pick], dtype=np.int64)


def mixed_negatives(seed: int, step: int, n_chunks: int, k: int, n_degree: int, n_entities: int,
                    batch_h: np.ndarray, batch_t: np.ndarray, neg_side: int) -> np.ndarray:
    """[n_chunks, k] corrupting ids: slots 0 .. n_degree-1 of every chunk degree-proportional (from the batch), the
    others uniform over all entities.  Slot j of either kind is the same id that the all-degree / all-uniform
    generator gives for slot j."""
    uni = uniform_negatives(seed, step, n_chunks, k, n_entities)
    if n_degree == 0:
        return uni
    deg = degree_negatives(seed, step, n_chunks, k, batch_h, batch_t, neg_side)
    return np.where(np.arange(k)[None, :] < n_degree, deg, uni)


def side_of_step(mode: str, step: int) -> int:
    """0 = tails corrupted, 1 = heads corrupted.  'alternate' starts with tails at step 0."""
    if mode == "tail":
        return 0
    if mode == "head":
        return 1
    if mode == "alternate":
        return step & 1
    raise ValueError(mode)
