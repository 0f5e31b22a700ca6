"""CPU oracle for the KGE mini-batch step (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this
package.  It is a ctypes wrapper around ``kge_oracle.c`` (plain C, fp64 arithmetic, one triple and one
negative at a time), which holds all of the training step's arithmetic; the only arithmetic written here is the
two-line definition of a link-prediction rank and of the Hit@k / MR / MRR averages (``ranks``, ``rank_metrics``,
paper Sec. 5), in numpy.  It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kge_oracle.c")
_LIB = os.path.join(_HERE, "libkge_oracle.so")
_LIB_OMP = os.path.join(_HERE, "libkge_oracle_omp.so")

TRANSE_L2, TRANSE_L1, DISTMULT, COMPLEX, ROTATE, RESCAL, TRANSR = 0, 1, 2, 3, 4, 5, 6
NEG_TAIL, NEG_HEAD = 0, 1
LOSS_IDS = {"logistic": 0, "ranking": 1}
MODEL_IDS = {"transe_l2": TRANSE_L2, "transe_l1": TRANSE_L1, "distmult": DISTMULT, "complex": COMPLEX,
             "rotate": ROTATE, "rescal": RESCAL, "transr": TRANSR}


def compile_oracle(src: str, lib: str, openmp: bool = False) -> str:
    """gcc, no fast-math, no contraction.  openmp: the all-cores build (timing baseline only)."""
    subprocess.run(["gcc", "-O2", "-Wall", "-Wextra", "-ffp-contract=off", *(["-fopenmp"] if openmp else []),
                    "-shared", "-fPIC", "-o", lib, src, "-lm"], check=True)
    return lib


def build(force: bool = False, openmp: bool = False) -> str:
    """Compile kge_oracle.c and return the library path.  With force both builds are made: the parity oracle
    (single thread) and the OpenMP build that the benchmark times on all host cores."""
    for lib, omp in ((_LIB, False), (_LIB_OMP, True)):
        wanted = force or omp == openmp
        if wanted and (force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC)):
            compile_oracle(_SRC, lib, omp)
    return _LIB_OMP if openmp else _LIB


class _Params(ctypes.Structure):
    _fields_ = [("model", ctypes.c_int32), ("ent_dim", ctypes.c_int32), ("rel_dim", ctypes.c_int32),
                ("neg_side", ctypes.c_int32), ("tables_f64", ctypes.c_int32), ("bf16_inputs", ctypes.c_int32),
                ("rotate_squared", ctypes.c_int32), ("split_form", ctypes.c_int32), ("loss", ctypes.c_int32),
                ("gamma", ctypes.c_double), ("adv_temperature", ctypes.c_double)]


_lib = None
_lib_omp = None


def bind(path: str):
    """Load a build of kge_oracle.c and declare its entry points."""
    lib = ctypes.CDLL(path)
    vp, i64, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double
    lib.ko_round_bf16.restype = dbl
    lib.ko_round_bf16.argtypes = [dbl]
    lib.ko_threads.restype = ctypes.c_int
    lib.ko_threads.argtypes = []
    lib.ko_loss_grad.restype = ctypes.c_int
    lib.ko_loss_grad.argtypes = [ctypes.POINTER(_Params), vp, vp, vp, vp, vp, i64, vp, i64, i64, vp,
                                 vp, vp, vp, vp, vp, i64, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.ko_dedup.restype = i64
    lib.ko_dedup.argtypes = [vp, i64, vp, vp]
    lib.ko_adagrad_rows.restype = None
    lib.ko_adagrad_rows.argtypes = [vp, vp, vp, i64, ctypes.c_int, vp, dbl, dbl, ctypes.c_int]
    lib.ko_train_step.restype = ctypes.c_int
    lib.ko_train_step.argtypes = [ctypes.POINTER(_Params), vp, vp, i64, vp, vp, i64, vp, vp, vp, i64,
                                  vp, i64, i64, dbl, dbl, ctypes.c_int, ctypes.c_int, vp, vp, vp,
                                  vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    return lib


def _load(openmp: bool = False):
    global _lib, _lib_omp
    if openmp:
        if _lib_omp is None:
            _lib_omp = bind(build(openmp=True))
        return _lib_omp
    if _lib is None:
        _lib = bind(build())
    return _lib


def threads(openmp: bool = False) -> int:
    """Workers the chosen build spreads a mini-batch over (1 for the parity oracle)."""
    return int(_load(openmp).ko_threads())


def round_bf16(x) -> np.ndarray:
    """The oracle's bfloat16 rounding (nearest, ties to even, of the value held as float32), element by element."""
    lib = _load()
    a = np.asarray(x, dtype=np.float64)
    return np.array([lib.ko_round_bf16(float(v)) for v in a.reshape(-1)], dtype=np.float64).reshape(a.shape)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _ids(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int64)


def _params(model, ent_dim, rel_dim, neg_side, gamma, adv_temperature=0.0, tables_f64=False, bf16_inputs=False,
            rotate_squared=False, split_form=False, loss="logistic") -> _Params:
    m = MODEL_IDS[model] if isinstance(model, str) else int(model)
    return _Params(m, int(ent_dim), int(rel_dim), int(neg_side), int(tables_f64), int(bf16_inputs),
                   int(rotate_squared), int(split_form), LOSS_IDS[loss], float(gamma), float(adv_temperature))


def loss_and_grad(model, E, R, h, r, t, neg, k, chunk, neg_side, gamma, adv_temperature=0.0, w_fixed=None,
                  want_grad=True, bf16_inputs=False, rotate_squared=False, split_form=False, loss="logistic"):
    """Loss, scores, weights and (dense) gradients of one mini-batch.

    E, R: float32 or float64 2-D arrays.  Returns a dict with ``loss`` (float), ``pos`` [b], ``neg`` [b,k],
    ``w`` [b,k] and, if wanted, ``dE``, ``dR`` with the shapes of E and R (float64).
    """
    lib = _load()
    f64 = E.dtype == np.float64
    assert R.dtype == E.dtype and E.dtype in (np.float32, np.float64)
    E = np.ascontiguousarray(E)
    R = np.ascontiguousarray(R)
    h, r, t, neg = _ids(h), _ids(r), _ids(t), _ids(neg).reshape(-1)
    b = h.shape[0]
    assert neg.shape[0] == (b // chunk) * k
    p = _params(model, E.shape[1], R.shape[1], neg_side, gamma, adv_temperature, f64, bf16_inputs, rotate_squared,
                split_form, loss)
    loss = ctypes.c_double(0.0)
    pos = np.zeros(b, np.float64)
    negs = np.zeros((b, k), np.float64)
    w = np.zeros((b, k), np.float64)
    dE = np.zeros(E.shape, np.float64) if want_grad else None
    dR = np.zeros(R.shape, np.float64) if want_grad else None
    aE = np.zeros(E.shape, np.float64) if want_grad else None
    aR = np.zeros(R.shape, np.float64) if want_grad else None
    wf = None if w_fixed is None else np.ascontiguousarray(w_fixed, dtype=np.float64)
    rc = lib.ko_loss_grad(ctypes.byref(p), _ptr(E), _ptr(R), _ptr(h), _ptr(r), _ptr(t), b, _ptr(neg), k, chunk,
                          _ptr(wf), ctypes.addressof(loss), _ptr(pos), _ptr(negs), _ptr(w),
                          None, E.shape[0], _ptr(dE), _ptr(aE), None, R.shape[0], _ptr(dR), _ptr(aR), None, None)
    if rc != 0:
        raise ValueError(f"ko_loss_grad failed with {rc}")
    out = {"loss": loss.value, "pos": pos, "neg": negs, "w": w}
    if want_grad:
        out["dE"], out["dR"], out["absE"], out["absR"] = dE, dR, aE, aR
    return out


def scores(model, E, R, h, r, t, neg, k, chunk, neg_side, gamma, **kw):
    """Positive scores [b] and negative scores [b,k] (float64)."""
    o = loss_and_grad(model, E, R, h, r, t, neg, k, chunk, neg_side, gamma, want_grad=False, **kw)
    return o["pos"], o["neg"]


def dedup(keys):
    """Distinct values (ascending) and their multiplicities, both int64."""
    lib = _load()
    keys = _ids(keys).reshape(-1)
    n = keys.shape[0]
    uniq = np.zeros(max(n, 1), np.int64)
    cnt = np.zeros(max(n, 1), np.int64)
    u = lib.ko_dedup(_ptr(keys), n, _ptr(uniq), _ptr(cnt))
    return uniq[:u].copy(), cnt[:u].copy()


def adagrad_rows(table, state, ids, grad, lr, eps, rowwise=False):
    """In-place Adagrad on rows ``ids`` (or all rows when ids is None) of float32 table/state.  rowwise: state is
    one float per row, fed with the mean of the squared gradient elements of the row."""
    lib = _load()
    assert table.dtype == np.float32 and state.dtype == np.float32 and table.flags.c_contiguous
    grad = np.ascontiguousarray(grad, dtype=np.float64)
    if ids is None:
        n = table.shape[0]
        idp = None
    else:
        ids = _ids(ids)
        n = ids.shape[0]
        idp = _ptr(ids)
    assert state.shape == ((table.shape[0],) if rowwise else table.shape)
    lib.ko_adagrad_rows(_ptr(table), _ptr(state), idp, n, table.shape[1], _ptr(grad), float(lr), float(eps),
                        int(rowwise))


def train_step(model, E, SE, R, SR, h, r, t, neg, k, chunk, neg_side, gamma, lr, eps=1e-10, adv_temperature=0.0,
               dense=False, bf16_inputs=False, rotate_squared=False, want_scores=False, report=False, rowwise=False,
               loss="logistic", openmp=False):
    """One step, in place on float32 E, SE, R, SR.  Returns loss (and scores when asked).

    report=True (touched-rows mode) returns ``(loss, rep)`` where rep holds, for the distinct rows of the step,
    ``ent_ids``, ``dE`` (their summed gradient rows), ``absE`` (magnitudes of the terms, per element) and ``maxE``
    (largest share of a single negative pair in that element), and the same for relations: what the tests need to
    bound rounding effects, not part of the method.  openmp=True runs the all-cores build (timing baseline; same
    terms, summed per thread first)."""
    lib = _load(openmp)
    for a in (E, SE, R, SR):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    h, r, t, neg = _ids(h), _ids(r), _ids(t), _ids(neg).reshape(-1)
    b = h.shape[0]
    assert neg.shape[0] == (b // chunk) * k
    p = _params(model, E.shape[1], R.shape[1], neg_side, gamma, adv_temperature, False, bf16_inputs, rotate_squared,
                False, loss)
    loss = ctypes.c_double(0.0)
    pos = np.zeros(b, np.float64) if want_scores else None
    negs = np.zeros((b, k), np.float64) if want_scores else None
    rep = None
    extra = [None] * 10
    if report:
        assert not dense
        nk = 2 * b + neg.shape[0]
        rep = {"ent_ids": np.zeros(nk, np.int64), "dE": np.zeros((nk, E.shape[1])), "absE": np.zeros((nk, E.shape[1])),
               "rel_ids": np.zeros(b, np.int64), "dR": np.zeros((b, R.shape[1])), "absR": np.zeros((b, R.shape[1])),
               "maxE": np.zeros((nk, E.shape[1])), "maxR": np.zeros((b, R.shape[1]))}
        ne, nr = ctypes.c_int64(0), ctypes.c_int64(0)
        extra = [_ptr(rep["ent_ids"]), ctypes.addressof(ne), _ptr(rep["dE"]), _ptr(rep["absE"]),
                 _ptr(rep["rel_ids"]), ctypes.addressof(nr), _ptr(rep["dR"]), _ptr(rep["absR"]),
                 _ptr(rep["maxE"]), _ptr(rep["maxR"])]
    rc = lib.ko_train_step(ctypes.byref(p), _ptr(E), _ptr(SE), E.shape[0], _ptr(R), _ptr(SR), R.shape[0],
                           _ptr(h), _ptr(r), _ptr(t), b, _ptr(neg), k, chunk, float(lr), float(eps), int(dense),
                           int(rowwise),
                           ctypes.addressof(loss), _ptr(pos), _ptr(negs), *extra)
    if rc != 0:
        raise ValueError(f"ko_train_step failed with {rc}")
    if report:
        for key, n in (("ent_ids", ne.value), ("dE", ne.value), ("absE", ne.value), ("maxE", ne.value),
                       ("rel_ids", nr.value), ("dR", nr.value), ("absR", nr.value), ("maxR", nr.value)):
            rep[key] = rep[key][:n]
        return loss.value, rep
    if want_scores:
        return loss.value, pos, negs
    return loss.value


def ranks(pos, neg):
    """Link-prediction rank of every positive among its negatives (paper Sec. 5, no filtering):
    rank_i = 1 + #{j : neg[i, j] > pos[i]}.  pos [b], neg [b, k] scores; int64 [b]."""
    pos = np.asarray(pos, dtype=np.float64)
    neg = np.asarray(neg, dtype=np.float64)
    return 1 + (neg > pos[:, None]).sum(axis=1).astype(np.int64)


def rank_metrics(rank):
    """Hit@1, Hit@3, Hit@10 (shares of ranks <= 1, 3, 10), MR (mean rank), MRR (mean reciprocal rank)."""
    rank = np.asarray(rank, dtype=np.float64)
    return np.array([(rank <= 1).mean(), (rank <= 3).mean(), (rank <= 10).mean(), rank.mean(), (1.0 / rank).mean()])
