"""ctypes binding of libkge (include/kge.h): argument marshalling only.

Every function below has the name and the argument order of the C entry point it calls.  Tensors are torch
CUDA (ROCm) tensors; the binding checks dtype, device and contiguity and passes ``data_ptr()`` and the
current HIP stream.  Nothing is computed here, and there is no fallback: if libkge.so cannot be loaded the
import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("KGE_LIBRARY", os.path.join(_HERE, "libkge.so"))  # KGE_LIBRARY: another build of the same library

KGE_TRANSE_L2, KGE_TRANSE_L1, KGE_DISTMULT, KGE_COMPLEX, KGE_ROTATE, KGE_RESCAL, KGE_TRANSR = 0, 1, 2, 3, 4, 5, 6
KGE_NEG_TAIL, KGE_NEG_HEAD = 0, 1
KGE_OK, KGE_ERR_INVALID_ARG, KGE_ERR_UNSUPPORTED, KGE_ERR_WORKSPACE, KGE_ERR_DEVICE, KGE_ERR_INDEX_RANGE = \
    0, -1, -2, -3, -4, -5
LOSS_IDS = {"logistic": 0, "ranking": 1}
MODEL_IDS = {"transe_l2": KGE_TRANSE_L2, "transe_l1": KGE_TRANSE_L1, "distmult": KGE_DISTMULT,
             "complex": KGE_COMPLEX, "rotate": KGE_ROTATE, "rescal": KGE_RESCAL, "transr": KGE_TRANSR}

EXPORTS = ("kge_create", "kge_destroy", "kge_train_step", "kge_train_steps", "kge_score", "kge_get_dedup",
           "kge_check_indices", "kge_last_error", "kge_workspace_bytes", "kge_profile", "kge_profile_read",
           "kge_profile_slot_name", "kge_sample_steps", "kge_rank", "kge_rank_metrics", "kge_graph_captures", "kge_score_noalloc")
KGE_PROF_SLOTS = 9


class kge_sampler(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("triples", ctypes.c_void_p), ("n_triples", ctypes.c_int64),
                ("num_entities", ctypes.c_int64), ("batch", ctypes.c_int32), ("n_chunks", ctypes.c_int32),
                ("neg_per_chunk", ctypes.c_int32), ("n_degree", ctypes.c_int32), ("side_mode", ctypes.c_int32)]


class kge_config(ctypes.Structure):
    _fields_ = [("model", ctypes.c_int32), ("device", ctypes.c_int32),
                ("num_entities", ctypes.c_int64), ("num_relations", ctypes.c_int64),
                ("ent_dim", ctypes.c_int32), ("rel_dim", ctypes.c_int32),
                ("max_batch", ctypes.c_int32), ("max_neg_per_chunk", ctypes.c_int32), ("max_chunks", ctypes.c_int32),
                ("gemm_input", ctypes.c_int32), ("adagrad_mode", ctypes.c_int32),
                ("adagrad_eps", ctypes.c_float), ("adv_temperature", ctypes.c_float),
                ("validate_indices", ctypes.c_int32), ("loss", ctypes.c_int32)]


class KgeError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libkge error {code}: {text}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        import importlib.util
        spec = importlib.util.spec_from_file_location("_kge_build", os.path.join(_HERE, "csrc", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    lib.kge_create.restype = ctypes.c_int
    lib.kge_create.argtypes = [ctypes.POINTER(kge_config), ctypes.POINTER(vp)]
    lib.kge_destroy.restype = None
    lib.kge_destroy.argtypes = [vp]
    lib.kge_train_step.restype = ctypes.c_int
    lib.kge_train_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, i64, i64, i32, f32, f32, vp, vp]
    lib.kge_train_steps.restype = ctypes.c_int
    lib.kge_train_steps.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, i64, i64, vp, i64, f32, f32, vp, vp]
    lib.kge_profile.restype = ctypes.c_int
    lib.kge_profile.argtypes = [vp, i32]
    lib.kge_profile_read.restype = ctypes.c_int
    lib.kge_profile_read.argtypes = [vp, vp, vp]
    lib.kge_profile_slot_name.restype = ctypes.c_char_p
    lib.kge_profile_slot_name.argtypes = [i32]
    lib.kge_score.restype = ctypes.c_int
    lib.kge_score.argtypes = [vp, vp, vp, vp, vp, vp, i64, vp, i64, i64, i32, f32, vp, vp, vp]
    lib.kge_score_noalloc.restype = ctypes.c_int
    lib.kge_score_noalloc.argtypes = [ctypes.POINTER(kge_config), vp, vp, vp, vp, vp, i64, vp, i64, i64, i32, f32, vp, vp, vp]
    lib.kge_get_dedup.restype = ctypes.c_int
    lib.kge_get_dedup.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.kge_check_indices.restype = ctypes.c_int
    lib.kge_check_indices.argtypes = [vp, vp]
    lib.kge_last_error.restype = ctypes.c_char_p
    lib.kge_last_error.argtypes = [vp]
    lib.kge_workspace_bytes.restype = i64
    lib.kge_workspace_bytes.argtypes = [vp]
    lib.kge_graph_captures.restype = i64
    lib.kge_graph_captures.argtypes = [vp]
    lib.kge_rank.restype = ctypes.c_int
    lib.kge_rank.argtypes = [vp, vp, vp, vp, vp, vp, i64, vp, i64, i64, i32, f32, vp, vp]
    lib.kge_rank_metrics.restype = ctypes.c_int
    lib.kge_rank_metrics.argtypes = [vp, i64, vp, vp]
    lib.kge_sample_steps.restype = ctypes.c_int
    lib.kge_sample_steps.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, vp]
    return lib


_lib = _load()


def _dev_ptr(x: Optional[torch.Tensor], dtype, name: str):
    if x is None:
        return None
    if not isinstance(x, torch.Tensor) or not x.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if x.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {x.dtype}")
    if not x.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(x.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(ctx, rc: int):
    if rc != KGE_OK:
        text = _lib.kge_last_error(ctx)
        raise KgeError(rc, text.decode() if text else "")


def kge_rank(ctx, ent, rel, h, r, t, b, neg, k, chunk, neg_side, gamma, rank_out, hip_stream=None) -> None:
    f, i = torch.float32, torch.int64
    rc = _lib.kge_rank(ctx, _dev_ptr(ent, f, "ent"), _dev_ptr(rel, f, "rel"), _dev_ptr(h, i, "h"), _dev_ptr(r, i, "r"),
                       _dev_ptr(t, i, "t"), int(b), _dev_ptr(neg, i, "neg"), int(k), int(chunk), int(neg_side),
                       float(gamma), _stream(hip_stream), _dev_ptr(rank_out, torch.int32, "rank_out"))
    _check(ctx, rc)


def kge_rank_metrics(ranks, metrics_out, hip_stream=None) -> None:
    """metrics_out: device float64 [5] = Hit@1, Hit@3, Hit@10, MR, MRR of the device int32 ranks."""
    rc = _lib.kge_rank_metrics(_dev_ptr(ranks, torch.int32, "ranks"), int(ranks.numel()),
                               _dev_ptr(metrics_out, torch.float64, "metrics_out"), _stream(hip_stream))
    _check(None, rc)


SIDE_MODES = {"tail": 0, "head": 1, "alternate": 2}


def kge_sample_steps(seed, triples, num_entities, batch, n_chunks, neg_per_chunk, n_degree, side_mode, first_step,
                     n_steps, h, r, t, neg, sides=None, hip_stream=None) -> None:
    """Ids of steps first_step .. first_step + n_steps - 1 into the device tensors h, r, t [n_steps, batch],
    neg [n_steps, n_chunks * neg_per_chunk] and (optionally) sides [n_steps] int32."""
    i = torch.int64
    sp = kge_sampler(int(seed) & 0xFFFFFFFFFFFFFFFF, _dev_ptr(triples, i, "triples"), int(triples.shape[0]),
                     int(num_entities), int(batch), int(n_chunks), int(neg_per_chunk), int(n_degree),
                     SIDE_MODES[side_mode] if isinstance(side_mode, str) else int(side_mode))
    rc = _lib.kge_sample_steps(ctypes.byref(sp), int(first_step), int(n_steps), _dev_ptr(h, i, "h"),
                               _dev_ptr(r, i, "r"), _dev_ptr(t, i, "t"), _dev_ptr(neg, i, "neg"),
                               _dev_ptr(sides, torch.int32, "sides"), _stream(hip_stream))
    _check(None, rc)


def kge_create(cfg: kge_config) -> ctypes.c_void_p:
    out = ctypes.c_void_p()
    rc = _lib.kge_create(ctypes.byref(cfg), ctypes.byref(out))
    _check(None, rc)
    return out


def kge_destroy(ctx) -> None:
    _lib.kge_destroy(ctx)


def kge_train_step(ctx, ent, ent_state, rel, rel_state, h, r, t, b, neg, k, chunk, neg_side, gamma, lr,
                   hip_stream=None, loss_out=None) -> None:
    f, i = torch.float32, torch.int64
    rc = _lib.kge_train_step(ctx, _dev_ptr(ent, f, "ent"), _dev_ptr(ent_state, f, "ent_state"),
                             _dev_ptr(rel, f, "rel"), _dev_ptr(rel_state, f, "rel_state"),
                             _dev_ptr(h, i, "h"), _dev_ptr(r, i, "r"), _dev_ptr(t, i, "t"), int(b),
                             _dev_ptr(neg, i, "neg"), int(k), int(chunk), int(neg_side), float(gamma), float(lr),
                             _stream(hip_stream), _dev_ptr(loss_out, f, "loss_out"))
    _check(ctx, rc)


def kge_train_steps(ctx, ent, ent_state, rel, rel_state, h, r, t, b, neg, k, chunk, neg_sides, n_steps, gamma, lr,
                    hip_stream=None, loss_out=None) -> None:
    """h, r, t: device int64 [n_steps, b]; neg: device int64 [n_steps, (b/chunk)*k]; neg_sides: host sequence (a
    contiguous numpy int32 array is passed as it is) or None."""
    f, i = torch.float32, torch.int64
    sides = None
    if neg_sides is not None:
        import numpy as np
        keep = np.ascontiguousarray(neg_sides, dtype=np.int32)  # alive until the call returns (it copies them)
        if keep.shape != (int(n_steps),):
            raise ValueError("neg_sides must have one entry per step")
        sides = keep.ctypes.data_as(ctypes.c_void_p)
    rc = _lib.kge_train_steps(ctx, _dev_ptr(ent, f, "ent"), _dev_ptr(ent_state, f, "ent_state"),
                              _dev_ptr(rel, f, "rel"), _dev_ptr(rel_state, f, "rel_state"),
                              _dev_ptr(h, i, "h"), _dev_ptr(r, i, "r"), _dev_ptr(t, i, "t"), int(b),
                              _dev_ptr(neg, i, "neg"), int(k), int(chunk), sides, int(n_steps), float(gamma),
                              float(lr), _stream(hip_stream), _dev_ptr(loss_out, f, "loss_out"))
    _check(ctx, rc)


def kge_profile(ctx, enable) -> None:
    _check(ctx, _lib.kge_profile(ctx, int(bool(enable))))


def kge_profile_read(ctx):
    """Returns ({slot name: summed kernel milliseconds}, steps covered)."""
    ms = (ctypes.c_double * KGE_PROF_SLOTS)()
    steps = ctypes.c_int64(0)
    _check(ctx, _lib.kge_profile_read(ctx, ms, ctypes.byref(steps)))
    return {kge_profile_slot_name(s): ms[s] for s in range(KGE_PROF_SLOTS)}, int(steps.value)


def kge_profile_slot_name(slot) -> str:
    return _lib.kge_profile_slot_name(int(slot)).decode()


def kge_score(ctx, ent, rel, h, r, t, b, neg, k, chunk, neg_side, gamma, hip_stream=None, pos_out=None,
              neg_out=None) -> None:
    f, i = torch.float32, torch.int64
    rc = _lib.kge_score(ctx, _dev_ptr(ent, f, "ent"), _dev_ptr(rel, f, "rel"), _dev_ptr(h, i, "h"),
                        _dev_ptr(r, i, "r"), _dev_ptr(t, i, "t"), int(b), _dev_ptr(neg, i, "neg"), int(k), int(chunk),
                        int(neg_side), float(gamma), _stream(hip_stream), _dev_ptr(pos_out, f, "pos_out"),
                        _dev_ptr(neg_out, f, "neg_out"))
    _check(ctx, rc)


def kge_score_noalloc(cfg: kge_config, ent, rel, h, r, t, b, neg, k, chunk, neg_side, gamma, hip_stream=None,
                      pos_out=None, neg_out=None) -> None:
    f, i = torch.float32, torch.int64
    rc = _lib.kge_score_noalloc(ctypes.byref(cfg), _dev_ptr(ent, f, "ent"), _dev_ptr(rel, f, "rel"),
                                _dev_ptr(h, i, "h"), _dev_ptr(r, i, "r"), _dev_ptr(t, i, "t"), int(b),
                                _dev_ptr(neg, i, "neg"), int(k), int(chunk), int(neg_side), float(gamma),
                                _stream(hip_stream), _dev_ptr(pos_out, f, "pos_out"), _dev_ptr(neg_out, f, "neg_out"))
    _check(None, rc)


def kge_get_dedup(ctx, which, uniq_out, count_out, n_unique_out, hip_stream=None) -> None:
    rc = _lib.kge_get_dedup(ctx, int(which), _dev_ptr(uniq_out, torch.int64, "uniq_out"),
                            _dev_ptr(count_out, torch.int32, "count_out"),
                            _dev_ptr(n_unique_out, torch.int64, "n_unique_out"), _stream(hip_stream))
    _check(ctx, rc)


def kge_check_indices(ctx, hip_stream=None) -> None:
    _check(ctx, _lib.kge_check_indices(ctx, _stream(hip_stream)))


def kge_last_error(ctx) -> str:
    text = _lib.kge_last_error(ctx)
    return text.decode() if text else ""


def kge_workspace_bytes(ctx) -> int:
    return int(_lib.kge_workspace_bytes(ctx))


def kge_graph_captures(ctx) -> int:
    return int(_lib.kge_graph_captures(ctx))


class KgeContext:
    """Owns one kge_ctx; a convenience over the functions above (still marshalling only)."""

    def __init__(self, model, num_entities, num_relations, ent_dim, rel_dim=None, max_batch=1024,
                 max_neg_per_chunk=256, max_chunks=None, device=0, gemm_input=0, adv_temperature=0.0,
                 adagrad_eps=0.0, validate_indices=False, adagrad_mode=0, loss="logistic"):
        m = MODEL_IDS[model] if isinstance(model, str) else int(model)
        if rel_dim is None:
            rel_dim = {KGE_ROTATE: ent_dim // 2, KGE_RESCAL: ent_dim * ent_dim,
                       KGE_TRANSR: ent_dim + ent_dim * ent_dim}.get(m, ent_dim)
        if max_chunks is None:
            max_chunks = max_batch
        self.cfg = kge_config(m, int(device), int(num_entities), int(num_relations), int(ent_dim), int(rel_dim),
                              int(max_batch), int(max_neg_per_chunk), int(max_chunks), int(gemm_input),
                              int(adagrad_mode),
                              float(adagrad_eps), float(adv_temperature), int(bool(validate_indices)),
                              LOSS_IDS[loss])
        self.ctx = kge_create(self.cfg)

    def train_step(self, ent, ent_state, rel, rel_state, h, r, t, neg, k, chunk, neg_side, gamma, lr, loss_out=None,
                   stream=None):
        kge_train_step(self.ctx, ent, ent_state, rel, rel_state, h, r, t, h.numel(), neg, k, chunk, neg_side, gamma,
                       lr, stream, loss_out)

    def train_steps(self, ent, ent_state, rel, rel_state, h, r, t, neg, k, chunk, neg_sides, gamma, lr, loss_out=None,
                    stream=None):
        kge_train_steps(self.ctx, ent, ent_state, rel, rel_state, h, r, t, h.shape[1], neg, k, chunk, neg_sides,
                        h.shape[0], gamma, lr, stream, loss_out)

    def profile(self, enable):
        kge_profile(self.ctx, enable)

    def profile_read(self):
        return kge_profile_read(self.ctx)

    def score(self, ent, rel, h, r, t, neg, k, chunk, neg_side, gamma, pos_out=None, neg_out=None, stream=None):
        kge_score(self.ctx, ent, rel, h, r, t, h.numel(), neg, k, chunk, neg_side, gamma, stream, pos_out, neg_out)

    def rank(self, ent, rel, h, r, t, neg, k, chunk, neg_side, gamma, rank_out=None, stream=None):
        if rank_out is None:
            rank_out = torch.empty(h.numel(), dtype=torch.int32, device=h.device)
        kge_rank(self.ctx, ent, rel, h, r, t, h.numel(), neg, k, chunk, neg_side, gamma, rank_out, stream)
        return rank_out

    def get_dedup(self, which: int, n_keys: int):
        dev = torch.device("cuda", self.cfg.device)
        uniq = torch.empty(n_keys, dtype=torch.int64, device=dev)
        cnt = torch.empty(n_keys, dtype=torch.int32, device=dev)
        n = torch.zeros(1, dtype=torch.int64, device=dev)
        kge_get_dedup(self.ctx, which, uniq, cnt, n)
        torch.cuda.synchronize(dev)
        u = int(n.item())
        return uniq[:u].clone(), cnt[:u].clone()

    def check_indices(self):
        kge_check_indices(self.ctx)

    def workspace_bytes(self) -> int:
        return kge_workspace_bytes(self.ctx)

    def graph_captures(self) -> int:
        return kge_graph_captures(self.ctx)

    def close(self):
        if self.ctx is not None:
            kge_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
