"""Pins for the oracle's score functions (Table 1 of the paper) and for the chunk layout of joint negative
sampling (Sec. 3.3).  CPU only."""
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_scores.txt")
MODELS = ["transe_l2", "transe_l1", "distmult", "complex", "rotate", "rescal"]


def _vec(txt):
    out = []
    for tok in txt.split():
        tok = tok.replace("PI", "math.pi")
        out.append(float(eval(tok, {"math": math})))
    return np.array(out, dtype=np.float64)


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            model, gamma, h, r, t, want, _ = [c.strip() for c in line.split(";", 6)]
            rows.append((model, float(gamma), _vec(h), _vec(r), _vec(t), float(want)))
    return rows


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: f"{r[0]}-{r[5]}")
def test_hand_worked_scores(row):
    model, gamma, h, r, t, want = row
    squared = model == "rotate_squared"
    model = "rotate" if squared else model
    E = np.stack([h, t])
    # relation rows may be shorter than entity rows (RotatE); pad nothing, pass as their own table
    R = r[None, :]
    for dtype, tol in ((np.float64, 1e-12), (np.float32, 1e-6)):
        pos, _ = oracle.scores(model, E.astype(dtype), R.astype(dtype), [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1,
                               oracle.NEG_TAIL, gamma, rotate_squared=squared)
        assert abs(pos[0] - want) <= tol * max(1.0, abs(want)), (model, pos[0], want)


def _rand_problem(model, rng, n_ent=23, n_rel=5, D=8, b=12, chunk=4, k=5):
    Dr = D // 2 if model == "rotate" else (D * D if model == "rescal" else D)
    E = rng.normal(size=(n_ent, D))
    R = rng.uniform(-math.pi, math.pi, size=(n_rel, Dr)) if model == "rotate" else rng.normal(size=(n_rel, Dr))
    h = rng.integers(0, n_ent, b)
    r = rng.integers(0, n_rel, b)
    t = rng.integers(0, n_ent, b)
    neg = rng.integers(0, n_ent, (b // chunk, k))
    return E, R, h, r, t, neg, chunk, k


def _split_scores_numpy(model, E, R, h, r, t, neg, chunk, k, side, gamma):
    """Sec. 3.3: o depends on the uncorrupted entity and the relation; the (o, n) pairs of one group are then a
    matrix product (DistMult, ComplEx, TransE-L2 via |o|^2 + |n|^2 - 2 o.n) or an elementwise reduction."""
    b, D = h.shape[0], E.shape[1]
    C = D // 2
    a = E[t] if side == 1 else E[h]
    rr = R[r]
    if model in ("transe_l2", "transe_l1"):
        o = a - rr if side == 1 else a + rr
    elif model == "distmult":
        o = a * rr
    elif model == "rescal":  # h^T M n = (M^T h) . n ;  n^T M t = n . (M t)
        M = rr.reshape(b, D, D)
        o = np.einsum("bxc,bc->bx", M, a) if side == 1 else np.einsum("bx,bxc->bc", a, M)
    else:
        if model == "rotate":
            rc = np.cos(rr) + 1j * np.sin(rr)
        else:
            rc = rr[:, :C] + 1j * rr[:, C:]
        ac = a[:, :C] + 1j * a[:, C:]
        oc = ac * (np.conj(rc) if side == 1 else rc)
        o = np.concatenate([oc.real, oc.imag], axis=1)
    out = np.zeros((b, k))
    for c in range(b // chunk):
        Oc = o[c * chunk:(c + 1) * chunk]
        Nc = E[neg[c]]
        if model in ("distmult", "complex", "rescal"):
            S = Oc @ Nc.T
        elif model == "transe_l2":
            d2 = (Oc * Oc).sum(1)[:, None] + (Nc * Nc).sum(1)[None, :] - 2.0 * (Oc @ Nc.T)
            S = gamma - np.sqrt(np.maximum(d2, 0.0))
        elif model == "transe_l1":
            S = gamma - np.abs(Oc[:, None, :] - Nc[None, :, :]).sum(-1)
        else:
            q = (Oc[:, None, :C] - Nc[None, :, :C]) + 1j * (Oc[:, None, C:] - Nc[None, :, C:])
            S = gamma - np.abs(q).sum(-1)
        out[c * chunk:(c + 1) * chunk] = S
    return out


@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("model", MODELS)
def test_per_pair_scores_equal_split_form(model, side):
    """The oracle scores every pair from the Table 1 formula; Sec. 3.3's split form, evaluated here with
    numpy matrix products, must give the same numbers."""
    rng = np.random.default_rng(7 + side)
    E, R, h, r, t, neg, chunk, k = _rand_problem(model, rng)
    pos, sneg = oracle.scores(model, E, R, h, r, t, neg, k, chunk, side, 3.5)
    want = _split_scores_numpy(model, E, R, h, r, t, neg, chunk, k, side, 3.5)
    np.testing.assert_allclose(sneg, want, rtol=1e-10, atol=1e-10)
    # the oracle's own split path (used for bf16 emulation) agrees with its per-pair path
    _, sneg2 = oracle.scores(model, E, R, h, r, t, neg, k, chunk, side, 3.5, split_form=True)
    np.testing.assert_allclose(sneg2, sneg, rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("model", MODELS)
def test_negative_equal_to_positive_entity_reproduces_positive_score(model):
    """A corrupting entity equal to the true tail (head) gives the positive's score: ties the negative path to
    the positive path and the chunk indexing (group c uses neg[c])."""
    rng = np.random.default_rng(3)
    E, R, h, r, t, neg, chunk, k = _rand_problem(model, rng)
    b = h.shape[0]
    for side in (0, 1):
        for i in range(b):
            c, j = i // chunk, i % k
            neg2 = neg.copy()
            neg2[c, j] = h[i] if side == 1 else t[i]
            pos, sneg = oracle.scores(model, E, R, h, r, t, neg2, k, chunk, side, 2.0)
            assert abs(sneg[i, j] - pos[i]) < 1e-12


def test_chunk_members_share_negatives_and_row_count_law():
    """Sec. 3.3: the b positives touch (b/g)*k corrupting rows, not b*k; two positives of one group that agree
    in (h, r) get identical negative scores, and changing another group's list does not affect them."""
    rng = np.random.default_rng(11)
    E, R, h, r, t, neg, chunk, k = _rand_problem("transe_l2", rng)
    assert neg.size == (h.shape[0] // chunk) * k
    h[1], r[1] = h[0], r[0]
    _, s0 = oracle.scores("transe_l2", E, R, h, r, t, neg, k, chunk, 0, 1.0)
    np.testing.assert_array_equal(s0[0], s0[1])
    neg2 = neg.copy()
    neg2[1] = (neg2[1] + 1) % E.shape[0]
    _, s1 = oracle.scores("transe_l2", E, R, h, r, t, neg2, k, chunk, 0, 1.0)
    np.testing.assert_array_equal(s0[:chunk], s1[:chunk])
    assert not np.array_equal(s0[chunk:2 * chunk], s1[chunk:2 * chunk])


def test_transe_translation_invariance_and_rotate_isometry():
    """Closed-form invariants: TransE scores do not change when the same vector is added to h and t;
    RotatE with all phases zero equals the sum of moduli of h - t; rotating h and t by a common phase and
    keeping theta leaves RotatE unchanged."""
    rng = np.random.default_rng(5)
    D = 6
    E = rng.normal(size=(4, D))
    R = rng.normal(size=(1, D))
    shift = rng.normal(size=D)
    E2 = E.copy()
    E2[0] += shift
    E2[1] += shift
    for m in ("transe_l2", "transe_l1"):
        p1, _ = oracle.scores(m, E, R, [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1, 0, 9.0)
        p2, _ = oracle.scores(m, E2, R, [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1, 0, 9.0)
        assert abs(p1[0] - p2[0]) < 1e-12
    C = D // 2
    Rz = np.zeros((1, C))
    p, _ = oracle.scores("rotate", E, Rz, [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1, 0, 9.0)
    want = 9.0 - np.abs((E[0, :C] - E[1, :C]) + 1j * (E[0, C:] - E[1, C:])).sum()
    assert abs(p[0] - want) < 1e-12
    Rt = rng.uniform(-3, 3, size=(1, C))
    phase = np.exp(1j * 0.7)
    Ec = (E[:, :C] + 1j * E[:, C:]) * phase
    E3 = np.concatenate([Ec.real, Ec.imag], axis=1)
    p1, _ = oracle.scores("rotate", E, Rt, [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1, 0, 9.0)
    p2, _ = oracle.scores("rotate", E3, Rt, [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1, 0, 9.0)
    assert abs(p1[0] - p2[0]) < 1e-12


def test_complex_reduces_to_distmult_for_real_embeddings():
    """ComplEx with zero imaginary parts is DistMult on the real parts (textbook special case)."""
    rng = np.random.default_rng(9)
    C = 5
    Er = rng.normal(size=(6, C))
    Rr = rng.normal(size=(2, C))
    E = np.concatenate([Er, np.zeros_like(Er)], axis=1)
    R = np.concatenate([Rr, np.zeros_like(Rr)], axis=1)
    h, r, t = [0, 1, 2], [0, 1, 1], [3, 4, 5]
    neg = np.array([[1, 5]])
    pc, nc = oracle.scores("complex", E, R, h, r, t, neg, 2, 3, 0, 0.0)
    pd, nd = oracle.scores("distmult", Er, Rr, h, r, t, neg, 2, 3, 0, 0.0)
    np.testing.assert_allclose(pc, pd, atol=1e-13)
    np.testing.assert_allclose(nc, nd, atol=1e-13)


def test_rescal_with_diagonal_matrices_is_distmult():
    """M_r = diag(r) turns h^T M_r t into DistMult's sum_d h_d r_d t_d: scores, loss and the entity gradients coincide,
    and the diagonal of dL/dM_r is DistMult's relation gradient (off-diagonal entries are h_a t_c terms, not zero)."""
    rng = np.random.default_rng(11)
    E, R, h, r, t, neg, chunk, k = _rand_problem("distmult", rng)
    D = E.shape[1]
    Rm = np.zeros((R.shape[0], D * D))
    for i in range(R.shape[0]):
        Rm[i] = np.diag(R[i]).reshape(-1)
    for side in (0, 1):
        for loss in ("logistic", "ranking"):
            a = oracle.loss_and_grad("distmult", E, R, h, r, t, neg, k, chunk, side, 0.4, loss=loss)
            m = oracle.loss_and_grad("rescal", E, Rm, h, r, t, neg, k, chunk, side, 0.4, loss=loss)
            np.testing.assert_allclose(m["pos"], a["pos"], rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(m["neg"], a["neg"], rtol=1e-12, atol=1e-12)
            assert abs(m["loss"] - a["loss"]) < 1e-12
            np.testing.assert_allclose(m["dE"], a["dE"], rtol=1e-10, atol=1e-12)
            diag = m["dR"].reshape(-1, D, D)[:, np.arange(D), np.arange(D)]
            np.testing.assert_allclose(diag, a["dR"], rtol=1e-10, atol=1e-12)


def test_transr_with_identity_projections_is_the_squared_transe_distance():
    """M_r = identity: gamma - f_TransR = |h + r - t|^2 = (gamma - f_TransE-L2)^2, for positives and negatives on both
    sides; and projecting both entities with the same matrix makes the score invariant under a common shift of h and t
    (M (h + s) - M (t + s) = M h - M t), whatever the matrix."""
    rng = np.random.default_rng(12)
    E, R, h, r, t, neg, chunk, k = _rand_problem("transe_l2", rng)
    D = E.shape[1]
    Rt = np.concatenate([R, np.tile(np.eye(D).reshape(-1), (R.shape[0], 1))], axis=1)
    for side in (0, 1):
        p2, n2 = oracle.scores("transe_l2", E, R, h, r, t, neg, k, chunk, side, 3.0)
        pr, nr = oracle.scores("transr", E, Rt, h, r, t, neg, k, chunk, side, 3.0)
        np.testing.assert_allclose(3.0 - pr, (3.0 - p2) ** 2, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(3.0 - nr, (3.0 - n2) ** 2, rtol=1e-12, atol=1e-12)
    Rm = np.concatenate([R, rng.normal(size=(R.shape[0], D * D))], axis=1)
    a = oracle.scores("transr", E, Rm, h, r, t, neg, k, chunk, 0, 3.0)
    b = oracle.scores("transr", E + rng.normal(size=(1, D)), Rm, h, r, t, neg, k, chunk, 0, 3.0)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-10, atol=1e-10)
