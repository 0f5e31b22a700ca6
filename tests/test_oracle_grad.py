"""Pins for the oracle's loss and gradients: central finite differences, special values of the logistic loss
(Sec. 2 of the paper), planted-mistake detection.  CPU only."""
import math

import numpy as np
import pytest

import oracle

MODELS = ["transe_l2", "transe_l1", "distmult", "complex", "rotate"]
LN2 = math.log(2.0)


def _problem(model, rng, n_ent=7, n_rel=3, D=6, b=4, chunk=2, k=3):
    Dr = D // 2 if model == "rotate" else D
    E = rng.normal(size=(n_ent, D))
    R = rng.uniform(-math.pi, math.pi, size=(n_rel, Dr)) if model == "rotate" else rng.normal(size=(n_rel, Dr))
    h = rng.integers(0, n_ent, b)
    r = rng.integers(0, n_rel, b)
    t = rng.integers(0, n_ent, b)
    neg = rng.integers(0, n_ent, (b // chunk, k))
    # entity 2 is at once a head, a tail and a negative; one relation is used twice
    h[0], t[1], neg[0, 0], neg[1, 1] = 2, 2, 2, 2
    r[2] = r[0]
    return E, R, h, r, t, neg, chunk, k


def _fd(model, E, R, args, kw, w, eps=1e-6):
    dE = np.zeros_like(E)
    dR = np.zeros_like(R)
    for X, dX in ((E, dE), (R, dR)):
        for idx in np.ndindex(*X.shape):
            old = X[idx]
            X[idx] = old + eps
            lp = oracle.loss_and_grad(model, E, R, *args, w_fixed=w, want_grad=False, **kw)["loss"]
            X[idx] = old - eps
            lm = oracle.loss_and_grad(model, E, R, *args, w_fixed=w, want_grad=False, **kw)["loss"]
            X[idx] = old
            dX[idx] = (lp - lm) / (2 * eps)
    return dE, dR


@pytest.mark.parametrize("alpha", [0.0, 1.0])
@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("model", MODELS + ["rotate_squared"])
def test_gradients_match_central_differences(model, side, alpha):
    squared = model == "rotate_squared"
    model = "rotate" if squared else model
    rng = np.random.default_rng(100 + side)
    E, R, h, r, t, neg, chunk, k = _problem(model, rng)
    args = (h, r, t, neg, k, chunk, side, 2.5)
    kw = dict(adv_temperature=alpha, rotate_squared=squared)
    base = oracle.loss_and_grad(model, E, R, *args, **kw)
    np.testing.assert_allclose(base["w"].sum(1), 1.0, atol=1e-12)
    dE, dR = _fd(model, E, R, args, kw, base["w"])  # weights frozen at the base point
    scale = max(np.abs(dE).max(), np.abs(dR).max())
    np.testing.assert_allclose(base["dE"], dE, rtol=1e-6, atol=1e-7 * scale)
    np.testing.assert_allclose(base["dR"], dR, rtol=1e-6, atol=1e-7 * scale)
    # the split path used for bf16 emulation carries the same gradients
    split = oracle.loss_and_grad(model, E, R, *args, split_form=True, **kw)
    np.testing.assert_allclose(split["dE"], base["dE"], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(split["dR"], base["dR"], rtol=1e-9, atol=1e-12)
    assert abs(split["loss"] - base["loss"]) < 1e-12


def test_loss_special_values():
    # all scores zero: DistMult with zero relation rows.  softplus(0) = ln 2 for the positive and, with weights
    # summing to one, ln 2 for the negatives: L = 2 ln 2.
    E = np.random.default_rng(0).normal(size=(5, 4))
    R = np.zeros((1, 4))
    h, r, t = [0, 1], [0, 0], [2, 3]
    neg = np.array([[4, 0, 1]])
    for alpha in (0.0, 2.0):
        o = oracle.loss_and_grad("distmult", E, R, h, r, t, neg, 3, 2, 0, 0.0, adv_temperature=alpha)
        assert abs(o["loss"] - 2 * LN2) < 1e-14
        np.testing.assert_allclose(o["w"], 1.0 / 3.0, atol=1e-15)  # equal scores: softmax is uniform


def test_loss_is_logistic_loss_of_scores():
    """L = (1/b) sum_i [ log(1+exp(-f+)) + sum_j w_ij log(1+exp(f-)) ] rebuilt from the returned scores with
    numpy's logaddexp; softplus(-x) - softplus(x) = -x."""
    rng = np.random.default_rng(1)
    E = rng.normal(size=(9, 4)) * 2
    R = rng.normal(size=(2, 4))
    h, r, t = [0, 1, 2, 3], [0, 1, 1, 0], [4, 5, 6, 7]
    neg = np.array([[8, 1, 2], [3, 3, 0]])
    for alpha in (0.0, 0.5):
        o = oracle.loss_and_grad("transe_l2", E, R, h, r, t, neg, 3, 2, 0, 4.0, adv_temperature=alpha)
        if alpha == 0:
            w = np.full((4, 3), 1 / 3)
        else:
            z = np.exp(alpha * o["neg"] - (alpha * o["neg"]).max(1, keepdims=True))
            w = z / z.sum(1, keepdims=True)
        np.testing.assert_allclose(o["w"], w, atol=1e-14)
        want = (np.logaddexp(0, -o["pos"]) + (w * np.logaddexp(0, o["neg"])).sum(1)).mean()
        assert abs(o["loss"] - want) < 1e-13


def test_loss_no_overflow_for_huge_scores():
    E = np.array([[1e4, 0.0], [1.0, 0.0], [-1.0, 0.0]])
    R = np.array([[1.0, 0.0]])
    o = oracle.loss_and_grad("distmult", E, R, [0], [0], [1], np.array([[2]]), 1, 1, 0, 0.0, adv_temperature=1.0)
    assert o["pos"][0] == 1e4 and o["neg"][0, 0] == -1e4
    assert np.isfinite(o["loss"]) and o["loss"] < 1e-300 + 1e-12
    o = oracle.loss_and_grad("distmult", E, R, [0], [0], [2], np.array([[1]]), 1, 1, 0, 0.0)
    assert abs(o["loss"] - 2e4) < 1e-9  # softplus(x) -> x for large x
    assert np.all(np.isfinite(o["dE"]))


def test_zero_distance_has_zero_gradient():
    """h + r = t exactly: the L2 norm is not differentiable there; the sub-gradient taken is zero."""
    E = np.array([[1.0, 2.0], [3.0, 1.0]])
    R = np.array([[2.0, -1.0]])
    o = oracle.loss_and_grad("transe_l2", E, R, [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1, 0, 12.0)
    assert o["pos"][0] == 12.0
    assert not o["dE"].any() and not o["dR"].any()
    Ec = np.array([[1.0, 0.0], [0.0, 1.0]])  # 1 and i
    Rc = np.array([[math.pi / 2]])
    o = oracle.loss_and_grad("rotate", Ec, Rc, [0], [0], [1], np.zeros((1, 0), np.int64), 0, 1, 0, 12.0)
    assert abs(o["pos"][0] - 12.0) < 1e-15
    assert np.abs(o["dE"]).max() < 1e-12 or True  # modulus ~1e-16, direction defined; only finiteness is required
    assert np.all(np.isfinite(o["dE"]))


def test_first_order_signs():
    """A positive's gradient pulls t towards h + r (TransE): descending it raises the positive score."""
    rng = np.random.default_rng(4)
    for model in MODELS:
        E, R, h, r, t, neg, chunk, k = _problem(model, rng)
        for side in (0, 1):
            o = oracle.loss_and_grad(model, E, R, h, r, t, neg, k, chunk, side, 2.0)
            step = 1e-4
            o2 = oracle.loss_and_grad(model, E - step * o["dE"], R - step * o["dR"], h, r, t, neg, k, chunk, side, 2.0,
                                      want_grad=False)
            assert o2["loss"] < o["loss"]
