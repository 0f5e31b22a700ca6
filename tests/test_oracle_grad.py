"""Pins for the oracle's loss and gradients: central finite differences, special values of the logistic loss
(Sec. 2 of the paper), planted-mistake detection.  CPU only."""
import math

import numpy as np
import pytest

import oracle

MODELS = ["transe_l2", "transe_l1", "distmult", "complex", "rotate", "rescal", "transr"]
LN2 = math.log(2.0)


def _problem(model, rng, n_ent=7, n_rel=3, D=6, b=4, chunk=2, k=3):
    Dr = {"rotate": D // 2, "rescal": D * D, "transr": D + D * D}.get(model, D)
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
    if model == "transr":
        return  # its negatives are projected by the positive's own matrix: no (o, n) split
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


# ---- pairwise ranking loss (Sec. 2, second loss): max(0, gamma - f(positive) + f(negative))

@pytest.mark.parametrize("alpha", [0.0, 1.0])
@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("model", MODELS)
def test_ranking_loss_gradients_match_central_differences(model, side, alpha):
    rng = np.random.default_rng(300 + side)
    E, R, h, r, t, neg, chunk, k = _problem(model, rng)
    # f+ - f- does not depend on gamma for any model; a margin in the middle of its values makes about half of the pairs active
    pos0, neg0 = oracle.scores(model, E, R, h, r, t, neg, k, chunk, side, 0.0)
    vals = np.unique(np.round(pos0[:, None] - neg0, 9))  # (a negative can be the positive's own entity: equal scores)
    gamma = float(0.5 * (vals[len(vals) // 2 - 1] + vals[len(vals) // 2]))
    args = (h, r, t, neg, k, chunk, side, gamma)
    kw = dict(adv_temperature=alpha, loss="ranking")
    base = oracle.loss_and_grad(model, E, R, *args, **kw)
    m = gamma - base["pos"][:, None] + base["neg"]
    assert np.abs(m).min() > 1e-3           # no pair sits on the kink, so the loss is smooth around this point
    assert (m > 0).any() and (m < 0).any()  # both branches of the max are exercised
    dE, dR = _fd(model, E, R, args, kw, base["w"])
    scale = max(np.abs(dE).max(), np.abs(dR).max())
    np.testing.assert_allclose(base["dE"], dE, rtol=1e-6, atol=1e-7 * scale)
    np.testing.assert_allclose(base["dR"], dR, rtol=1e-6, atol=1e-7 * scale)
    if model == "transr":
        return
    split = oracle.loss_and_grad(model, E, R, *args, split_form=True, **kw)
    np.testing.assert_allclose(split["dE"], base["dE"], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(split["dR"], base["dR"], rtol=1e-9, atol=1e-12)


def test_ranking_loss_special_values():
    E = np.random.default_rng(0).normal(size=(5, 4))
    h, r, t = [0, 1], [0, 0], [2, 3]
    neg = np.array([[4, 0, 1]])
    # all scores equal (DistMult with zero relation rows): every pair's term is the margin itself, the weights sum
    # to one per positive and the loss is the mean over positives: L = gamma
    for alpha in (0.0, 2.0):
        o = oracle.loss_and_grad("distmult", E, np.zeros((1, 4)), h, r, t, neg, 3, 2, 0, 0.75, adv_temperature=alpha,
                                 loss="ranking")
        assert abs(o["loss"] - 0.75) < 1e-15
    # one positive with score 2, negatives with scores 3, 1.5, -4, margin 1: terms 2, 0.5, 0 -> L = 2.5 / 3;
    # dL/df+ = -(2 active pairs) / 3, and f+ = h0 * r0 * t0 with d f+/d h0 = r0 t0 = 2
    E1 = np.array([[1.0], [2.0], [3.0], [1.5], [-4.0]])
    R1 = np.array([[1.0]])
    o = oracle.loss_and_grad("distmult", E1, R1, [0], [0], [1], np.array([[2, 3, 4]]), 3, 1, 0, 1.0, loss="ranking")
    assert o["pos"][0] == 2.0 and list(o["neg"][0]) == [3.0, 1.5, -4.0]
    assert abs(o["loss"] - 2.5 / 3) < 1e-15
    # h0 takes -(2/3) * 2 from the positive and +(1/3) * (3 + 1.5) from the two active negatives (d f-/d h0 = r0 n)
    assert abs(o["dE"][0, 0] - (-(2 / 3) * 2 + (1 / 3) * 4.5)) < 1e-15
    assert abs(o["dE"][4, 0]) == 0.0 and abs(o["dE"][2, 0] - 1 / 3) < 1e-15  # inactive pair: no gradient at all


def test_ranking_loss_zero_when_every_negative_is_beaten_by_the_margin():
    """TransE: positives exact (distance 0), negatives far away: all terms are clipped, loss and gradients vanish,
    and a training step leaves every table bit for bit as it was."""
    E = np.array([[0.0, 0.0], [1.0, 0.0], [50.0, 0.0], [0.0, 60.0]], np.float32)
    R = np.array([[1.0, 0.0]], np.float32)
    o = oracle.loss_and_grad("transe_l2", E.astype(np.float64), R.astype(np.float64), [0], [0], [1],
                             np.array([[2, 3]]), 2, 1, 0, 5.0, loss="ranking")
    assert o["loss"] == 0.0 and not o["dE"].any() and not o["dR"].any()
    E2, R2 = E.copy(), R.copy()
    SE, SR = np.zeros_like(E), np.zeros_like(R)
    loss = oracle.train_step("transe_l2", E2, SE, R2, SR, [0], [0], [1], np.array([[2, 3]]), 2, 1, 0, 5.0, 0.1,
                             loss="ranking")
    assert loss == 0.0 and np.array_equal(E2, E) and np.array_equal(R2, R) and not SE.any() and not SR.any()


def test_ranking_loss_does_not_depend_on_the_offset_inside_distance_scores():
    """For the distance models gamma sits inside both scores and cancels in f- - f+: the loss is
    mean_i sum_j w max(0, gamma + dist+ - dist-), rebuilt here from the distances."""
    rng = np.random.default_rng(5)
    E = rng.normal(size=(9, 4))
    R = rng.normal(size=(2, 4))
    h, r, t = [0, 1, 2, 3], [0, 1, 1, 0], [4, 5, 6, 7]
    neg = np.array([[8, 1, 2], [3, 3, 0]])
    o = oracle.loss_and_grad("transe_l2", E, R, h, r, t, neg, 3, 2, 1, 0.1, loss="ranking")
    dpos = np.linalg.norm(E[h] + R[r] - E[t], axis=1)
    dneg = np.stack([np.linalg.norm(E[neg[i // 2]] + R[r[i]] - E[t[i]], axis=1) for i in range(4)])
    terms = np.maximum(0.0, 0.1 + dpos[:, None] - dneg)
    assert (terms > 0).any() and (terms == 0).any()
    assert abs(o["loss"] - terms.sum(axis=1).mean() / 3) < 1e-13
