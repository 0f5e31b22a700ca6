"""Pins for the oracle's duplicate handling and Adagrad update (step 4 of the mini-batch loop, Sec. 3.1).
CPU only."""
import math

import numpy as np
import pytest

import oracle


def test_dedup_against_brute_force():
    rng = np.random.default_rng(0)
    for n in (1, 2, 17, 300):
        keys = rng.integers(0, max(2, n // 3), n)
        uniq, cnt = oracle.dedup(keys)
        assert np.all(np.diff(uniq) > 0)
        assert cnt.sum() == n
        for u, c in zip(uniq, cnt):  # O(n^2) count
            assert c == sum(1 for x in keys if x == u)
        assert set(uniq.tolist()) == set(keys.tolist())
    uniq, cnt = oracle.dedup(np.zeros(0, np.int64))
    assert uniq.size == 0 and cnt.size == 0
    big = np.array([2 ** 40 + 3, 5, 2 ** 40 + 3, 86_054_150], dtype=np.int64)
    uniq, cnt = oracle.dedup(big)
    assert uniq.tolist() == [5, 86_054_150, 2 ** 40 + 3] and cnt.tolist() == [1, 1, 2]


def test_adagrad_closed_form_constant_gradient():
    """Constant gradient g for T steps from S = 0: theta_T = theta_0 - lr * sum_tau g / (sqrt(tau) |g| + eps)."""
    g = np.array([[0.5, -2.0, 1e-3, 0.0]])
    th0 = np.array([[1.0, 2.0, 3.0, 4.0]], dtype=np.float32)
    th = th0.copy()
    st = np.zeros_like(th)
    lr, eps, T = 0.1, 1e-10, 7
    for _ in range(T):
        oracle.adagrad_rows(th, st, None, g, lr, eps)
    want = th0.astype(np.float64) - lr * sum(g / (math.sqrt(tau) * np.abs(g) + eps) for tau in range(1, T + 1))
    np.testing.assert_allclose(th, want, rtol=3e-7)
    np.testing.assert_allclose(st, T * g * g, rtol=3e-7)
    assert th[0, 3] == th0[0, 3] and st[0, 3] == 0.0  # zero gradient: bit-unchanged


def test_first_step_moves_by_lr_times_sign():
    g = np.array([[3.0, -1e-4, 7e2]])
    th = np.zeros((1, 3), np.float32)
    st = np.zeros_like(th)
    oracle.adagrad_rows(th, st, None, g, 0.25, 1e-10)
    np.testing.assert_allclose(th, -0.25 * np.sign(g), rtol=1e-5)


def _small_step_inputs(model="transe_l2"):
    rng = np.random.default_rng(2)
    n_ent, n_rel, D = 40, 4, 8
    Dr = D // 2 if model == "rotate" else D
    E = rng.uniform(-0.3, 0.3, (n_ent, D)).astype(np.float32)
    R = rng.uniform(-0.3, 0.3, (n_rel, Dr)).astype(np.float32)
    h = rng.integers(0, 10, 8)
    r = rng.integers(0, n_rel, 8)
    t = rng.integers(0, 10, 8)
    neg = rng.integers(0, 10, (2, 3))
    return E, R, h, r, t, neg


def test_duplicates_are_summed_before_squaring():
    """An entity hit twice in one step gets S = (g1 + g2)^2, not g1^2 + g2^2: compare one step with the row
    duplicated against the Adagrad rule applied by numpy to the summed dense gradient."""
    for model in ("transe_l2", "distmult", "complex", "rotate"):
        E, R, h, r, t, neg = _small_step_inputs(model)
        h[:] = 3  # every positive shares its head
        g = oracle.loss_and_grad(model, E, R, h, r, t, neg, 3, 4, 0, 2.0)
        E1, R1 = E.copy(), R.copy()
        SE, SR = np.zeros_like(E), np.zeros_like(R)
        oracle.train_step(model, E1, SE, R1, SR, h, r, t, neg, 3, 4, 0, 2.0, 0.1)
        np.testing.assert_allclose(SE, g["dE"] ** 2, rtol=2e-7, atol=0)
        wantE = E - 0.1 * g["dE"] / (np.sqrt(g["dE"] ** 2) + 1e-10)
        np.testing.assert_allclose(E1, wantE, rtol=2e-6, atol=1e-7)
        np.testing.assert_allclose(SR, g["dR"] ** 2, rtol=2e-7, atol=0)


@pytest.mark.parametrize("model", ["transe_l2", "transe_l1", "distmult", "complex", "rotate"])
def test_dense_update_equals_touched_rows_update_bit_for_bit(model):
    E, R, h, r, t, neg = _small_step_inputs(model)
    outs = []
    for dense in (True, False):
        E1, R1 = E.copy(), R.copy()
        SE, SR = np.zeros_like(E), np.zeros_like(R)
        losses = [oracle.train_step(model, E1, SE, R1, SR, h, r, t, neg, 3, 4, s % 2, 2.0, 0.1, dense=dense,
                                    adv_temperature=0.5) for s in range(3)]
        outs.append((E1, SE, R1, SR, losses))
    for a, b in zip(outs[0][:4], outs[1][:4]):
        assert a.tobytes() == b.tobytes()
    assert outs[0][4] == outs[1][4]
    # rows outside the batch keep their bits (only rows of the mini-batch are updated, Sec. 2)
    touched = np.unique(np.concatenate([h, t, neg.ravel()]))
    mask = np.ones(E.shape[0], bool)
    mask[touched] = False
    assert outs[0][0][mask].tobytes() == E[mask].tobytes()
    assert not outs[0][1][mask].any()


def test_train_step_rejects_bad_ids():
    E, R, h, r, t, neg = _small_step_inputs()
    SE, SR = np.zeros_like(E), np.zeros_like(R)
    h2 = h.copy()
    h2[0] = E.shape[0]
    with pytest.raises(ValueError):
        oracle.train_step("transe_l2", E, SE, R, SR, h2, r, t, neg, 3, 4, 0, 2.0, 0.1)
    with pytest.raises(ValueError):
        oracle.train_step("transe_l2", E, SE, R, SR, h[:7], r[:7], t[:7], neg[:1], 3, 4, 0, 2.0, 0.1)


# ---- row-wise state: one accumulator per row, fed with the mean of the squared gradient elements

def test_rowwise_adagrad_hand_example_and_closed_form():
    """g = (3, -4, 0, 0): mean g^2 = 25/4, so the first step divides by 5/2: x -= lr * g * 2/5.  Constant g for T
    steps: S_T = T * mean g^2 and x_T = x_0 - lr * g * sum_tau 1 / (sqrt(tau * mean g^2) + eps)."""
    g = np.array([[3.0, -4.0, 0.0, 0.0]])
    th0 = np.array([[1.0, 2.0, 3.0, 4.0]], dtype=np.float32)
    th, st = th0.copy(), np.zeros(1, np.float32)
    oracle.adagrad_rows(th, st, None, g, 0.5, 1e-10, rowwise=True)
    np.testing.assert_allclose(th, [[1.0 - 0.6, 2.0 + 0.8, 3.0, 4.0]], rtol=3e-7)
    assert st[0] == np.float32(6.25)
    assert th[0, 2] == th0[0, 2] and th[0, 3] == th0[0, 3]   # zero elements of a touched row do not move
    th, st = th0.copy(), np.zeros(1, np.float32)
    lr, eps, T = 0.1, 1e-10, 6
    for _ in range(T):
        oracle.adagrad_rows(th, st, None, g, lr, eps, rowwise=True)
    want = th0.astype(np.float64) - lr * g * sum(1.0 / (math.sqrt(tau * 6.25) + eps) for tau in range(1, T + 1))
    np.testing.assert_allclose(th, want, rtol=3e-7)
    np.testing.assert_allclose(st, [T * 6.25], rtol=3e-7)


def test_rowwise_equals_elementwise_when_all_elements_have_the_same_magnitude():
    g = np.array([[0.5, -0.5, 0.5, -0.5], [2.0, 2.0, -2.0, 2.0]])
    th_e = np.arange(8, dtype=np.float32).reshape(2, 4)
    th_r = th_e.copy()
    st_e, st_r = np.zeros_like(th_e), np.zeros(2, np.float32)
    for _ in range(4):
        oracle.adagrad_rows(th_e, st_e, None, g, 0.3, 1e-10)
        oracle.adagrad_rows(th_r, st_r, None, g, 0.3, 1e-10, rowwise=True)
    assert th_e.tobytes() == th_r.tobytes()
    assert np.array_equal(st_e[:, 0], st_r)


def test_rowwise_step_sums_duplicates_first_and_leaves_other_rows_alone():
    for model in ("transe_l2", "distmult", "complex", "rotate"):
        E, R, h, r, t, neg = _small_step_inputs(model)
        h[:] = 3
        g = oracle.loss_and_grad(model, E, R, h, r, t, neg, 3, 4, 0, 2.0)
        outs = []
        for dense in (True, False):
            E1, R1 = E.copy(), R.copy()
            SE, SR = np.zeros(E.shape[0], np.float32), np.zeros(R.shape[0], np.float32)
            oracle.train_step(model, E1, SE, R1, SR, h, r, t, neg, 3, 4, 0, 2.0, 0.1, rowwise=True, dense=dense)
            outs.append((E1, SE, R1, SR))
        for a, b in zip(*outs):
            assert a.tobytes() == b.tobytes()                 # dense == touched rows, bit for bit
        E1, SE, R1, SR = outs[0]
        ms = (g["dE"] ** 2).mean(axis=1)
        np.testing.assert_allclose(SE, ms, rtol=3e-7, atol=0)  # mean of the SUMMED gradient's squares
        wantE = E - 0.1 * g["dE"] / (np.sqrt(ms)[:, None] + 1e-10)
        touched = ms > 0
        np.testing.assert_allclose(E1[touched], wantE[touched], rtol=2e-6, atol=1e-7)
        assert E1[~touched].tobytes() == E[~touched].tobytes()
