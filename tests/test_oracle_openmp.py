"""The all-cores build of the oracle (the benchmark's CPU baseline: the same C file compiled with OpenMP, positives
dealt to the threads, thread-private accumulators added up afterwards) against the single-thread parity oracle:
the same terms in another order of summation.  CPU only."""
import numpy as np
import pytest

import oracle
from harness import configs


@pytest.mark.parametrize("model,alpha,loss", [("transe_l2", 0.0, "logistic"), ("complex", 1.0, "logistic"),
                                               ("rotate", 1.0, "ranking"), ("distmult", 0.0, "logistic")])
def test_all_cores_build_equals_the_single_thread_oracle(model, alpha, loss):
    w = configs.TINY.scaled(name="omp-" + model, model=model, rel_dim=32 if model == "rotate" else 64,
                            side_mode="alternate", adv_temperature=alpha, loss=loss,
                            gamma=0.5 if loss == "ranking" else 12.0)
    bs = configs.BatchStream(w)
    E, R = configs.init_tables(w)
    SE, SR = np.zeros_like(E), np.zeros_like(R)
    assert oracle.threads() == 1 and oracle.threads(openmp=True) >= 1
    for s in range(3):
        h, r, t, neg, side = bs.step(s)
        # both builds start every step from the single-thread run's tables, so that a last-bit difference of one step
        # is not fed into the next
        E2, SE2, R2, SR2 = E.copy(), SE.copy(), R.copy(), SR.copy()
        args = (h, r, t, neg, w.neg_per_chunk, w.chunk, side, w.gamma, w.lr)
        kw = dict(adv_temperature=alpha, loss=loss, report=True)
        l1, r1 = oracle.train_step(model, E, SE, R, SR, *args, **kw)
        l2, r2 = oracle.train_step(model, E2, SE2, R2, SR2, *args, openmp=True, **kw)
        assert abs(l1 - l2) <= 1e-13 * max(1.0, abs(l1))
        assert np.array_equal(r1["ent_ids"], r2["ent_ids"]) and np.array_equal(r1["rel_ids"], r2["rel_ids"])
        for key in ("dE", "dR", "absE", "absR"):
            scale = np.abs(r1[key]).max() + 1e-300
            np.testing.assert_allclose(r2[key], r1[key], rtol=1e-10, atol=1e-13 * scale)
        np.testing.assert_array_equal(r2["maxE"], r1["maxE"])  # a maximum does not depend on the order
        # stored tables: float32 roundings of values that agree to 1e-13 may differ in the last bit
        np.testing.assert_allclose(E2, E, rtol=3e-7, atol=1e-9)
        np.testing.assert_allclose(R2, R, rtol=3e-7, atol=1e-9)
