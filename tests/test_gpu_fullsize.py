"""Parity at the size and in the launch configuration that bench.py times, for every named configuration at its full
entity count: the Freebase-scale TransE-L2 and ComplEx steps with the full 86,054,151 x 400 entity table and its
Adagrad state resident in HBM (256.5 GiB), 'medium' (2.5 M entities, RotatE, in-batch degree negatives,
self-adversarial weights) and 'large' (5 M entities, TransE-L2 with bf16 operands).

The oracle cannot hold these tables, and does not need to: a step reads and writes only the rows its ids name.  For
every checked step the rows of the distinct ids are copied from the device into a compact host table, the ids are
renumbered by their rank among the distinct ids (which keeps their order, so the duplicate reduction sees the same
runs), and the oracle performs the step on the compact table.  Every element of every touched row is then compared
as in the small-size tests.  The rest of the table is covered by a property: rows outside the batch keep their bits.

Launch configuration: bench.py drives kge_train_steps on a side stream, which replays HIP graphs of 1, 2, 4, 8,
16 and 32 steps.  The
same steps are therefore run a second time through kge_train_steps from the same rows, and must reproduce the
step-by-step result bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from harness import configs, graphs
from parity_util import ALLOWANCE_SHARE, EMB_TOL, SCORE_TOL, rounding_allowance

pytestmark = pytest.mark.gpu

N_CHECKED = 3   # steps checked one by one against the oracle
N_REPLAY = 95   # steps run again through kge_train_steps (replayed graphs of 1, 2, 4, 8, 16, 32, 32 steps)


def _compact(ids_list):
    """distinct ids (ascending) and a function that renumbers an id array by rank among them"""
    uniq = np.unique(np.concatenate([np.asarray(x).reshape(-1) for x in ids_list]))
    return uniq, (lambda x: np.searchsorted(uniq, x).astype(np.int64))


def _rows(t: torch.Tensor, ids: np.ndarray) -> np.ndarray:
    return t[torch.from_numpy(ids).cuda()].cpu().numpy()


@pytest.mark.parametrize("w", [configs.FREEBASE_TRANSE, configs.FREEBASE_COMPLEX, configs.MEDIUM, configs.LARGE],
                         ids=lambda w: w.name)
def test_full_size_step_with_the_whole_table_resident(w):
    import paper_2004_08532_amd as kge

    dev = torch.device("cuda", 0)
    need = 2 * (w.n_entities * w.ent_dim + w.n_relations * w.rel_dim) * 4
    torch.cuda.empty_cache()  # give back what earlier tests left in the allocator's cache
    free, _ = torch.cuda.mem_get_info(dev)
    if need + (4 << 30) > free:
        pytest.skip(f"needs {need / 2**30:.1f} GiB of HBM, {free / 2**30:.1f} GiB free")

    # positives straight from the generating distribution (an i.i.d. triple list sampled with replacement is the same
    # thing), so that the 16 M / 20 M triples of 'medium' / 'large' need not be drawn on the host first
    bs = configs.BatchStream(w, materialise=False)
    n_steps = N_CHECKED + N_REPLAY
    h, r, t, neg, sides = bs.steps(0, n_steps)
    neg = neg.reshape(n_steps, -1)
    E, R = configs.init_tables(w, device=dev)
    SE, SR = torch.zeros_like(E), torch.zeros_like(R)
    ctx = kge.KgeContext(w.model, w.n_entities, w.n_relations, w.ent_dim, w.rel_dim, max_batch=w.batch,
                         max_neg_per_chunk=w.neg_per_chunk, max_chunks=w.n_chunks, gemm_input=int(w.bf16_inputs),
                         adv_temperature=w.adv_temperature)
    floor = graphs.init_bound(w.gamma, w.ent_dim)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    dh, dr, dt, dn = (torch.from_numpy(x).to(dev) for x in (h, r, t, neg))
    stats = {"elements": 0, "needed_allowance": 0, "worst_ratio": 0.0}
    try:
        # rows that no step of this test names must keep their bits: a sample of them
        rng = np.random.default_rng(7)
        named = np.unique(np.concatenate([h.reshape(-1), t.reshape(-1), neg.reshape(-1)]))
        probe = np.setdiff1d(rng.integers(0, w.n_entities, 4096), named)
        probe = np.concatenate([probe, np.setdiff1d(np.array([0, w.n_entities - 1]), named)])
        probe_before = _rows(E, probe)

        # ---- steps checked one by one against the oracle on compact tables
        for s in range(N_CHECKED):
            ent_ids, renum = _compact([h[s], t[s], neg[s]])
            rel_ids = np.unique(r[s])
            Ec, SEc = _rows(E, ent_ids), _rows(SE, ent_ids)
            Rh, SRh = R.cpu().numpy(), SR.cpu().numpy()
            S_prev = {"E": SEc.astype(np.float64), "R": SRh[rel_ids].astype(np.float64)}
            ctx.train_step(E, SE, R, SR, dh[s], dr[s], dt[s], dn[s], w.neg_per_chunk, w.chunk, int(sides[s]), w.gamma,
                           w.lr, loss_out=loss)
            torch.cuda.synchronize()
            want_loss, rep = oracle.train_step(w.model, Ec, SEc, Rh, SRh, renum(h[s]), r[s], renum(t[s]),
                                               renum(neg[s]).reshape(w.n_chunks, -1), w.neg_per_chunk, w.chunk,
                                               int(sides[s]), w.gamma, w.lr, report=True,
                                               adv_temperature=w.adv_temperature, bf16_inputs=w.bf16_inputs)
            got_loss = float(loss.item())
            assert abs(got_loss - want_loss) <= SCORE_TOL * max(1.0, abs(want_loss)), (s, got_loss, want_loss)
            assert np.array_equal(rep["ent_ids"], np.arange(ent_ids.shape[0])) and np.array_equal(rep["rel_ids"], rel_ids)
            uniq, cnt = ctx.get_dedup(0, 2 * w.batch + neg.shape[1])
            ou, oc = oracle.dedup(np.concatenate([h[s], t[s], neg[s]]))
            assert np.array_equal(uniq.cpu().numpy(), ou) and np.array_equal(cnt.cpu().numpy().astype(np.int64), oc)
            for name, ids, want, want_s, devt, devs, g, A, M in (
                    ("E", ent_ids, Ec, SEc, E, SE, rep["dE"], rep["absE"], rep["maxE"]),
                    ("R", rel_ids, Rh[rel_ids], SRh[rel_ids], R, SR, rep["dR"], rep["absR"], rep["maxR"])):
                got = _rows(devt, ids).astype(np.float64)
                got_s = _rows(devs, ids).astype(np.float64)
                want, want_s = want.astype(np.float64), want_s.astype(np.float64)
                du, ds = rounding_allowance(g, A, S_prev[name], w.lr, 1e-10, M if w.bf16_inputs else None)
                base = EMB_TOL * np.maximum(np.abs(want), floor)
                ratio = np.abs(got - want) / (base + du)
                stats["elements"] += ratio.size
                stats["needed_allowance"] += int((np.abs(got - want) > base).sum())
                stats["worst_ratio"] = max(stats["worst_ratio"], float(ratio.max()))
                assert ratio.max() <= 1.0, (s, name, float(ratio.max()))
                s_ratio = np.abs(got_s - want_s) / (1e-5 * want_s + ds + 1e-30)
                assert s_ratio.max() <= 1.0, (s, name + " state", float(s_ratio.max()))
        print("\n[parity]", w.name, "full table", stats)
        assert stats["needed_allowance"] <= max(4, ALLOWANCE_SHARE["default"] * stats["elements"]), stats

        # ---- the launch configuration of the benchmark: kge_train_steps on a side stream (replayed graphs) must give
        # the bits of step-by-step calls.  Rows named by these steps are saved, the steps run one by one, the results
        # saved, the rows restored, and the same steps run again through kge_train_steps.
        lo, hi = N_CHECKED, n_steps
        ent_ids = np.unique(np.concatenate([h[lo:hi].reshape(-1), t[lo:hi].reshape(-1), neg[lo:hi].reshape(-1)]))
        rel_ids = np.unique(r[lo:hi])
        ei, ri = torch.from_numpy(ent_ids).cuda(), torch.from_numpy(rel_ids).cuda()
        saved = [E[ei].clone(), SE[ei].clone(), R[ri].clone(), SR[ri].clone()]
        losses_a = torch.zeros(hi - lo, dtype=torch.float32, device=dev)
        for s in range(lo, hi):
            ctx.train_step(E, SE, R, SR, dh[s], dr[s], dt[s], dn[s], w.neg_per_chunk, w.chunk, int(sides[s]), w.gamma,
                           w.lr, loss_out=losses_a[s - lo:s - lo + 1])
        torch.cuda.synchronize()
        result_a = [E[ei].clone(), SE[ei].clone(), R[ri].clone(), SR[ri].clone()]
        E[ei], SE[ei], R[ri], SR[ri] = saved
        losses_b = torch.zeros(hi - lo, dtype=torch.float32, device=dev)
        stream = torch.cuda.Stream(device=dev)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            ctx.train_steps(E, SE, R, SR, dh[lo:hi], dr[lo:hi], dt[lo:hi], dn[lo:hi], w.neg_per_chunk, w.chunk,
                            sides[lo:hi].tolist(), w.gamma, w.lr, loss_out=losses_b)
        torch.cuda.synchronize()
        for a, b_ in zip(result_a, [E[ei], SE[ei], R[ri], SR[ri]]):
            assert torch.equal(a, b_)
        assert torch.equal(losses_a, losses_b)

        assert np.array_equal(_rows(E, probe), probe_before)
        assert float(SE[torch.from_numpy(probe).cuda()].abs().max()) == 0.0
    finally:
        ctx.close()
        del E, SE, R, SR
        torch.cuda.empty_cache()
