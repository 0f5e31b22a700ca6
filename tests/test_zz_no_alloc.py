"""kge_score_noalloc, the entry point for callers that cannot allocate device memory: its scratch is a fixed array in
the library's device image.  Checked through the C ABI against kge_score (same kernels, so the bits must agree) and
against the oracle, on two calls in a row of which the second is smaller, for every model it serves."""
import numpy as np
import pytest
import torch

import oracle
from harness import configs
from parity_util import SCORE_TOL, dev, rel_err

pytestmark = pytest.mark.gpu

MODELS = ["transe_l2", "transe_l1", "distmult", "complex", "rotate"]


def _workload(model, batch, chunk, k):
    return configs.Workload(name="noalloc-" + model, model=model, n_entities=517, n_relations=11, n_triples=4000,
                            s_entity=1.0, s_relation=None, ent_dim=72, rel_dim=36 if model == "rotate" else 72,
                            batch=batch, chunk=chunk, neg_per_chunk=k, neg_mode="uniform", side_mode="alternate",
                            gamma=6.0, lr=0.1, steps=2, seed=5)


@pytest.mark.parametrize("model", MODELS)
def test_noalloc_scores_equal_kge_score_on_two_calls_in_a_row(model):
    import paper_2004_08532_amd as kge
    big, small = _workload(model, 90, 45, 37), _workload(model, 30, 15, 5)
    E, R = configs.init_tables(big)
    dE, dR = dev(E), dev(R)
    ctx = kge.KgeContext(model, big.n_entities, big.n_relations, big.ent_dim, big.rel_dim, max_batch=big.batch,
                         max_neg_per_chunk=big.neg_per_chunk, max_chunks=big.n_chunks)
    try:
        for w, side in ((big, 0), (small, 1)):  # the second call is smaller: stale scratch beyond its rows must not matter
            h, r, t, neg, _ = configs.BatchStream(w).step(0)
            b, k = w.batch, w.neg_per_chunk
            dh, dr, dt, dn = dev(h), dev(r), dev(t), dev(neg.reshape(-1))
            want_pos = torch.empty(b, device="cuda")
            want_neg = torch.empty((b, k), device="cuda")
            ctx.score(dE, dR, dh, dr, dt, dn, k, w.chunk, side, w.gamma, pos_out=want_pos, neg_out=want_neg)
            got_pos = torch.full((b,), float("nan"), device="cuda")
            got_neg = torch.full((b, k), float("nan"), device="cuda")
            kge.kge_score_noalloc(ctx.cfg, dE, dR, dh, dr, dt, b, dn, k, w.chunk, side, w.gamma, None, got_pos, got_neg)
            torch.cuda.synchronize()
            assert torch.equal(got_pos, want_pos) and torch.equal(got_neg, want_neg)
            opos, oneg = oracle.scores(model, E, R, h, r, t, neg, k, w.chunk, side, w.gamma)
            assert rel_err(got_pos.cpu().numpy(), opos, 1.0) <= SCORE_TOL
            assert rel_err(got_neg.cpu().numpy(), oneg, 1.0) <= SCORE_TOL
        # positives only
        got_pos = torch.full((small.batch,), float("nan"), device="cuda")
        kge.kge_score_noalloc(ctx.cfg, dE, dR, dh, dr, dt, small.batch, None, 0, small.chunk, 1, small.gamma, None,
                              got_pos, None)
        torch.cuda.synchronize()
        assert torch.equal(got_pos, want_pos)
    finally:
        ctx.close()


def test_noalloc_rejects_what_does_not_fit_its_scratch_and_what_it_does_not_serve():
    import paper_2004_08532_amd as kge
    w = _workload("distmult", 64, 32, 8)
    E, R = configs.init_tables(w)
    dE, dR = dev(E), dev(R)
    cfg = kge.kge_config(kge.KGE_DISTMULT, 0, w.n_entities, w.n_relations, w.ent_dim, w.rel_dim, 0, 0, 0, 0, 0, 0.0, 0.0,
                         0, 0)
    b, k = 8192, 4096  # 4 * 72 * (8192 + 4096) bytes = 3.4 MiB fits; with 4 chunks 4 * 72 * (8192 + 16384) = 6.8 MiB fits;
    ids = torch.zeros(b, dtype=torch.int64, device="cuda")
    negs = torch.zeros(8 * k, dtype=torch.int64, device="cuda")
    pos = torch.empty(b, device="cuda")
    out = torch.empty((b, k), device="cuda")
    kge.kge_score_noalloc(cfg, dE, dR, ids, ids, ids, b, negs, k, b // 4, 0, 1.0, None, pos, out)  # 6.8 MiB: runs
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    before = out.clone()
    with pytest.raises(kge.KgeError) as e:  # 8 chunks: 4 * 72 * (8192 + 32768) = 11.3 MiB > 8 MiB
        kge.kge_score_noalloc(cfg, dE, dR, ids, ids, ids, b, negs, k, b // 8, 0, 1.0, None, pos, out)
    assert e.value.code == kge.KGE_ERR_WORKSPACE and "8 MiB" in str(e.value)
    torch.cuda.synchronize()
    assert torch.equal(out, before)  # nothing was enqueued
    bad = kge.kge_config(kge.KGE_RESCAL, 0, w.n_entities, w.n_relations, 8, 64, 0, 0, 0, 0, 0, 0.0, 0.0, 0, 0)
    with pytest.raises(kge.KgeError) as e:
        kge.kge_score_noalloc(bad, dE, dR, ids, ids, ids, 8, negs, 4, 8, 0, 1.0, None, pos, out)
    assert e.value.code == kge.KGE_ERR_UNSUPPORTED
    cfg.gemm_input = 1
    with pytest.raises(kge.KgeError) as e:
        kge.kge_score_noalloc(cfg, dE, dR, ids, ids, ids, 8, negs, 4, 8, 0, 1.0, None, pos, out)
    assert e.value.code == kge.KGE_ERR_UNSUPPORTED


def test_noalloc_makes_no_device_allocation():
    """torch's allocator statistics cannot see a hipMalloc made by the library, but the device's free memory can:
    it must not move across calls (after the first, which may load kernels)."""
    import paper_2004_08532_amd as kge
    w = _workload("transe_l2", 90, 45, 37)
    E, R = configs.init_tables(w)
    dE, dR = dev(E), dev(R)
    cfg = kge.kge_config(kge.KGE_TRANSE_L2, 0, w.n_entities, w.n_relations, w.ent_dim, w.rel_dim, 0, 0, 0, 0, 0, 0.0, 0.0,
                         0, 0)
    h, r, t, neg, _ = configs.BatchStream(w).step(0)
    dh, dr, dt, dn = dev(h), dev(r), dev(t), dev(neg.reshape(-1))
    pos = torch.empty(w.batch, device="cuda")
    out = torch.empty((w.batch, w.neg_per_chunk), device="cuda")
    kge.kge_score_noalloc(cfg, dE, dR, dh, dr, dt, w.batch, dn, w.neg_per_chunk, w.chunk, 0, w.gamma, None, pos, out)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(20):
        kge.kge_score_noalloc(cfg, dE, dR, dh, dr, dt, w.batch, dn, w.neg_per_chunk, w.chunk, 0, w.gamma, None, pos, out)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
