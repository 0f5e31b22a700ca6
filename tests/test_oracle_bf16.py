"""Pins for the oracle's bfloat16 rounding and for its bf16_inputs branch (operands of the Sec. 3.3 products rounded
to bfloat16, fp32 accumulation emulated in fp64).  CPU only.

round_bf16 is fixed by exact values (ties, carries, the largest finite number, inf / nan) and by two conversions
that share nothing with it: torch's CPU float32 -> bfloat16 cast and a numpy routine on the bit patterns.  The
bf16_inputs scores, loss and gradients are rebuilt in numpy from the Sec. 3.3 split -- o from the kept entity and the
relation, the (o, n) pairs of a group as matrix products -- on operands rounded by the numpy routine.  A copy of the
oracle with a truncating rounding, and one that leaves the backward coefficient unrounded, must fail these tests.
"""
import os

import numpy as np
import pytest
import torch

import oracle

MODELS = ["transe_l2", "distmult", "complex"]


def bf16_bits(x):
    """float32 -> bfloat16 -> float64 on the bit patterns: keep the upper 16 bits and go one up when the discarded
    half is above one half of the last kept bit, or exactly one half and the last kept bit is odd."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    upper, lower = u >> 16, u & 0xFFFF
    up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    special = (upper & 0x7F80) == 0x7F80  # inf / nan keep their bits
    out = np.where(special, u & 0xFFFF0000, (upper + up.astype(np.uint64)) << 16).astype(np.uint32)
    return out.view(np.float32).astype(np.float64).reshape(f.shape)


def test_round_bf16_exact_values():
    two = 2.0
    cases = [
        (1.0, 1.0), (0.0, 0.0), (-2.5, -2.5),                     # representable: unchanged
        (1 + two ** -8, 1.0),                                      # tie, last kept bit even: down
        (1 + 3 * two ** -8, 1 + two ** -6),                        # tie, last kept bit odd: up to the even neighbour
        (-(1 + two ** -8), -1.0), (-(1 + 3 * two ** -8), -(1 + two ** -6)),   # ties are symmetric in sign
        (1 + two ** -8 + two ** -23, 1 + two ** -7),               # just above a tie: up
        (1 + two ** -8 - two ** -23 * 0.5, 1.0),                   # fp64 value below the tie that fp32 rounds ONTO it
        (1 + two ** -7 - two ** -23, 1 + two ** -7),               # just below the next number
        (2 - two ** -8, 2.0),                                      # tie with carry into the exponent
        (two ** -126, two ** -126),                                # smallest normal
        (two ** -133 + two ** -141, two ** -133),                  # subnormal, a tie on the subnormal grid: even
        (3.3895313892515355e38, 3.3895313892515355e38),            # largest finite bfloat16
        (3.4028234663852886e38, np.inf),                           # largest finite float32 rounds up to inf
        (np.inf, np.inf), (-np.inf, -np.inf),
    ]
    for x, want in cases:
        got = float(oracle.round_bf16(x))
        assert got == want and np.signbit(got) == np.signbit(want), (x, got, want)
    assert np.isnan(float(oracle.round_bf16(np.nan)))
    assert np.signbit(float(oracle.round_bf16(-0.0)))
    # the value is first held as float32 (the library forms o in fp32): 1 + 2^-8 - 2^-25 is below the tie in fp64 but
    # IS the tie once stored as float32, so it goes to the even neighbour 1.0 and not up
    assert float(oracle.round_bf16(1 + two ** -8 - two ** -25)) == 1.0


def _finite_bit_patterns(rng, n):
    u = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
    u = u[(u & 0x7F800000) != 0x7F800000]  # no inf / nan
    return u.view(np.float32).astype(np.float64)


def test_round_bf16_against_two_independent_conversions():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.normal(size=20000), rng.normal(size=5000) * 1e-3, rng.normal(size=5000) * 1e4,
        # every tie and near-tie around a stretch of bfloat16 numbers
        (1.0 + np.arange(0, 1024) * 2.0 ** -10), -(0.75 + np.arange(0, 1024) * 2.0 ** -11),
        _finite_bit_patterns(rng, 20000),
    ])
    got = oracle.round_bf16(x)
    bits = bf16_bits(x)
    via_torch = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, bits)
    assert np.array_equal(got, via_torch)
    ties = np.abs(x.astype(np.float32).view(np.uint32) & 0xFFFF) == 0x8000
    assert ties.sum() > 100  # the sample does exercise the tie rule


# ------------------------------------------------------------------------------------------------------------------
# the bf16_inputs branch against the products of Sec. 3.3 written out in numpy


def _problem(model, rng, n_ent=29, n_rel=5, D=8, b=12, chunk=4, k=5):
    E = rng.normal(size=(n_ent, D)).astype(np.float32)
    R = rng.normal(size=(n_rel, D)).astype(np.float32)
    h = rng.integers(0, n_ent, b)
    r = rng.integers(0, n_rel, b)
    t = rng.integers(0, n_ent, b)
    neg = rng.integers(0, n_ent, (b // chunk, k))
    h[0], t[1], neg[0, 0], neg[1, 1] = 2, 2, 2, 2  # one entity as head, tail and corrupting entity
    return E, R, h, r, t, neg, chunk, k


def _phi(model, a, rr, side):
    C = a.shape[1] // 2
    if model == "transe_l2":
        return a - rr if side == 1 else a + rr
    if model == "distmult":
        return a * rr
    rc = rr[:, :C] + 1j * rr[:, C:]
    oc = (a[:, :C] + 1j * a[:, C:]) * (np.conj(rc) if side == 1 else rc)
    return np.concatenate([oc.real, oc.imag], axis=1)


def _phi_backward(model, a, rr, go, side):
    """ga = J_a^T go, gr = J_r^T go of o = phi(a, r), from the closed forms (TransE: identities; DistMult: the other
    factor; ComplEx: multiplication by the conjugate)."""
    C = a.shape[1] // 2
    if model == "transe_l2":
        return go, (-go if side == 1 else go)
    if model == "distmult":
        return go * rr, go * a
    rc = rr[:, :C] + 1j * rr[:, C:]
    ac = a[:, :C] + 1j * a[:, C:]
    gc = go[:, :C] + 1j * go[:, C:]  # gradient as (d/d re) + i (d/d im)
    if side == 1:   # o = a conj(r):  d/da = g r ;  d/dr = conj(g) a  (g enters conjugated because r does)
        ga, gr = gc * rc, np.conj(gc) * ac
    else:           # o = a r:        d/da = g conj(r) ;  d/dr = g conj(a)
        ga, gr = gc * np.conj(rc), gc * np.conj(ac)
    return np.concatenate([ga.real, ga.imag], 1), np.concatenate([gr.real, gr.imag], 1)


def _rebuild(model, E, R, h, r, t, neg, chunk, k, side, gamma, alpha, rnd=bf16_bits, round_w=True):
    """Negative scores, loss and the negatives' share of the gradients with bf16 operands, chunk by chunk as matrix
    products: S = Ob Nb^T (DistMult, ComplEx) or gamma - sqrt(|Ob|^2 + |Nb|^2 - 2 Ob Nb^T) (TransE-L2); backward
    dO = W Nb, dN = W^T Ob (for TransE-L2 with W = round(c / dist) and the two row-scaled correction terms)."""
    b, D = h.shape[0], E.shape[1]
    E64, R64 = E.astype(np.float64), R.astype(np.float64)
    a = E64[t] if side == 1 else E64[h]
    Ob = rnd(_phi(model, a, R64[r], side))
    dE, dR = np.zeros_like(E64), np.zeros_like(R64)
    S = np.zeros((b, k))
    GO = np.zeros((b, D))
    for c in range(b // chunk):
        rows = slice(c * chunk, (c + 1) * chunk)
        Nb = rnd(E64[neg[c]])
        G = Ob[rows] @ Nb.T
        if model == "transe_l2":
            d2 = (Ob[rows] ** 2).sum(1)[:, None] + (Nb ** 2).sum(1)[None, :] - 2.0 * G
            dist = np.sqrt(np.maximum(d2, 0.0))
            S[rows] = gamma - dist
        else:
            S[rows] = G
    if alpha > 0:
        z = alpha * S
        w = np.exp(z - z.max(1, keepdims=True))
        w /= w.sum(1, keepdims=True)
    else:
        w = np.full((b, k), 1.0 / k)
    neg_loss = (w * np.logaddexp(0.0, S)).sum() / b
    cneg = w / (1.0 + np.exp(-S)) / b
    for c in range(b // chunk):
        rows = slice(c * chunk, (c + 1) * chunk)
        Nb = rnd(E64[neg[c]])
        if model == "transe_l2":
            dist = gamma - S[rows]
            with np.errstate(divide="ignore", invalid="ignore"):
                W = np.where(dist > 0, cneg[rows] / dist, 0.0)
            if round_w:
                W = rnd(W)
            # d(gamma - |o - n|)/do = -(o - n)/dist:  dO = -(rowsum(W) o - W N),  dN = +(W^T O - colsum(W) n)
            GO[rows] = -(W.sum(1)[:, None] * Ob[rows] - W @ Nb)
            dN = W.T @ Ob[rows] - W.sum(0)[:, None] * Nb
        else:
            W = rnd(cneg[rows]) if round_w else cneg[rows]
            GO[rows] = W @ Nb
            dN = W.T @ Ob[rows]
        np.add.at(dE, neg[c], dN)
    ga, gr = _phi_backward(model, a, R64[r], GO, side)
    np.add.at(dE, t if side == 1 else h, ga)
    np.add.at(dR, r, gr)
    return S, neg_loss, dE, dR


def _check_bf16_branch(model, side, alpha, **kw):
    rng = np.random.default_rng(7 + side)
    E, R, h, r, t, neg, chunk, k = _problem(model, rng)
    gamma = 3.0
    got = oracle.loss_and_grad(model, E, R, h, r, t, neg, k, chunk, side, gamma, adv_temperature=alpha,
                               bf16_inputs=True)
    # the positives' part is not rounded: the same batch without negatives gives it (pinned by finite differences)
    pos_only = oracle.loss_and_grad(model, E, R, h, r, t, np.zeros((h.shape[0] // chunk, 0), np.int64), 0, chunk, side,
                                    gamma)
    S, neg_loss, dE, dR = _rebuild(model, E, R, h, r, t, neg, chunk, k, side, gamma, alpha, **kw)
    np.testing.assert_allclose(got["neg"], S, rtol=1e-11, atol=1e-11)
    assert abs(got["loss"] - pos_only["loss"] - neg_loss) <= 1e-12
    scale = np.abs(dE).max()
    np.testing.assert_allclose(got["dE"] - pos_only["dE"], dE, rtol=1e-9, atol=1e-12 * scale)
    np.testing.assert_allclose(got["dR"] - pos_only["dR"], dR, rtol=1e-9, atol=1e-12 * scale)
    return got, S


@pytest.mark.parametrize("alpha", [0.0, 1.0])
@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("model", MODELS)
def test_bf16_branch_equals_the_split_products_on_rounded_operands(model, side, alpha):
    got, S = _check_bf16_branch(model, side, alpha)
    # and the rounding matters at this size: the unrounded scores differ visibly
    rng = np.random.default_rng(7 + side)
    E, R, h, r, t, neg, chunk, k = _problem(model, rng)
    plain = oracle.scores(model, E, R, h, r, t, neg, k, chunk, side, 3.0)[1]
    assert np.abs(plain - S).max() > 1e-4


def test_rebuild_distinguishes_the_readings_it_is_meant_to_pin():
    """The numpy rebuild with another rounding rule, or with unrounded backward coefficients, does not match the
    oracle: so the comparison above does pin the rule and the W = round(c / dist) reading."""
    def truncate(x):
        u = np.asarray(x, dtype=np.float64).astype(np.float32).view(np.uint32) & np.uint32(0xFFFF0000)
        return u.view(np.float32).astype(np.float64)

    for kw in (dict(rnd=truncate), dict(round_w=False)):
        for model in MODELS:
            with pytest.raises(AssertionError):
                _check_bf16_branch(model, 0, 0.0, **kw)


# ------------------------------------------------------------------------------------------------------------------
# planted mistakes in a copy of the oracle must fail the comparisons above


PLANTS = {
    "truncating-rounding": ("    u += 0x7fffu + lsb;\n", "    (void)lsb;\n"),
    "ties-away-from-zero": ("    u += 0x7fffu + lsb;\n", "    (void)lsb; u += 0x8000u;\n"),
    "coefficient-not-rounded": ("                    cneg = round_bf16(cneg);\n", "                    cneg = cneg;\n"),
    "transe-coefficient-rounded-before-the-division": (
        "                    double wq = dist > 0 ? round_bf16(cneg / dist) : 0.0;\n",
        "                    double wq = dist > 0 ? round_bf16(cneg) / dist : 0.0;\n"),
    "o-not-rounded": ("        if (p->bf16_inputs) for (int d = 0; d < De; ++d) ov[d] = round_bf16(ov[d]);\n", ""),
}


@pytest.fixture
def planted(tmp_path, monkeypatch):
    def plant(name):
        old, new = PLANTS[name]
        src = open(os.path.join(os.path.dirname(oracle.__file__), "kge_oracle.c")).read()
        assert src.count(old) == 1, name
        path = tmp_path / f"{name}.c"
        path.write_text(src.replace(old, new))
        lib = oracle.compile_oracle(str(path), str(tmp_path / f"{name}.so"))
        monkeypatch.setattr(oracle, "_lib", oracle.bind(lib))
    return plant


@pytest.mark.parametrize("name", list(PLANTS))
def test_planted_mistakes_in_the_bf16_branch_are_caught(planted, name):
    planted(name)
    failures = 0
    for check in (test_round_bf16_exact_values, test_round_bf16_against_two_independent_conversions,
                  lambda: _check_bf16_branch("transe_l2", 0, 0.0), lambda: _check_bf16_branch("distmult", 1, 1.0),
                  lambda: _check_bf16_branch("complex", 0, 0.0)):
        try:
            check()
        except AssertionError:
            failures += 1
    assert failures > 0, name
