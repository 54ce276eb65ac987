"""Pins of the oracle's diagnostic outputs: `margin` (how far a uniform lay from the nearest
decision threshold: it decides which nodes the GPU parity tests exempt from bit-exactness),
`flags`, and the batch driver's `resid_mass`.

Expected values are worked out by hand from the printed procedures (Alg. 1: "r_i < p(x_i)/q(x_i)";
Alg. 3's four tests; Alg. 2's residuals; the inverse CDF) on distributions small enough to do on
paper; the arithmetic is shown beside each case.  A margin in the wrong units, scaled, or stuck at
0 or infinity fails here.
"""
import numpy as np
import pytest

import oracle

INF = float("inf")


# ----------------------------------------------------------------- inverse CDF
def test_icdf_margin_is_distance_to_the_interval_ends_over_W():
    # w = [1, 2, 1]: W = 4, token 1 owns [1, 3) of the running sum
    w = np.array([1.0, 2.0, 1.0])
    x, W, m = oracle.icdf(w, 0.3)            # t = 1.2: 0.2 above the lower end, 1.8 below the upper
    assert (x, W) == (1, 4.0) and m == pytest.approx(0.2 / 4, rel=1e-12)
    x, _, m = oracle.icdf(w, 0.7)            # t = 2.8: 0.2 below the upper end
    assert x == 1 and m == pytest.approx(0.2 / 4, rel=1e-12)
    x, _, m = oracle.icdf(w, 0.1)            # t = 0.4 inside token 0's [0, 1)
    assert x == 0 and m == pytest.approx(0.4 / 4, rel=1e-12)
    x, _, m = oracle.icdf(w, 0.9)            # t = 3.6 inside token 2's [3, 4)
    assert x == 2 and m == pytest.approx(0.4 / 4, rel=1e-12)


@pytest.mark.parametrize("eps", [1e-7, 1e-3])
def test_icdf_margin_next_to_a_boundary(eps):
    # boundary between tokens 0 and 1 at u = 0.25; u a distance eps to either side of it
    w = np.array([1.0, 2.0, 1.0])
    for u, tok in ((0.25 - eps, 0), (0.25 + eps, 1)):
        x, _, m = oracle.icdf(w, u)
        assert x == tok and m == pytest.approx(eps, rel=1e-6)
        assert (m < 1e-6) == (eps < 1e-6)   # the band the parity tests use


def test_icdf_margin_without_mass_and_at_the_rounding_fallback():
    assert oracle.icdf(np.zeros(3), 0.4) == (-1, 0.0, INF)
    # zero-weight tokens do not move the ends: w = [0, 1, 0, 1], u = 0.5 sits on the boundary of
    # token 1's [0, 1) and token 3's [1, 2): the running sum 1 is not > 1, so token 3, margin 0
    x, W, m = oracle.icdf(np.array([0.0, 1.0, 0.0, 1.0]), 0.5)
    assert (x, W, m) == (3, 2.0, 0.0)


# ----------------------------------------------------------------- Alg. 1 accept tests
P2, Q2 = np.array([0.5, 0.5]), np.array([0.25, 0.75])      # p(1)/q(1) = 2/3, p(0)/q(0) = 2


def test_rrs_margin_of_an_accepted_draft():
    r = oracle.rrs_verify(P2, Q2, [1], [0.6], 0.5)
    assert r["outcome"] == 0 and r["token"] == 1 and r["flags"] == 0
    assert r["margin"] == pytest.approx(2 / 3 - 0.6, rel=1e-12)     # no draw happened: this test alone


def test_rrs_margin_is_the_minimum_over_the_tests_reached():
    # r = 0.7 > 2/3: rejected (margin 0.7 - 2/3 = 0.0333); residual max(p - q, 0) = [0.25, 0],
    # normalised [1, 0]; the draw with u lands in token 0's [0, 1): margin min(u, 1 - u)
    r = oracle.rrs_verify(P2, Q2, [1], [0.7], 0.5)
    assert r["outcome"] == -1 and r["token"] == 0
    assert r["margin"] == pytest.approx(0.7 - 2 / 3, rel=1e-9)
    r = oracle.rrs_verify(P2, Q2, [1], [0.7], 0.01)
    assert r["margin"] == pytest.approx(0.01, rel=1e-12)
    r = oracle.rrs_verify(P2, Q2, [1], [0.7], 0.995)
    assert r["margin"] == pytest.approx(0.005, rel=1e-9)
    # a test that is never reached contributes nothing: draft 0 accepted at once (ratio 2)
    r = oracle.rrs_verify(P2, Q2, [0, 1], [0.5, 2 / 3], 0.5)
    assert r["outcome"] == 0 and r["margin"] == pytest.approx(2 - 0.5, rel=1e-12)


@pytest.mark.parametrize("eps", [1e-7, 1e-3])
def test_rrs_margin_next_to_the_threshold(eps):
    for r0, oc in ((2 / 3 - eps, 0), (2 / 3 + eps, -1)):
        r = oracle.rrs_verify(P2, Q2, [1], [r0], 0.5)
        assert r["outcome"] == oc and r["margin"] == pytest.approx(eps, rel=1e-6)
        assert (r["margin"] < 1e-6) == (eps < 1e-6)


def test_rrs_second_round_margin_uses_the_residual_and_the_rescaled_draft():
    # round 1 rejects token 1 (r = 0.9, margin 0.2333).  Residual p = [1, 0].
    # With replacement: round 2 on token 0 tests r < 1 / 0.25 = 4: margin |0.5 - 4| = 3.5.
    r = oracle.rrs_verify(P2, Q2, [1, 0], [0.9, 0.5], 0.5)
    assert r["outcome"] == 1 and r["token"] == 0
    assert r["margin"] == pytest.approx(0.9 - 2 / 3, rel=1e-9)
    # Without replacement q becomes [1, 0]: round 2 tests r < 1 / 1: margin |0.99 - 1| = 0.01.
    r = oracle.rrs_verify(P2, Q2, [1, 0], [0.9, 0.99], 0.5, without_replacement=True)
    assert r["outcome"] == 1 and r["margin"] == pytest.approx(0.01, rel=1e-9)
    # the same second test with replacement is far from its threshold 4
    r = oracle.rrs_verify(P2, Q2, [1, 0], [0.9, 0.99], 0.5)
    assert r["outcome"] == 1 and r["margin"] == pytest.approx(0.9 - 2 / 3, rel=1e-9)


# ----------------------------------------------------------------- Alg. 3: its four tests
# p = [.5, .1, .4], q = [.4, .4, .2], hub a = 0, D = 1 - q(a) = .6:
#   Q(x,a) = [0, .4, .2]              Q(a,x) = q(a) q(x) / D = [0, 4/15, 2/15]
#   p'  = max(p - Q(.,a), 0) = [.5, 0, .2]        Q'(.,a) = max(Q(.,a) - p, 0) = [0, .3, 0]   S_xa = .3
#   p'' = max(p' - Q(a,.), 0) = [-, 0, 1/15]      Q'(a,.) = max(Q(a,.) - p', 0) = [0, 4/15, 0] S_ax = 4/15
PA, QA = np.array([0.5, 0.1, 0.4]), np.array([0.4, 0.4, 0.2])


def test_spechub_margins_pair_x_a():
    # pair (1, a): test 1  r0 < p(1)/Q(1,a) = .25; test 2  r1 < (p(a) - S_ax)/S_xa = (7/30)/.3 = 7/9
    r = oracle.spechub_verify(PA, QA, 0, 1, 0, 0.2, 0.9, 0.5)
    assert (r["outcome"], r["token"], r["flags"]) == (0, 1, 0)
    assert r["margin"] == pytest.approx(0.05, rel=1e-9)
    r = oracle.spechub_verify(PA, QA, 0, 1, 0, 0.5, 0.7, 0.5)
    assert (r["outcome"], r["token"]) == (1, 0)
    assert r["margin"] == pytest.approx(7 / 9 - 0.7, rel=1e-9)        # min(.25, .0778)
    r = oracle.spechub_verify(PA, QA, 0, 1, 0, 0.26, 0.7, 0.5)
    assert r["margin"] == pytest.approx(0.01, rel=1e-9)               # min(.01, .0778)
    # both rejected: the draw from p'' = [0, 0, 1/15] lands in token 2's interval, u = .3 from its end
    r = oracle.spechub_verify(PA, QA, 0, 1, 0, 0.5, 0.9, 0.3)
    assert (r["outcome"], r["token"]) == (-1, 2)
    assert r["resid_mass"] == pytest.approx(1 / 15, rel=1e-12)
    assert r["margin"] == pytest.approx(0.9 - 7 / 9, rel=1e-9)        # min(.25, .1222, .3)
    r = oracle.spechub_verify(PA, QA, 0, 1, 0, 0.5, 0.9, 0.04)
    assert r["margin"] == pytest.approx(0.04, rel=1e-9)


def test_spechub_margins_pair_a_x():
    # pair (a, 2): test 1  r0 < p'(2)/Q(a,2) = .2/(2/15) = 1.5 (always accepted); margin |r0 - 1.5|
    r = oracle.spechub_verify(PA, QA, 0, 0, 2, 0.9, 0.5, 0.5)
    assert (r["outcome"], r["token"]) == (1, 2) and r["margin"] == pytest.approx(0.6, rel=1e-9)
    # pair (a, 1): test 1  r0 < p'(1)/Q(a,1) = 0: rejected, margin r0; test 2  r1 < p(a)/S_ax = 1.875
    r = oracle.spechub_verify(PA, QA, 0, 0, 1, 0.3, 0.95, 0.5)
    assert (r["outcome"], r["token"]) == (0, 0)
    assert r["margin"] == pytest.approx(0.3, rel=1e-9)                # min(.3, .925)
    r = oracle.spechub_verify(PA, QA, 0, 0, 1, 0.999, 0.95, 0.5)
    assert r["margin"] == pytest.approx(1.875 - 0.95, rel=1e-9)       # min(.999, .925)


@pytest.mark.parametrize("eps", [1e-7, 1e-3])
def test_spechub_margin_next_to_the_hub_threshold(eps):
    for r1, oc in ((7 / 9 - eps, 1), (7 / 9 + eps, -1)):
        r = oracle.spechub_verify(PA, QA, 0, 1, 0, 0.5, r1, 0.5)
        assert r["outcome"] == oc and r["margin"] == pytest.approx(eps, rel=1e-6)
        assert (r["margin"] < 1e-6) == (eps < 1e-6)


# ----------------------------------------------------------------- draft margins
def test_draft_margins():
    # q = [.4, .4, .2]: u0 = .5 draws token 1 (interval [.4, .8)): margin .1, pair (1, a)
    assert oracle.spechub_draft(QA, 0, 0.5, 0.123)[:3] == (1, 0, 0)
    assert oracle.spechub_draft(QA, 0, 0.5, 0.123)[3] == pytest.approx(0.1, rel=1e-9)
    # u0 = .1 draws the hub ([0, .4), margin .1); the second draw over [0, .4, .2] (W = .6) with
    # u1 = .5: t = .3 in token 1's [0, .4): margin min(.3, .1)/.6 = 1/6: node margin .1
    x1, x2, fl, m = oracle.spechub_draft(QA, 0, 0.1, 0.5)
    assert (x1, x2, fl) == (0, 1, 0) and m == pytest.approx(0.1, rel=1e-9)
    # u1 = .66: t = .396, .004 below the boundary .4 between tokens 1 and 2: .004/.6
    x1, x2, fl, m = oracle.spechub_draft(QA, 0, 0.2, 0.66)
    assert (x1, x2) == (0, 1) and m == pytest.approx(0.004 / 0.6, rel=1e-6)
    # k draws: the minimum over the draws
    xs, fl, m = oracle.rrs_draft(QA, [0.5, 0.79, 0.3])
    assert list(xs) == [1, 1, 0] and fl == 0 and m == pytest.approx(0.01, rel=1e-6)
    # without replacement the second draw is over [.4, 0, .2] (W = .6): u = .67 -> t = .402 in token
    # 2's [.4, .6): margin .002/.6, below the first draw's .1
    xs, fl, m = oracle.rrs_draft(QA, [0.5, 0.67], without_replacement=True)
    assert list(xs) == [1, 2] and m == pytest.approx(0.002 / 0.6, rel=1e-6)


# ----------------------------------------------------------------- flags
def test_flags_are_zero_on_ordinary_rows_and_set_where_defined():
    rng = np.random.default_rng(0)
    Bn, N, V, k = 40, 3, 12, 2
    p = rng.dirichlet(np.full(V, 0.5), size=(Bn, N)).astype(np.float32)
    q = rng.dirichlet(np.full(V, 0.5), size=(Bn, N)).astype(np.float32)
    u_d = oracle.philox_uniform(3, 1, Bn * N, k).reshape(Bn, N, k)
    u_v = oracle.philox_uniform(3, 2, Bn * N, k + 1).reshape(Bn, N, k + 1)
    for method in (oracle.SPECHUB, oracle.RRS, oracle.RRSW):
        kw = dict(dtype=oracle.FP32, kind=oracle.PROBS, k=k, depth=2)
        od = oracle.batch_draft(method, q, u_d, **kw)
        ov = oracle.batch_verify(method, p, q, od["tokens"], u_v, **kw)
        assert (od["flags"] == 0).all() and (ov["flags"] == 0).all()
        assert np.isfinite(ov["margin"]).all() and (ov["margin"] > 0).all()
        assert np.isinf(od["margin"][:, 1:]).all() and np.isfinite(od["margin"][:, 0]).all()
    pm = np.array([0.2, 0.5, 0.3])
    # a token outside the vocabulary; a pair without the hub
    assert oracle.spechub_verify(pm, QA, 0, 0, 7, .5, .5, .5)["flags"] == oracle.FLAG_BAD_TOKEN
    assert oracle.spechub_verify(pm, QA, 0, 1, 2, .5, .5, .5)["flags"] == oracle.FLAG_BAD_PAIR
    assert oracle.rrs_verify(pm, QA, [1, -1], [.5, .5], .5)["flags"] == oracle.FLAG_BAD_TOKEN
    # the whole draft mass on the hub
    q1 = np.array([0.0, 1.0, 0.0])
    assert oracle.spechub_draft(q1, 1, 0.5, 0.5) == (1, 1, oracle.FLAG_DEGENERATE_HUB, 0.5)
    assert oracle.spechub_verify(pm, q1, 1, 1, 1, .9, .5, .5)["flags"] == oracle.FLAG_DEGENERATE_HUB
    # p == q: a rejection (only possible with r >= 1, handed in here) leaves a residual without mass
    r = oracle.rrs_verify(pm, pm, [1], [1.5], .5)
    assert r["flags"] == oracle.FLAG_ZERO_RESIDUAL and r["outcome"] == -1
    # RRSw: nothing left to draft from after the only token with draft mass is rejected
    r = oracle.rrs_verify(pm, q1, [1, 1], [0.9, 0.5], .5, without_replacement=True)
    assert r["flags"] & oracle.FLAG_Q_EXHAUSTED
    assert oracle.rrs_draft(q1, [0.5, 0.5], without_replacement=True)[:2][1] == oracle.FLAG_Q_EXHAUSTED


# ----------------------------------------------------------------- batch resid_mass (RRS)
def test_batch_rrs_resid_mass_is_the_product_of_the_rounds_rejection_masses():
    """Alg. 1: after a rejection the target becomes norm(max(p - q, 0)); the mass taken out of p
    by i rejections is the product of the rounds' sums.  p = [.5, .5], q = [.25, .75]:
    round 1 leaves max(p - q, 0) = [.25, 0], mass 1 - alpha = .25; the next residual is
    max([1, 0] - [.25, .75], 0) = [.75, 0], mass .75 (with replacement)."""
    k, N = 2, 3
    p = np.tile(np.array([0.5, 0.5], np.float32), (4, N, 1))
    q = np.tile(np.array([0.25, 0.75], np.float32), (4, N, 1))
    toks = np.array([[-1, 1, 1], [-1, 1, 0], [-1, 0, 1], [-1, 1, 1]], np.int32)
    u = np.zeros((4, N, k + 1), np.float32)
    u[0, 0] = [0.9, 0.9, 0.5]       # both rejected (token 1: ratio 2/3, then 0)
    u[1, 0] = [0.9, 0.5, 0.5]       # second accepted (token 0 of the residual: ratio 4)
    u[2, 0] = [0.5, 0.5, 0.5]       # first accepted (token 0: ratio 2)
    u[3, 0] = [0.9, 0.9, 0.5]
    kw = dict(dtype=oracle.FP32, kind=oracle.PROBS, k=k, depth=2)
    ov = oracle.batch_verify(oracle.RRS, p, q, toks, u, **kw)
    assert list(ov["outcome"][:, 0]) == [-1, 1, 0, -1]
    np.testing.assert_allclose(ov["resid_mass"][:, 0], [0.25 * 0.75, 0.25, 1.0, 0.25 * 0.75], rtol=1e-12)
    # leaves: the mass of p itself
    np.testing.assert_allclose(ov["resid_mass"][:, 1:], 1.0, rtol=1e-12)
    # without replacement: after rejecting token 1, q = [1, 0]; max([1, 0] - [1, 0], 0) has no mass,
    # which is flagged and changes nothing (the product stays .25)
    ov = oracle.batch_verify(oracle.RRSW, p, q, toks, u, **kw)
    assert ov["resid_mass"][0, 0] == pytest.approx(0.25, rel=1e-12)
    # general check against 1 - alpha_i computed here: the k-fold residual of random rows
    rng = np.random.default_rng(4)
    V = 9
    pr = rng.dirichlet(np.ones(V), size=(6, N)).astype(np.float32)
    qr = rng.dirichlet(np.ones(V), size=(6, N)).astype(np.float32)
    tk = np.full((6, N), -1, np.int32)
    ur = np.full((6, N, k + 1), 0.5, np.float32)
    ur[:, :, :k] = 1.0              # r = 1 never accepts where p <= q; pick over-drafted tokens
    for b in range(6):
        over = np.argsort(pr[b, 0].astype(np.float64) - qr[b, 0].astype(np.float64))[:2]
        tk[b, 1:] = over
    ov = oracle.batch_verify(oracle.RRS, pr, qr, tk, ur, **kw)
    for b in range(6):
        P, Q = pr[b, 0].astype(np.float64), qr[b, 0].astype(np.float64)
        want = 1.0
        for _ in range(k):
            alpha = np.minimum(P, Q).sum()          # Theorem 3's alpha of the current pair
            want *= P.sum() - alpha
            P = np.maximum(P - Q, 0.0)
            P /= P.sum()
        assert ov["outcome"][b, 0] == -1
        assert ov["resid_mass"][b, 0] == pytest.approx(want, rel=1e-12)
