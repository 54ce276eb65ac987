"""Pins of the fp64 oracle to what the paper and the mathematics fix.

Nothing here compares the oracle with itself: expectations are the paper's
printed numbers (tests/golden), its closed forms retyped from the text,
library routines (scipy's LP solver and softmax), and exact integration of the
oracle's samplers over their uniforms (tests/probe.py).
"""
import os

import numpy as np
import pytest
import scipy.optimize
import scipy.special

import oracle
from probe import (ONE_MINUS, accept_threshold, measure, rrs_branches,
                   rrs_output_distribution, rrs_tuple_distribution,
                   spechub_branches, spechub_output_distribution,
                   spechub_pair_distribution)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_pair(rng, V, sharp=1.0):
    p = rng.dirichlet(np.full(V, 0.5 * sharp))
    q = 0.6 * p + 0.4 * rng.dirichlet(np.full(V, 0.5 * sharp))
    return p, q / q.sum()


# ----------------------------------------------------------------- softmax
def test_softmax_equals_library_routine():
    rng = np.random.default_rng(1)
    for T in (0.3, 0.7, 1.0, 2.5):
        l = rng.normal(0, 3, 257)
        np.testing.assert_allclose(oracle.softmax(l, T), scipy.special.softmax(l / T),
                                   rtol=1e-13, atol=0)


def test_softmax_shift_invariance_and_limit():
    l = np.array([1.0, 2.0, 3.0, -50.0])
    np.testing.assert_allclose(oracle.softmax(l, 1.0), oracle.softmax(l + 1000.0, 1.0), rtol=1e-12)
    cold = oracle.softmax(l, 1e-3)
    assert cold[2] == pytest.approx(1.0) and cold[:2].sum() < 1e-300 + 1e-12


# ----------------------------------------------------------------- inverse CDF
def test_icdf_interval_measures_equal_normalised_weights():
    rng = np.random.default_rng(2)
    w = rng.random(9)
    w[[2, 5]] = 0.0                      # zero-weight tokens are never returned
    m = measure(lambda u: oracle.icdf(w, u)[0], 9)
    np.testing.assert_allclose(m, w / w.sum(), atol=1e-13)
    assert oracle.icdf(w, 0.0)[0] == 0 and oracle.icdf(w, ONE_MINUS)[0] == 8
    assert oracle.icdf(np.zeros(4), 0.3)[0] == -1


def test_icdf_textbook_case():
    w = np.array([0.1, 0.2, 0.3, 0.4])
    for u, x in ((0.0, 0), (0.0999, 0), (0.1001, 1), (0.2999, 1), (0.3001, 2), (0.61, 3)):
        assert oracle.icdf(w, u)[0] == x


# ----------------------------------------------------------------- SpecHub: Q
@pytest.mark.parametrize("V", [3, 5, 8])
def test_spechub_pair_sampler_realises_Q(V):
    """Sec. 4: Q(x,a) = q(x), Q(a,x) = q(a) q(x) / (1 - q(a)), 0 elsewhere."""
    rng = np.random.default_rng(10 + V)
    for _ in range(5):
        _, q = random_pair(rng, V)
        a = int(np.argmax(q))
        dist = spechub_pair_distribution(q, a)
        assert abs(sum(dist.values()) - 1) < 1e-12
        for (x1, x2), pr in dist.items():
            assert (x1 == a) != (x2 == a)
            if x2 == a:
                assert pr == pytest.approx(q[x1], abs=1e-12)
            else:
                assert pr == pytest.approx(q[a] * q[x2] / (1 - q[a]), abs=1e-12)
        assert len(dist) == 2 * (V - 1)


# ----------------------------------------------------------------- SpecHub: closed forms
@pytest.mark.parametrize("V", [3, 4, 6, 8])
def test_spechub_acceptance_masses_match_closed_forms(V):
    """App. B.2: per token x != a the first draft transports min(p,q), the second
    min(p - min(p,q), q(a)q(x)/(1-q(a))), the residual keeps
    max(p - q - q(a)q(x)/(1-q(a)), 0); the hub is emitted with probability p(a)
    (Corollary 1) and the emitted token follows p (Theorem 2)."""
    rng = np.random.default_rng(20 + V)
    for trial in range(6):
        p, q = random_pair(rng, V, sharp=0.5 + trial * 0.4)
        a = int(np.argmax(q))
        out, acc = spechub_output_distribution(p, q, a)
        c = q[a] / (1 - q[a])
        first = np.minimum(p, q)
        second = np.minimum(p - first, c * q)
        resid = np.maximum(p - q - c * q, 0)
        for arr in (first, second, resid):
            arr[a] = 0
        np.testing.assert_allclose(acc["xa"], first, atol=1e-12)
        np.testing.assert_allclose(acc["ax"], second, atol=1e-12)
        np.testing.assert_allclose(acc["resid"], resid, atol=1e-12)
        assert acc["hub_ax"] + acc["hub_xa"] == pytest.approx(p[a], abs=1e-12)
        np.testing.assert_allclose(out, p, atol=1e-12)
        # hub order (App. B.1): pairs (a,.) draw on p(a) first
        S_ax = np.sum(np.maximum(c * q - np.maximum(p - q, 0), 0)) - max(c * q[a] - max(p[a] - q[a], 0), 0)
        assert acc["hub_ax"] == pytest.approx(min(p[a], S_ax), abs=1e-12)


def test_spechub_unbiased_config1_shape():
    """Exact output distribution on rows of the tiny configuration (V = 16)."""
    rng = np.random.default_rng(0)
    for _ in range(3):
        p = rng.dirichlet(np.full(16, 0.3))
        q = 0.7 * p + 0.3 * rng.dirichlet(np.full(16, 0.3))
        out, _ = spechub_output_distribution(p, q)
        np.testing.assert_allclose(out, p, atol=1e-12)


def test_spechub_unbiased_for_any_hub():
    """The proof of Theorem 2 never uses that a is the argmax."""
    rng = np.random.default_rng(5)
    p, q = random_pair(rng, 5)
    for a in range(5):
        out, _ = spechub_output_distribution(p, q, a)
        np.testing.assert_allclose(out, p, atol=1e-12)


def test_spechub_resid_mass_and_w_output():
    rng = np.random.default_rng(6)
    p, q = random_pair(rng, 7)
    a = int(np.argmax(q))
    x = (a + 1) % 7
    r = oracle.spechub_verify(p, q, a, x, a, 0.5, 0.5, 0.5, want_w=True)
    c = q[a] / (1 - q[a])
    w = np.maximum(p - q - c * q, 0)
    w[a] = 0
    np.testing.assert_allclose(r["w"], w, atol=1e-15)
    assert r["resid_mass"] == pytest.approx(w.sum(), abs=1e-15)


# ----------------------------------------------------------------- SpecHub: LP optimality
def sparse_lp_optimum(p, q, a):
    """Simplified LP of Sec. 3.2 restricted to the pairs SpecHub populates."""
    V = len(p)
    others = [x for x in range(V) if x != a]
    nv = 4 * len(others)  # per x: pi(x,a,x), pi(x,a,a), pi(a,x,x), pi(a,x,a)
    A, b = [], []
    c = q[a] / (1 - q[a])
    for i, x in enumerate(others):
        row = np.zeros(nv); row[4 * i] = row[4 * i + 1] = 1; A.append(row); b.append(q[x])
        row = np.zeros(nv); row[4 * i + 2] = row[4 * i + 3] = 1; A.append(row); b.append(c * q[x])
        row = np.zeros(nv); row[4 * i] = row[4 * i + 2] = 1; A.append(row); b.append(p[x])
    row = np.zeros(nv)
    for i in range(len(others)):
        row[4 * i + 1] = row[4 * i + 3] = 1
    A.append(row); b.append(p[a])
    res = scipy.optimize.linprog(-np.ones(nv), A_ub=np.array(A), b_ub=np.array(b),
                                 bounds=(0, None), method="highs")
    assert res.status == 0
    return -res.fun


@pytest.mark.parametrize("V", [3, 5, 8])
def test_spechub_plan_is_lp_optimal(V):
    """Sec. 4: the closed-form plan solves the LP on the sparse Q; 1 - optimum
    is the mass SpecHub leaves to the residual."""
    rng = np.random.default_rng(30 + V)
    for _ in range(8):
        p, q = random_pair(rng, V)
        a = int(np.argmax(q))
        x = (a + 1) % V
        rm = oracle.spechub_verify(p, q, a, x, a, 0.5, 0.5, 0.5)["resid_mass"]
        assert 1 - rm == pytest.approx(sparse_lp_optimum(p, q, a), abs=1e-9)
        _, acc = spechub_output_distribution(p, q, a)
        assert acc["resid"].sum() == pytest.approx(rm, abs=1e-12)


# ----------------------------------------------------------------- worked example
def read_worked_example():
    vals = {}
    for line in open(os.path.join(GOLDEN, "worked_example.txt")):
        if line.startswith("#") or "=" not in line:
            continue
        k, v = line.split("=")
        vals[k.strip()] = [float(t) for t in v.split()]
    return np.array(vals["p"]), np.array(vals["q"]), vals["rrsw_transport_cost"][0]


def test_worked_example_rrsw_cost():
    p, q, cost = read_worked_example()
    out, per_round = rrs_output_distribution(p, q, 2, without_replacement=True)
    assert 1 - per_round.sum() == pytest.approx(cost, abs=1e-12)
    np.testing.assert_allclose(out, p, atol=1e-12)


def test_worked_example_spechub_and_rrs():
    """Same pair: by the formulas of Sec. 4 SpecHub transports everything
    (min(p,q) = [.,.3,.2]; second draft min([.3,.1],[.3,.2]) = [.3,.1]; hub
    takes p(a) = .1), and RRS with replacement loses (1-a1)(1-a2) with
    a1 = .6, residual [0,.75,.25] vs q -> a2 = .5."""
    p, q, _ = read_worked_example()
    out, acc = spechub_output_distribution(p, q)
    assert acc["resid"].sum() == pytest.approx(0.0, abs=1e-12)
    np.testing.assert_allclose(acc["xa"], [0, 0.3, 0.2], atol=1e-12)
    np.testing.assert_allclose(acc["ax"], [0, 0.3, 0.1], atol=1e-12)
    np.testing.assert_allclose(out, p, atol=1e-12)
    _, per_round = rrs_output_distribution(p, q, 2, without_replacement=False)
    assert 1 - per_round.sum() == pytest.approx(0.2, abs=1e-12)


# ----------------------------------------------------------------- RRS / RRSw
@pytest.mark.parametrize("wo", [False, True])
def test_rrs_draft_tuple_distribution(wo):
    """Sec. 3.3: Q = prod q(x_i) with replacement;
    prod q(x_i) / prod_{i<k} (1 - sum_{j<=i} q(x_j)) without."""
    rng = np.random.default_rng(40)
    _, q = random_pair(rng, 5)
    dist = rrs_tuple_distribution(q, 3, wo)
    assert abs(sum(dist.values()) - 1) < 1e-12
    for xs, pr in dist.items():
        if wo:
            assert len(set(xs)) == 3
            expect = q[xs[0]] * q[xs[1]] * q[xs[2]] / ((1 - q[xs[0]]) * (1 - q[xs[0]] - q[xs[1]]))
        else:
            expect = q[xs[0]] * q[xs[1]] * q[xs[2]]
        assert pr == pytest.approx(expect, abs=1e-12)


@pytest.mark.parametrize("wo", [False, True])
@pytest.mark.parametrize("V,k", [(4, 1), (8, 2), (5, 3), (4, 4)])
def test_rrs_unbiased(V, k, wo):
    if wo and k >= V:
        pytest.skip("cannot draw k distinct tokens")
    rng = np.random.default_rng(50 + 10 * V + k)
    for _ in range(3):
        p, q = random_pair(rng, V)
        out, _ = rrs_output_distribution(p, q, k, wo)
        np.testing.assert_allclose(out, p, atol=1e-12)


def test_single_draft_acceptance_is_sum_min():
    """Sec. 2 / Theorem 3: the first draft is accepted with probability sum min(p,q)."""
    rng = np.random.default_rng(60)
    p, q = random_pair(rng, 8)
    _, per_round = rrs_output_distribution(p, q, 1, False)
    np.testing.assert_allclose(per_round[0], np.minimum(p, q), atol=1e-12)
    assert per_round.sum() == pytest.approx(np.minimum(p, q).sum(), abs=1e-12)


def test_rrs_second_draft_closed_form():
    """Proof of Theorem 3: second-draft acceptance of x under RRS is
    min(p(x) - min(p,q)(x), (1 - alpha) q(x))."""
    rng = np.random.default_rng(61)
    for _ in range(4):
        p, q = random_pair(rng, 6)
        _, per_round = rrs_output_distribution(p, q, 2, False)
        alpha = np.minimum(p, q).sum()
        np.testing.assert_allclose(per_round[1], np.minimum(p - np.minimum(p, q), (1 - alpha) * q),
                                   atol=1e-12)


def test_rrs_residual_and_masses():
    """Alg. 1: after one rejection the target is norm(max(p - q, 0))."""
    rng = np.random.default_rng(62)
    p, q = random_pair(rng, 6)
    x = int(np.argmax(q - p))
    r = oracle.rrs_verify(p, q, [x], [ONE_MINUS], 0.3, want_P=True)
    res = np.maximum(p - q, 0)
    assert r["outcome"] == -1
    np.testing.assert_allclose(r["P"], res / res.sum(), atol=1e-15)
    assert r["mass"][0] == pytest.approx(res.sum(), abs=1e-15)


def test_thm3_spechub_beats_rrs_second_draft():
    """Theorem 3: if q(a)/(1-q(a)) > 1 - alpha, SpecHub's second-draft acceptance
    of every x != a is at least RRS's."""
    rng = np.random.default_rng(63)
    checked = 0
    for _ in range(40):
        p, q = random_pair(rng, 5, sharp=0.6)
        a = int(np.argmax(q))
        alpha = np.minimum(p, q).sum()
        if q[a] / (1 - q[a]) <= 1 - alpha:
            continue
        _, acc = spechub_output_distribution(p, q, a)
        _, per_round = rrs_output_distribution(p, q, 2, False)
        mask = np.arange(5) != a
        assert np.all(acc["ax"][mask] >= per_round[1][mask] - 1e-12)
        checked += 1
    assert checked >= 10


# ----------------------------------------------------------------- limits / special cases
def test_p_equals_q_always_accepts_first():
    rng = np.random.default_rng(70)
    p, _ = random_pair(rng, 6)
    a = int(np.argmax(p))
    for x in range(6):
        if x == a:
            continue
        assert oracle.spechub_verify(p, p, a, x, a, ONE_MINUS, ONE_MINUS, 0.5)["outcome"] == 0
        assert oracle.rrs_verify(p, p, [x, a], [ONE_MINUS, 0.5], 0.5)["outcome"] == 0
    # pair (a, x): the non-hub token has no residual, the hub takes everything
    x = (a + 1) % 6
    t1, t2, _ = spechub_branches(p, p, a, (a, x))
    assert t1 == 0.0 and t2 == 1.0


def test_low_temperature_limit_is_top2_greedy():
    """Sec. 5.2: as T -> 0 SpecHub and RRSw both propose the top-2 tokens."""
    l = np.array([0.3, 2.0, 1.1, -0.5, 1.9])
    q = oracle.softmax(l, 0.01)
    a = oracle.argmax(q)
    assert a == 1
    for u0, u1 in ((0.2, 0.7), (0.9, 0.1), (0.5, 0.5)):
        x1, x2, _, _ = oracle.spechub_draft(q, a, u0, u1)
        assert {x1, x2} == {1, 4}
        xs, _, _ = oracle.rrs_draft(q, [u0, u1], without_replacement=True)
        assert set(int(t) for t in xs) == {1, 4}


def test_k1_rrs_equals_single_draft_speculative_sampling():
    rng = np.random.default_rng(71)
    p, q = random_pair(rng, 6)
    for x in range(6):
        thr, res = rrs_branches(p, q, [x], False)
        assert thr[0] == pytest.approx(min(1.0, p[x] / q[x]), abs=1e-12)
        if thr[0] < 1:
            r = np.maximum(p - q, 0)
            np.testing.assert_allclose(res, r / r.sum(), atol=1e-12)


def test_degenerate_point_mass_draft():
    """All draft mass on the hub (reading: single-draft case on a)."""
    q = np.array([0.0, 1.0, 0.0, 0.0])
    p = np.array([0.2, 0.5, 0.1, 0.2])
    x1, x2, fl, _ = oracle.spechub_draft(q, 1, 0.4, 0.4)
    assert (x1, x2) == (1, 1) and fl & oracle.FLAG_DEGENERATE_HUB
    thr = accept_threshold(lambda r: oracle.spechub_verify(p, q, 1, 1, 1, r, 0.5, 0.5)["outcome"] == 0)
    assert thr == pytest.approx(0.5, abs=1e-12)
    m = measure(lambda u: oracle.spechub_verify(p, q, 1, 1, 1, ONE_MINUS, 0.5, u)["token"], 4)
    np.testing.assert_allclose(m, [0.4, 0, 0.2, 0.4], atol=1e-12)


def test_bad_inputs_are_flagged_not_trapped():
    p = np.array([0.2, 0.5, 0.3])
    q = np.array([0.3, 0.4, 0.3])
    r = oracle.spechub_verify(p, q, 1, 0, 2, 0.5, 0.5, 0.5)
    assert r["outcome"] == -2 and r["flags"] & oracle.FLAG_BAD_PAIR
    r = oracle.spechub_verify(p, q, 1, 7, 1, 0.5, 0.5, 0.5)
    assert r["outcome"] == -3 and r["flags"] & oracle.FLAG_BAD_TOKEN
    r = oracle.rrs_verify(p, q, [0, -1], [0.5, 0.5], 0.5)
    assert r["outcome"] == -3


# ----------------------------------------------------------------- toy experiment (soft pin)
def test_toy_table_soft_pin():
    """App. D: V = 50, p = softmax(u_p/T), q = softmax((lam u_p + (1-lam) u_q)/T).
    Reading: with the printed Unif(0,1) logits the table is not reproduced; with
    standard normal logits it is, within the spread of a 100-pair mean.  Soft
    statistical pin on the RRS and SpecHub columns (both analytic)."""
    rows = [[float(t) for t in line.split()] for line in open(os.path.join(GOLDEN, "toy_table.txt"))
            if line.strip() and not line.startswith("#")]
    rng = np.random.default_rng(123)
    for T, lam, rrs_ref, _, _, _, hub_ref in rows:
        acc_rrs, acc_hub = [], []
        for _ in range(400):
            up, uq = rng.normal(size=50), rng.normal(size=50)
            p = oracle.softmax(up, T)
            q = oracle.softmax(lam * up + (1 - lam) * uq, T)
            a = oracle.argmax(q)
            x = (a + 1) % 50
            acc_hub.append(1 - oracle.spechub_verify(p, q, a, x, a, 0.5, 0.5, 0.5)["resid_mass"])
            x = int(np.argmax(q - p))        # over-sampled: rejected by a uniform next to 1
            m = oracle.rrs_verify(p, q, [x, x], [ONE_MINUS, ONE_MINUS], 0.5)["mass"]
            acc_rrs.append(1 - m[0] * m[1])
        # the table averages 100 pairs; allow 3 standard errors of such a mean
        se_rrs = np.std(acc_rrs) / 10
        se_hub = np.std(acc_hub) / 10
        assert abs(np.mean(acc_rrs) - rrs_ref) < 3 * se_rrs + 0.01
        assert abs(np.mean(acc_hub) - hub_ref) < 3 * se_hub + 0.01


# ----------------------------------------------------------------- tree walk
def test_tree_walk_binary_depth3():
    # nodes: 0; 1,2; 3,4,5,6.  accept slot 1 at the root, slot 0 at node 2, node 5 is a leaf
    outcome = [1, -1, 0, -1, -1, -1, -1]
    token = [20, 11, 50, 13, 14, 77, 16]
    d, em = oracle.tree_walk(outcome, token, k=2, depth=3)
    assert d == 2 and list(em) == [20, 50, 77]
    outcome[0] = -1
    d, em = oracle.tree_walk(outcome, token, k=2, depth=3)
    assert d == 0 and list(em) == [20, -1, -1]
    outcome[0], outcome[1] = 0, -1
    d, em = oracle.tree_walk(outcome, token, k=2, depth=3)
    assert d == 1 and list(em) == [20, 11, -1]


def test_tree_walk_general_topology():
    # root has children 1,2; node 1 has children 3,4; node 2 is a leaf
    fc = [1, 3, -1, -1, -1]
    d, em = oracle.tree_walk([0, 1, -1, -1, -1], [5, 6, 7, 8, 9], k=2, depth=3, first_child=fc)
    assert d == 2 and list(em) == [5, 6, 9]
    d, em = oracle.tree_walk([1, 1, -1, -1, -1], [5, 6, 7, 8, 9], k=2, depth=3, first_child=fc)
    assert d == 1 and list(em) == [5, 7, -1]


def test_tokens_per_step_arithmetic_of_the_paper():
    """Tables of Sec. 5 / App. E: on a 3-node tree tokens/step = 1 + first + second
    draft acceptance (SpecHub .4248 + .166 vs 1.5997 printed at T = 1)."""
    assert 1 + 0.4248 + 0.166 == pytest.approx(1.5997, abs=0.01)
    assert 1 + 0.4344 + 0.1021 == pytest.approx(1.5432, abs=0.01)
    assert 1 + 0.4418 + 0.1140 == pytest.approx(1.5521, abs=0.01)


# ----------------------------------------------------------------- Philox
def test_philox_known_answers():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        np.testing.assert_array_equal(oracle.philox4x32_10(w[0:4], w[4:6]), np.array(w[6:10], np.uint32))


def test_philox_uniform_layout_and_range():
    u, words = oracle.philox_uniform(7, 3, rows=5, slots=6, want_words=True)
    for r in range(5):
        for s in range(6):
            o = oracle.philox4x32_10([r, 0, s >> 2, 3], [7, 0])
            assert words[r, s] == o[s & 3]
            assert u[r, s] == np.float32((int(o[s & 3]) >> 8) * 2.0 ** -24)
    big = oracle.philox_uniform(1, 0, rows=20000, slots=4)
    assert big.min() >= 0.0 and big.max() < 1.0
    assert abs(big.mean() - 0.5) < 0.005
    hist, _ = np.histogram(big, bins=16, range=(0, 1))
    assert np.all(np.abs(hist / big.size - 1 / 16) < 0.004)
