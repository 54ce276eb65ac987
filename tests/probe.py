"""Exact integration of the oracle's samplers over their uniforms.

The oracle's samplers are deterministic functions of the uniforms they are
handed.  Each accept test is a threshold in its uniform and each inverse-CDF
draw is a non-decreasing step function of its uniform, so the probability of
every branch can be measured, to fp64 resolution, by bisection on the
uniforms alone.  This treats the sampler as a black box: nothing of its
arithmetic is retyped here.
"""
from __future__ import annotations

import numpy as np

import oracle

ONE_MINUS = float(np.nextafter(1.0, 0.0))


def accept_threshold(f):
    """f(r) is True for r below an unknown threshold in [0,1]; return it."""
    if not f(0.0):
        return 0.0
    if f(ONE_MINUS):
        return 1.0
    lo, hi = 0.0, ONE_MINUS
    for _ in range(64):
        mid = 0.5 * (lo + hi)
        if f(mid):
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def step_intervals(g):
    """g(u) is a non-decreasing integer step function on [0,1); return
    [(value, lo, hi)] of its constant pieces (pieces of measure 0 are dropped)."""
    jumps = []  # (position, value on the right), in increasing position

    def rec(lo, vlo, hi, vhi):
        if vlo == vhi:
            return
        mid = 0.5 * (lo + hi)
        if hi - lo < 2e-16 or mid <= lo or mid >= hi:
            jumps.append((mid, vhi))
            return
        vm = g(mid)
        rec(lo, vlo, mid, vm)
        rec(mid, vm, hi, vhi)

    v0 = g(0.0)
    rec(0.0, v0, ONE_MINUS, g(ONE_MINUS))
    res, prev, v = [], 0.0, v0
    for b, vr in jumps:
        res.append((v, prev, b))
        prev, v = b, vr
    res.append((v, prev, 1.0))
    return res


def measure(g, V):
    m = np.zeros(V)
    for v, lo, hi in step_intervals(g):
        m[v] += hi - lo
    return m


# ------------------------------------------------------------------ SpecHub
def spechub_pair_distribution(q, a):
    """{(x1, x2): probability} of the oracle's pair sampler."""
    dist = {}
    for x, lo, hi in step_intervals(lambda u0: oracle.spechub_draft(q, a, u0, 0.5)[0]):
        if x != a:
            dist[(x, a)] = dist.get((x, a), 0.0) + (hi - lo)
        else:
            u0 = 0.5 * (lo + hi)
            for y, lo1, hi1 in step_intervals(lambda u1: oracle.spechub_draft(q, a, u0, u1)[1]):
                dist[(a, y)] = dist.get((a, y), 0.0) + (hi - lo) * (hi1 - lo1)
    return dist


def spechub_branches(p, q, a, pair):
    """Branch probabilities of the oracle's verifier for one sampled pair:
    (P[non-hub token accepted], P[hub accepted | first rejected],
     residual token distribution given both rejected)."""
    x1, x2 = pair
    V = len(p)
    nonhub_slot = 0 if x2 == a and x1 != a else 1

    def oc(r0, r1, u=0.5):
        return oracle.spechub_verify(p, q, a, x1, x2, r0, r1, u)

    t1 = accept_threshold(lambda r0: oc(r0, ONE_MINUS)["outcome"] == nonhub_slot)
    t2 = accept_threshold(lambda r1: oc(ONE_MINUS, r1)["outcome"] == 1 - nonhub_slot)
    if t1 < 1.0 and t2 < 1.0:
        res = measure(lambda u: oc(ONE_MINUS, ONE_MINUS, u)["token"], V)
    else:
        res = np.zeros(V)
    return t1, t2, res


def spechub_output_distribution(p, q, a=None):
    """Distribution of the emitted token and the per-slot acceptance masses."""
    p = np.asarray(p, float)
    q = np.asarray(q, float)
    V = len(p)
    if a is None:
        a = oracle.argmax(q)
    out = np.zeros(V)
    acc = dict(xa=np.zeros(V), ax=np.zeros(V), hub_ax=0.0, hub_xa=0.0, resid=np.zeros(V))
    for pair, Qp in spechub_pair_distribution(q, a).items():
        t1, t2, res = spechub_branches(p, q, a, pair)
        x = pair[0] if pair[1] == a and pair[0] != a else pair[1]
        fam = "xa" if pair[1] == a and pair[0] != a else "ax"
        acc[fam][x] += Qp * t1
        acc["hub_" + fam] += Qp * (1 - t1) * t2
        acc["resid"] += Qp * (1 - t1) * (1 - t2) * res
        out[x] += Qp * t1
        out[a] += Qp * (1 - t1) * t2
        out += Qp * (1 - t1) * (1 - t2) * res
    return out, acc


# ------------------------------------------------------------------ RRS / RRSw
def rrs_tuple_distribution(q, k, without_replacement):
    """{tuple: probability} of the oracle's k-draft sampler."""
    dist = {}

    def rec(prefix_u, prefix_x, prob):
        i = len(prefix_u)
        if i == k:
            dist[tuple(prefix_x)] = dist.get(tuple(prefix_x), 0.0) + prob
            return

        def g(ui):
            us = prefix_u + [ui] + [0.5] * (k - i - 1)
            return int(oracle.rrs_draft(q, us, without_replacement)[0][i])

        for x, lo, hi in step_intervals(g):
            if hi > lo:
                rec(prefix_u + [0.5 * (lo + hi)], prefix_x + [x], prob * (hi - lo))

    rec([], [], 1.0)
    return dist


def rrs_branches(p, q, xs, without_replacement):
    """([P(accept in round i | rounds < i rejected)], residual distribution)."""
    k = len(xs)
    V = len(p)
    thr = []
    for i in range(k):
        def f(ri, i=i):
            r = [ONE_MINUS] * k
            r[i] = ri
            return oracle.rrs_verify(p, q, xs, r, 0.5, without_replacement)["outcome"] == i
        # rounds before i must really reject for round i to be reached
        reached = all(t < 1.0 for t in thr)
        thr.append(accept_threshold(f) if reached else 0.0)
    if all(t < 1.0 for t in thr):
        res = measure(lambda u: oracle.rrs_verify(p, q, xs, [ONE_MINUS] * k, u,
                                                  without_replacement)["token"], V)
    else:
        res = np.zeros(V)
    return thr, res


def rrs_output_distribution(p, q, k, without_replacement):
    """Distribution of the emitted token, and acceptance mass per round and token."""
    p = np.asarray(p, float)
    q = np.asarray(q, float)
    V = len(p)
    out = np.zeros(V)
    per_round = np.zeros((k, V))
    for xs, Pt in rrs_tuple_distribution(q, k, without_replacement).items():
        thr, res = rrs_branches(p, q, list(xs), without_replacement)
        alive = Pt
        for i in range(k):
            per_round[i, xs[i]] += alive * thr[i]
            out[xs[i]] += alive * thr[i]
            alive *= 1 - thr[i]
        out += alive * res
    return out, per_round
