"""Pins of the oracle's multi-candidate verification (several candidates at one position, each
from a proposal of its own; Method, "Sampling and Verification", the recursion over consecutive
rejections; appendix "Theoretical Justification").

What is fixed outside the oracle:
  * the theorem itself: whatever the proposals, the emitted token follows the (warped) target
    distribution.  The oracle is treated as a black box in its uniforms: for every candidate
    tuple its accept thresholds and the breakpoints of its final inverse-CDF draw are found by
    bisection over float32 uniforms, which gives the exact output law up to 2^-24 per term;
  * the closed form of the two-proposal law from the appendix, evaluated with rationals, which
    also decides between the two readings of the residual update (subtract the rejected
    candidate's own proposal, as the derivation and the general form do, or the first proposal
    twice, as one displayed equation prints);
  * the one-candidate case, which is the already pinned orc_spec_sample;
  * the greedy case and the total-variation identity for the residual mass.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

ONE_BELOW = float(np.nextafter(np.float32(1.0), np.float32(0.0)))


def warped(l, temperature, top_k):
    """Target / proposal distribution after temperature and top-k, by library routines."""
    z = torch.from_numpy(np.asarray(l, np.float32)) * np.float32(1.0 / temperature)
    if top_k < z.numel():
        kth = torch.topk(z, top_k).values[-1]
        z = torch.where(z >= kth, z, torch.tensor(-np.inf))
    return torch.softmax(z.double(), 0).numpy()


def bisect_u(pred):
    """Smallest float32 u in [0, 1) with pred(u) true (pred monotone false -> true), or 1.0."""
    lo, hi = np.float32(0.0), np.float32(ONE_BELOW)
    if pred(float(lo)):
        return 0.0
    if not pred(float(hi)):
        return 1.0
    while True:
        mid = np.float32((np.float64(lo) + np.float64(hi)) / 2)
        if mid == lo or mid == hi:
            return float(hi)
        if pred(float(mid)):
            hi = mid
        else:
            lo = mid


def output_law(p_l, q_l, temperature, top_k):
    """Law of the emitted token, integrating the oracle over its uniforms exactly."""
    m, n = q_l.shape
    qs = [warped(q_l[i], temperature, top_k) for i in range(m)]
    law = np.zeros(n)
    accept_mass = np.zeros(m + 1)
    for tup in itertools.product(range(n), repeat=m):
        w = float(np.prod([qs[i][tup[i]] for i in range(m)]))
        if w == 0.0:
            continue
        reach = 1.0   # probability of having rejected candidates 0..i-1
        u = [0.0] * m
        for i in range(m):
            # accepted at step i iff u_i below a threshold, earlier ones rejected (u = just below 1)
            def rejected(x, i=i):
                uu = list(u)
                uu[i] = x
                return oracle.multi_verify(p_l, q_l, tup, uu, 0.5, temperature, top_k)[0] != i
            t = bisect_u(rejected)
            law[tup[i]] += w * reach * t
            accept_mass[i] += w * reach * t
            reach *= 1.0 - t
            u[i] = ONE_BELOW
            if reach == 0.0:
                break
        if reach == 0.0:
            continue
        # all rejected: the final draw is an inverse CDF over ascending index, monotone in u_final
        edges = [0.0]
        for j in range(1, n):
            edges.append(bisect_u(lambda x, j=j: oracle.multi_verify(p_l, q_l, tup, u, x, temperature, top_k)[1] >= j))
        edges.append(1.0)
        assert oracle.multi_verify(p_l, q_l, tup, u, 0.5, temperature, top_k)[0] == m
        for j in range(n):
            law[j] += w * reach * max(0.0, edges[j + 1] - edges[j])
        accept_mass[m] += w * reach
    return law, accept_mass


@pytest.mark.parametrize("m,n,temperature,top_k", [(2, 5, 1.0, 5), (3, 4, 1.0, 4), (2, 6, 0.7, 4), (1, 6, 1.3, 6)])
def test_output_law_is_the_target_distribution(m, n, temperature, top_k):
    rng = np.random.default_rng(100 * m + n)
    p_l = (rng.standard_normal(n) * 1.5).astype(np.float32)
    q_l = (rng.standard_normal((m, n)) * 1.5).astype(np.float32)
    law, accept_mass = output_law(p_l, q_l, temperature, top_k)
    ref = warped(p_l, temperature, top_k)
    assert abs(law.sum() - 1.0) < 1e-5
    np.testing.assert_allclose(law, ref, rtol=0, atol=2e-6)
    # the first candidate is accepted with probability sum min(p, q_1)
    q1 = warped(q_l[0], temperature, top_k)
    assert abs(accept_mass[0] - np.minimum(ref, q1).sum()) < 2e-6
    if m > 1:
        assert accept_mass[1] > 1e-3   # the distinct second proposal does get used


def two_proposal_law(p, q1, q2, subtract_second):
    """Closed form of the appendix for one candidate from each of two proposals (rationals)."""
    def norm(v):
        s = sum(v)
        return [x / s for x in v]
    n = len(p)
    alpha1 = 1 - sum(p[x] - min(q1[x], p[x]) for x in range(n))
    p1 = norm([max(Fraction(0), p[x] - q1[x]) for x in range(n)])
    alpha2 = 1 - sum(p1[x] - min(q2[x], p1[x]) for x in range(n))
    sub = q2 if subtract_second else q1
    p2 = norm([max(Fraction(0), p1[x] - sub[x]) for x in range(n)])
    return [min(q1[x], p[x]) + (1 - alpha1) * min(q2[x], p1[x]) + (1 - alpha1) * (1 - alpha2) * p2[x] for x in range(n)]


def test_closed_form_fixes_the_reading_of_the_second_residual():
    p = [Fraction(1, 10), Fraction(2, 10), Fraction(3, 10), Fraction(4, 10)]
    q1 = [Fraction(4, 10), Fraction(3, 10), Fraction(2, 10), Fraction(1, 10)]
    q2 = [Fraction(1, 4), Fraction(1, 4), Fraction(1, 8), Fraction(3, 8)]
    assert two_proposal_law(p, q1, q2, subtract_second=True) == p          # exact
    assert two_proposal_law(p, q1, q2, subtract_second=False) != p         # the printed variant is not exact
    # and the oracle follows the exact one: same numbers through logits
    p_l = np.log(np.array([float(x) for x in p])).astype(np.float32)
    q_l = np.log(np.array([[float(x) for x in q1], [float(x) for x in q2]])).astype(np.float32)
    law, _ = output_law(p_l, q_l, 1.0, 4)
    np.testing.assert_allclose(law, [float(x) for x in p], rtol=0, atol=2e-6)


def test_one_candidate_is_the_single_draft_rule():
    rng = np.random.default_rng(7)
    n = 300
    for trial in range(200):
        p_l = (rng.standard_normal(n) * 2).astype(np.float32)
        q_l = (rng.standard_normal((1, n)) * 2).astype(np.float32)
        top_k = int(rng.choice([n, 50, 7]))
        temperature = float(rng.choice([1.0, 0.8]))
        qd = warped(q_l[0], temperature, top_k)
        cand = int(rng.choice(n, p=qd))
        u_acc, u_fin = float(rng.random(dtype=np.float32)), float(rng.random(dtype=np.float32))
        idx, tok = oracle.multi_verify(p_l, q_l, [cand], [u_acc], u_fin, temperature, top_k)
        a, toks = oracle.spec_sample(np.stack([p_l, p_l]), q_l, [cand], [u_acc], u_fin, temperature, top_k)
        assert (idx == 0) == (a == 1)
        if idx == 0:
            assert tok == cand
        else:
            assert tok == toks[0]


def test_greedy_candidates():
    rng = np.random.default_rng(3)
    n, m = 50, 3
    for trial in range(50):
        p_l = rng.standard_normal(n).astype(np.float32)
        q_l = rng.standard_normal((m, n)).astype(np.float32)
        if trial % 2:
            q_l[1, :] = p_l   # the second proposal agrees with the target
        cand = q_l.argmax(1)
        u = rng.random(m, dtype=np.float32)
        idx, tok = oracle.multi_verify(p_l, q_l, cand, u, 0.3, 0.0, n)
        hits = [i for i in range(m) if cand[i] == p_l.argmax()]
        assert idx == (hits[0] if hits else m)
        assert tok == p_l.argmax()


def test_residual_mass_is_total_variation_distance():
    rng = np.random.default_rng(11)
    n, m = 64, 2
    p_l = rng.standard_normal(n).astype(np.float32)
    q_l = rng.standard_normal((m, n)).astype(np.float32)
    p, q1, q2 = warped(p_l, 1.0, n), warped(q_l[0], 1.0, n), warped(q_l[1], 1.0, n)
    idx, tok, resid = oracle.multi_verify(p_l, q_l, [0, 1], [ONE_BELOW, ONE_BELOW], 0.1, 1.0, n, want_resid=True)
    assert abs(resid[0] - 0.5 * np.abs(p - q1).sum()) < 1e-12
    if idx >= 1:
        p1 = np.maximum(0, p - q1)
        p1 /= p1.sum()
        assert abs(resid[1] - (1 - np.minimum(p1, q2).sum())) < 1e-12


def rejection_curves(rows, m, n, top_k, seed, verify):
    """Residual masses 1 - alpha_j of every step for the same proposal repeated and for distinct
    proposals; the candidates are tokens the target gives no mass, so every step is evaluated."""
    rng = np.random.Generator(np.random.PCG64(seed))
    same, distinct = [], []
    for r in range(rows):
        p = (rng.standard_normal(n) * 1.5).astype(np.float32)
        qd = (p[None, :] + rng.standard_normal((m, n))).astype(np.float32)
        qs = np.repeat(qd[:1], m, axis=0)
        out = int(np.argmin(p))
        for q, acc in ((qs, same), (qd, distinct)):
            idx, tok, resid = verify(p, q, [out] * m, [ONE_BELOW] * m, 0.5, 1.0, top_k)
            assert idx == m
            acc.append(resid)
    return np.array(same), np.array(distinct)


def test_rejection_probability_same_proposal_stalls_distinct_proposals_do_not():
    # Experiment, the paragraph on the rejection probability r(x) and its figure: with one proposal
    # used again and again the residual reaches a fixed point (1 - alpha_j -> 1, r stops falling);
    # distinct proposals keep lowering r = prod_j (1 - alpha_j).
    m = 8
    same, distinct = rejection_curves(12, m, 2048, 200, 5,
                                      lambda *a: oracle.multi_verify(*a, want_resid=True))
    assert np.all((same > 0) & (same <= 1)) and np.all((distinct > 0) & (distinct <= 1))
    np.testing.assert_allclose(same[:, 0], distinct[:, 0], rtol=0, atol=0)   # the first step is the same
    ms, md = same.mean(0), distinct.mean(0)
    assert np.all(np.diff(ms) > 0) and ms[-1] > 0.97            # approaches the fixed point
    r_same, r_dist = np.cumprod(same, 1).mean(0), np.cumprod(distinct, 1).mean(0)
    assert np.all(r_dist[1:] < r_same[1:])
    assert r_same[-1] / r_same[-2] > 0.97                       # r has stopped falling
    assert r_dist[-1] < 0.5 * r_same[-1]
    # the fixed point itself: with q repeated for ever what survives is the target's mass where it
    # exceeds every multiple of q that fits under it - in the limit the mass p puts where q has none
    p = np.array([0.5, 0.3, 0.2, 0.0])
    q = np.array([0.0, 0.6, 0.2, 0.2])
    lp = np.log(np.maximum(p, 1e-300)).astype(np.float32)
    lq = np.log(np.maximum(q, 1e-300)).astype(np.float32)
    idx, tok, resid = oracle.multi_verify(lp, np.repeat(lq[None], 6, 0), [3] * 6, [ONE_BELOW] * 6, 0.0, 1.0, 4, want_resid=True)
    # step 1: sum max(0, p - q) = 0.5; afterwards the residual is the point mass on token 0, q(0) = 0
    np.testing.assert_allclose(resid, [0.5, 1, 1, 1, 1, 1], rtol=0, atol=1e-6)
    assert idx == 6 and tok == 0
