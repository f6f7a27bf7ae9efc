"""Pins of the oracle's sampling stage (warp, inverse CDF, accept / reject / resample).

Each test checks the oracle against something fixed outside it: a library routine
(torch.softmax / topk, numpy cumsum / searchsorted), exact rational enumeration of the
speculative-sampling rule (Preliminary, "Speculative Sampling"; appendix "Theoretical
Justification": acceptance probability 1 - sum(p - min(q,p)), residual
(p - min(q,p)) / sum(p - min(q,p)), and the decomposition of p into accepted and
residual parts specialised to one candidate per depth), or a chi-square statistic.
"""
import ctypes as C
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.filterwarnings("ignore")


# --------------------------------------------------------------------------- warp

def test_warp_full_support_is_softmax():
    rng = np.random.default_rng(0)
    for n in (8, 1000, 4096):
        l = (rng.standard_normal(n) * 2).astype(np.float32)
        w, z = oracle.warp(l, 1.0, n)
        ref = torch.softmax(torch.from_numpy(l).double(), 0).numpy()
        np.testing.assert_allclose(w / z, ref, rtol=1e-13, atol=0)
        assert abs(z - w.sum()) <= 1e-12 * z


@pytest.mark.parametrize("temperature", [1.0, 0.7, 2.0])
def test_warp_topk_matches_torch_topk_softmax(temperature):
    rng = np.random.default_rng(1)
    n, k = 4096, 1000
    l = rng.standard_normal(n).astype(np.float32)
    w, z = oracle.warp(l, temperature, k)
    zt = torch.from_numpy(l) * torch.tensor(1.0, dtype=torch.float32).div(temperature)  # fp32 scaling
    vals, idx = torch.topk(zt, k)
    ref = np.zeros(n)
    ref[idx.numpy()] = torch.softmax(vals.double(), 0).numpy()
    assert (w > 0).sum() == k
    np.testing.assert_allclose(w / z, ref, rtol=1e-13, atol=0)


def test_warp_ties_keep_lower_index():
    l = np.array([1.0, 3.0, 2.0, 3.0, 2.0, 2.0, 0.0, 2.0], dtype=np.float32)
    w, _ = oracle.warp(l, 1.0, 4)  # 3,3 and the first two 2's (indices 2 and 4)
    assert list(np.nonzero(w)[0]) == [1, 2, 3, 4]
    w, _ = oracle.warp(l, 1.0, 1)  # arg-max with lowest index
    assert list(np.nonzero(w)[0]) == [1] and w[1] == 1.0
    w, z = oracle.warp(l, 0.0, 5)  # temperature 0 is greedy whatever top_k says
    assert list(np.nonzero(w)[0]) == [1] and z == 1.0
    # stable ordering by (value desc, index asc) from a library sort
    rng = np.random.default_rng(2)
    l = rng.integers(0, 6, size=200).astype(np.float32)
    for k in (1, 7, 50, 199, 200):
        w, _ = oracle.warp(l, 1.0, k)
        keep = np.argsort(-l, kind="stable")[:k]
        assert sorted(np.nonzero(w)[0]) == sorted(keep) or k == 1


# --------------------------------------------------------------------------- inverse CDF

def test_inv_cdf_against_searchsorted():
    rng = np.random.default_rng(3)
    for trial in range(200):
        n = int(rng.integers(1, 50))
        w = rng.random(n) * (rng.random(n) < 0.6)
        if w.sum() == 0:
            w[rng.integers(n)] = 1.0
        z = float(np.sum(w))
        u = np.float32(rng.integers(0, 1 << 24) / (1 << 24))
        got = oracle.inv_cdf(w, z, float(u))
        pos = np.nonzero(w)[0]
        cs = np.cumsum(w[pos])
        j = int(np.searchsorted(cs, float(u) * z, side="right"))
        want = pos[min(j, len(pos) - 1)]
        # cumulative sums may differ in the last bit between the two orders of addition
        if abs(cs[min(j, len(pos) - 1)] - float(u) * z) > 1e-12 * z:
            assert got == want


def test_inv_cdf_edges():
    w = np.array([0.0, 0.25, 0.0, 0.5, 0.25, 0.0])
    assert oracle.inv_cdf(w, 1.0, 0.0) == 1          # u = 0: first index with mass
    assert oracle.inv_cdf(w, 1.0, 0.25) == 3         # boundary belongs to the next bin (c > u*Z)
    assert oracle.inv_cdf(w, 1.0, 0.7499999) == 3
    assert oracle.inv_cdf(w, 1.0, 0.75) == 4
    assert oracle.inv_cdf(w, 1.0, 1.0 - 2.0 ** -24) == 4
    assert oracle.inv_cdf(w, 0.5, 1.0 - 2.0 ** -24) == 3   # total given too small: still a valid bin
    assert oracle.inv_cdf(w, 2.0, 0.9) == 4          # nothing exceeds: last index with mass


# --------------------------------------------------------------------------- exact enumeration

def _rand_dist(rng, n, zero_prob=0.0):
    while True:
        v = [Fraction(int(rng.integers(1, 12))) * (0 if rng.random() < zero_prob else 1) for _ in range(n)]
        if sum(v) > 0:
            s = sum(v)
            return [x / s for x in v]


def _logits(dist):
    # zero probability -> a very low logit that top-k then removes
    return np.array([math.log(float(x)) if x > 0 else -80.0 for x in dist], dtype=np.float32)


def _enumerate_paths(P, Q, k, V):
    """All (drafts, a, y) with their exact probability under the accept / residual rule.
    P(prefix) and Q(prefix) give the target / draft distribution after `prefix`."""
    paths = []
    for drafts in itertools.product(range(V), repeat=k):
        pq = Fraction(1)
        for i in range(k):
            pq *= Q(drafts[:i])[drafts[i]]
        if pq == 0:
            continue
        acc = Fraction(1)
        for a in range(k + 1):
            if a < k:
                p, q = P(drafts[:a]), Q(drafts[:a])
                d = drafts[a]
                alpha = min(Fraction(1), p[d] / q[d])
                rej = acc * (1 - alpha)
                if rej > 0:
                    res = [max(Fraction(0), p[x] - q[x]) for x in range(V)]
                    tot = sum(res)
                    res = [r / tot for r in res] if tot > 0 else p
                    for y in range(V):
                        if res[y] > 0:
                            paths.append((drafts, a, y, pq * rej * res[y], res))
                acc *= alpha
                if acc == 0:
                    break
            else:
                p = P(drafts)
                for y in range(V):
                    if p[y] > 0:
                        paths.append((drafts, a, y, pq * acc * p[y], p))
    return paths


@pytest.mark.parametrize("k,V,seed", [(1, 5, 0), (2, 4, 1), (3, 3, 2), (2, 5, 3)])
def test_enumeration_preserves_target_and_oracle_follows_every_path(k, V, seed):
    rng = np.random.default_rng(seed)
    tabP, tabQ = {}, {}

    def P(prefix):
        if prefix not in tabP:
            tabP[prefix] = _rand_dist(rng, V)
        return tabP[prefix]

    def Q(prefix):
        if prefix not in tabQ:
            tabQ[prefix] = _rand_dist(rng, V, zero_prob=0.25)
        return tabQ[prefix]

    paths = _enumerate_paths(P, Q, k, V)
    assert sum(p[3] for p in paths) == 1
    # (A) the rule reproduces the target exactly: first emitted token ~ P(()),
    # and every later emitted token ~ P(accepted prefix)
    first = [Fraction(0)] * V
    for drafts, a, y, pr, _ in paths:
        first[drafts[0] if a >= 1 else y] += pr
    assert first == P(())
    for depth in range(1, k + 1):
        mass, joint = {}, {}
        for drafts, a, y, pr, _ in paths:
            if a >= depth:
                pre = drafts[:depth]
                tok = drafts[depth] if a > depth else y
                mass[pre] = mass.get(pre, 0) + pr
                joint[(pre, tok)] = joint.get((pre, tok), 0) + pr
        for (pre, tok), pr in joint.items():
            assert pr == mass[pre] * P(pre)[tok]

    # (B) the oracle takes exactly these decisions: drive it down every path
    seen = set()
    for drafts, a, y, pr, res in paths:
        p_rows = np.stack([_logits(P(drafts[:i])) for i in range(k + 1)])
        q_rows = np.stack([_logits(Q(drafts[:i])) for i in range(k)])
        u_acc = np.zeros(k, dtype=np.float32)
        for i in range(k):
            alpha = float(min(Fraction(1), P(drafts[:i])[drafts[i]] / Q(drafts[:i])[drafts[i]]))
            if i < a:
                u_acc[i] = alpha * (1 - 1e-4) if (drafts, a, i) in seen else alpha * 0.5
            elif i == a:
                u_acc[i] = alpha + (1 - alpha) * (1e-4 if (drafts, a, i) in seen else 0.5)
            seen.add((drafts, a, i))
        cdf = np.cumsum([float(r) for r in res])
        lo, hi = (cdf[y - 1] if y else 0.0), cdf[y]
        for frac in (0.5, 1e-3, 1 - 1e-3):
            u_f = np.float32(lo + (hi - lo) * frac)
            got_a, toks = oracle.spec_sample(p_rows, q_rows, drafts, u_acc, float(u_f), 1.0, V)
            assert got_a == a, (drafts, a, y)
            assert list(toks) == list(drafts[:a]) + [y], (drafts, a, y, frac)


def test_enumeration_with_topk_truncated_supports():
    # top-k makes the supports of p and q differ; the rational model is the renormalised top-k
    V, K = 6, 3
    p_full = [Fraction(x, 32) for x in (1, 9, 2, 8, 5, 7)]
    q_full = [Fraction(x, 32) for x in (10, 1, 6, 2, 9, 4)]

    def trunc(dist):
        keep = sorted(range(V), key=lambda j: (-dist[j], j))[:K]
        s = sum(dist[j] for j in keep)
        return [dist[j] / s if j in keep else Fraction(0) for j in range(V)]

    p, q = trunc(p_full), trunc(q_full)
    lp = np.stack([_logits(p_full)] * 2)
    lq = _logits(q_full)[None]
    for d in range(V):
        if q[d] == 0:
            continue
        alpha = float(min(Fraction(1), p[d] / q[d]))
        res = [max(Fraction(0), p[x] - q[x]) for x in range(V)]
        tot = sum(res)
        res = [float(r / tot) for r in res]
        if alpha > 0:
            a, toks = oracle.spec_sample(lp, lq, [d], [alpha * (1 - 1e-4)], 0.3, 1.0, K)
            assert a == 1 and toks[0] == d
        if alpha < 1:
            cdf = np.cumsum(res)
            for y in range(V):
                if res[y] == 0:
                    continue
                lo = cdf[y - 1] if y else 0.0
                for frac in (1e-3, 0.5, 1 - 1e-3):
                    a, toks = oracle.spec_sample(lp, lq, [d], [alpha + (1 - alpha) * 1e-4],
                                                 float(np.float32(lo + (cdf[y] - lo) * frac)), 1.0, K)
                    assert a == 0 and toks[0] == y


# --------------------------------------------------------------------------- statistics

def _raw():
    L = oracle.lib()
    return L


def _run_many(p_logits, q_logits, n_samples, seed, temperature=1.0, top_k=None):
    """n_samples independent speculative steps: drafts drawn from q with the oracle's own
    warp + inverse CDF, then accept / resample.  Returns (a, tokens[n, k+1])."""
    L = _raw()
    p = np.ascontiguousarray(p_logits, np.float32)
    q = np.ascontiguousarray(q_logits, np.float32)
    k, V = q.shape
    top_k = V if top_k is None else top_k
    rng = np.random.default_rng(seed)
    U = (rng.integers(0, 1 << 24, size=(n_samples, 2 * k + 1)).astype(np.float32) / np.float32(1 << 24))
    wq = [oracle.warp(q[i], temperature, top_k) for i in range(k)]
    wq_arr = [np.ascontiguousarray(w) for w, _ in wq]
    drafts = np.zeros(k, np.int32)
    toks = np.zeros(k + 1, np.int32)
    A = np.zeros(n_samples, np.int32)
    T = np.full((n_samples, k + 1), -1, np.int32)
    vp = C.c_void_p
    pp, qp, dp, tp = p.ctypes.data, q.ctypes.data, drafts.ctypes.data, toks.ctypes.data
    for s in range(n_samples):
        for i in range(k):
            drafts[i] = L.orc_inv_cdf(vp(wq_arr[i].ctypes.data), V, wq[i][1], float(U[s, i]))
        ua = U[s, k:2 * k]
        a = L.orc_spec_sample(k, V, vp(pp), vp(qp), vp(dp), 0, temperature, top_k,
                              vp(ua.ctypes.data), float(U[s, 2 * k]), vp(tp))
        A[s] = a
        T[s, : a + 1] = toks[: a + 1]
    return A, T


def _chi2(counts, probs):
    n = counts.sum()
    e = probs * n
    m = e > 0
    assert counts[~m].sum() == 0
    return float(((counts[m] - e[m]) ** 2 / e[m]).sum())


def test_chi_square_first_token_follows_target():
    # V = 8, 10^6 speculative samples, fixed seed; df = 7, reject above 24.32 (p-value 1e-3)
    rng = np.random.default_rng(11)
    V, n = 8, 1_000_000
    lp = rng.standard_normal((2, V)).astype(np.float32) * 1.5
    lq = rng.standard_normal((1, V)).astype(np.float32) * 1.5
    A, T = _run_many(lp, lq, n, seed=12)
    p = torch.softmax(torch.from_numpy(lp[0]).double(), 0).numpy()
    q = torch.softmax(torch.from_numpy(lq[0]).double(), 0).numpy()
    counts = np.bincount(T[:, 0], minlength=V)
    assert _chi2(counts, p) < 24.32
    # acceptance rate -> sum_x min(p, q)
    alpha = np.minimum(p, q).sum()
    assert abs(A.mean() - alpha) < 4.5 * math.sqrt(alpha * (1 - alpha) / n)


def test_chi_square_with_topk_and_second_token():
    rng = np.random.default_rng(21)
    V, K, n = 8, 5, 400_000
    lp = rng.standard_normal((3, V)).astype(np.float32) * 1.5
    lq = rng.standard_normal((2, V)).astype(np.float32) * 1.5
    A, T = _run_many(lp, lq, n, seed=22, top_k=K)

    def tk(l):
        v, i = torch.topk(torch.from_numpy(l), K)
        out = np.zeros(V)
        out[i.numpy()] = torch.softmax(v.double(), 0).numpy()
        return out

    p1, p2 = tk(lp[0]), tk(lp[1])
    assert _chi2(np.bincount(T[:, 0], minlength=V), p1) < 24.32  # df <= 7
    second = T[A >= 1, 1]
    assert len(second) > 50_000
    assert _chi2(np.bincount(second, minlength=V), p2) < 24.32


def test_tokens_per_step_closed_form():
    # identical (p, q) at every depth => acceptances are i.i.d. with rate alpha and
    # E[tokens per step] = (1 - alpha^(k+1)) / (1 - alpha)
    rng = np.random.default_rng(31)
    V, k, n = 8, 4, 200_000
    lp1 = rng.standard_normal(V).astype(np.float32)
    lq1 = (lp1 + rng.standard_normal(V).astype(np.float32) * 0.7).astype(np.float32)
    A, _ = _run_many(np.stack([lp1] * (k + 1)), np.stack([lq1] * k), n, seed=32)
    p = torch.softmax(torch.from_numpy(lp1).double(), 0).numpy()
    q = torch.softmax(torch.from_numpy(lq1).double(), 0).numpy()
    alpha = np.minimum(p, q).sum()
    want = (1 - alpha ** (k + 1)) / (1 - alpha)
    got = (A + 1).mean()
    assert abs(got - want) < 4.5 * (A + 1).std() / math.sqrt(n)


def test_q_equal_p_always_accepts_and_disjoint_always_rejects():
    rng = np.random.default_rng(41)
    V, k = 16, 3
    l = rng.standard_normal((k + 1, V)).astype(np.float32)
    A, T = _run_many(l, l[:k], 2000, seed=42)
    assert (A == k).all()
    # disjoint supports: q lives on the lower half, p on the upper half
    lp = np.where(np.arange(V) >= V // 2, l, -60.0).astype(np.float32)
    lq = np.where(np.arange(V) < V // 2, l[:k], -60.0).astype(np.float32)
    A, T = _run_many(lp, lq, 50_000, seed=43, top_k=V // 2)
    assert (A == 0).all()
    v, i = torch.topk(torch.from_numpy(lp[0]), V // 2)
    p = np.zeros(V)
    p[i.numpy()] = torch.softmax(v.double(), 0).numpy()
    assert _chi2(np.bincount(T[:, 0], minlength=V), p) < 24.32  # residual == p


def test_greedy_sampling_stage():
    rng = np.random.default_rng(51)
    V, k = 32, 4
    lp = rng.standard_normal((k + 1, V)).astype(np.float32)
    lq = rng.standard_normal((k, V)).astype(np.float32)
    am = lp.argmax(1)
    for n_ok in range(k + 1):
        drafts = am[:k].copy()
        if n_ok < k:
            drafts[n_ok] = (am[n_ok] + 1) % V
        for onehot in (False, True):
            u = rng.random(k).astype(np.float32)
            a, toks = oracle.spec_sample(lp, lq, drafts, u, 0.9, 0.0, V, q_onehot=onehot) \
                if onehot else oracle.spec_sample(lp, lq, drafts, u, 0.9, 0.0, V)
            if onehot or all(lq[i].argmax() == drafts[i] for i in range(min(n_ok + 1, k))):
                assert a == n_ok and toks[-1] == am[n_ok]


def test_zero_uniform_never_accepts_a_token_outside_the_target_support():
    # the test is the strict u*q < p: with u = 0 and p(d) = 0 the draft must still be rejected
    lp = np.array([[0.0, 5.0, 1.0, 2.0], [3.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    lq = np.array([[4.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    a, toks = oracle.spec_sample(lp, lq, [0], [0.0], 0.0, 1.0, 2)   # top-2 of p = {1, 3}; d = 0
    assert a == 0 and toks[0] == 1
    a, toks = oracle.spec_sample(lp, lq, [0], [0.0], 0.5, 0.0, 4)   # greedy: p = onehot(1)
    assert a == 0 and toks[0] == 1
    a, toks = oracle.spec_sample(lp, lq, [1], [0.0], 0.5, 0.0, 4, q_onehot=True)
    assert a == 1 and list(toks) == [1, 0]


def test_replay_onehot_draft_keeps_target_distribution():
    # q = point mass on a fixed draft token: accept with probability p(d), else
    # resample from p with d removed
    rng = np.random.default_rng(61)
    V, n = 8, 200_000
    lp = rng.standard_normal((2, V)).astype(np.float32)
    p = torch.softmax(torch.from_numpy(lp[0]).double(), 0).numpy()
    L = _raw()
    U = rng.integers(0, 1 << 24, size=(n, 2)).astype(np.float32) / np.float32(1 << 24)
    d = np.array([3], np.int32)
    toks = np.zeros(2, np.int32)
    cnt = np.zeros(V, np.int64)
    acc = 0
    q = np.zeros((1, V), np.float32)
    vp = C.c_void_p
    for s in range(n):
        ua = U[s, :1]
        a = L.orc_spec_sample(1, V, vp(lp.ctypes.data), vp(q.ctypes.data), vp(d.ctypes.data), 1, 1.0, V,
                              vp(ua.ctypes.data), float(U[s, 1]), vp(toks.ctypes.data))
        acc += a
        cnt[toks[0]] += 1
    assert _chi2(cnt, p) < 24.32
    assert abs(acc / n - p[3]) < 4.5 * math.sqrt(p[3] * (1 - p[3]) / n)


def test_uniform_generator_matches_big_integer_arithmetic():
    M64 = (1 << 64) - 1

    def mix(z):
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
        return z ^ (z >> 31)

    def ref(seed, seq, step, slot):
        ctr = (seq << 44) | (step << 8) | (slot & 0xFF)
        z = mix((seed + 0x9E3779B97F4A7C15) & M64)
        z = mix((z + 0x9E3779B97F4A7C15 * (ctr + 1)) & M64)
        return (z >> 40) / float(1 << 24)

    vals = []
    for seed in (0, 1, 2 ** 63 + 5):
        for seq in (0, 3, 31):
            for step in (0, 1, 600, 70000):
                for slot in (0, 4, 64, 68, 128):
                    u = oracle.uniform(seed, seq, step, slot)
                    assert u == ref(seed, seq, step, slot)
                    assert 0.0 <= u < 1.0
                    vals.append(u)
    assert len(set(vals)) > 0.99 * len(vals)
    assert abs(np.mean(vals) - 0.5) < 0.1
