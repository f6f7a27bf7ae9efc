"""Pins of the oracle's tree verification (Method, "Spatial Sampling Pool": the candidate tree as
a Cartesian product; "Sampling and Verification": the walk).

Fixed outside the oracle:
  * the tree's shape: node counts sum_j prod_{i<=j} m_i, every root-to-leaf path is one element
    of the Cartesian product, every prefix of a node is a node;
  * one candidate per depth is the chain of the single-draft rule (the already pinned
    orc_spec_sample), one depth is the already pinned multi-candidate rule;
  * greedy decoding: the walk emits the arg-max continuation, whatever the candidates;
  * the point of the method: the emitted tokens follow the target's autoregressive law - a
    chi-square test over all sequences of length D + 1 of a tabular target, the walk's output
    completed with draws from the target where it stopped early.
"""
import itertools

import numpy as np

import oracle
from oracle import tree


def test_tree_is_the_cartesian_product():
    for m_depth in ((3,), (2, 3), (3, 3), (2, 1, 2), (1, 1, 1, 1), (4, 2, 3)):
        nodes = tree.tree_nodes(m_depth)
        assert nodes[0] == ()
        assert len(nodes) == 1 + sum(int(np.prod(m_depth[:j])) for j in range(1, len(m_depth) + 1))
        assert len(set(nodes)) == len(nodes)
        leaves = [p for p in nodes if len(p) == len(m_depth)]
        assert sorted(leaves) == sorted(itertools.product(*[range(m) for m in m_depth]))
        for p in nodes:
            assert all(p[:i] in nodes for i in range(len(p)))
            assert all(0 <= d < m_depth[j] for j, d in enumerate(p))
        depths = [len(p) for p in nodes]
        assert depths == sorted(depths)   # depth by depth, so a parent always comes before its children


class Table:
    """A tabular target: logits after any prefix, by a seeded draw per prefix."""

    def __init__(self, n, seed, scale=1.0):
        self.n, self.seed, self.scale, self.memo = n, seed, scale, {}

    def logits(self, prefix):
        prefix = tuple(int(t) for t in prefix)
        if prefix not in self.memo:
            rng = np.random.default_rng([self.seed, len(prefix), *prefix])
            self.memo[prefix] = (rng.standard_normal(self.n) * self.scale).astype(np.float32)
        return self.memo[prefix]

    def node_logits(self, m_depth, cand):
        return np.stack([self.logits([cand[j][i] for j, i in enumerate(p)]) for p in tree.tree_nodes(m_depth)])


def test_one_candidate_per_depth_is_the_chain_rule():
    rng = np.random.default_rng(5)
    n, D = 40, 3
    for trial in range(300):
        tab = Table(n, trial)
        top_k = int(rng.choice([n, 10]))
        q = (rng.standard_normal((D, n)) * 1.5).astype(np.float32)
        if trial % 3 == 0:
            q[0] = tab.logits(())                      # a good first proposal: longer chains
        cand = []
        for j in range(D):
            w, z = oracle.warp(q[j], 1.0, top_k)
            cand.append([oracle.inv_cdf(w, z, float(rng.random(dtype=np.float32)))])
        u_acc = rng.random((D, 1), dtype=np.float32)
        u_fin = rng.random(D + 1, dtype=np.float32)
        node_logits = tab.node_logits([1] * D, cand)   # nodes: root, (0), (0,0), (0,0,0) = the chain's rows
        acc, toks, path = tree.tree_walk(node_logits, [1] * D, [q[j:j + 1] for j in range(D)], cand, u_acc, u_fin, 1.0, top_k)
        # the chain rule draws its one final uniform where it stops
        a, ref = oracle.spec_sample(node_logits, q, [c[0] for c in cand], u_acc[:, 0], float(u_fin[acc]), 1.0, top_k)
        assert acc == a and toks == list(ref[:a + 1])


def test_one_depth_is_the_multi_candidate_rule():
    rng = np.random.default_rng(6)
    n, m = 30, 3
    for trial in range(100):
        p = (rng.standard_normal(n) * 1.5).astype(np.float32)
        q = (p + rng.standard_normal((m, n))).astype(np.float32)
        cand = [int(c) for c in rng.integers(0, n, m)]
        u = rng.random(m, dtype=np.float32)
        u_fin = rng.random(2, dtype=np.float32)
        nl = np.stack([p] + [rng.standard_normal(n).astype(np.float32) for _ in range(m)])
        acc, toks, path = tree.tree_walk(nl, [m], [q], [cand], [u], u_fin, 1.0, n)
        idx, tok = oracle.multi_verify(p, q, cand, u, float(u_fin[0]), 1.0, n)
        if idx == m:
            assert (acc, toks) == (0, [tok])
        else:   # accepted: the extra token comes from the accepted child's row
            w, z = oracle.warp(nl[1 + idx], 1.0, n)
            assert (acc, toks, path) == (1, [tok, oracle.inv_cdf(w, z, float(u_fin[1]))], (idx,))


def test_greedy_walk_is_the_argmax_continuation():
    rng = np.random.default_rng(7)
    n, m_depth = 12, (3, 2, 2)
    longest = 0
    for trial in range(200):
        tab = Table(n, 1000 + trial)
        best = []
        for j in range(len(m_depth) + 1):
            best.append(int(np.argmax(tab.logits(best))))
        cand = [[int(c) for c in rng.integers(0, n, m)] for m in m_depth]
        for j in range(trial % 4):   # plant the right token somewhere in the first depths
            if j < len(m_depth):
                cand[j][int(rng.integers(0, m_depth[j]))] = best[j]
        q = [(rng.standard_normal((m, n))).astype(np.float32) for m in m_depth]
        for j, m in enumerate(m_depth):   # greedy proposals are point masses on their candidates
            for i in range(m):
                q[j][i, cand[j][i]] = 50.0
        u_acc = [rng.random(m, dtype=np.float32) for m in m_depth]
        acc, toks, path = tree.tree_walk(tab.node_logits(m_depth, cand), m_depth, q, cand, u_acc,
                                         rng.random(len(m_depth) + 1, dtype=np.float32), 0.0, n)
        assert toks == best[:acc + 1]
        expect = 0
        while expect < len(m_depth) and best[expect] in cand[expect]:
            expect += 1
        assert acc == expect
        longest = max(longest, acc)
    assert longest == 3


def test_emitted_tokens_follow_the_autoregressive_law():
    n, m_depth, top_k = 4, (2, 2), 4
    D = len(m_depth)
    tab = Table(n, 77, scale=1.2)
    rng = np.random.default_rng(8)
    # proposals do not depend on the path (as in the method: the pool of a position is fixed before the pass)
    q = [(rng.standard_normal((m, n)) * 1.2).astype(np.float32) for m in m_depth]
    qd = [[oracle.warp(q[j][i], 1.0, top_k) for i in range(m)] for j, m in enumerate(m_depth)]
    samples = 60000
    counts = np.zeros((n,) * (D + 1))
    accepted_hist = np.zeros(D + 1, dtype=int)
    soft = lambda l: np.exp(l.astype(np.float64) - l.max()) / np.exp(l.astype(np.float64) - l.max()).sum()
    for _ in range(samples):
        cand = [[oracle.inv_cdf(*qd[j][i], float(rng.random(dtype=np.float32))) for i in range(m)] for j, m in enumerate(m_depth)]
        u_acc = [rng.random(m, dtype=np.float32) for m in m_depth]
        acc, toks, _ = tree.tree_walk(tab.node_logits(m_depth, cand), m_depth, q, cand, u_acc,
                                      rng.random(D + 1, dtype=np.float32), 1.0, top_k)
        accepted_hist[acc] += 1
        while len(toks) < D + 1:   # where the walk stopped the target itself goes on
            toks.append(int(rng.choice(n, p=soft(tab.logits(toks)))))
        counts[tuple(toks)] += 1
    law = np.zeros_like(counts)
    for seq in itertools.product(range(n), repeat=D + 1):
        pr = 1.0
        for j in range(D + 1):
            pr *= soft(tab.logits(seq[:j]))[seq[j]]
        law[seq] = pr
    chi2 = ((counts - samples * law) ** 2 / (samples * law)).sum()
    # 63 degrees of freedom: 99.9 % quantile 103.4
    assert chi2 < 103.4, chi2
    assert (accepted_hist > 0).all()
    # the marginal of the first token alone (3 degrees of freedom, 99.9 % quantile 16.27)
    first = counts.sum(axis=(1, 2))
    p0 = soft(tab.logits(()))
    assert ((first - samples * p0) ** 2 / (samples * p0)).sum() < 16.27


def test_guidance_routine_is_the_formula_of_the_guided_rows():
    # the routine the tree oracle combines two streams with (Experiment, "Model and Benchmark": guidance
    # scale): lu + s (lc - lu), against the formula in fp64 and its special cases
    rng = np.random.default_rng(9)
    lc = (rng.standard_normal(4096) * 3).astype(np.float32)
    lu = (rng.standard_normal(4096) * 3).astype(np.float32)
    for scale in (3.0, 4.0, 1.5):
        out = oracle.guide(lc, lu, scale)
        ref = lu.astype(np.float64) + scale * (lc.astype(np.float64) - lu.astype(np.float64))
        assert out.dtype == np.float32
        np.testing.assert_allclose(out, ref, rtol=3e-7, atol=1e-6)   # one rounding of the difference, one of the result
    np.testing.assert_array_equal(oracle.guide(lc, lu, 0.0), lu)       # scale 0: the unconditional stream
    np.testing.assert_array_equal(oracle.guide(lc, lc, 3.0), lc)       # equal streams: unchanged
    # scale 1 gives back the conditional stream up to the rounding of the difference
    np.testing.assert_allclose(oracle.guide(lc, lu, 1.0), lc, rtol=0, atol=1e-6)
    # the direction matters: a larger scale moves further from the unconditional stream
    assert np.all(np.abs(oracle.guide(lc, lu, 4.0) - lu) >= np.abs(oracle.guide(lc, lu, 2.0) - lu) - 1e-6)
