"""CPU oracle of the whole drafting and verification scheme over one image (Method, overview figure:
dual-direction heads -> speculation cache -> spatial sampling pool -> candidate tree -> verification;
"Sampling and Verification").

TEST INFRASTRUCTURE ONLY, like the rest of this package.  The loop takes the paper's steps one after
the other with the pieces defined in this package - the heads and the cache of `oracle.spatial`, the
tree and its walk of `oracle.tree`, the model of `oracle.Oracle` fed row by row - and nothing else: no
masks, no batching, no moved cache entries.  One prompt, no guidance.

Per pass, from n committed tokens (T = position a hidden state predicts):
  1. the heads on the hidden states of the rows committed by the pass before (first pass: the last
     condition row, T = 0); horizontal head j proposes position T + j, vertical head d position T + d * IW;
  2. every vertical prediction goes to the cache under the position it points to;
  3. the pool at position n + j, j = 0 .. HD - 1: the cached vertical predictions for it in ascending
     depth, then horizontal head j + 1 of the last committed row;
  4. one candidate per pool member by inverse CDF from the member's warped distribution;
  5. the target distribution after every node of the candidate tree, the walk (multi-candidate rule
     per depth), commit of the accepted candidates and the extra token.
When fewer positions are left than the widest tree has nodes, ordinary steps with one draft token of the
model's own draft head finish the image.  Uniforms: `oracle.uniform(seed, 0, step, slot)` with step =
pass number from 1 (the ordinary steps go on counting), slot 8 j + i for the candidate of member i at
depth j + 1, 64 + 8 j + i for its acceptance test, 128 + j for the draw after a rejection at depth j + 1
(j = HD: the extra token); step 0 slot 128 samples token 0; an ordinary step uses slots 0, 64, 128.
"""
from __future__ import annotations

import numpy as np

import oracle
from oracle import spatial, tree


def generate_spatial(orc: "oracle.Oracle", E: np.ndarray, cond: np.ndarray, n_cond: int, IH: int, IW: int, samp_lo: int,
                     W_heads: np.ndarray, W_out: np.ndarray, HD: int, VSD: int, temperature: float, top_k: int, seed: int):
    """E: embedding table [V, d]; W_heads [HD + VSD, d, d], W_out [V_s, d] (fp32 / fp64 arrays holding the
    heads' bf16 values).  Returns (grid [N] of vocabulary ids, dict(passes, accepted, tail_steps))."""
    N, C, lo = IH * IW, n_cond, samp_lo
    u = lambda step, slot: oracle.uniform(seed, 0, step, slot)  # noqa: E731
    orc.prefill(cond, None, temperature, top_k, 1.0, [u(0, 128)])
    cache = spatial.SpecCache(IW, IH, VSD)
    h_rows, positions, n, step = [np.asarray(orc.h_prev()[0], np.float64)], [0], 1, 0
    max_nodes = sum((VSD + 1) ** j for j in range(HD + 1))
    passes = accepted = tail = 0
    while n + max_nodes <= N:
        step += 1
        _, q_all = spatial.spatial_heads(np.stack(h_rows), W_heads, W_out)            # [rows, heads, V_s]
        for i, T in enumerate(positions):
            cache.push(T, [q_all[i, HD + dv] for dv in range(VSD)])
        pools = [cache.pool(n + j, q_all[-1, j]) for j in range(HD)]
        m_depth = [len(p) for p in pools]
        cand = []
        for j, pool in enumerate(pools):
            row = []
            for i, (_, logits) in enumerate(pool):
                w, z = oracle.warp(logits, temperature, top_k)
                row.append(int(oracle.inv_cdf(w, z, u(step, 8 * j + i))))
            cand.append(row)
        root, base = int(orc.grid()[0, n - 1]), C + n - 1
        node_logits = tree.tree_logits(orc, E, 0, base, root, [[lo + c for c in row] for row in cand], m_depth)
        a, toks, _ = tree.tree_walk(node_logits, m_depth, [np.stack([r for _, r in pool]) for pool in pools], cand,
                                    [[u(step, 64 + 8 * j + i) for i in range(m_depth[j])] for j in range(HD)],
                                    [u(step, 128 + j) for j in range(HD + 1)], temperature, top_k)
        # the rows that were committed - the root and the accepted candidates, fed one after the other -
        # give the hidden states the heads read next
        fed = [root] + [lo + t for t in toks[:a]]
        h_rows = [np.asarray(orc.forward_row(0, base + r, E[t], want_logits=False)[0], np.float64) for r, t in enumerate(fed)]
        orc.force(np.array([n], dtype=np.int32), np.array([[lo + t for t in toks]], dtype=np.int32))
        positions = [n + i for i in range(a + 1)]
        n += a + 1
        passes += 1
        accepted += a
    while n < N:
        step += 1
        orc.draft(1, [[u(step, 0)]])
        na, _ = orc.verify(1, [[u(step, 64)]], [u(step, 128)])
        n += int(na[0]) + 1
        tail += 1
    return orc.grid()[0].copy(), dict(passes=passes, accepted=accepted, tail_steps=tail)
