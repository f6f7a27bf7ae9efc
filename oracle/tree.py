"""CPU oracle of tree verification (Method, "Spatial Sampling Pool": the candidate tree as the
Cartesian product of the per-position samples; "Sampling and Verification": candidates of one
depth verified in order, the walk goes one depth down on an acceptance and ends with a draw from
the updated target on a rejection).

TEST INFRASTRUCTURE ONLY, like the rest of this package.  Nothing here masks or batches: a node's
target distribution is what the model gives after its path has been fed token by token, and the
walk calls the multi-candidate rule once per depth.
"""
from __future__ import annotations

import itertools
from typing import List, Sequence, Tuple

import numpy as np

import oracle


def tree_nodes(m_depth: Sequence[int]) -> List[Tuple[int, ...]]:
    """Nodes of the candidate tree as tuples of candidate indices (one per depth passed), the root
    first, then depth by depth, each depth in lexicographic order: depth j holds the Cartesian
    product of the first j candidate lists."""
    nodes: List[Tuple[int, ...]] = [()]
    for j in range(1, len(m_depth) + 1):
        nodes += list(itertools.product(*[range(m) for m in m_depth[:j]]))
    return nodes


def tree_logits(orc: "oracle.Oracle", E: np.ndarray, seq: int, base_pos: int, root_token: int,
                cand: Sequence[Sequence[int]], m_depth: Sequence[int], uncond_seq: int = -1,
                cfg_scale: float = 1.0) -> np.ndarray:
    """Target logits after every node: the root's row (the last committed token, at absolute
    position base_pos) and then the node's candidates, one row each at the following positions, fed
    through the model one after the other.  E: the embedding table [V, d].  With guidance
    (uncond_seq >= 0) the same rows go through the unconditional sequence as well and the two are
    combined as everywhere else (Experiment, "Model and Benchmark").  Returns [nodes, V_s]."""
    out = []
    for path in tree_nodes(m_depth):
        toks = [root_token] + [cand[j][i] for j, i in enumerate(path)]
        lg = lu = None
        for r, t in enumerate(toks):
            last = r == len(toks) - 1
            _, lg = orc.forward_row(seq, base_pos + r, E[t], want_logits=last)
            if uncond_seq >= 0:
                _, lu = orc.forward_row(uncond_seq, base_pos + r, E[t], want_logits=last)
        out.append(oracle.guide(lg, lu, cfg_scale) if uncond_seq >= 0 else lg)
    return np.stack(out)


def tree_walk(node_logits: np.ndarray, m_depth: Sequence[int], pool_logits: Sequence[np.ndarray],
              cand: Sequence[Sequence[int]], u_acc: Sequence[Sequence[float]], u_final: Sequence[float],
              temperature: float, top_k: int):
    """node_logits [nodes, n] in tree_nodes order; pool_logits[j] [m_j, n]: the proposals the
    candidates cand[j] of depth j + 1 were drawn from; u_acc[j] [m_j]; u_final [D + 1] (entry j
    for a rejection at depth j + 1, entry D for the extra token after D acceptances).
    Returns (accepted, tokens emitted (accepted + 1 of them), path of candidate indices)."""
    nodes = tree_nodes(m_depth)
    index = {p: i for i, p in enumerate(nodes)}
    path: Tuple[int, ...] = ()
    tokens: List[int] = []
    D = len(m_depth)
    for j in range(D):
        p_row = node_logits[index[path]]
        m = m_depth[j]
        idx, tok = oracle.multi_verify(p_row, np.asarray(pool_logits[j])[:m], list(cand[j])[:m], list(u_acc[j])[:m],
                                       float(u_final[j]), temperature, top_k)
        tokens.append(tok)
        if idx == m:
            return len(path), tokens, path
        assert tok == cand[j][idx]
        path = path + (idx,)
    w, z = oracle.warp(node_logits[index[path]], temperature, top_k)
    tokens.append(oracle.inv_cdf(w, z, float(u_final[D])))
    return D, tokens, path
