"""Pins of the oracle's loop over the whole drafting and verification scheme (Method, overview figure;
"Sampling and Verification"; appendix "Theoretical Justification").

The loop only composes pieces that have pins of their own (heads, cache, pool, tree, walk, the model fed
row by row), so what is fixed here, outside the loop, is what must hold for the composition:
  * verification is lossless: at temperature 0 the image is the token-by-token arg-max image whatever
    the heads propose (random heads; and heads whose horizontal proposal is always right, which makes
    every pass commit HD + 1 tokens);
  * the bookkeeping: tokens committed = 1 + sum over passes of (accepted + 1) + the ordinary steps' tokens,
    every token inside the sampled slice, the same seed gives the same image, another seed another one;
  * the first token is the prefill's draw with step 0, slot 128 - the same as the chain's;
  * losslessness with sampling: the distribution of the second token given the first over many seeds is
    the target's, computed here from the model fed row by row, with a pool of two members at the second token.
"""
import numpy as np

import oracle
import synth
from oracle import scheme


def setup(seed_heads=3, HD=2, VSD=2, **kw):
    s = synth.CONFIGS[0].replace(**kw)
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    E = synth.blob_tensor(s, blob, "E")
    _, wh, wo = synth.make_spatial_heads(seed_heads, 1, HD + VSD, s.d_model, s.v_s)
    Wh, Wo = synth.bf16_bits_to_f32(wh), synth.bf16_bits_to_f32(wo)
    max_nodes = sum((VSD + 1) ** j for j in range(HD + 1))
    orc = oracle.Oracle.from_shape(s, blob, batch=1, k_max=max(max_nodes - 1, s.k))
    return s, blob, cond, E, Wh, Wo, orc


def run(s, cond, E, Wh, Wo, orc, HD, VSD, T, seed):
    return scheme.generate_spatial(orc, E, cond, s.n_cond, s.grid_h, s.grid_w, s.samp_lo, Wh, Wo, HD, VSD, T, s.top_k, seed)


def test_greedy_image_is_the_argmax_image_whatever_the_heads_propose():
    s, blob, cond, E, Wh, Wo, orc = setup(grid_h=6, grid_w=6)
    ref, _ = orc.generate(cond, None, 0, 0.0, s.top_k, 1.0, 1)
    grid, st = run(s, cond, E, Wh, Wo, orc, 2, 2, 0.0, 5)
    np.testing.assert_array_equal(grid, ref[0])
    assert st["passes"] > 0 and 1 + st["passes"] + st["accepted"] + st["tail_steps"] >= s.n_img - 1


def test_sampled_images_bookkeeping_and_seeds():
    s, blob, cond, E, Wh, Wo, orc = setup(HD=2, VSD=1, grid_h=4, grid_w=6)
    g1, st1 = run(s, cond, E, Wh, Wo, orc, 2, 1, 1.0, 7)
    g2, st2 = run(s, cond, E, Wh, Wo, orc, 2, 1, 1.0, 7)
    g3, _ = run(s, cond, E, Wh, Wo, orc, 2, 1, 1.0, 8)
    np.testing.assert_array_equal(g1, g2)
    assert st1 == st2 and not np.array_equal(g1, g3)
    assert ((g1 >= s.samp_lo) & (g1 < s.samp_lo + s.v_s)).all()
    # the first token is the chain's: the prefill's draw with step 0, slot 128
    chain, _ = orc.generate(cond, None, s.k, 1.0, s.top_k, 1.0, 7)
    assert g1[0] == chain[0, 0]
    # the widest tree has 1 + 2 + 4 = 7 nodes: tree passes run while 7 positions are left, ordinary steps after
    assert st1["passes"] >= (s.n_img - 7) // 3 and st1["tail_steps"] >= 1


def test_the_second_token_follows_the_target_distribution():
    # Lossless verification (appendix "Theoretical Justification"): whatever the two proposals of a pool are, the
    # token the pass commits is distributed as the target.  A 4 x 1 image (IW = 1: the vertical head of depth 1 and
    # the horizontal head both point to the next position, so the pool at position 1 has two members and the second
    # candidate meets the residual of the first), top-k 2, one layer: the distribution of token 1 given token 0 over
    # 300 seeds against the exact one from the model fed row by row.
    s, blob, cond, E, Wh, Wo, orc = setup(HD=1, VSD=1, n_layers=1, grid_h=4, grid_w=1, k=1, top_k=2)
    runs, seen = 300, {}
    for seed in range(1, runs + 1):
        g, st = run(s, cond, E, Wh, Wo, orc, 1, 1, 1.0, seed)
        seen.setdefault(int(g[0]), []).append(int(g[1]))
    assert len(seen) == 2, "top-k 2 leaves two first tokens"
    checked = 0
    for t0, seconds in seen.items():
        orc.prefill(cond, None, 1.0, s.top_k, 1.0, [0.5])            # conditions back in the cache; position 0 is fed below
        _, lg = orc.forward_row(0, s.n_cond, E[t0])
        w1, z1 = oracle.warp(lg, 1.0, s.top_k)
        support = {s.samp_lo + int(t): float(w1[t] / z1) for t in np.nonzero(w1)[0]}
        assert len(support) == 2 and set(seconds) <= set(support), "a token outside the target's support was committed"
        for t1, pr in support.items():
            sigma = (pr * (1 - pr) / len(seconds)) ** 0.5
            assert abs(seconds.count(t1) / len(seconds) - pr) < 4 * sigma + 1e-9, (t0, t1, pr, seconds.count(t1) / len(seconds))
            checked += 1
    assert checked == 4
