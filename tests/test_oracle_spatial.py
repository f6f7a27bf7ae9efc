"""Pins of the oracle's spatial drafting structures (Method, "Dual Direction Drafting Heads" and
"Spatial Sampling Pool"; appendix "Draft Heads Structure and Memory Overhead").

What is fixed outside the oracle:
  * the head: special weights for which it reduces to a library routine or a hand value (zero
    weights, a multiple of the identity, a single nonzero entry that tells W from its transpose,
    a head index that tells the heads apart), and torch's silu for the activation;
  * the cache size the paper prints, IW * VSD * (VSD + 1) / 2: the oracle's live entries reach it
    exactly and never pass it, whatever the accept lengths;
  * the definition of VertSpec: the pool at t holds exactly the predictions made from
    t - delta * IW with depth delta, checked against a scan of the whole history of predictions
    that is written here, not taken from the oracle.
"""
import json
import os

import numpy as np
import pytest
import torch

import synth
from oracle import spatial

GOLDEN = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_values.json")))


def test_paper_values_fix_the_head_shape_and_the_cache_size():
    # the 134 MB the appendix quotes are four d x d fp16 matrices at the 7B model's hidden size: heads
    # without output layers of their own (the reading the head oracle and kernels follow)
    s = synth.CONFIGS[4]
    h, wh, wo = synth.make_spatial_heads(0, 1, 4, 64, 16)
    assert wh.shape == (4, 64, 64) and wh.dtype == np.uint16        # one square matrix per head, 2 bytes a weight
    head_bytes = 4 * s.d_model * s.d_model * 2
    assert abs(head_bytes / 1e6 - GOLDEN["draft_heads_fp16_megabytes"]["value"]) < 0.5
    assert 4 * s.d_model * s.d_model / s.n_params() < GOLDEN["draft_heads_fraction_of_base_model_below"]["value"]
    # a head with an output layer of its own would be far beyond both figures
    assert (4 * (s.d_model * s.d_model + s.vocab * s.d_model)) * 2 / 1e6 > 10 * GOLDEN["draft_heads_fp16_megabytes"]["value"]
    for IW, VSD, entries in GOLDEN["speculation_cache_entries"]["examples"]:
        assert spatial.cache_entries(IW, VSD) == entries


def test_head_special_weights():
    rng = np.random.default_rng(1)
    rows, d, V, n_heads = 3, 8, 11, 4
    h = rng.standard_normal((rows, d))
    W_out = rng.standard_normal((V, d))
    W = np.zeros((n_heads, d, d))
    W[1] = 0.7 * np.eye(d)
    W[2][2, 5] = 1.0          # output feature 2 reads input feature 5
    W[3] = rng.standard_normal((d, d))
    g, logits = spatial.spatial_heads(h, W, W_out)
    # zero weights: silu(0) = 0, the head is the model's own output layer
    np.testing.assert_allclose(g[:, 0], h, rtol=0, atol=0)
    np.testing.assert_allclose(logits[:, 0], (torch.from_numpy(h) @ torch.from_numpy(W_out).T).numpy(), rtol=1e-6)
    # a multiple of the identity: elementwise
    ref = torch.from_numpy(h) + torch.nn.functional.silu(torch.from_numpy(0.7 * h))
    np.testing.assert_allclose(g[:, 1], ref.numpy(), rtol=1e-14)
    # a single entry: only feature 2 changes, by silu of input feature 5
    exp = h.copy()
    exp[:, 2] += torch.nn.functional.silu(torch.from_numpy(h[:, 5])).numpy()
    np.testing.assert_allclose(g[:, 2], exp, rtol=1e-14)
    # a general head against torch's linear layer (weights are [out, in])
    lin = torch.nn.functional.linear(torch.from_numpy(h), torch.from_numpy(W[3]))
    ref = torch.from_numpy(h) + torch.nn.functional.silu(lin)
    np.testing.assert_allclose(g[:, 3], ref.numpy(), rtol=1e-13)
    np.testing.assert_allclose(logits[:, 3], torch.nn.functional.linear(ref, torch.from_numpy(W_out)).numpy(), rtol=1e-6)
    assert logits.dtype == np.float32 and logits.shape == (rows, n_heads, V)


def test_head_hand_value():
    # d = 2, one head, one row, by hand: W h = (1*1 + 2*(-1), 0.5*1 + 0*(-1)) = (-1, 0.5)
    h = np.array([[1.0, -1.0]])
    W = np.array([[[1.0, 2.0], [0.5, 0.0]]])
    W_out = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    s = lambda x: x / (1.0 + np.exp(-x))
    g0, g1 = 1.0 + s(-1.0), -1.0 + s(0.5)
    g, logits = spatial.spatial_heads(h, W, W_out)
    np.testing.assert_allclose(g[0, 0], [g0, g1], rtol=1e-15)
    np.testing.assert_allclose(logits[0, 0], np.float32([g0, g1, g0 + g1]), rtol=1e-7)


@pytest.mark.parametrize("IW,IH,VSD", [(6, 9, 1), (6, 9, 2), (5, 12, 3), (24, 24, 2), (7, 3, 4)])
def test_cache_size_formula_and_vertspec_definition(IW, IH, VSD):
    rng = np.random.default_rng(IW * 100 + VSD)
    cache = spatial.SpecCache(IW, IH, VSD)
    history = []   # every vertical prediction ever made: (source position, depth)
    live_max = 0
    for T in range(IW * IH):
        # before T is committed its pool is read (as it would be while drafting)
        pool = cache.pool(T, ("horizontal", T))
        expect = [(dv, (T - dv * IW, dv)) for dv in range(1, VSD + 1) if (T - dv * IW, dv) in history]
        assert pool == expect + [(0, ("horizontal", T))]
        # rows of the image that no earlier row points to have no vertical members
        if T < IW:
            assert len(pool) == 1
        if T >= VSD * IW:
            assert len(pool) == VSD + 1
        # a drafting step looks a few positions ahead as well; what it finds there is final already
        ahead = T + int(rng.integers(1, IW))
        if ahead < IW * IH:
            got = cache.vert_spec(ahead)
            assert got == [(dv, (ahead - dv * IW, dv)) for dv in range(1, VSD + 1) if (ahead - dv * IW, dv) in history]
        cache.push(T, [(T, d) for d in range(1, VSD + 1)])
        history += [(T, d) for d in range(1, VSD + 1)]
        live = sum(1 for (src, d) in history if T < src + d * IW < IW * IH)
        assert live == len(cache.store)
        live_max = max(live_max, live)
        assert len(cache.store) <= spatial.cache_entries(IW, VSD)
    assert cache.peak == live_max
    if IH > VSD:   # enough rows for every depth to be outstanding at once
        assert cache.peak == spatial.cache_entries(IW, VSD)
    assert spatial.cache_entries(IW, VSD) == IW * sum(range(1, VSD + 1))
    assert len(cache.store) == 0   # everything made was consumed or fell off the image
