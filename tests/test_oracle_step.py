"""Pins of the oracle's whole speculate-and-verify step and generation loop.

Fixed points used: speculative decoding preserves the target model's output (Method,
"Sampling and Verification"), so with greedy decoding the speculative token sequence is
the plain token-by-token sequence whatever the drafts are; a step with no drafts is a
plain autoregressive step; a non-speculative run has accept length 1 (Experiment,
"Metrics"); raster-order neighbours x_{T-1} and x_{T-IW} (Preliminary, "Attention
Sinking").  The plain autoregressive reference is driven from the test through single
target rows only.
"""
import numpy as np
import pytest

import oracle
import synth


def ar_reference(shape, blob, cond, uniforms, temperature, top_k):
    """Token-by-token decoding using only forward_row + warp + inv_cdf."""
    o = oracle.Oracle.from_shape(shape, blob, batch=1)
    C, N = shape.n_cond, shape.n_img
    E = synth.blob_tensor(shape, blob, "E").astype(np.float64)
    for t in range(C):
        h, lg = o.forward_row(0, t, cond[0, t].astype(np.float64), want_logits=(t == C - 1))
    toks = []
    for t in range(N):
        w, z = oracle.warp(lg, temperature, top_k)
        toks.append(shape.samp_lo + oracle.inv_cdf(w, z, float(uniforms[t])))
        if t + 1 < N:
            h, lg = o.forward_row(0, C + t, E[toks[-1]])
    return np.array(toks, dtype=np.int32)


@pytest.fixture(scope="module")
def micro(micro_shape):
    blob = synth.make_weights(micro_shape, seed=0, std=0.3)
    cond = synth.make_cond(micro_shape, seed=2)
    return micro_shape, blob, cond


@pytest.mark.parametrize("k", [0, 1, 2, 3, 4])
def test_greedy_speculative_equals_plain_ar(micro, k):
    s, blob, cond = micro
    ref = ar_reference(s, blob, cond, np.zeros(s.n_img), 0.0, s.top_k)
    o = oracle.Oracle.from_shape(s, blob, k_max=4)
    grid, st = o.generate(cond, None, k, 0.0, s.top_k, 1.0, seed=3)
    assert (grid[0] == ref).all()
    assert st["tokens"] == s.n_img - 1 and st["steps"] == st["iters"]
    if k == 0:
        assert st["accepted"] == 0 and st["steps"] == s.n_img - 1  # accept length 1


@pytest.mark.parametrize("k", [1, 3, 4])
def test_greedy_with_adversarial_drafts_equals_plain_ar(micro, k):
    s, blob, cond = micro
    ref = ar_reference(s, blob, cond, np.zeros(s.n_img), 0.0, s.top_k)
    rng = np.random.default_rng(k)
    o = oracle.Oracle.from_shape(s, blob, k_max=4)
    o.prefill(cond, None, 0.0, s.top_k, 1.0, [0.5])
    total_acc = 0
    while o.n()[0] < s.n_img:
        n = int(o.n()[0])
        # random drafts, sometimes the true continuation so that acceptances occur too
        d = rng.integers(0, s.vocab, size=(1, k)).astype(np.int32)
        for i in range(k):
            if n + i < s.n_img and rng.random() < 0.5:
                d[0, i] = ref[n + i]
            else:
                break
        o.draft_forced(k, d, point_mass=bool(rng.integers(2)))
        na, toks = o.verify(k, rng.random((1, k)), rng.random(1))
        total_acc += int(na[0])
        assert (o.grid()[0, : o.n()[0]] == ref[: o.n()[0]]).all()
    assert total_acc > 0


def test_no_draft_step_is_plain_sampled_ar(micro):
    s, blob, cond = micro
    u = synth.make_uniforms(5, s.n_img)
    ref = ar_reference(s, blob, cond, u, 1.0, 17)
    o = oracle.Oracle.from_shape(s, blob)
    o.prefill(cond, None, 1.0, 17, 1.0, u[:1])
    for t in range(1, s.n_img):
        o.draft(0, None)
        na, toks = o.verify(0, None, u[t:t + 1])
        assert na[0] == 0 and toks[0, 0] == ref[t]
    assert (o.grid()[0] == ref).all()


def test_replay_of_greedy_tokens_accepts_everything(micro):
    s, blob, cond = micro
    k = 3
    ref = ar_reference(s, blob, cond, np.zeros(s.n_img), 0.0, s.top_k)
    o = oracle.Oracle.from_shape(s, blob)
    o.prefill(cond, None, 0.0, s.top_k, 1.0, [0.0])
    steps = 0
    while o.n()[0] < s.n_img:
        n = int(o.n()[0])
        k_eff = min(k, s.n_img - n - 1)
        d = np.zeros((1, k), np.int32)
        d[0, :k_eff] = ref[n:n + k_eff]
        o.draft_forced(k, d, point_mass=True)
        na, toks = o.verify(k, np.full((1, k), 0.999), [0.0])
        assert na[0] == k_eff                      # tokens per step == k_eff + 1 exactly
        assert list(toks[0, : k_eff + 1]) == list(ref[n:n + k_eff + 1])
        steps += 1
    assert o.n()[0] == s.n_img and steps == -(-(s.n_img - 1) // (k + 1))


def test_draft_reads_left_and_upper_neighbours(micro):
    s, blob, cond = micro
    k, IW = 3, s.grid_w
    rng = np.random.default_rng(9)
    o = oracle.Oracle.from_shape(s, blob)
    o.prefill(cond, None, 1.0, s.top_k, 1.0, [0.3])
    while o.n()[0] < s.n_img:
        n = int(o.n()[0])
        grid = o.grid()[0]
        g = o.h_prev()[0]
        u = rng.random((1, k)).astype(np.float32)
        d = o.draft(k, u)[0]
        lq = o.draft_logits()[0]
        k_eff = min(k, s.n_img - n - 1)
        for i in range(1, k + 1):
            if i > k_eff:
                assert d[i - 1] == -1            # no draft beyond the last grid position
                continue
            t = n - 1 + i
            left = grid[n - 1] if i == 1 else d[i - 2]      # raster predecessor, also at column 0
            up = grid[t - IW] if t >= IW else -1            # first image row: no upper neighbour
            g, lg = o.draft_head(g, int(left), int(up))
            assert (lg == lq[i - 1]).all()
            w, z = oracle.warp(lg, 1.0, s.top_k)
            assert d[i - 1] == oracle.inv_cdf(w, z, float(u[0, i - 1]))
        o.verify(k, rng.random((1, k)), rng.random(1))


def test_verify_commits_and_rewinds_cache(micro):
    s, blob, cond = micro
    k = 3
    rng = np.random.default_rng(13)
    o = oracle.Oracle.from_shape(s, blob)
    o.prefill(cond, None, 1.0, s.top_k, 1.0, [0.7])
    E = synth.blob_tensor(s, blob, "E").astype(np.float64)
    shadow = oracle.Oracle.from_shape(s, blob)  # fed strictly token by token
    for t in range(s.n_cond):
        h_sh, lg_sh = shadow.forward_row(0, t, cond[0, t].astype(np.float64))
    fed = 0
    while o.n()[0] < s.n_img:
        n0 = int(o.n()[0])
        d = o.draft(k, rng.random((1, k)))[0]
        ua, uf = rng.random((1, k)).astype(np.float32), rng.random(1).astype(np.float32)
        na, toks = o.verify(k, ua, uf)
        a = int(na[0])
        k_eff = min(k, s.n_img - n0 - 1)
        assert 0 <= a <= k_eff and o.n()[0] == n0 + a + 1
        assert list(toks[0, :a]) == list(d[:a]) and (toks[0, a + 1:] == -1).all()
        # h_prev is the hidden state of the row that produced the last committed token,
        # computed as if the committed tokens had been fed one by one
        grid = o.grid()[0]
        while fed < o.n()[0] - 1:
            h_sh, lg_sh = shadow.forward_row(0, s.n_cond + fed, E[grid[fed]])
            fed += 1
        np.testing.assert_allclose(o.h_prev()[0], h_sh, rtol=1e-12, atol=1e-13)
        # the emitted token is a draw from the target row a (or its residual)
        lp = o.logits()[0]
        np.testing.assert_allclose(lp[a], lg_sh, rtol=1e-5, atol=1e-6)
    assert fed == s.n_img - 1


def test_generate_is_the_loop_of_draft_and_verify(micro):
    s, blob, cond = micro
    k, seed = 3, 77
    o = oracle.Oracle.from_shape(s, blob)
    grid, st = o.generate(cond, None, k, 1.0, 20, 1.0, seed)
    m = oracle.Oracle.from_shape(s, blob)
    m.prefill(cond, None, 1.0, 20, 1.0, [oracle.uniform(seed, 0, 0, oracle.SLOT_FINAL)])
    step, acc = 0, 0
    while m.n()[0] < s.n_img:
        step += 1
        m.draft(k, [[oracle.uniform(seed, 0, step, oracle.SLOT_DRAFT + i) for i in range(k)]])
        na, _ = m.verify(k, [[oracle.uniform(seed, 0, step, oracle.SLOT_ACC + i) for i in range(k)]],
                         [oracle.uniform(seed, 0, step, oracle.SLOT_FINAL)])
        acc += int(na[0])
    assert (m.grid() == grid).all()
    assert st == dict(steps=step, accepted=acc, tokens=s.n_img - 1, iters=step)


def test_guidance_combines_two_streams(micro):
    s, blob, cond = micro
    sc = s.replace(cfg_scale=2.5)
    unc = synth.make_cond(s, seed=3)
    k = 2
    o = oracle.Oracle.from_shape(sc, blob)
    oc = oracle.Oracle.from_shape(s, blob)   # conditional stream alone
    ou = oracle.Oracle.from_shape(s, blob)   # unconditional stream alone
    o.prefill(cond, unc, 1.0, 10, 2.5, [0.4])
    oc.prefill(cond, None, 1.0, 10, 1.0, [0.4])
    ou.prefill(unc, None, 1.0, 10, 1.0, [0.4])
    x0 = int(o.grid()[0, 0])
    # force both single-stream oracles onto the guided run's tokens and compare logits
    d = o.draft(k, [[0.2, 0.6]])
    na, toks = o.verify(k, [[0.0, 0.0]], [0.5])   # u_acc = 0 accepts whenever p(d) > 0
    lp = o.logits()[0]
    E = synth.blob_tensor(s, blob, "E").astype(np.float64)
    rows = [x0] + list(d[0])
    for r, tok in enumerate(rows):
        _, lc = oc.forward_row(0, s.n_cond + r, E[tok])
        _, lu = ou.forward_row(0, s.n_cond + r, E[tok])
        want = (lu.astype(np.float64) + 2.5 * (lc.astype(np.float64) - lu.astype(np.float64)))
        np.testing.assert_allclose(lp[r], want, rtol=1e-5, atol=1e-6)
    hp = o.h_prev()
    assert hp.shape[0] == 2 and not np.allclose(hp[0], hp[1])


def test_force_equals_generated_state(micro):
    s, blob, cond = micro
    k = 3
    o = oracle.Oracle.from_shape(s, blob)
    grid, _ = o.generate(cond, None, k, 1.0, 20, 1.0, 5)
    f = oracle.Oracle.from_shape(s, blob)
    f.prefill(cond, None, 1.0, 20, 1.0, [oracle.uniform(5, 0, 0, oracle.SLOT_FINAL)])
    assert f.grid()[0, 0] == grid[0, 0]
    n = 1
    while n < s.n_img - 2:
        cnt = min(k + 1, s.n_img - 2 - n)
        f.force([n], grid[:, n:n + cnt])
        n += cnt
    assert f.n()[0] == s.n_img - 2 and (f.grid()[0, :n] == grid[0, :n]).all()
    # rewinding and forcing again gives the same hidden state
    h1 = f.h_prev().copy()
    f.force([n - 2], grid[:, n - 2:n])
    np.testing.assert_allclose(f.h_prev(), h1, rtol=1e-12, atol=1e-13)


def test_batch_prompts_are_independent(micro):
    s, blob, _ = micro
    cond = synth.make_cond(s, seed=2, batch=3)
    o = oracle.Oracle.from_shape(s, blob, batch=3)
    grid, st = o.generate(cond, None, 2, 1.0, 20, 1.0, 9)
    assert st["tokens"] == 3 * (s.n_img - 1)
    o1 = oracle.Oracle.from_shape(s, blob, batch=1)
    g0, _ = o1.generate(cond[:1], None, 2, 1.0, 20, 1.0, 9)
    assert (g0[0] == grid[0]).all()   # sequence index 0 draws the same uniforms


def test_argument_checks(micro):
    s, blob, cond = micro
    o = oracle.Oracle.from_shape(s, blob)
    with pytest.raises(RuntimeError):
        o.draft(2, [[0.1, 0.2]])                      # draft before prefill
    with pytest.raises(RuntimeError):
        o.prefill(cond, None, 1.0, s.vocab + 1, 1.0, [0.1])
    o.prefill(cond, None, 1.0, 5, 1.0, [0.1])
    with pytest.raises(RuntimeError):
        o.verify(2, [[0.1, 0.2]], [0.3])              # verify before draft
    with pytest.raises(RuntimeError):
        o.draft(s.grid_w + 1, np.zeros((1, s.grid_w + 1)))   # k beyond the grid width / k_max
