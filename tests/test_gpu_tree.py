"""GPU parity of tree verification (Method, "Spatial Sampling Pool": the candidate tree;
"Sampling and Verification": the walk) against the oracle: the rows of the target pass over the
tree against the model fed path by path, the walk's result, and - through the steps that follow -
the cache entries and the hidden state the call leaves behind.

fp32 configuration: everything exact.  bf16: node logits within 2e-2, the walk exact on the GPU's
own logits, and the ordinary step after the tree step within 2e-2 of the oracle's (which only holds
if the accepted path's keys and values were moved to the right entries).  The oracle always commits
its own walk's tokens; a GPU result that differs (bf16) is forced onto them before the next step.

Inputs are seeded and synthetic: the proposals of depth j are the target's logits after the first
candidates of the depths before (from the oracle) plus noise of half the logits' standard deviation
- drafts that are right fairly often -, candidates drawn from them by inverse CDF, uniforms on the 2^-24 grid.
"""
import numpy as np
import pytest

import oracle
import synth
from oracle import tree

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    import paper_2510_25739_amd as H
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return H


def uni(rng, *shp):
    return (rng.integers(0, 1 << 24, size=shp).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)


def build_pools(orc, E, s, n, grid, m_depth, rng, T, K, sigma=0.5):
    """Proposals and candidates for every prompt: cand [D, B, m_max], q [D, B, m_max, V_s]."""
    B, D, m_max = len(n), len(m_depth), max(m_depth)
    cand = np.zeros((D, B, m_max), dtype=np.int32)
    q = np.zeros((D, B, m_max, s.v_s), dtype=np.float32)
    for b in range(B):
        base = s.n_cond + int(n[b]) - 1
        toks = [int(grid[b, n[b] - 1])]
        for j in range(D):
            lg = None
            for r, t in enumerate(toks):
                _, lg = orc.forward_row(b, base + r, E[t], want_logits=(r == len(toks) - 1))
            noise = rng.standard_normal((m_depth[j], s.v_s)).astype(np.float32) * np.float32(sigma * lg.std())
            q[j, b, :m_depth[j]] = lg[None, :] + noise
            for i in range(m_depth[j]):
                w, z = oracle.warp(q[j, b, i], T, K)
                cand[j, b, i] = oracle.inv_cdf(w, z, float(uni(rng, 1)[0]))
            toks.append(s.samp_lo + int(cand[j, b, 0]))
    return cand, q


def n_nodes_of(m_depth):
    return len(tree.tree_nodes(m_depth))


def same_committed(hk, orc):
    """Committed tokens agree (entries beyond n are whatever the workspace held)."""
    n = orc.n()
    np.testing.assert_array_equal(hk.n(), n)
    g, o = hk.grid(), orc.grid()
    for b in range(len(n)):
        np.testing.assert_array_equal(g[b, :n[b]], o[b, :n[b]])


def force_rows(obj, grid, n0, rows):
    """Forces prompt b onto the tokens rows[b] from position n0[b]; the forced call takes one count for all
    prompts, so the shorter ones start further back and feed tokens that are committed already."""
    cnt = max(len(r) for r in rows)
    begin, data = [], []
    for b, own in enumerate(rows):
        pad = cnt - len(own)
        begin.append(int(n0[b]) - pad)
        data.append([int(t) for t in grid[b, n0[b] - pad:n0[b]]] + [int(t) for t in own])
    assert min(begin) >= 1
    obj.force(np.array(begin, dtype=np.int32), np.array(data, dtype=np.int32))


def tree_step(H, hk, orc, E, s, m_depth, rng, T, K):
    """One tree step on both sides from the same committed state.  The oracle commits its own result
    (the tokens fed one after the other: no mask, no moved cache entries); where the GPU's result
    differs (bf16 only: the two walks saw slightly different rows) the GPU is forced onto the oracle's
    tokens.  Returns what was compared; "same": the GPU's tokens were the oracle's."""
    import torch
    B, D = hk.batch, len(m_depth)
    n, grid = orc.n().copy(), orc.grid()
    cand, q = build_pools(orc, E, s, n, grid, m_depth, rng, T, K)
    u_acc, u_fin = uni(rng, D, B, max(m_depth)), uni(rng, D + 1, B)
    na, toks = hk.verify_tree(m_depth, cand, torch.from_numpy(q).to("cuda:0"), u_acc, u_fin)
    nn = n_nodes_of(m_depth)
    lg_g = hk.tree_logits(nn)
    out = dict(err=0.0, acc=[], same=True)
    o_rows = []
    for b in range(B):
        cb = [[int(c) for c in cand[j, b, :m_depth[j]]] for j in range(D)]
        lg_o = tree.tree_logits(orc, E, b, s.n_cond + int(n[b]) - 1, int(grid[b, n[b] - 1]),
                                [[s.samp_lo + c for c in row] for row in cb], m_depth,
                                uncond_seq=B + b if s.use_cfg else -1, cfg_scale=s.cfg_scale)
        out["err"] = max(out["err"], float(np.abs(lg_g[b].astype(np.float64) - lg_o).max()))
        args = (m_depth, [q[j, b] for j in range(D)], cb, [u_acc[j, b] for j in range(D)], u_fin[:, b], T, K)
        # the walk on the GPU's own rows must give the GPU's result exactly
        a_s, t_s, _ = tree.tree_walk(lg_g[b], *args)
        assert na[b] == a_s and list(toks[b, :a_s + 1]) == [s.samp_lo + t for t in t_s], (na[b], toks[b], a_s, t_s)
        assert (toks[b, a_s + 1:] == -1).all()
        a_o, t_o, _ = tree.tree_walk(lg_o, *args)
        out["same"] = out["same"] and (a_o == a_s and t_o == t_s)
        out["acc"].append(a_o)
        o_rows.append([s.samp_lo + t for t in t_o])
    force_rows(orc, grid, n, o_rows)
    if not out["same"]:
        force_rows(hk, grid, n, o_rows)
    same_committed(hk, orc)
    return out


def chain_step(hk, orc, s, k, rng, exact):
    """An ordinary draft + verify step on both sides; returns the largest logit error."""
    B = hk.batch
    ud, ua, uf = uni(rng, B, k), uni(rng, B, k), uni(rng, B)
    d_o, d_g = orc.draft(k, ud), hk.draft(k, ud)
    if exact:
        np.testing.assert_array_equal(d_g, d_o)
    elif not np.array_equal(d_g, d_o):   # a draft that differs changes the inputs of the ones after it: same drafts first
        hk.draft_forced(k, np.where(d_o >= 0, d_o, s.samp_lo).astype(np.int32), False)
    err = float(np.abs(hk.draft_logits(k) - orc.draft_logits()).max())
    na_g, t_g = hk.verify(k, ua, uf)
    na_o, t_o = orc.verify(k, ua, uf)
    err = max(err, float(np.abs(hk.logits(k + 1) - orc.logits()).max()))
    if exact:
        np.testing.assert_array_equal(na_g, na_o)
        np.testing.assert_array_equal(t_g, t_o)
    elif not (np.array_equal(na_g, na_o) and np.array_equal(t_g, t_o)):
        force_rows(hk, orc.grid(), orc.n() - (na_o + 1), [t_o[b, :na_o[b] + 1] for b in range(B)])
    return err


def start(H, s, k_max, batch=1, path=1):
    blob = synth.make_weights(s, seed=0)
    hk = H.Hawk(H.HawkConfig.from_shape(s, batch=batch, k_max=k_max))
    hk.load(blob)
    hk.set_path(path)   # 1: the persistent kernel where it applies, 0: one kernel per operation
    orc = oracle.Oracle.from_shape(s, blob, batch=batch, k_max=k_max)
    cond = synth.make_cond(s, seed=2, batch=batch)
    unc = synth.make_cond(s, seed=3, batch=batch) if s.use_cfg else None
    u0 = synth.make_uniforms(9, (batch,))
    hk.prefill(cond, unc, s.grid_h, s.grid_w, s.temperature, s.top_k, s.cfg_scale, u0)
    orc.prefill(cond, unc, s.temperature, s.top_k, s.cfg_scale, u0)
    E = synth.blob_tensor(s, blob, "E").astype(np.float64)
    return hk, orc, E


@pytest.mark.parametrize("m_depth", [(3, 3), (2, 2, 2), (4,), (1, 1, 1, 1), (2, 3, 1)])
def test_tree_steps_fp32_exact(H, m_depth):
    s = synth.CONFIGS[0].replace(top_k=64)   # top-k 64 of 4096: drafts get accepted often enough to walk deep
    hk, orc, E = start(H, s, k_max=14)
    np.testing.assert_array_equal(hk.grid()[:, 0], orc.grid()[:, 0])
    rng = np.random.Generator(np.random.PCG64(sum(m_depth) * 7 + len(m_depth)))
    nn, accs, moved = n_nodes_of(m_depth), [], 0
    while orc.n()[0] + nn <= s.n_img:
        r = tree_step(H, hk, orc, E, s, m_depth, rng, s.temperature, s.top_k)
        assert r["err"] < 1e-4 and r["same"]
        accs.append(r["acc"][0])
        # an ordinary step from the state the tree step left: exact only if the cache entries of the
        # accepted path and the kept hidden state are the right ones
        if orc.n()[0] + s.k + 1 <= s.n_img:
            chain_step(hk, orc, s, s.k, rng, exact=True)
    print("accepted per tree step:", accs)
    assert max(accs) >= min(2, len(m_depth)) and min(accs) == 0


@pytest.mark.parametrize("m_depth", [(63,), (1,) * 8, (7, 7), (3, 3, 3)])
def test_tree_extreme_shapes_fp32_exact(H, m_depth):
    # the largest tree (64 nodes: 63 candidates at one depth), the deepest (8 depths), 57 and 40 nodes
    s = synth.CONFIGS[0].replace(top_k=64, grid_h=12, grid_w=12)
    hk, orc, E = start(H, s, k_max=63)
    np.testing.assert_array_equal(hk.grid()[:, 0], orc.grid()[:, 0])
    rng = np.random.Generator(np.random.PCG64(len(m_depth) * 100 + m_depth[0]))
    accs = []
    for _ in range(3):
        if orc.n()[0] + n_nodes_of(m_depth) > s.n_img:
            break
        r = tree_step(H, hk, orc, E, s, m_depth, rng, s.temperature, s.top_k)
        assert r["err"] < 1e-4 and r["same"]
        accs.append(r["acc"][0])
        chain_step(hk, orc, s, s.k, rng, exact=True)
    print("accepted per tree step:", accs)
    assert len(accs) >= 2


def test_tree_steps_with_guidance_fp32_exact(H):
    # classifier-free guidance: both streams go through the tree pass, every target row is guided
    s = synth.CONFIGS[0].replace(top_k=64, cfg_scale=2.0)
    hk, orc, E = start(H, s, k_max=12)
    np.testing.assert_array_equal(hk.grid()[:, 0], orc.grid()[:, 0])
    rng = np.random.Generator(np.random.PCG64(17))
    accs = []
    while orc.n()[0] + 13 <= s.n_img:
        r = tree_step(H, hk, orc, E, s, (3, 3), rng, s.temperature, s.top_k)
        assert r["err"] < 1e-4 and r["same"]
        accs.append(r["acc"][0])
        if orc.n()[0] + s.k + 1 <= s.n_img:
            chain_step(hk, orc, s, s.k, rng, exact=True)   # both streams' cache entries are in place
    print("accepted per tree step:", accs)
    assert max(accs) == 2


def test_tree_step_two_prompts_fp32(H):
    s = synth.CONFIGS[0].replace(top_k=64)
    hk, orc, E = start(H, s, k_max=12, batch=2)
    rng = np.random.Generator(np.random.PCG64(21))
    chain_step(hk, orc, s, s.k, rng, exact=True)   # the prompts stand at different positions afterwards
    seen = set()
    for _ in range(4):
        r = tree_step(H, hk, orc, E, s, (3, 3), rng, s.temperature, s.top_k)
        assert r["err"] < 1e-4 and r["same"]
        seen.update(r["acc"])   # the prompts accept different numbers of candidates
        chain_step(hk, orc, s, s.k, rng, exact=True)
    assert len(seen) > 1


def test_tree_step_two_prompts_bf16(H):
    # two prompts, 7-node trees: 14 rows on the persistent kernel
    s = synth.CONFIGS[2].replace(n_layers=4)
    hk, orc, E = start(H, s, k_max=12, batch=2)
    if not np.array_equal(hk.grid()[:, 0], orc.grid()[:, 0]):
        pytest.skip("token 0 differs in bf16 for this seed")
    rng = np.random.Generator(np.random.PCG64(22))
    worst = chain_step(hk, orc, s, s.k, rng, exact=False)
    same_committed(hk, orc)
    seen, agree = set(), 0
    for _ in range(4):
        r = tree_step(H, hk, orc, E, s, (2, 2), rng, s.temperature, s.top_k)
        assert hk.last_path() == 1
        seen.update(r["acc"])
        agree += int(r["same"])
        worst = max(worst, r["err"], chain_step(hk, orc, s, s.k, rng, exact=False))
        same_committed(hk, orc)
    print(f"max-abs logit error {worst:.2e}, accepted counts seen {sorted(seen)}, steps with the oracle's tokens {agree}/4")
    assert worst < 2e-2 and agree >= 1


@pytest.mark.parametrize("path,m_depth", [(1, (3, 3)), (0, (3, 3)), (1, (5, 2)), (1, (2, 2, 1)), (1, (2, 2)), (1, (4, 1))])
def test_tree_steps_bf16(H, path, m_depth):
    # the XL shape at four layers: node logits within tolerance, the walk exact on the GPU's own rows,
    # and the ordinary steps in between stay within tolerance (keys and values of the accepted path in place);
    # on the persistent kernel (trees of up to 16 rows; one row per attention job up to 10 rows, two beyond)
    # and with one kernel per operation
    s = synth.CONFIGS[2].replace(n_layers=4)
    hk, orc, E = start(H, s, k_max=15, path=path)
    if hk.grid()[0, 0] != orc.grid()[0, 0]:
        pytest.skip("token 0 differs in bf16 for this seed")
    rng = np.random.Generator(np.random.PCG64(4))
    worst, accs, agree = 0.0, [], 0
    for step in range(6):
        r = tree_step(H, hk, orc, E, s, m_depth, rng, s.temperature, s.top_k)
        assert hk.last_path() == path
        worst = max(worst, r["err"])
        agree += int(r["same"])
        a = r["acc"][0]
        accs.append(a)
        ce = chain_step(hk, orc, s, s.k, rng, exact=False)
        print(f"step {step}: tree rows {r['err']:.2e}, accepted {a}, same tokens {r['same']}, ordinary step after it {ce:.2e}")
        worst = max(worst, ce)
    print(f"max-abs logit error {worst:.2e}, accepted {accs}, walks identical to the oracle's {agree}/6")
    assert worst < 2e-2
    assert max(accs) >= 1 and agree >= 2   # steps with the same tokens also check the moved cache entries


@pytest.mark.parametrize("m_depth,path", [((3, 3), 0), ((2, 2), 1)])
def test_tree_steps_with_guidance_bf16(H, m_depth, path):
    # the XL shape at four layers with guidance 4.0 (the batched configuration's scale), one prompt: 26 rows
    # per pass run one kernel per operation, 14 rows (two streams of a 7-node tree) on the persistent kernel
    s = synth.CONFIGS[3].replace(n_layers=4, batch=1)
    hk, orc, E = start(H, s, k_max=12)
    if hk.grid()[0, 0] != orc.grid()[0, 0]:
        pytest.skip("token 0 differs in bf16 for this seed")
    rng = np.random.Generator(np.random.PCG64(12))
    worst, accs = 0.0, []
    for step in range(4):
        r = tree_step(H, hk, orc, E, s, m_depth, rng, s.temperature, s.top_k)
        assert hk.last_path() == path
        a = r["acc"][0]
        accs.append(a)
        ce = chain_step(hk, orc, s, s.k, rng, exact=False)
        print(f"step {step}: tree rows {r['err']:.2e}, accepted {a}, ordinary step after it {ce:.2e}")
        worst = max(worst, r["err"], ce)
    assert worst < 2e-2


def test_tree_step_full_depth_bf16(H):
    # the XL configuration at its full depth (36 layers), the tree the timing helper uses (13 rows)
    s = synth.CONFIGS[2]
    hk, orc, E = start(H, s, k_max=12)
    if hk.grid()[0, 0] != orc.grid()[0, 0]:
        pytest.skip("token 0 differs in bf16 for this seed")
    rng = np.random.Generator(np.random.PCG64(8))
    worst = 0.0
    for step in range(2):
        r = tree_step(H, hk, orc, E, s, (3, 3), rng, s.temperature, s.top_k)
        a = r["acc"][0]
        ce = chain_step(hk, orc, s, s.k, rng, exact=False)
        print(f"step {step}: tree rows {r['err']:.2e}, accepted {a}, ordinary step after it {ce:.2e}")
        worst = max(worst, r["err"], ce)
    assert worst < 2e-2


@pytest.mark.parametrize("cfg,m_depth,path", [(0, (2, 2), 1), (0, (3, 2, 1), 1), (1, (3, 3), 1), (1, (3, 3), 0), (1, (3, 4), 1)])
def test_greedy_tree_decoding_is_plain_greedy_decoding(H, cfg, m_depth, path):
    # whole images: with temperature 0 the tokens must be those of token-by-token arg-max decoding,
    # whatever the candidates are (some are planted from the reference so that the walk goes deep,
    # the others are random); the image's last positions, where the tree no longer fits, are ordinary steps
    import torch
    s = synth.CONFIGS[cfg]
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    nn = n_nodes_of(m_depth)
    hk = H.Hawk(H.HawkConfig.from_shape(s, batch=1, k_max=max(nn - 1, s.k)))
    hk.load(blob)
    hk.set_path(path)
    ref, _ = hk.generate(cond, None, s.grid_h, s.grid_w, 0, 0.0, s.top_k, 1.0, 1)
    hk.prefill(cond, None, s.grid_h, s.grid_w, 0.0, s.top_k, 1.0, np.array([0.5], np.float32))
    rng = np.random.Generator(np.random.PCG64(cfg + 40))
    D, m_max = len(m_depth), max(m_depth)
    accs = []
    while hk.n()[0] < s.n_img:
        n = int(hk.n()[0])
        if n + nn > s.n_img:
            hk.draft(1, uni(rng, 1, 1))
            hk.verify(1, uni(rng, 1, 1), uni(rng, 1))
            continue
        cand = rng.integers(0, s.v_s, size=(D, 1, m_max)).astype(np.int32)
        for j in range(D):
            if rng.random() < 0.8:
                cand[j, 0, int(rng.integers(0, m_depth[j]))] = ref[0, n + j] - s.samp_lo
        q = torch.zeros((D, 1, m_max, s.v_s), device="cuda:0")
        q.scatter_(3, torch.from_numpy(cand.astype(np.int64)).to("cuda:0")[..., None], 50.0)   # point masses on the candidates
        na, toks = hk.verify_tree(m_depth, cand, q, uni(rng, D, 1, m_max), uni(rng, D + 1, 1))
        accs.append(int(na[0]))
        expect = 0
        while expect < D and ref[0, n + expect] - s.samp_lo in cand[expect, 0, :m_depth[expect]]:
            expect += 1
        assert na[0] == expect
    np.testing.assert_array_equal(hk.grid(), ref)
    print("accepted per tree step, histogram:", np.bincount(accs, minlength=D + 1))
    assert max(accs) == D


def test_tree_rejects_what_it_cannot_run(H):
    s = synth.CONFIGS[0]
    hk, orc, E = start(H, s, k_max=6)
    import torch
    def call(m_depth):
        D, m = len(m_depth), max(m_depth)
        q = torch.zeros((D, 1, m, s.v_s), device="cuda:0")
        return hk.verify_tree(m_depth, np.zeros((D, 1, m), np.int32), q, np.zeros((D, 1, m), np.float32),
                              np.zeros((D + 1, 1), np.float32))
    with pytest.raises(H.HawkError):
        call((3, 3))          # 13 nodes, the context has room for 7 rows
    with pytest.raises(H.HawkError):
        call((1,) * 9)        # deeper than 8
    na, toks = call((2, 2))   # 7 nodes: fits
    assert na[0] >= 0
    # near the end of the image the tree no longer fits
    rng = np.random.Generator(np.random.PCG64(3))
    while hk.n()[0] + 7 <= s.n_img:
        hk.draft(s.k, uni(rng, 1, s.k))
        hk.verify(s.k, uni(rng, 1, s.k), uni(rng, 1))
    if hk.n()[0] < s.n_img:
        with pytest.raises(H.HawkError):
            call((2, 2))
