"""The whole drafting and verification scheme chained on the GPU (Method, overview figure: dual-
direction heads -> speculation cache -> spatial sampling pool -> candidate tree -> verification),
image by image, with every intermediate staying in device memory.

What is checked: at temperature 0 the image must be the token-by-token arg-max image whatever the
heads propose (random head weights; in a second run the horizontal proposal is replaced by the
reference's token, which makes the walk go to full depth every step); and at every step the rows
the cache hands out are, bit for bit, the rows that were pushed for those positions and depths
(a dictionary kept by the test: a check of where rows go - what the rows hold is checked against the
oracle in the tests of the heads), with the member counts and order the definition of the pool gives.
"""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    import paper_2510_25739_amd as H
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return H


@pytest.mark.parametrize("perfect_horizontal", [False, True])
def test_whole_scheme_greedy_image(H, perfect_horizontal):
    import torch
    s = synth.CONFIGS[1]                     # B-shaped bf16: 12 layers, d = 768, 16 x 16 image, 16384-entry vocabulary
    HD, VSD = 2, 2
    n_heads, m_max, IW, IH, v_s, C = HD + VSD, VSD + 1, s.grid_w, s.grid_h, s.v_s, s.n_cond
    max_nodes = 1 + m_max + m_max * m_max
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    hk = H.Hawk(H.HawkConfig.from_shape(s, batch=1, k_max=max_nodes - 1))
    hk.load(blob)
    ref, _ = hk.generate(cond, None, IH, IW, 0, 0.0, s.top_k, 1.0, 1)
    _, wh, wo = synth.make_spatial_heads(3, 1, n_heads, s.d_model, v_s)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    Wh, Wo = dev(wh.view(np.int16)).view(torch.bfloat16), dev(wo.view(np.int16)).view(torch.bfloat16)
    rng = np.random.Generator(np.random.PCG64(2))
    uni = lambda *shp: (rng.integers(0, 1 << 24, size=shp).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)

    hk.prefill(cond, None, IH, IW, 0.0, s.top_k, 1.0, uni(1))
    cache = H.SpecCache(IW, IH, VSD, v_s)
    pushed = {}   # (position pointed to, depth) -> the row pushed for it
    # the hidden state that predicted position 0: the last condition row of the prefill
    h_rows, positions, n = hk.last_hidden(C)[C - 1:C].clone(), [0], 1
    accepted, steps = [], 0
    while n + max_nodes <= s.n_img:
        q_all = H.spatial_heads(h_rows.contiguous(), Wh, Wo)                      # [rows, heads, V_s]: heads 0..HD-1 horizontal
        cache.push(dev(np.array(positions, np.int32)), q_all.view(-1)[HD * v_s:], n_heads * v_s)
        for i, T in enumerate(positions):
            for d in range(1, VSD + 1):
                pushed[(T + d * IW, d)] = q_all[i, HD + d - 1].cpu().numpy()
        targets = [n - 1 + j for j in range(1, HD + 1)]                           # the positions the last row's horizontal heads point to
        q_h = q_all[-1, :HD].contiguous()
        if perfect_horizontal:
            q_h = torch.zeros_like(q_h)
            for j, t in enumerate(targets):
                q_h[j, int(ref[0, t]) - s.samp_lo] = 50.0
        logits, m, delta = cache.pool(dev(np.array(targets, np.int32)), q_h.view(-1), v_s)
        m_host = [int(x) for x in m.cpu()]
        for j, t in enumerate(targets):                                          # bit for bit the rows pushed for t, nearest row first
            want = [(dv, pushed[(t, dv)]) for dv in range(1, VSD + 1) if (t, dv) in pushed] + [(0, q_h[j].cpu().numpy())]
            assert m_host[j] == len(want) == min(VSD, t // IW) + 1
            assert delta[j].cpu().tolist() == [dv for dv, _ in want] + [-1] * (m_max - len(want))
            for i, (_, row) in enumerate(want):
                assert np.array_equal(logits[j, i].cpu().numpy(), row)
        cand = H.sample_rows(logits.view(HD * m_max, v_s), dev(uni(HD * m_max)), 0.0, s.top_k, skip=delta.view(-1))
        cand = np.maximum(cand.view(HD, 1, m_max).cpu().numpy(), 0)
        na, toks = hk.verify_tree(tuple(m_host), cand[:, :, :max(m_host)],
                                  logits[:, :max(m_host)].contiguous().view(HD, 1, max(m_host), v_s),
                                  uni(HD, 1, max(m_host)), uni(HD + 1, 1))
        a = int(na[0])
        nodes = 1 + m_host[0] + m_host[0] * m_host[1]
        path = [int(x) for x in hk.tree_path()[0, :a]]
        # the rows that were committed: the root and the accepted candidates; their hidden states feed the heads next
        h_rows = hk.last_hidden(nodes)[[0] + path].clone()
        positions = [n + i for i in range(a + 1)]
        np.testing.assert_array_equal(toks[0, :a + 1], ref[0, n:n + a + 1])
        n += a + 1
        accepted.append(a)
        steps += 1
    while n < s.n_img:                                                            # the last positions: ordinary steps
        hk.draft(1, uni(1, 1))
        na, _ = hk.verify(1, uni(1, 1), uni(1))
        n += int(na[0]) + 1
    np.testing.assert_array_equal(hk.grid(), ref)
    print(f"{steps} tree steps, accepted per step: histogram {np.bincount(accepted, minlength=HD + 1)}")
    if perfect_horizontal:
        assert min(accepted) == HD          # every step walks to full depth: 3 tokens per pass
