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


# ----------------------------------------------------------------------------- the loop inside the library

def heads_for(s, HD, VSD, seed=3):
    import torch
    _, wh, wo = synth.make_spatial_heads(seed, 1, HD + VSD, s.d_model, s.v_s)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    return (dev(wh.view(np.int16)).view(torch.bfloat16), dev(wo.view(np.int16)).view(torch.bfloat16),
            synth.bf16_bits_to_f32(wh), synth.bf16_bits_to_f32(wo))


@pytest.mark.parametrize("HD,VSD,grid", [(2, 2, (8, 8)), (1, 1, (4, 6)), (3, 1, (6, 5)), (2, 0, (4, 6))])
def test_library_loop_fp32_images_equal_the_oracle_loop(H, HD, VSD, grid):
    # hawk_generate_spatial against oracle.scheme.generate_spatial on the fp32 configuration, sampled
    # (temperature 1, top-k of the configuration) with the same counter-based uniforms: identical images and
    # pass statistics.  (The heads' logits differ by ~2e-5 between the two sides - fp32 accumulation against
    # fp64 -, so a draw or an acceptance test within that distance of a boundary could differ; none does for
    # these seeds.)
    import oracle
    from oracle import scheme
    s = synth.CONFIGS[0].replace(grid_h=grid[0], grid_w=grid[1])
    max_nodes = sum((VSD + 1) ** j for j in range(HD + 1))
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    E = synth.blob_tensor(s, blob, "E")
    Wh_d, Wo_d, Wh, Wo = heads_for(s, HD, VSD)
    hk = H.Hawk(H.HawkConfig.from_shape(s, batch=1, k_max=max(max_nodes - 1, s.k)))
    hk.load(blob)
    orc = oracle.Oracle.from_shape(s, blob, batch=1, k_max=max(max_nodes - 1, s.k))
    for seed in (11, 12):
        g_o, st_o = scheme.generate_spatial(orc, E, cond, s.n_cond, s.grid_h, s.grid_w, s.samp_lo, Wh, Wo, HD, VSD,
                                            s.temperature, s.top_k, seed)
        g_g, st_g = hk.generate_spatial(cond, s.grid_h, s.grid_w, s.temperature, s.top_k, Wh_d, Wo_d, HD, VSD, seed)
        np.testing.assert_array_equal(g_g[0], g_o)
        assert {k: st_g[k] for k in st_o} == st_o and st_g["tokens"] == s.n_img
        assert st_g["passes"] > 0
    hk.close()
    orc.close()


@pytest.mark.parametrize("path", [0, 1])
def test_library_loop_greedy_image_bf16(H, path):
    # bf16 configuration 1 at reduced depth: at temperature 0 the library's loop commits the arg-max image,
    # whatever the heads propose (verification is lossless); path 1 runs the tree rows on the persistent kernel
    s = synth.CONFIGS[1].replace(n_layers=3, n_cond=24, grid_h=8, grid_w=8)
    HD, VSD = 2, 2
    max_nodes = sum((VSD + 1) ** j for j in range(HD + 1))
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    Wh_d, Wo_d, _, _ = heads_for(s, HD, VSD)
    hk = H.Hawk(H.HawkConfig.from_shape(s, batch=1, k_max=max_nodes - 1))
    hk.load(blob)
    hk.set_path(path)
    ref, _ = hk.generate(cond, None, s.grid_h, s.grid_w, 0, 0.0, s.top_k, 1.0, 1)
    g, st = hk.generate_spatial(cond, s.grid_h, s.grid_w, 0.0, s.top_k, Wh_d, Wo_d, HD, VSD, 5)
    np.testing.assert_array_equal(g, ref)
    assert st["passes"] > 0 and 1 + st["passes"] + st["accepted"] <= s.n_img
    hk.close()


def test_library_loop_rejects_what_it_cannot_run(H):
    s = synth.CONFIGS[0]
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    Wh_d, Wo_d, _, _ = heads_for(s, 2, 2)
    hk = H.Hawk(H.HawkConfig.from_shape(s, batch=1, k_max=s.k))        # room for 5 rows: the 13-row tree does not fit
    hk.load(blob)
    with pytest.raises(H.HawkError) as e:
        hk.generate_spatial(cond, s.grid_h, s.grid_w, 1.0, s.top_k, Wh_d, Wo_d, 2, 2, 1)
    assert e.value.code == -1
    hk.close()
    sg = s.replace(cfg_scale=2.0)
    hk2 = H.Hawk(H.HawkConfig.from_shape(sg, batch=1, k_max=12))       # a context with guidance
    hk2.load(blob)
    with pytest.raises(H.HawkError) as e:
        hk2.generate_spatial(cond, s.grid_h, s.grid_w, 1.0, s.top_k, Wh_d, Wo_d, 2, 2, 1)
    assert e.value.code == -1 and "guidance" in str(e.value)
    hk2.close()
    L = H.load_library()
    cfg = H.HawkConfig.from_shape(s, batch=1, k_max=12)
    import ctypes as C
    assert L.hawk_generate_spatial_workspace_bytes(C.byref(cfg), s.grid_w, 0, 2) == 0
    assert L.hawk_generate_spatial_workspace_bytes(C.byref(cfg), s.grid_w, 2, 8) == 0
    assert L.hawk_generate_spatial_workspace_bytes(C.byref(cfg), s.grid_w, 2, 2) > 0
