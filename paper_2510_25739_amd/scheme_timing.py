"""Decodes one image with the whole drafting and verification scheme chained on the GPU - dual-
direction heads, speculation cache, sampling pool, one candidate per pool member, tree step -
driven from Python through the binding (one synchronisation per step: the tree step's read-back),
and reports passes, tokens per pass and image tokens per second, the figures quoted in the design
notes: python -m paper_2510_25739_amd.scheme_timing [config]"""
import json
import sys
import time


def decode_image(H, hk, s, cond, Wh, Wo, HD, VSD, temperature, seed, reference=None):
    """One image.  reference (a token grid [1, N]): the horizontal proposals are replaced by point
    masses on its tokens, i.e. a draft head that is always right (the walk then goes to full depth)."""
    import numpy as np
    import torch
    dev = "cuda:0"
    n_heads, m_max, IW, IH, v_s, C = HD + VSD, VSD + 1, s.grid_w, s.grid_h, s.v_s, s.n_cond
    max_nodes = sum(m_max ** j for j in range(HD + 1))
    rng = np.random.Generator(np.random.PCG64(seed))
    uni = lambda *shp: (rng.integers(0, 1 << 24, size=shp).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)
    hk.prefill(cond, None, IH, IW, temperature, s.top_k, 1.0, uni(1))
    cache = H.SpecCache(IW, IH, VSD, v_s)
    h_rows, positions, n = hk.last_hidden(C)[C - 1:C].clone(), [0], 1
    passes, accepted = 0, 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while n + max_nodes <= s.n_img:
        q_all = H.spatial_heads(h_rows, Wh, Wo)
        cache.push(torch.tensor(positions, dtype=torch.int32, device=dev), q_all.view(-1)[HD * v_s:], n_heads * v_s)
        targets = torch.arange(n, n + HD, dtype=torch.int32, device=dev)
        q_h = q_all[-1, :HD].contiguous()
        if reference is not None:
            q_h.zero_()
            q_h[torch.arange(HD), torch.from_numpy(reference[0, n:n + HD].astype(np.int64) - s.samp_lo)] = 50.0
        logits, m, delta = cache.pool(targets, q_h.view(-1), v_s)
        cand = H.sample_rows(logits.view(HD * m_max, v_s), torch.from_numpy(uni(HD * m_max)).to(dev), temperature, s.top_k,
                             skip=delta.view(-1))
        m_host = [min(VSD, (n - 1 + j) // IW) + 1 for j in range(1, HD + 1)]     # members exist once their source row does
        mm = max(m_host)
        cand_h = np.maximum(cand.view(HD, 1, m_max).cpu().numpy(), 0)[:, :, :mm]
        na, _ = hk.verify_tree(tuple(m_host), cand_h, logits[:, :mm].contiguous().view(HD, 1, mm, v_s), uni(HD, 1, mm),
                               uni(HD + 1, 1))
        a = int(na[0])
        nodes = sum(int(np.prod(m_host[:j])) for j in range(HD + 1))
        path = [int(x) for x in hk.tree_path()[0, :a]]
        h_rows = hk.last_hidden(nodes)[[0] + path].clone()
        positions = [n + i for i in range(a + 1)]
        n += a + 1
        passes += 1
        accepted += a
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tokens = n - 1
    while n < s.n_img:   # the last positions, where the tree no longer fits: ordinary steps (not timed)
        hk.draft(1, uni(1, 1))
        na, _ = hk.verify(1, uni(1, 1), uni(1))
        n += int(na[0]) + 1
    return {"passes": passes, "tokens": tokens, "tokens_per_pass": tokens / max(passes, 1), "ms_per_pass": dt * 1e3 / max(passes, 1),
            "tokens_per_s": tokens / dt}


def bench_scheme(H, s, blob, cond, HD=2, VSD=2):
    import numpy as np
    import torch
    m_max = VSD + 1
    max_nodes = sum(m_max ** j for j in range(HD + 1))
    s1 = s.replace(cfg_scale=1.0, batch=1)
    hk = H.Hawk(H.HawkConfig.from_shape(s1, batch=1, k_max=max(max_nodes - 1, s.k)))
    hk.load(blob)
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7)
    Wh = (torch.randn(HD + VSD, s.d_model, s.d_model, device="cuda:0", generator=g) * 0.02).to(torch.bfloat16)
    Wo = (torch.randn(s.v_s, s.d_model, device="cuda:0", generator=g) * 0.04).to(torch.bfloat16)
    ref, _ = hk.generate(cond[:1], None, s.grid_h, s.grid_w, 0, 0.0, s.top_k, 1.0, 1)
    # the same loop inside the library (hawk_generate_spatial): one call per image, prefill included
    hk.generate_spatial(cond[:1], s.grid_h, s.grid_w, s.temperature, s.top_k, Wh, Wo, HD, VSD, 1)   # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _, st = hk.generate_spatial(cond[:1], s.grid_h, s.grid_w, s.temperature, s.top_k, Wh, Wo, HD, VSD, 2)
    dt = time.perf_counter() - t0
    library = {"passes": st["passes"], "accepted": st["accepted"], "tail_steps": st["tail_steps"], "tokens": st["tokens"],
               "ms_per_image_with_prefill": dt * 1e3, "tokens_per_s_with_prefill": st["tokens"] / dt}
    t0 = time.perf_counter()
    hk.prefill(cond[:1], None, s.grid_h, s.grid_w, s.temperature, s.top_k, 1.0, [0.5])
    hk.synchronize()
    t_prefill = time.perf_counter() - t0
    library["ms_per_pass"] = (dt - t_prefill) * 1e3 / max(st["passes"] + st["tail_steps"], 1)
    library["tokens_per_s"] = (st["tokens"] - 1) / (dt - t_prefill)
    out = {"config": f"{s.name}: HD={HD}, VSD={VSD}, trees up to {max_nodes} rows, one prompt, no guidance, driven from Python",
           "library_loop_random_heads": library,
           "random_heads": decode_image(H, hk, s1, cond[:1], Wh, Wo, HD, VSD, s.temperature, 1),
           "perfect_horizontal_greedy": decode_image(H, hk, s1, cond[:1], Wh, Wo, HD, VSD, 0.0, 2, reference=ref)}
    same = bool(np.array_equal(hk.grid(), ref))
    out["perfect_horizontal_greedy"]["image_equals_argmax_decoding"] = same
    hk.close()
    return out


def main():
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import synth
    import paper_2510_25739_amd as H
    s = synth.CONFIGS[int(sys.argv[1]) if len(sys.argv) > 1 else 2]
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    print(json.dumps({"whole_scheme": bench_scheme(H, s, blob, cond)}))


if __name__ == "__main__":
    main()
