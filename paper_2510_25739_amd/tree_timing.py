"""Times hawk_verify_tree (one target pass over a candidate tree, the walk, the commit) at a
configuration's shape with synthetic proposals, next to the ordinary verify step of the same
context, the figures quoted in the design notes:
python -m paper_2510_25739_amd.tree_timing [config]"""
import json
import sys
import time


def bench_tree(H, s, blob, cond, m_depth=(3, 3), steps=20, uncond=None):
    """Milliseconds per call (host clock around the synchronous call), synthetic proposals N(0, 1.5^2)
    and candidates drawn from them on the GPU; k_max is sized for the tree's rows."""
    import numpy as np
    import torch
    n_nodes, width = 1, 1
    for m in m_depth:
        width *= m
        n_nodes += width
    D, m_max = len(m_depth), max(m_depth)
    hk = H.Hawk(H.HawkConfig.from_shape(s if uncond is not None else s.replace(cfg_scale=1.0), batch=1,
                                        k_max=max(n_nodes - 1, s.k)))
    hk.load(blob)
    rng = np.random.Generator(np.random.PCG64(1))
    uni = lambda *shp: (rng.integers(0, 1 << 24, size=shp).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)
    hk.prefill(cond[:1], None if uncond is None else uncond[:1], s.grid_h, s.grid_w, s.temperature, s.top_k,
               s.cfg_scale if uncond is not None else 1.0, uni(1))
    g = torch.Generator(device="cuda:0")
    g.manual_seed(3)
    out = {"rows": n_nodes, "m_depth": list(m_depth)}
    t_tree, t_chain, acc = [], [], []
    for i in range(steps):
        q = torch.randn(D, 1, m_max, s.v_s, device="cuda:0", generator=g) * 1.5
        cand = H.sample_rows(q.view(D * m_max, s.v_s), torch.from_numpy(uni(D * m_max)).to("cuda:0"), s.temperature,
                             s.top_k).view(D, 1, m_max).cpu().numpy()
        ua, uf = uni(D, 1, m_max), uni(D + 1, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        na, _ = hk.verify_tree(m_depth, cand, q, ua, uf)
        t_tree.append((time.perf_counter() - t0) * 1e3)
        acc.append(int(na[0]))
        hk.draft(s.k, uni(1, s.k))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        hk.verify(s.k, uni(1, s.k), uni(1))
        t_chain.append((time.perf_counter() - t0) * 1e3)
    out["ms_tree_step"] = float(np.median(t_tree[2:]))
    out["ms_chain_verify"] = float(np.median(t_chain[2:]))
    out["chain_path"] = "persistent kernel" if hk.last_path() == 1 else "one kernel per operation"
    out["accepted_mean"] = float(np.mean(acc))
    hk.close()
    return out


def main():
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import synth
    import paper_2510_25739_amd as H
    s = synth.CONFIGS[int(sys.argv[1]) if len(sys.argv) > 1 else 2].replace(batch=1)
    blob = synth.make_weights(s, seed=0)
    cond = synth.make_cond(s, seed=2, batch=1)
    unc = synth.make_cond(s, seed=3, batch=1) if s.use_cfg else None
    shapes = ((3, 3), (2, 2), (3,)) if len(sys.argv) < 3 else (tuple(int(x) for x in sys.argv[2].split("x")),)
    print(json.dumps({"tree": [bench_tree(H, s, blob, cond, m, uncond=unc) for m in shapes]}))


if __name__ == "__main__":
    main()
