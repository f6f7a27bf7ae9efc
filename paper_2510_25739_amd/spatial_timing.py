"""Times one drafting step of the spatial structures (dual-direction heads, speculation cache push,
pool gather, candidate draws, multi-candidate verification) at a configuration's shape, the figures
quoted in the design notes and the profile summary:
python -m paper_2510_25739_amd.spatial_timing [config]"""
import json
import sys


def _time(fn, reps):
    import torch
    for _ in range(5):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def bench_spatial_draft(H, s, HD=2, VSD=2, reps=50):
    """Microseconds per call, HIP events on the launch stream, synthetic inputs (hidden states
    N(0,1), head matrices N(0, 0.02^2), output rows N(0, 0.04^2)): the heads on the k+1 rows of one
    verify pass of every sequence, the push of those rows' vertical predictions, the pools of the HD
    positions ahead, one candidate per pool member and their verification."""
    import torch
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(11)
    d, v_s, IW, IH = s.d_model, s.v_s, s.grid_w, s.grid_h
    rows, n_heads, m_max = (s.k + 1) * s.n_seq, HD + VSD, VSD + 1
    h = torch.randn(rows, d, device=dev, generator=g)
    Wh = (torch.randn(n_heads, d, d, device=dev, generator=g) * 0.02).to(torch.bfloat16)
    Wo = (torch.randn(v_s, d, device=dev, generator=g) * 0.04).to(torch.bfloat16)
    cache = H.SpecCache(IW, IH, VSD, v_s)
    T = (IH // 2) * IW + IW // 2
    # the rows above the walk's position filled once, so that the pools below are complete
    warm = torch.randn(IW, n_heads, v_s, device=dev, generator=g) * 1.5
    for r in range(VSD, 0, -1):
        cache.push(torch.arange(T - r * IW, T - r * IW + IW, dtype=torch.int32, device=dev), warm.view(-1)[HD * v_s:],
                   n_heads * v_s)
    pos = torch.arange(T, T + s.k + 1, dtype=torch.int32, device=dev)
    target = torch.arange(T + s.k + 1, T + s.k + 1 + HD, dtype=torch.int32, device=dev)
    u = torch.rand(HD * m_max, device=dev, generator=g)
    u_acc = torch.rand(HD, m_max, device=dev, generator=g)
    u_fin = torch.rand(HD, device=dev, generator=g)
    ws = torch.empty(H.multi_verify_workspace_bytes(HD, m_max), dtype=torch.uint8, device=dev)
    q = H.spatial_heads(h, Wh, Wo)
    logits, m, delta = cache.pool(target, q.view(-1)[s.k * n_heads * v_s:], v_s)
    cand = H.sample_rows(logits.view(HD * m_max, v_s), u, s.temperature, s.top_k, skip=delta.view(-1)).view(HD, m_max)
    p = (logits[:, 0] + torch.randn(HD, v_s, device=dev, generator=g)).contiguous()

    def step():
        qq = H.spatial_heads(h, Wh, Wo)
        cache.push(pos, qq.view(-1)[HD * v_s:], n_heads * v_s)
        lg, mm, dl = cache.pool(target, qq.view(-1)[s.k * n_heads * v_s:], v_s)
        cd = H.sample_rows(lg.view(HD * m_max, v_s), u, s.temperature, s.top_k, skip=dl.view(-1)).view(HD, m_max)
        return H.multi_verify(p, lg, cd, u_acc, u_fin, s.temperature, s.top_k, m_rows=mm, workspace=ws)

    t = {
        "heads": _time(lambda: H.spatial_heads(h, Wh, Wo), reps),
        "cache_push": _time(lambda: cache.push(pos, q.view(-1)[HD * v_s:], n_heads * v_s), reps),
        "pool": _time(lambda: cache.pool(target, q.view(-1)[s.k * n_heads * v_s:], v_s), reps),
        "sample_rows": _time(lambda: H.sample_rows(logits.view(HD * m_max, v_s), u, s.temperature, s.top_k,
                                                   skip=delta.view(-1)), reps),
        "multi_verify": _time(lambda: H.multi_verify(p, logits, cand, u_acc, u_fin, s.temperature, s.top_k, m_rows=m,
                                                     workspace=ws), reps),
        "whole_step": _time(step, reps),
    }
    weight_bytes = (n_heads * d * d + v_s * d) * 2
    io_bytes = rows * d * 4 + rows * n_heads * v_s * 4
    return {"us": t, "heads_bytes": weight_bytes + io_bytes, "heads_GB/s": (weight_bytes + io_bytes) / (t["heads"] * 1e-6) / 1e9,
            "cache_bytes": H.spec_cache_bytes(IW, VSD, v_s), "pool_members": [int(x) for x in m.cpu()],
            "config": f"{s.name}: HD={HD} horizontal + VSD={VSD} vertical heads on {rows} rows, d={d}, slice {v_s}, "
                      f"image {IH}x{IW}, top-k {s.top_k}"}


def main():
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import synth
    import paper_2510_25739_amd as H
    s = synth.CONFIGS[int(sys.argv[1]) if len(sys.argv) > 1 else 2]
    print(json.dumps({"spatial_draft": bench_spatial_draft(H, s)}))


if __name__ == "__main__":
    main()
