"""Times hawk_multi_verify on synthetic logit rows (the figures quoted in the design notes and the
profile summary): python -m paper_2510_25739_amd.multi_verify_timing [config]"""
import json
import sys


def bench_multi_verify(H, s, rows_list=(6, 192), m=2, reps=50):
    """hawk_multi_verify (two candidates per position, one per head, each from its own proposal) on
    synthetic logit rows of the configuration's vocabulary slice: microseconds per launch, HIP events
    on the launch stream.  Rows: one sequence's k+1 positions, and the batched configuration's 192."""
    import torch
    out = {}
    g = torch.Generator(device="cuda:0")
    g.manual_seed(5)
    n = s.v_s
    for rows in rows_list:
        p = torch.randn(rows, n, device="cuda:0", generator=g) * 1.5
        q = (p[:, None, :] + torch.randn(rows, m, n, device="cuda:0", generator=g)).contiguous()
        cand = q.argmax(2).to(torch.int32).contiguous()
        u_acc = torch.rand(rows, m, device="cuda:0", generator=g)
        u_fin = torch.rand(rows, device="cuda:0", generator=g)
        ws = torch.empty(H.multi_verify_workspace_bytes(rows, m), dtype=torch.uint8, device="cuda:0")
        timed = {}
        for name, w in (("one_launch", None), ("two_launches", ws)):
            for _ in range(5):
                H.multi_verify(p, q, cand, u_acc, u_fin, s.temperature, s.top_k, workspace=w)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                idx, tok = H.multi_verify(p, q, cand, u_acc, u_fin, s.temperature, s.top_k, workspace=w)
            e1.record()
            torch.cuda.synchronize()
            timed[name] = e0.elapsed_time(e1) * 1e3 / reps
        us = timed["two_launches"]
        out[f"rows_{rows}"] = {"us_per_launch": us, "us_one_launch": timed["one_launch"], "logit_bytes": rows * (m + 1) * n * 4,
                               "GB/s": rows * (m + 1) * n * 4 / (us * 1e-6) / 1e9,
                               "rejected_all_frac": float((idx == m).float().mean())}
    out["config"] = f"m={m} candidates per position, slice {n}, top-k {s.top_k}, T={s.temperature}"
    return out



def main():
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import synth
    import paper_2510_25739_amd as H
    s = synth.CONFIGS[int(sys.argv[1]) if len(sys.argv) > 1 else 2]
    out = {"m2": bench_multi_verify(H, s, rows_list=(1, 6, 32, 192), m=2),
           "m4": bench_multi_verify(H, s, rows_list=(6, 192), m=4)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
