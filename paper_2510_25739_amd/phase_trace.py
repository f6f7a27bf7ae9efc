"""Stage table of the persistent target-pass kernels from their own time stamps (hawk_phase_trace).

    python -m paper_2510_25739_amd.phase_trace [--config 2|4] [--path 1|2] [--kv 400] [--launches 3]

Configuration 2 (XL shape, one prompt, k = 5) or 4 (7B shape with guidance; every layer repeats layer 0's
weights): the image is teacher-forced until the cache holds
about --kv positions, then --launches traced steps run; the table averages the last launch's layers
(the first three are skipped).  --path 1: the kernel laid out on the XCDs; --path 2: the grid-barrier
kernel.  Times are in microseconds (the stamps tick at 100 MHz, so single figures are +-0.01 us and the
means over 33 layers finer).  Tracing itself costs a few per cent of the launch.
"""
import argparse
import ctypes as C
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import synth  # noqa: E402
import paper_2510_25739_amd as H  # noqa: E402

NAMES = ["A qkv", "B attention", "C wo", "D w1|w3", "E w2"]


def xcd_table(hk, L):
    out = np.zeros(2 * 512 * 16, dtype=np.uint64)
    hk._chk(hk._L.hawk_phase_trace(hk._h, 0, out.ctypes.data_as(C.c_void_p), out.size), "hawk_phase_trace")
    tr = out.reshape(2, 512, 16).astype(np.int64)
    # slots: compute waves 0 stage entry, 1 input in LDS (barrier crossed), 3 products done, 2 stores of the
    # partial sums issued, 4 stores acknowledged; IO waves 8 stage entry, 9 flags seen, 10 input staged
    # (attention: 9 queries seen, 11 .. 14 see the print below, 10 output rows stored and flag raised), 12 partial sums of the wave's strip all there, 11 epilogue
    # done and flag raised
    for wg, name in ((0, "workgroup 0 (XCD 0, unit 0)"), (1, "workgroup 248 (XCD 0, unit 31)")):
        t = tr[wg]
        print(f"{name}: {(t[5 * L, 11] - t[0, 8]) / 100.0:.1f} us from the first stage's entry to the last stamp")
        total = 0.0
        for k in range(5):
            rows = t[k:5 * L:5][3:]
            nxt = t[k + 1:5 * L + 1:5][3:]
            d = lambda a, b: float(np.mean(rows[:, b] - rows[:, a])) / 100.0  # noqa: E731
            both = (nxt[:len(rows), 9] > 0) & (rows[:len(nxt), 9] > 0)   # a unit without a job in a stage leaves no stamp
            length = float(np.mean((nxt[:len(rows), 9] - rows[:len(nxt), 9])[both])) / 100.0 if both.any() else float("nan")
            total += length
            if k == 1:
                job = rows[:, 10] > rows[:, 9]
                pub = float(np.mean((rows[:, 10] - rows[:, 9])[job])) / 100.0 if job.any() else float("nan")
                dj = lambda a, b: float(np.mean((rows[:, b] - rows[:, a])[job])) / 100.0 if job.any() else float("nan")  # noqa: E731
                print(f"  {NAMES[k]:12s} stage {length:5.2f} | queries seen -> rows stored, flag raised {pub:5.2f}: queries in LDS "
                      f"{dj(9, 11):5.2f} cached positions {dj(11, 12):5.2f} rows of this pass {dj(12, 13):5.2f} "
                      f"waves' parts in LDS {dj(13, 14):5.2f} merged and stored {dj(14, 10):5.2f}")
                continue
            job = rows[:, 12] > rows[:, 10]
            g = float(np.mean((rows[:, 12] - rows[:, 10])[job])) / 100.0 if job.any() else float("nan")
            e = float(np.mean((rows[:, 11] - rows[:, 12])[job])) / 100.0 if job.any() else float("nan")
            print(f"  {NAMES[k]:12s} stage {length:5.2f} | IO: flags {d(8, 9):5.2f} staging {d(9, 10):5.2f} "
                  f"partials there after {g:5.2f} epilogue+flag {e:5.2f} | compute: at barrier {d(0, 1):5.2f} "
                  f"products {d(1, 3):5.2f} stores issued {d(3, 2):5.2f} acknowledged {d(2, 4):5.2f}")
        print(f"  layer {total:6.2f} us")


def barrier_table(hk, L):
    nst = 5 * L + 3
    tr = hk.phase_trace(False, nst).astype(np.int64)
    arr = hk.last_arrivals.astype(np.int64)
    for wg in (0, 1):
        t = tr[wg]
        last = np.nonzero(t[:, 6])[0].max()
        print(f"workgroup {wg * 128}, first IO wave: {(t[last, 6] - t[0, 0]) / 100.0:.1f} us over {last + 1} stages")
        for k in range(5):
            rows = t[1 + k:1 + 5 * L:5][3:]
            d = lambda a, b: float(np.mean(rows[:, b] - rows[:, a])) / 100.0  # noqa: E731
            print(f"  {NAMES[k]:12s} barrier wait {d(0, 1):5.2f} staging {d(1, 2):5.2f} sync {d(2, 3):5.2f} products {d(3, 4):5.2f} "
                  f"epilogue {d(4, 5):5.2f} arrival {d(5, 6):5.2f} | total {d(0, 6):5.2f}")
    total = 0.0
    print("stage = median over workgroups of 'release seen', next stage's minus this stage's; spread = last arrival - median arrival")
    for k in range(5):
        phs = [1 + 5 * l + k for l in range(4, min(L, 50) - 1) if 1 + 5 * l + k + 1 < 256]
        length = np.mean([(np.median(arr[1, ph + 1]) - np.median(arr[1, ph])) / 100.0 for ph in phs])
        spread = np.mean([(arr[0, ph].max() - np.median(arr[0, ph])) / 100.0 for ph in phs])
        lat = np.mean([(np.median(arr[1, ph + 1]) - arr[0, ph].max()) / 100.0 for ph in phs])
        total += length
        print(f"  {NAMES[k]:12s} stage {length:5.2f} | spread {spread:5.2f} | last arrival -> release seen {lat:5.2f}")
    print(f"  layer {total:6.2f} us")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2, choices=(2, 4))
    ap.add_argument("--path", type=int, default=1, choices=(1, 2))
    ap.add_argument("--kv", type=int, default=400)
    ap.add_argument("--launches", type=int, default=3)
    a = ap.parse_args()
    s = synth.CONFIGS[a.config]
    hk = H.Hawk(H.HawkConfig.from_shape(s))
    hk.load(synth.make_weights(s, seed=0, repeat_layer0=(a.config == 4)))
    hk.set_path(a.path)
    unc = synth.make_cond(s, seed=3) if s.use_cfg else None
    hk.prefill(synth.make_cond(s, seed=2), unc, s.grid_h, s.grid_w, 1.0, s.top_k, s.cfg_scale, [0.5])
    filler = np.random.default_rng(7).integers(0, s.v_s, size=(1, s.n_img)).astype(np.int32)
    n = 1
    while n + s.n_cond < a.kv and n + s.k + 1 < s.n_img:
        hk.force([n], filler[:, n:n + s.k + 1])
        n += s.k + 1
    hk.phase_trace(True)
    ms = hk.run_steps(s.k, a.launches, 1, False, timed=True)
    kern = hk.last_kernel()
    print(f"configuration {a.config}, cache length ~{n + s.n_cond}, {a.launches} traced steps: (draft, verify, kernel) ms = {ms}; kernel {kern} "
          f"({'laid out on the XCDs' if kern == 2 else 'grid barriers'})")
    (xcd_table if kern == 2 else barrier_table)(hk, s.n_layers)
    hk.close()


if __name__ == "__main__":
    main()
