"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): a driver in C
(tests/sanitize_oracle_main.c) linked with oracle/hawk_oracle.c runs the generation loop, the calls
one by one up to the end of the image, re-synchronisation and the context-free routines on the micro
model with guidance and two prompts; it must end cleanly, and its generated image must be the one
the ordinary build of the oracle produces."""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("asan") / "oracle_asan")
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fopenmp", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "tests", "sanitize_oracle_main.c"), os.path.join(ROOT, "oracle", "hawk_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True, cwd=ROOT)
    return exe


@pytest.mark.parametrize("guided,dtype", [(False, "fp32"), (True, "bf16")])
def test_oracle_runs_clean_under_address_and_ub_sanitizers(driver, micro_shape, tmp_path, guided, dtype):
    s = micro_shape.replace(dtype=dtype, cfg_scale=2.0 if guided else 1.0, samp_lo=3 if guided else 0,
                            samp_n=32 if guided else 0)
    batch, k, top_k, seed = 2, 3, 10, 7
    blob = synth.make_weights(s, seed=0, std=0.3)
    cond = synth.make_cond(s, seed=2, batch=batch)
    unc = synth.make_cond(s, seed=3, batch=batch) if guided else None
    path = str(tmp_path / "in.bin")
    with open(path, "wb") as f:
        hdr = [s.samp_lo, s.samp_n, batch, int(guided), s.n_cond, s.grid_h, s.grid_w, 4, k, top_k, s.d_model, seed, s.v_s,
               0, 0, 0]
        f.write(struct.pack("<16i", *hdr))
        f.write(struct.pack("<4f", 1.0, s.cfg_scale, s.rms_eps, s.rope_theta))
        b = np.ascontiguousarray(blob, dtype=np.uint8)
        f.write(struct.pack("<q", b.nbytes))
        f.write(b.tobytes())
        f.write(np.ascontiguousarray(cond, dtype=np.float32).tobytes())
        if guided:
            f.write(np.ascontiguousarray(unc, dtype=np.float32).tobytes())
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, path], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "Sanitizer" not in r.stderr, r.stderr[-4000:]
    lines = r.stdout.strip().splitlines()
    assert lines[-1] == "OK"
    got = np.array(lines[0].split()[1:], dtype=np.int32).reshape(batch, s.n_img)
    o = oracle.Oracle(blob, batch=batch, use_cfg=guided, max_cond=s.n_cond, grid_h=s.grid_h, grid_w=s.grid_w, k_max=4,
                      samp_lo=s.samp_lo, samp_n=s.samp_n, rms_eps=s.rms_eps, rope_theta=s.rope_theta)
    ref, st = o.generate(cond, unc, k, 1.0, top_k, s.cfg_scale, seed)
    np.testing.assert_array_equal(got, ref)
    assert [int(x) for x in lines[1].split()[1:]] == [st["steps"], st["accepted"], st["tokens"], st["iters"]]
