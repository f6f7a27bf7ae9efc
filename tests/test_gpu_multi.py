"""GPU parity of hawk_multi_verify (several candidates per position, each from its own proposal;
Method, "Sampling and Verification"; appendix "Theoretical Justification") against the oracle:
accepted index and emitted token bit-exact, residual masses to fp64 rounding.

Inputs are seeded and synthetic: target logits N(0, 1.5^2) per entry, each proposal = target +
N(0, sigma^2) noise (a draft head that is right most of the time), candidates drawn from their
own warped proposal with the oracle's inverse CDF, uniforms on the 2^-24 grid.
"""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    import paper_2510_25739_amd as H
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return H


def make_rows(seed, rows, m, n, temperature, top_k, sigma=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    uni = lambda *shp: (rng.integers(0, 1 << 24, size=shp).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)
    p = (rng.standard_normal((rows, n)) * 1.5).astype(np.float32)
    q = (p[:, None, :] + sigma * rng.standard_normal((rows, m, n))).astype(np.float32)
    cand = np.zeros((rows, m), dtype=np.int32)
    u_draw = uni(rows, m)
    for r in range(rows):
        for i in range(m):
            w, z = oracle.warp(q[r, i], temperature, top_k)
            cand[r, i] = oracle.inv_cdf(w, z, float(u_draw[r, i]))
    return p, q, cand, uni(rows, m), uni(rows)


def run_both(H, p, q, cand, u_acc, u_fin, temperature, top_k):
    import torch
    dev = "cuda:0"
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    args = (t(p), t(q), t(cand), t(u_acc), t(u_fin), temperature, top_k)
    idx, tok, resid = H.multi_verify(*args, want_resid=True)
    # the two-launch form (rows' selections in parallel, statistics in a caller-provided workspace)
    # must give the same result, to the bit
    rows, m = cand.shape
    ws = torch.empty(H.multi_verify_workspace_bytes(rows, m), dtype=torch.uint8, device=dev)
    idx2, tok2, resid2 = H.multi_verify(*args, want_resid=True, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(tok, tok2) and torch.equal(resid, resid2)
    idx, tok, resid = idx.cpu().numpy(), tok.cpu().numpy(), resid.cpu().numpy()
    o_idx, o_tok, o_res = np.zeros(rows, np.int32), np.zeros(rows, np.int32), np.zeros((rows, m))
    for r in range(rows):
        o_idx[r], o_tok[r], o_res[r] = oracle.multi_verify(p[r], q[r], cand[r], u_acc[r], float(u_fin[r]), temperature,
                                                           top_k, want_resid=True)
    return (idx, tok, resid), (o_idx, o_tok, o_res)


CASES = [
    # rows, m, n, temperature, top_k, sigma
    (64, 2, 16384, 1.0, 1000, 1.0),     # the paper's case: one vertical and one horizontal candidate, top-k 1000
    (48, 4, 16384, 1.0, 1000, 1.5),     # longer chains of rejections
    (48, 3, 4096, 0.8, 4096, 1.0),      # whole vocabulary kept, four entries per thread
    (48, 2, 1000, 1.0, 50, 1.0),        # ragged row
    (32, 3, 5000, 1.3, 1000, 2.0),      # ragged row, sixteen entries per thread
    (32, 2, 8192, 1.0, 2000, 1.0),      # the 7B configuration's slice and top-k
    (32, 1, 300, 1.0, 300, 1.0),        # a single candidate
    (16, 2, 16384, 1.0, 3000, 1.0),     # top-k beyond the list capacity: dense form, sixteen entries per thread
    (32, 3, 16384, 0.0, 1000, 0.3),     # greedy by temperature
    (32, 2, 16384, 1.0, 1, 0.3),        # greedy by top-k
]


@pytest.mark.parametrize("rows,m,n,temperature,top_k,sigma", CASES)
def test_multi_verify_matches_oracle(H, rows, m, n, temperature, top_k, sigma):
    oracle.margins(reset=True)
    p, q, cand, u_acc, u_fin = make_rows(1000 + n + m, rows, m, n, temperature, top_k, sigma)
    (idx, tok, resid), (o_idx, o_tok, o_res) = run_both(H, p, q, cand, u_acc, u_fin, temperature, top_k)
    print("accepted index histogram", np.bincount(o_idx, minlength=m + 1), "margins", oracle.margins())
    np.testing.assert_array_equal(idx, o_idx)
    np.testing.assert_array_equal(tok, o_tok)
    np.testing.assert_allclose(resid, o_res, rtol=1e-11, atol=1e-13)
    if temperature > 0 and top_k > 1 and m > 1:
        assert (o_idx > 0).any(), "the case should exercise the recursion"


def test_multi_verify_edge_candidates(H):
    # candidates outside the proposal's kept set (q(s) = 0: accepted iff p^(i)(s) > 0), candidates the
    # target gives no mass (always rejected), uniforms 0 and 1 - 2^-24, identical proposals
    rows, m, n, top_k = 16, 3, 4096, 64
    p, q, cand, u_acc, u_fin = make_rows(77, rows, m, n, 1.0, top_k)
    order_p = np.argsort(-p, axis=1)
    for r in range(rows):
        cand[r, 0] = order_p[r, n - 1 - r]          # far outside both kept sets
        if r % 2:
            cand[r, 1] = order_p[r, r]               # inside the target's kept set
        q[r, 2] = q[r, 1]                            # the same proposal twice
    u_acc[::4, :] = 0.0
    u_acc[1::4, :] = np.float32(1.0) - np.float32(2.0 ** -24)
    u_fin[0], u_fin[1] = 0.0, np.float32(1.0) - np.float32(2.0 ** -24)
    (idx, tok, resid), (o_idx, o_tok, o_res) = run_both(H, p, q, cand, u_acc, u_fin, 1.0, top_k)
    np.testing.assert_array_equal(idx, o_idx)
    np.testing.assert_array_equal(tok, o_tok)
    np.testing.assert_allclose(resid, o_res, rtol=1e-11, atol=1e-13)


def test_short_pools_all_rejected_leave_no_unwritten_residual(H):
    # positions with fewer candidates than m (a sampling pool near the top of the image) whose
    # candidates are all rejected: every residual entry beyond the row's own count must read -1,
    # whatever the output buffer held before; all three kernel forms
    import torch
    dev = "cuda:0"
    for n, top_k in ((16384, 1000), (16384, 3000)):
        rows, m = 12, 3
        p, q, cand, u_acc, u_fin = make_rows(31 + top_k, rows, m, n, 1.0, top_k)
        cand[:] = np.argmin(p, axis=1).astype(np.int32)[:, None]      # no target mass: always rejected
        m_rows = np.array([r % (m + 1) for r in range(rows)], dtype=np.int32)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        args = (t(p), t(q), t(cand), t(u_acc), t(u_fin), 1.0, top_k)
        for ws in (None, torch.empty(H.multi_verify_workspace_bytes(rows, m), dtype=torch.uint8, device=dev)):
            junk = torch.full((rows, m), 7.0, dtype=torch.float64, device=dev)   # what torch.empty hands out next
            del junk
            idx, tok, resid = H.multi_verify(*args, want_resid=True, workspace=ws, m_rows=t(m_rows))
            idx, tok, resid = idx.cpu().numpy(), tok.cpu().numpy(), resid.cpu().numpy()
            for r in range(rows):
                mr = int(m_rows[r])
                if mr == 0:
                    w, z = oracle.warp(p[r], 1.0, top_k)
                    assert idx[r] == 0 and tok[r] == oracle.inv_cdf(w, z, float(u_fin[r]))
                    assert (resid[r] == -1.0).all()
                    continue
                oi, ot, ores = oracle.multi_verify(p[r], q[r, :mr], cand[r, :mr], u_acc[r, :mr], float(u_fin[r]), 1.0,
                                                   top_k, want_resid=True)
                assert oi == mr and idx[r] == mr and tok[r] == ot
                np.testing.assert_allclose(resid[r, :mr], ores, rtol=1e-11, atol=1e-13)
                assert (resid[r, mr:] == -1.0).all(), (r, mr, resid[r])


def test_candidates_outside_the_slice_are_rejected(H):
    # a device-side candidate that is no token of the slice must not be read through: it is rejected,
    # with the residual of an ordinary rejection (the residual does not depend on the candidate)
    import torch
    dev = "cuda:0"
    for n, top_k in ((4096, 64), (16384, 3000)):
        rows, m = 8, 2
        p, q, cand, u_acc, u_fin = make_rows(91 + n, rows, m, n, 1.0, top_k)
        ref_cand = cand.copy()
        ref_cand[:, 0] = np.argmin(p, axis=1)          # what the oracle sees instead: a token without target mass
        bad = cand.copy()
        bad[0::2, 0] = n + 5
        bad[1::2, 0] = -3
        u_acc[:, 0] = 0.0                               # anything with mass would be accepted
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        for ws in (None, torch.empty(H.multi_verify_workspace_bytes(rows, m), dtype=torch.uint8, device=dev)):
            idx, tok, resid = H.multi_verify(t(p), t(q), t(bad), t(u_acc), t(u_fin), 1.0, top_k, want_resid=True, workspace=ws)
            idx, tok, resid = idx.cpu().numpy(), tok.cpu().numpy(), resid.cpu().numpy()
            for r in range(rows):
                oi, ot, ores = oracle.multi_verify(p[r], q[r], ref_cand[r], u_acc[r], float(u_fin[r]), 1.0, top_k,
                                                   want_resid=True)
                assert oi >= 1 and idx[r] == oi and tok[r] == ot
                np.testing.assert_allclose(resid[r], ores, rtol=1e-11, atol=1e-13)


def test_multi_verify_rejects_bad_arguments(H):
    import torch
    L = H.load_library()
    z = torch.zeros(8, device="cuda:0")
    ptr = z.data_ptr()
    assert L.hawk_multi_verify(None, ptr, ptr, ptr, ptr, None, 1, 1, 8, 1.0, 8, ptr, ptr, None, None, 0, None) == -1
    assert L.hawk_multi_verify(ptr, ptr, ptr, ptr, ptr, None, 1, 0, 8, 1.0, 8, ptr, ptr, None, None, 0, None) == -1
    assert L.hawk_multi_verify(ptr, ptr, ptr, ptr, ptr, None, 1, 1, 16385, 1.0, 8, ptr, ptr, None, None, 0, None) == -1
    assert L.hawk_multi_verify(ptr, ptr, ptr, ptr, ptr, None, 0, 1, 8, 1.0, 8, ptr, ptr, None, None, 0, None) == 0


def test_rejection_probability_curve_matches_oracle(H):
    # Experiment, the rejection probability r = prod_j (1 - alpha_j) against the number of candidates:
    # the same proposal repeated against distinct proposals, 8 steps, all evaluated (the candidates
    # are tokens without target mass), residual masses from the kernel against the oracle's
    import torch
    rows, m, n, top_k = 24, 8, 16384, 1000
    rng = np.random.Generator(np.random.PCG64(5))
    p = (rng.standard_normal((rows, n)) * 1.5).astype(np.float32)
    qd = (p[:, None, :] + rng.standard_normal((rows, m, n))).astype(np.float32)
    qs = np.repeat(qd[:, :1], m, axis=1).copy()
    cand = np.repeat(np.argmin(p, axis=1).astype(np.int32)[:, None], m, axis=1).copy()
    u_acc = np.full((rows, m), np.float32(1.0) - np.float32(2.0 ** -24), dtype=np.float32)
    u_fin = np.full(rows, 0.5, dtype=np.float32)
    curves = {}
    for name, q in (("same", qs), ("distinct", qd)):
        (idx, tok, resid), (o_idx, o_tok, o_res) = run_both(H, p, q, cand, u_acc, u_fin, 1.0, top_k)
        assert (o_idx == m).all()
        np.testing.assert_array_equal(idx, o_idx)
        np.testing.assert_array_equal(tok, o_tok)
        np.testing.assert_allclose(resid, o_res, rtol=1e-11, atol=0)
        curves[name] = np.cumprod(resid, 1).mean(0)
    print("r(m), same proposal    :", np.round(curves["same"], 4))
    print("r(m), distinct proposals:", np.round(curves["distinct"], 4))
    assert np.all(curves["distinct"][1:] < curves["same"][1:])
    assert curves["same"][-1] / curves["same"][-2] > 0.97
