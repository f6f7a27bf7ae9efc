"""The entry point that allocates nothing (hawk_multi_verify_static: the rows' statistics in the library's
fixed device array) against hawk_multi_verify with a caller-provided workspace: same index, token and
residual masses to the bit, through the C ABI, on two calls in a row - the second smaller, so that it
runs over what the first left in the array."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _rows(seed, rows, m, n):
    rng = np.random.Generator(np.random.PCG64(seed))
    uni = lambda *shp: (rng.integers(0, 1 << 24, size=shp).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)
    p = (rng.standard_normal((rows, n)) * 1.5).astype(np.float32)
    q = (p[:, None, :] + rng.standard_normal((rows, m, n))).astype(np.float32)
    cand = np.argsort(-q, axis=2)[:, :, 3].astype(np.int32)     # a likely token of each proposal
    m_rows = rng.integers(0, m + 1, size=rows).astype(np.int32)
    return p, q, cand, uni(rows, m), uni(rows), m_rows


def _call_both(H, torch, seed, rows, m, n, top_k):
    dev = "cuda:0"
    L = H.load_library()
    p, q, cand, u_acc, u_fin, m_rows = _rows(seed, rows, m, n)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    dp, dq, dc, dua, duf, dmr = t(p), t(q), t(cand), t(u_acc), t(u_fin), t(m_rows)
    out = {}
    for name in ("workspace", "static"):
        idx = torch.full((rows,), -7, dtype=torch.int32, device=dev)
        tok = torch.full((rows,), -7, dtype=torch.int32, device=dev)
        res = torch.full((rows, m), 7.0, dtype=torch.float64, device=dev)
        stream = torch.cuda.current_stream().cuda_stream
        if name == "workspace":
            ws = torch.empty(H.multi_verify_workspace_bytes(rows, m), dtype=torch.uint8, device=dev)
            rc = L.hawk_multi_verify(dp.data_ptr(), dq.data_ptr(), dc.data_ptr(), dua.data_ptr(), duf.data_ptr(),
                                     dmr.data_ptr(), rows, m, n, 1.0, top_k, idx.data_ptr(), tok.data_ptr(),
                                     res.data_ptr(), ws.data_ptr(), ws.numel(), stream)
        else:
            rc = L.hawk_multi_verify_static(dp.data_ptr(), dq.data_ptr(), dc.data_ptr(), dua.data_ptr(), duf.data_ptr(),
                                            dmr.data_ptr(), rows, m, n, 1.0, top_k, idx.data_ptr(), tok.data_ptr(),
                                            res.data_ptr(), stream)
        assert rc == 0, (name, rc)
        torch.cuda.synchronize()
        out[name] = (idx.cpu().numpy(), tok.cpu().numpy(), res.cpu().numpy())
    a, b = out["workspace"], out["static"]
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    assert np.array_equal(a[2], b[2])                   # the same kernels on the same records: identical bits
    assert (a[0] >= 0).all() and (a[0] <= m).all() and (a[1] >= 0).all() and (a[1] < n).all()
    return a


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    import paper_2510_25739_amd as H
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    first = _call_both(H, torch, 11, 48, 3, 16384, 1000)      # 192 logit rows of statistics
    second = _call_both(H, torch, 12, 5, 2, 8192, 2000)       # smaller, over the first call's leftovers
    assert len(first[0]) == 48 and len(second[0]) == 5
    # the limit: one record per logit row, 4096 of them; beyond it nothing is launched
    L = H.load_library()
    z = torch.zeros(8, device="cuda:0")
    ptr = z.data_ptr()
    assert L.hawk_multi_verify_static(ptr, ptr, ptr, ptr, ptr, None, 2048, 2, 8, 1.0, 8, ptr, ptr, None, None) == -3
    assert L.hawk_multi_verify_static(None, ptr, ptr, ptr, ptr, None, 1, 1, 8, 1.0, 8, ptr, ptr, None, None) == -1
    assert L.hawk_multi_verify_static(ptr, ptr, ptr, ptr, ptr, None, 0, 1, 8, 1.0, 8, ptr, ptr, None, None) == 0
