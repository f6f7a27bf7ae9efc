"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and the
entry points that need no GPU behave (workspace sizing, rejection of bad configurations)."""
import ctypes as C
import os
import re

import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def H():
    import paper_2510_25739_amd as H
    if not os.path.exists(H.lib_path()):
        from paper_2510_25739_amd import build
        build.build()
    return H


def test_every_declared_symbol_is_exported(H):
    hdr = open(os.path.join(ROOT, "include", "hawk.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(hawk_[a-z_]+)\s*\(", hdr))
    assert {"hawk_load", "hawk_prefill", "hawk_draft", "hawk_verify", "hawk_generate"} <= declared
    lib = C.CDLL(H.lib_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(H.hawk.EXPORTS), "binding and header list different calls"


def test_workspace_bytes_and_bad_configs(H):
    for s in synth.CONFIGS.values():
        cfg = H.HawkConfig.from_shape(s)
        n = H.workspace_bytes(cfg)
        kv = 2 * s.n_layers * s.n_seq * (s.n_cond + s.n_img) * s.d_model * (8 if s.dtype == "fp32" else 2)
        assert n > s.n_params() * s.itemsize + kv
        assert n < 3.6 * (s.n_params() * s.itemsize + kv) + (1 << 30)   # blob + three re-tiled copies of the weights
    good = H.HawkConfig.from_shape(synth.CONFIGS[0])
    for field, bad in (("d_model", 250), ("n_heads", 3), ("k_max", 64), ("samp_n", 5000), ("dtype", 7),
                       ("max_batch", 0), ("n_layers", 0), ("d_mlp", 1001)):
        cfg = H.HawkConfig.from_buffer_copy(good)
        setattr(cfg, field, bad)
        assert H.workspace_bytes(cfg) == 0, field


def test_create_rejects_bad_arguments_without_touching_the_device(H):
    lib = H.load_library()
    cfg = H.HawkConfig.from_shape(synth.CONFIGS[0])
    h = C.c_void_p()
    assert lib.hawk_create(C.byref(cfg), None, 1 << 30, None, C.byref(h)) == -1       # null workspace
    assert lib.hawk_create(C.byref(cfg), C.c_void_p(4096 + 8), 1 << 30, None, C.byref(h)) == -1  # misaligned
    assert lib.hawk_create(C.byref(cfg), C.c_void_p(4096), 16, None, C.byref(h)) == -3  # too small
    bad = H.HawkConfig.from_buffer_copy(cfg)
    bad.d_model = 7
    assert lib.hawk_create(C.byref(bad), C.c_void_p(4096), 1 << 30, None, C.byref(h)) == -1
    assert not h.value
    assert lib.hawk_load(None, None, 0) == -1
    assert lib.hawk_last_error(None) == b"null context"


def test_multi_verify_rejects_bad_arguments_before_any_launch(H):
    lib = C.CDLL(H.lib_path())
    fn = lib.hawk_multi_verify
    fn.restype = C.c_int
    fn.argtypes = [C.c_void_p] * 6 + [C.c_int] * 3 + [C.c_float, C.c_int] + [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
    one = C.c_void_p(16)   # never dereferenced: every call below fails validation first
    assert fn(None, one, one, one, one, None, 1, 1, 8, 1.0, 8, one, one, None, None, 0, None) == -1
    assert fn(one, one, one, one, one, None, 1, 0, 8, 1.0, 8, one, one, None, None, 0, None) == -1      # no candidates
    assert fn(one, one, one, one, one, None, 1, 1, 0, 1.0, 8, one, one, None, None, 0, None) == -1      # empty vocabulary
    assert fn(one, one, one, one, one, None, 1, 1, 8, -1.0, 8, one, one, None, None, 0, None) == -1     # negative temperature
    assert fn(one, one, one, one, one, None, 1, 1, 8, 1.0, 0, one, one, None, None, 0, None) == -1      # top_k < 1
    assert fn(one, one, one, one, one, None, -1, 1, 8, 1.0, 8, one, one, None, None, 0, None) == -1
    assert fn(one, one, one, one, one, None, 0, 1, 8, 1.0, 8, one, one, None, None, 0, None) == 0       # no rows: nothing to do
    ws = lib.hawk_multi_verify_workspace_bytes
    ws.restype, ws.argtypes = C.c_size_t, [C.c_int, C.c_int]
    assert ws(6, 2) == 6 * 3 * 24 and ws(12, 2) == 2 * ws(6, 2) and ws(0, 2) == 0   # one 24-byte record per logit row


def test_spec_cache_layout_holds_every_outstanding_prediction(H):
    # host logic of the speculation cache (Method, "Dual Direction Drafting Heads": the cache of
    # IW * VSD * (VSD + 1) / 2 entries): the slot arithmetic against a raster walk that keeps every
    # outstanding prediction in a plain dictionary
    for IW, IH, VSD, v_s in ((6, 9, 2, 32), (5, 12, 3, 8), (24, 24, 1, 16), (7, 5, 4, 4)):
        slots = IW * VSD * (VSD + 1) // 2
        tags = (slots * 4 + 255) // 256 * 256
        assert H.spec_cache_bytes(IW, VSD, v_s) == tags + slots * v_s * 4
        held = {}   # slot -> (target, depth) outstanding
        for T in range(IW * IH):
            for d in range(1, VSD + 1):           # what pointed to T is read before T is committed ...
                s = H.spec_cache_slot(IW, VSD, T, d)
                assert 0 <= s < slots
                if T - d * IW >= 0:
                    assert held.get(s) == (T, d)
            for d in range(1, VSD + 1):           # ... and its slot may be taken over right after
                t = T + d * IW
                if t < IW * IH:
                    s = H.spec_cache_slot(IW, VSD, t, d)
                    assert s not in held or held[s] == (T, d), "slot still holds an outstanding prediction"
                    held[s] = (t, d)
    assert H.spec_cache_slot(6, 2, 5, 3) == -1 and H.spec_cache_slot(6, 2, -1, 1) == -1
    assert H.spec_cache_bytes(0, 2, 8) == 0 and H.spec_cache_bytes(4, 17, 8) == 0


def test_tree_layout_is_the_cartesian_product(H):
    # host logic of tree verification (Method, "Spatial Sampling Pool": the candidate tree as a Cartesian
    # product): node order, parents, candidate indices and ancestor masks against the oracle's plain
    # enumeration of the product
    from oracle import tree
    for m_depth in ((3,), (2, 3), (3, 3), (5, 2), (2, 2, 1), (1, 1, 1, 1, 1, 1, 1, 1), (4, 2, 3), (63,), (2, 5)):
        parent, depth, cand, anc = H.tree_layout(m_depth)
        nodes = tree.tree_nodes(m_depth)
        assert len(parent) == len(nodes)
        index = {p: i for i, p in enumerate(nodes)}
        for i, path in enumerate(nodes):
            assert depth[i] == len(path)
            assert parent[i] == (index[path[:-1]] if path else -1)
            assert cand[i] == (path[-1] if path else -1)
            want = 0
            for j in range(len(path)):
                want |= 1 << index[path[:j]]
            assert int(anc[i]) == want
    for bad in ((), (0,), (64,), (8, 8), (1,) * 9):
        with pytest.raises(H.HawkError):
            H.tree_layout(bad)


def test_spatial_entry_points_reject_bad_arguments_before_any_launch(H):
    L = H.load_library()
    one = C.c_void_p(4096)   # never dereferenced: every call below fails validation first
    assert L.hawk_spatial_heads(None, one, one, 1, 4, 64, 16, one, None, one, 1 << 20, None) == -1
    assert L.hawk_spatial_heads(one, one, one, 1, 4, 60, 16, one, None, one, 1 << 20, None) == -1    # d % 64
    assert L.hawk_spatial_heads(one, one, one, 1, 4, 64, 24, one, None, one, 1 << 20, None) == -1    # V_s % 16
    assert L.hawk_spatial_heads(one, one, one, 1, 4, 64, 16, one, None, one, 16, None) == -1         # workspace too small
    assert L.hawk_spatial_heads(one, one, one, 0, 4, 64, 16, one, None, None, 0, None) == 0
    assert L.hawk_spatial_heads_workspace_bytes(6, 4, 1280) >= 6 * 4 * 1280 * 4 + 2 * 6 * 1280 * 2 + 2 * 24 * 1280 * 2
    assert L.hawk_spec_cache_reset(None, 4, 2, 8, None) == -1
    assert L.hawk_spec_cache_push(one, 4, 4, 2, 8, one, one, 8, 1, None) == -1     # row stride below VSD * V_s
    assert L.hawk_spec_cache_push(one, 4, 4, 2, 8, one, one, 16, 5, None) == -1    # more rows than a line holds
    assert L.hawk_spec_cache_push(one, 4, 4, 2, 8, one, one, 16, 0, None) == 0
    assert L.hawk_spec_pool(one, 4, 4, 2, 8, one, one, 4, 1, one, one, one, None) == -1   # stride below V_s
    assert L.hawk_spec_pool(one, 4, 4, 2, 8, one, one, 8, 0, one, one, one, None) == 0
    assert L.hawk_sample_rows(one, None, one, 1, 0, 1.0, 8, one, None) == -1
    assert L.hawk_sample_rows(one, None, one, 0, 8, 1.0, 8, one, None) == 0


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_25739_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f


def test_streaming_plan_covers_every_weight_tile_once(H):
    # host logic of the persistent kernel: job tables and tile descriptors
    for idx in (1, 2):
        s = synth.CONFIGS[idx]
        info = H.plan_info(H.HawkConfig.from_shape(s))
        assert info["supported"] == 1 and info["tables_ok"] == 1
        per_layer = (4 * s.d_model ** 2 + 3 * s.d_model * s.d_mlp) // 512     # 16x32 bf16 tiles
        assert info["layer_tiles"] == per_layer
        assert info["total_tiles"] == s.n_layers * per_layer + s.v_s * s.d_model // 512 + 3 * s.d_model ** 2 // 512
        mean = per_layer / info["workgroups"]
        # the owners of the residual strips stream the Wo and W2 strips on top of their share of the
        # other two stages (what bounds a stage is its own busiest workgroup, not the layer total)
        assert info["min_wg_tiles"] <= mean <= info["max_wg_tiles"] <= 2.6 * mean
    assert H.plan_info(H.HawkConfig.from_shape(synth.CONFIGS[0]))["supported"] == 0   # fp32: generic kernels
