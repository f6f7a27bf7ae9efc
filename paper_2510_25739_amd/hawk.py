"""ctypes binding of libhawk.so: argument marshalling only, same call names as the C ABI."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhawk.so")
_lib = None

HAWK_FP32, HAWK_BF16 = 0, 1


class HawkError(RuntimeError):
    def __init__(self, code: int, where: str, text: str = ""):
        super().__init__(f"{where} failed with code {code}: {text}")
        self.code = code


class HawkConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "d_model", "n_heads", "d_mlp", "vocab", "samp_lo", "samp_n", "max_cond",
        "max_grid_h", "max_grid_w", "max_batch", "k_max", "dtype", "use_cfg")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float)]

    @classmethod
    def from_shape(cls, s, *, batch: Optional[int] = None, k_max: Optional[int] = None):
        """From a synth.HawkShape-like object (duck typed: only attributes are read)."""
        return cls(n_layers=s.n_layers, d_model=s.d_model, n_heads=s.n_heads, d_mlp=s.d_mlp, vocab=s.vocab,
                   samp_lo=s.samp_lo, samp_n=s.samp_n, max_cond=s.n_cond, max_grid_h=s.grid_h,
                   max_grid_w=s.grid_w, max_batch=s.batch if batch is None else batch,
                   k_max=s.k if k_max is None else k_max, dtype=HAWK_FP32 if s.dtype == "fp32" else HAWK_BF16,
                   use_cfg=int(s.cfg_scale != 1.0), rms_eps=s.rms_eps, rope_theta=s.rope_theta)


class HawkStats(C.Structure):
    _fields_ = [("steps", C.c_int64), ("accepted", C.c_int64), ("tokens", C.c_int64), ("iters", C.c_int64),
                ("ms_prefill", C.c_float), ("ms_decode", C.c_float)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


EXPORTS = {
    "hawk_workspace_bytes": (C.c_size_t, [C.POINTER(HawkConfig)]),
    "hawk_plan_info": (C.c_int, [C.POINTER(HawkConfig), C.POINTER(C.c_int64)]),
    "hawk_create": (C.c_int, [C.POINTER(HawkConfig), C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]),
    "hawk_destroy": (None, [C.c_void_p]),
    "hawk_last_error": (C.c_char_p, [C.c_void_p]),
    "hawk_load": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t]),
    "hawk_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float,
                               C.c_int, C.c_float, C.c_void_p]),
    "hawk_draft": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]),
    "hawk_draft_forced": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int]),
    "hawk_verify": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hawk_generate": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                C.c_float, C.c_int, C.c_float, C.c_uint64, C.c_void_p, C.c_void_p,
                                C.POINTER(HawkStats)]),
    "hawk_run_steps": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_uint64, C.c_int, C.POINTER(C.c_float),
                                 C.POINTER(C.c_float), C.POINTER(C.c_float)]),
    "hawk_set_replay": (C.c_int, [C.c_void_p, C.c_void_p]),
    "hawk_get_stats": (C.c_int, [C.c_void_p, C.POINTER(HawkStats)]),
    "hawk_force": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]),
    "hawk_get_n": (C.c_int, [C.c_void_p, C.c_void_p]),
    "hawk_get_grid": (C.c_int, [C.c_void_p, C.c_void_p]),
    "hawk_get_logits": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int]),
    "hawk_get_draft_logits": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int]),
    "hawk_set_path": (C.c_int, [C.c_void_p, C.c_int]),
    "hawk_last_path": (C.c_int, [C.c_void_p]),
    "hawk_last_kernel": (C.c_int, [C.c_void_p]),
    "hawk_debug_raise_timeout": (C.c_int, [C.c_void_p]),
    "hawk_phase_trace": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t]),
    "hawk_tree_layout": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hawk_verify_tree": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p]),
    "hawk_get_tree_logits": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int]),
    "hawk_get_tree_path": (C.c_int, [C.c_void_p, C.c_void_p]),
    "hawk_last_hidden": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "hawk_multi_verify_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int]),
    "hawk_multi_verify": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                    C.c_int, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]),
    "hawk_multi_verify_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_int, C.c_int, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p]),
    "hawk_spatial_heads_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int]),
    "hawk_spatial_heads": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hawk_spec_cache_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int]),
    "hawk_spec_cache_slot": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int]),
    "hawk_spec_cache_reset": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "hawk_spec_cache_push": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                       C.c_size_t, C.c_int, C.c_void_p]),
    "hawk_spec_pool": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t,
                                 C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hawk_sample_rows": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_int,
                                   C.c_void_p, C.c_void_p]),
    "hawk_generate_spatial_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int, C.c_int, C.c_int]),
    "hawk_generate_spatial": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float, C.c_int, C.c_void_p,
                                        C.c_void_p, C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p,
                                        C.c_void_p]),
}


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> C.CDLL:
    """Loads the built HIP library; never falls back to anything else."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise HawkError(-4, "load_library", f"{_LIB_PATH} is missing: run `python __graft_entry__.py` "
                                                "(or paper_2510_25739_amd/build.py) first")
        L = C.CDLL(_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def workspace_bytes(cfg: HawkConfig) -> int:
    return int(load_library().hawk_workspace_bytes(C.byref(cfg)))


def plan_info(cfg: HawkConfig) -> dict:
    out = (C.c_int64 * 8)()
    rc = load_library().hawk_plan_info(C.byref(cfg), out)
    if rc != 0:
        raise HawkError(rc, "hawk_plan_info")
    keys = ("supported", "layer_tiles", "total_tiles", "min_wg_tiles", "max_wg_tiles", "lm_rounds", "tables_ok", "workgroups")
    return dict(zip(keys, [int(v) for v in out]))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def multi_verify_workspace_bytes(rows: int, m: int) -> int:
    return int(load_library().hawk_multi_verify_workspace_bytes(rows, m))


def multi_verify(p_logits, q_logits, cand, u_acc, u_final, temperature: float, top_k: int, want_resid: bool = False,
                 workspace=None, m_rows=None):
    """hawk_multi_verify on device tensors (torch, on the GPU): p_logits [rows, n] fp32, q_logits
    [rows, m, n] fp32, cand [rows, m] int32, u_acc [rows, m] fp32, u_final [rows] fp32.
    workspace: None, or a device uint8 tensor of at least multi_verify_workspace_bytes(rows, m) bytes.
    m_rows: None, or a device int32 tensor [rows] with each position's own number of candidates.
    Returns device tensors (index [rows] int32, token [rows] int32[, residual masses [rows, m] fp64]);
    the launch is asynchronous on torch's current stream."""
    import torch  # device memory and stream only
    rows, m, n = q_logits.shape
    for t, shape, dt in ((p_logits, (rows, n), torch.float32), (q_logits, (rows, m, n), torch.float32),
                         (cand, (rows, m), torch.int32), (u_acc, (rows, m), torch.float32),
                         (u_final, (rows,), torch.float32)) + (
                                 ((m_rows, (rows,), torch.int32),) if m_rows is not None else ()):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == dt and tuple(t.shape) == shape):
            raise HawkError(-1, "hawk_multi_verify", "arguments must be contiguous device tensors of the documented shapes")
    idx = torch.empty(rows, dtype=torch.int32, device=p_logits.device)
    tok = torch.empty(rows, dtype=torch.int32, device=p_logits.device)
    resid = torch.empty((rows, m), dtype=torch.float64, device=p_logits.device) if want_resid else None
    rc = load_library().hawk_multi_verify(p_logits.data_ptr(), q_logits.data_ptr(), cand.data_ptr(), u_acc.data_ptr(),
                                          u_final.data_ptr(), m_rows.data_ptr() if m_rows is not None else None,
                                          rows, m, n, float(temperature), int(top_k),
                                          idx.data_ptr(), tok.data_ptr(), resid.data_ptr() if want_resid else None,
                                          workspace.data_ptr() if workspace is not None else None,
                                          workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                          torch.cuda.current_stream(p_logits.device).cuda_stream)
    if rc != 0:
        raise HawkError(rc, "hawk_multi_verify")
    return (idx, tok, resid) if want_resid else (idx, tok)


def multi_verify_static(p_logits, q_logits, cand, u_acc, u_final, temperature: float, top_k: int, out_index, out_token,
                        out_resid=None, m_rows=None):
    """hawk_multi_verify_static: hawk_multi_verify without any allocation - the caller passes the output
    tensors too (out_index, out_token int32 [rows]; out_resid None or fp64 [rows, m]); the statistics go
    to the library's fixed device array.  At most 4096 logit rows (rows * (m + 1)) per call."""
    import torch  # stream handle only
    rows, m, n = q_logits.shape
    rc = load_library().hawk_multi_verify_static(p_logits.data_ptr(), q_logits.data_ptr(), cand.data_ptr(), u_acc.data_ptr(),
                                                 u_final.data_ptr(), m_rows.data_ptr() if m_rows is not None else None,
                                                 rows, m, n, float(temperature), int(top_k), out_index.data_ptr(),
                                                 out_token.data_ptr(), out_resid.data_ptr() if out_resid is not None else None,
                                                 torch.cuda.current_stream(p_logits.device).cuda_stream)
    if rc != 0:
        raise HawkError(rc, "hawk_multi_verify_static")


def tree_layout(m_depth):
    """hawk_tree_layout: (parent, depth, candidate, ancestors) arrays of the candidate tree's nodes."""
    md = _i32(m_depth)
    parent, depth, cand = (np.zeros(64, dtype=np.int32) for _ in range(3))
    anc = np.zeros(64, dtype=np.uint64)
    n = load_library().hawk_tree_layout(len(md), _p(md), _p(parent), _p(depth), _p(cand), _p(anc))
    if n < 0:
        raise HawkError(-1, "hawk_tree_layout", "bad tree shape")
    return parent[:n], depth[:n], cand[:n], anc[:n]


def _stream_of(t):
    import torch  # device memory and stream only
    return torch.cuda.current_stream(t.device).cuda_stream


def _dev_ok(t, dtype, shape=None):
    return t.is_cuda and t.is_contiguous() and t.dtype == dtype and (shape is None or tuple(t.shape) == tuple(shape))


def spatial_heads(h, W_heads, W_out, want_g: bool = False):
    """hawk_spatial_heads on device tensors: h [rows, d] fp32, W_heads [n_heads, d, d] bf16, W_out
    [V_s, d] bf16.  Returns q_logits [rows, n_heads, V_s] fp32 (and g [rows, n_heads, d] fp32)."""
    import torch  # device memory and stream only
    rows, d = h.shape
    n_heads, v_s = W_heads.shape[0], W_out.shape[0]
    if not (_dev_ok(h, torch.float32) and _dev_ok(W_heads, torch.bfloat16, (n_heads, d, d))
            and _dev_ok(W_out, torch.bfloat16, (v_s, d))):
        raise HawkError(-1, "hawk_spatial_heads", "arguments must be contiguous device tensors of the documented shapes")
    L = load_library()
    nws = int(L.hawk_spatial_heads_workspace_bytes(rows, n_heads, d))
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device=h.device)
    q = torch.empty((rows, n_heads, v_s), dtype=torch.float32, device=h.device)
    g = torch.empty((rows, n_heads, d), dtype=torch.float32, device=h.device) if want_g else None
    rc = L.hawk_spatial_heads(h.data_ptr(), W_heads.data_ptr(), W_out.data_ptr(), rows, n_heads, d, v_s, q.data_ptr(),
                              g.data_ptr() if want_g else None, ws.data_ptr(), nws, _stream_of(h))
    if rc != 0:
        raise HawkError(rc, "hawk_spatial_heads")
    return (q, g) if want_g else q


def spec_cache_bytes(IW: int, VSD: int, v_s: int) -> int:
    return int(load_library().hawk_spec_cache_bytes(IW, VSD, v_s))


def spec_cache_slot(IW: int, VSD: int, pos: int, depth: int) -> int:
    return int(load_library().hawk_spec_cache_slot(IW, VSD, pos, depth))


class SpecCache:
    """The speculation cache of one image in device memory (a torch uint8 tensor) and its calls."""

    def __init__(self, IW: int, IH: int, VSD: int, v_s: int, device: str = "cuda:0"):
        import torch  # device memory and stream only
        self._torch = torch
        self.IW, self.IH, self.VSD, self.v_s = IW, IH, VSD, v_s
        self._L = load_library()
        nbytes = spec_cache_bytes(IW, VSD, v_s)
        if nbytes == 0:
            raise HawkError(-1, "hawk_spec_cache_bytes", "invalid cache shape")
        self.mem = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.reset()

    def reset(self):
        rc = self._L.hawk_spec_cache_reset(self.mem.data_ptr(), self.IW, self.VSD, self.v_s, _stream_of(self.mem))
        if rc != 0:
            raise HawkError(rc, "hawk_spec_cache_reset")

    def push(self, pos, q_vert, row_stride: int):
        """pos [rows] int32; q_vert: a device fp32 tensor whose row r starts r * row_stride floats in."""
        torch = self._torch
        rows = pos.numel()
        if not (_dev_ok(pos, torch.int32) and q_vert.is_cuda and q_vert.dtype == torch.float32
                and q_vert.numel() >= (rows - 1) * row_stride + self.VSD * self.v_s):
            raise HawkError(-1, "hawk_spec_cache_push", "bad arguments")
        rc = self._L.hawk_spec_cache_push(self.mem.data_ptr(), self.IW, self.IH, self.VSD, self.v_s, pos.data_ptr(),
                                          q_vert.data_ptr(), row_stride, rows, _stream_of(self.mem))
        if rc != 0:
            raise HawkError(rc, "hawk_spec_cache_push")

    def pool(self, target, q_horiz, horiz_stride: int):
        """target [n] int32; q_horiz: device fp32 tensor, item i's horizontal logits i * horiz_stride
        floats in.  Returns pool_logits [n, VSD + 1, V_s], pool_m [n], pool_delta [n, VSD + 1]."""
        torch = self._torch
        n = target.numel()
        if not (_dev_ok(target, torch.int32) and q_horiz.is_cuda and q_horiz.dtype == torch.float32
                and q_horiz.numel() >= (n - 1) * horiz_stride + self.v_s):
            raise HawkError(-1, "hawk_spec_pool", "bad arguments")
        dev = self.mem.device
        logits = torch.empty((n, self.VSD + 1, self.v_s), dtype=torch.float32, device=dev)   # rows beyond the count stay unwritten
        m = torch.empty(n, dtype=torch.int32, device=dev)
        delta = torch.empty((n, self.VSD + 1), dtype=torch.int32, device=dev)
        rc = self._L.hawk_spec_pool(self.mem.data_ptr(), self.IW, self.IH, self.VSD, self.v_s, target.data_ptr(),
                                    q_horiz.data_ptr(), horiz_stride, n, logits.data_ptr(), m.data_ptr(),
                                    delta.data_ptr(), _stream_of(self.mem))
        if rc != 0:
            raise HawkError(rc, "hawk_spec_pool")
        return logits, m, delta


def sample_rows(logits, u, temperature: float, top_k: int, skip=None):
    """hawk_sample_rows on device tensors: logits [rows, n] fp32, u [rows] fp32, skip None or [rows] int32."""
    import torch  # device memory and stream only
    rows, n = logits.shape
    if not (_dev_ok(logits, torch.float32) and _dev_ok(u, torch.float32, (rows,))
            and (skip is None or _dev_ok(skip, torch.int32, (rows,)))):
        raise HawkError(-1, "hawk_sample_rows", "arguments must be contiguous device tensors of the documented shapes")
    out = torch.empty(rows, dtype=torch.int32, device=logits.device)
    rc = load_library().hawk_sample_rows(logits.data_ptr(), skip.data_ptr() if skip is not None else None, u.data_ptr(),
                                         rows, n, float(temperature), int(top_k), out.data_ptr(), _stream_of(logits))
    if rc != 0:
        raise HawkError(rc, "hawk_sample_rows")
    return out


class Hawk:
    """One context: device workspace (a torch uint8 tensor) + the C handle."""

    def __init__(self, cfg: HawkConfig, device: str = "cuda:0", stream=None):
        import torch  # device memory and stream only
        self._L = load_library()
        self.cfg = cfg
        nbytes = workspace_bytes(cfg)
        if nbytes == 0:
            raise HawkError(-1, "hawk_workspace_bytes", "invalid configuration")
        if not torch.cuda.is_available():
            raise HawkError(-4, "Hawk", "no GPU visible: the HIP path has no CPU fallback")
        self._torch = torch
        self._dev = torch.device(device)
        with torch.cuda.device(self._dev):
            self._ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self._dev)
            self._stream = stream if stream is not None else torch.cuda.current_stream(self._dev)
        base = self._ws.data_ptr()
        self._ws_ptr = (base + 255) & ~255
        h = C.c_void_p()
        rc = self._L.hawk_create(C.byref(cfg), C.c_void_p(self._ws_ptr), nbytes, C.c_void_p(self._stream.cuda_stream),
                                 C.byref(h))
        if rc != 0:
            raise HawkError(rc, "hawk_create")
        self._h = h
        self.v_s = cfg.samp_n if cfg.samp_n else cfg.vocab
        self.batch = 0
        self.n_img = 0

    # -- plumbing
    def _chk(self, rc, where):
        if rc != 0:
            raise HawkError(rc, where, self._L.hawk_last_error(self._h).decode())

    def close(self):
        if getattr(self, "_h", None):
            self._L.hawk_destroy(self._h)
            self._h = None
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def stream_handle(self) -> int:
        return int(self._stream.cuda_stream)

    # -- the C calls
    def set_path(self, path: int):
        self._chk(self._L.hawk_set_path(self._h, path), "hawk_set_path")

    def last_path(self) -> int:
        return int(self._L.hawk_last_path(self._h))

    def last_kernel(self) -> int:
        """0: one kernel per operation, 1: grid-barrier persistent kernel, 2: the kernel laid out on the XCDs."""
        return int(self._L.hawk_last_kernel(self._h))

    def debug_raise_timeout(self):
        """Test hook: sets the persistent kernels' error word from the host."""
        self._chk(self._L.hawk_debug_raise_timeout(self._h), "hawk_debug_raise_timeout")

    def phase_trace(self, enable: bool, n_stages: int = 0):
        """Switches the streaming kernel's stage time stamps; returns [4, n_stages, 8] uint64 if asked."""
        if n_stages <= 0:
            self._chk(self._L.hawk_phase_trace(self._h, int(enable), None, 0), "hawk_phase_trace")
            return None
        out = np.zeros(4 * 4096 * 8 + 2 * 256 * 256, dtype=np.uint64)
        self._chk(self._L.hawk_phase_trace(self._h, int(enable), _p(out), out.size), "hawk_phase_trace")
        self.last_arrivals = out[4 * 4096 * 8:].reshape(2, 256, 256)   # [arrive | release seen][stage][workgroup]
        return out[:4 * 4096 * 8].reshape(4, 4096, 8)[:, :n_stages]

    def load(self, blob: np.ndarray):
        blob = np.ascontiguousarray(blob, dtype=np.uint8)
        self._chk(self._L.hawk_load(self._h, _p(blob), blob.nbytes), "hawk_load")

    def prefill(self, cond, uncond, grid_h, grid_w, temperature, top_k, cfg_scale, u_first):
        cond = _f32(cond)
        unc = None if uncond is None else _f32(uncond)
        self.batch, self.n_img = cond.shape[0], grid_h * grid_w
        self._chk(self._L.hawk_prefill(self._h, _p(cond), _p(unc), cond.shape[0], cond.shape[1], grid_h, grid_w,
                                       temperature, top_k, cfg_scale, _p(_f32(u_first))), "hawk_prefill")

    def draft(self, k, u_draft, want=True):
        u = _f32(u_draft) if k > 0 else None
        out = np.full((self.batch, max(k, 1)), -1, dtype=np.int32) if want else None
        self._chk(self._L.hawk_draft(self._h, k, _p(u), _p(out) if (want and k > 0) else None), "hawk_draft")
        return None if out is None else out[:, :k]

    def draft_forced(self, k, tokens, point_mass):
        t = _i32(tokens) if k > 0 else None
        self._chk(self._L.hawk_draft_forced(self._h, k, _p(t), int(point_mass)), "hawk_draft_forced")

    def verify(self, k, u_acc, u_final, want=True):
        ua = _f32(u_acc) if k > 0 else None
        na = np.zeros(self.batch, dtype=np.int32) if want else None
        toks = np.zeros((self.batch, k + 1), dtype=np.int32) if want else None
        self._chk(self._L.hawk_verify(self._h, k, _p(ua), _p(_f32(u_final)), _p(na), _p(toks)), "hawk_verify")
        return na, toks

    def verify_tree(self, m_depth, cand, q_logits, u_acc, u_final):
        """hawk_verify_tree: m_depth [D]; cand [D, batch, m_max] int32 (host); q_logits a device fp32
        tensor [D, batch, m_max, V_s]; u_acc [D, batch, m_max], u_final [D + 1, batch] (host).
        Returns (accepted [batch], tokens [batch, D + 1])."""
        md = _i32(m_depth)
        D, m_max = len(md), int(md.max())
        cand, ua, uf = _i32(cand), _f32(u_acc), _f32(u_final)
        if cand.shape != (D, self.batch, m_max) or ua.shape != cand.shape or uf.shape != (D + 1, self.batch):
            raise HawkError(-1, "hawk_verify_tree", "host arrays do not have the documented shapes")
        if not (q_logits.is_cuda and q_logits.is_contiguous() and q_logits.dtype == self._torch.float32
                and tuple(q_logits.shape) == (D, self.batch, m_max, self.v_s)):
            raise HawkError(-1, "hawk_verify_tree", "q_logits must be a contiguous device fp32 tensor [D, batch, m_max, V_s]")
        na = np.zeros(self.batch, dtype=np.int32)
        toks = np.zeros((self.batch, D + 1), dtype=np.int32)
        self._chk(self._L.hawk_verify_tree(self._h, D, _p(md), _p(cand), C.c_void_p(q_logits.data_ptr()), _p(ua), _p(uf),
                                           _p(na), _p(toks)), "hawk_verify_tree")
        return na, toks

    def generate_spatial(self, cond, grid_h, grid_w, temperature, top_k, W_heads, W_out, HD, VSD, seed):
        """hawk_generate_spatial: the whole drafting and verification scheme over one image.  cond [1, n_cond, d]
        (host); W_heads [HD + VSD, d, d], W_out [V_s, d]: contiguous device bf16 tensors.  Returns (grid [1, N],
        dict(passes, accepted, tail_steps, tokens))."""
        torch = self._torch
        cond = _f32(cond)
        self.batch, self.n_img = 1, grid_h * grid_w
        d = self.cfg.d_model
        if not (W_heads.is_cuda and W_heads.is_contiguous() and W_heads.dtype == torch.bfloat16
                and tuple(W_heads.shape) == (HD + VSD, d, d) and W_out.is_cuda and W_out.is_contiguous()
                and W_out.dtype == torch.bfloat16 and tuple(W_out.shape) == (self.v_s, d)):
            raise HawkError(-1, "hawk_generate_spatial", "head weights must be contiguous device bf16 tensors [HD + VSD, d, d] and [V_s, d]")
        nbytes = int(self._L.hawk_generate_spatial_workspace_bytes(C.byref(self.cfg), grid_w, HD, VSD))
        if nbytes == 0:
            raise HawkError(-1, "hawk_generate_spatial_workspace_bytes", "bad arguments")
        ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=W_heads.device)
        base = (ws.data_ptr() + 255) & ~255
        grid = np.zeros((1, self.n_img), dtype=np.int32)
        stats = np.zeros(4, dtype=np.int64)
        self._chk(self._L.hawk_generate_spatial(self._h, _p(cond), cond.shape[1], grid_h, grid_w, float(temperature), int(top_k),
                                                C.c_void_p(W_heads.data_ptr()), C.c_void_p(W_out.data_ptr()), HD, VSD,
                                                C.c_uint64(seed), C.c_void_p(base), nbytes, _p(grid), _p(stats)),
                  "hawk_generate_spatial")
        return grid, dict(passes=int(stats[0]), accepted=int(stats[1]), tail_steps=int(stats[2]), tokens=int(stats[3]))

    def tree_path(self):
        out = np.zeros((self.batch, 8), dtype=np.int32)
        self._chk(self._L.hawk_get_tree_path(self._h, _p(out)), "hawk_get_tree_path")
        return out

    def last_hidden(self, rows_per_seq: int):
        """The hidden states of the last pass's rows as a device tensor view [sequences * rows_per_seq, d]
        (fp32 in the bf16 configurations, fp64 in the fp32 one) into the workspace: read only."""
        ptr, eb = C.c_void_p(), C.c_int()
        self._chk(self._L.hawk_last_hidden(self._h, C.byref(ptr), C.byref(eb)), "hawk_last_hidden")
        torch = self._torch
        n_seq = self.batch * (2 if self.cfg.use_cfg else 1)
        off = ptr.value - self._ws.data_ptr()
        nbytes = n_seq * rows_per_seq * self.cfg.d_model * eb.value
        return self._ws[off:off + nbytes].view(torch.float32 if eb.value == 4 else torch.float64).view(
            n_seq * rows_per_seq, self.cfg.d_model)

    def tree_logits(self, n_nodes):
        out = np.zeros((self.batch, n_nodes, self.v_s), dtype=np.float32)
        self._chk(self._L.hawk_get_tree_logits(self._h, _p(out), n_nodes), "hawk_get_tree_logits")
        return out

    def generate(self, cond, uncond, grid_h, grid_w, k, temperature, top_k, cfg_scale, seed, replay=None):
        cond = _f32(cond)
        unc = None if uncond is None else _f32(uncond)
        self.batch, self.n_img = cond.shape[0], grid_h * grid_w
        grid = np.zeros((self.batch, self.n_img), dtype=np.int32)
        rp = None if replay is None else _i32(replay)
        st = HawkStats()
        self._chk(self._L.hawk_generate(self._h, _p(cond), _p(unc), cond.shape[0], cond.shape[1], grid_h, grid_w, k,
                                        temperature, top_k, cfg_scale, seed, _p(rp), _p(grid), C.byref(st)),
                  "hawk_generate")
        return grid, st.as_dict()

    def run_steps(self, k, n_steps, seed, replay=False, timed=False):
        """Enqueues n_steps steps; with timed=True returns (ms_draft, ms_verify, ms_kernel) summed over them."""
        if timed:
            a, b, k_ = C.c_float(), C.c_float(), C.c_float()
            self._chk(self._L.hawk_run_steps(self._h, k, n_steps, seed, int(replay), C.byref(a), C.byref(b),
                                             C.byref(k_)), "hawk_run_steps")
            return a.value, b.value, k_.value
        self._chk(self._L.hawk_run_steps(self._h, k, n_steps, seed, int(replay), None, None, None), "hawk_run_steps")
        return None

    def set_replay(self, tokens):
        self._chk(self._L.hawk_set_replay(self._h, _p(_i32(tokens))), "hawk_set_replay")

    def stats(self):
        st = HawkStats()
        self._chk(self._L.hawk_get_stats(self._h, C.byref(st)), "hawk_get_stats")
        return st.as_dict()

    def synchronize(self):
        self._stream.synchronize()

    def force(self, n_from, tokens):
        t = _i32(tokens).reshape(self.batch, -1)
        self._chk(self._L.hawk_force(self._h, _p(_i32(n_from)), _p(t), t.shape[1]), "hawk_force")

    def n(self):
        out = np.zeros(self.batch, dtype=np.int32)
        self._chk(self._L.hawk_get_n(self._h, _p(out)), "hawk_get_n")
        return out

    def grid(self):
        out = np.zeros((self.batch, self.n_img), dtype=np.int32)
        self._chk(self._L.hawk_get_grid(self._h, _p(out)), "hawk_get_grid")
        return out

    def logits(self, rows):
        out = np.zeros((self.batch, rows, self.v_s), dtype=np.float32)
        self._chk(self._L.hawk_get_logits(self._h, _p(out), rows), "hawk_get_logits")
        return out

    def draft_logits(self, k):
        out = np.zeros((self.batch, k, self.v_s), dtype=np.float32)
        self._chk(self._L.hawk_get_draft_logits(self._h, _p(out), k), "hawk_get_draft_logits")
        return out
