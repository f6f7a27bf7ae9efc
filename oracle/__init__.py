"""ctypes front end of the CPU oracle (oracle/hawk_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's CPU
baseline leg.  The HIP library and its Python binding never import this package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hawk_oracle.c")
_HDR = os.path.join(_HERE, "hawk_oracle.h")
_SO = os.path.join(_HERE, "libhawk_oracle.so")

SLOT_DRAFT, SLOT_ACC, SLOT_FINAL = 0, 64, 128


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain x86-64 code so the library also runs on a
    different host CPU).  Rebuilds when a source is newer than the library."""
    stale = (not os.path.exists(_SO)) or any(
        os.path.getmtime(p) > os.path.getmtime(_SO) for p in (_SRC, _HDR))
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i32, f32, f64, u64, u32 = C.c_void_p, C.c_int, C.c_float, C.c_double, C.c_uint64, C.c_uint32
        sig = {
            "orc_load": (vp, [vp, C.c_size_t, i32, i32, f64, f64]),
            "orc_free_model": (None, [vp]),
            "orc_new_state": (vp, [vp, i32, i32, i32, i32, i32, i32]),
            "orc_free_state": (None, [vp]),
            "orc_prefill": (i32, [vp, vp, vp, i32, f32, i32, f32, vp]),
            "orc_draft": (i32, [vp, i32, vp, vp]),
            "orc_draft_forced": (i32, [vp, i32, vp, i32]),
            "orc_verify": (i32, [vp, i32, vp, vp, vp, vp]),
            "orc_force": (i32, [vp, vp, vp, i32]),
            "orc_generate": (i32, [vp, vp, vp, i32, i32, f32, i32, f32, u64, vp, vp]),
            "orc_get_n": (i32, [vp, vp]),
            "orc_get_grid": (i32, [vp, vp]),
            "orc_get_logits": (i32, [vp, vp]),
            "orc_get_draft_logits": (i32, [vp, vp]),
            "orc_get_hprev": (i32, [vp, vp]),
            "orc_uniform": (f32, [u64, u32, u32, u32]),
            "orc_warp": (f64, [vp, i32, f32, i32, vp]),
            "orc_inv_cdf": (i32, [vp, i32, f64, f32]),
            "orc_spec_sample": (i32, [i32, i32, vp, vp, vp, i32, f32, i32, vp, f32, vp]),
            "orc_multi_verify": (i32, [i32, i32, vp, vp, vp, f32, i32, vp, f32, vp, vp]),
            "orc_forward_row": (i32, [vp, i32, i32, vp, vp]),
            "orc_draft_head": (i32, [vp, vp, i32, i32, vp, vp]),
            "orc_guide": (None, [vp, vp, f32, i32, vp]),
            "orc_margins": (None, [vp, i32]),
            "orc_num_threads": (i32, []),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


# ---------------------------------------------------------------- building blocks

def uniform(seed: int, seq: int, step: int, slot: int) -> float:
    return float(lib().orc_uniform(seed, seq, step, slot))


def warp(logits, temperature: float, top_k: int):
    """(unnormalised weights fp64, their sum)."""
    l = _f32(logits)
    w = np.zeros(l.shape[0], dtype=np.float64)
    z = lib().orc_warp(_p(l), l.shape[0], temperature, top_k, _p(w))
    return w, float(z)


def inv_cdf(w, total: float, u: float) -> int:
    w = np.ascontiguousarray(w, dtype=np.float64)
    return int(lib().orc_inv_cdf(_p(w), w.shape[0], total, u))


def spec_sample(p_logits, q_logits, drafts, u_acc, u_final: float, temperature: float = 1.0,
                top_k: Optional[int] = None, q_onehot: bool = False):
    """(number accepted a, tokens emitted [a+1])."""
    p = _f32(p_logits)
    k_eff, n = p.shape[0] - 1, p.shape[1]
    q = _f32(q_logits) if (q_logits is not None and k_eff > 0) else np.zeros((1, n), np.float32)
    d = _i32(drafts) if k_eff > 0 else np.zeros(1, np.int32)
    ua = _f32(u_acc) if k_eff > 0 else np.zeros(1, np.float32)
    out = np.full(k_eff + 1, -1, dtype=np.int32)
    a = lib().orc_spec_sample(k_eff, n, _p(p), _p(q), _p(d), int(q_onehot), temperature,
                              n if top_k is None else top_k, _p(ua), u_final, _p(out))
    return int(a), out[: a + 1].copy()


def multi_verify(p_logits, q_logits, cand, u_acc, u_final: float, temperature: float = 1.0,
                 top_k: Optional[int] = None, want_resid: bool = False):
    """Several candidates at one position, each from its own proposal row of q_logits [m, n].

    Returns (index of the accepted candidate or m, emitted token[, residual masses [m]])."""
    p = _f32(p_logits)
    q = _f32(q_logits)
    m, n = q.shape
    assert p.shape == (n,)
    c = _i32(cand)
    ua = _f32(u_acc)
    assert c.shape == (m,) and ua.shape == (m,)
    tok = np.full(1, -1, dtype=np.int32)
    resid = np.zeros(m, dtype=np.float64) if want_resid else None
    a = lib().orc_multi_verify(m, n, _p(p), _p(q), _p(c), temperature, n if top_k is None else top_k, _p(ua),
                               u_final, _p(tok), _p(resid))
    return (int(a), int(tok[0]), resid) if want_resid else (int(a), int(tok[0]))


def guide(lc, lu, scale: float) -> np.ndarray:
    """Guided logits lu + scale * (lc - lu), by the oracle's own routine."""
    lc, lu = _f32(lc), _f32(lu)
    out = np.zeros_like(lc)
    lib().orc_guide(_p(lc), _p(lu), scale, lc.size, _p(out))
    return out


def num_threads() -> int:
    return int(lib().orc_num_threads())


def margins(reset: bool = False) -> np.ndarray:
    out = np.zeros(3, dtype=np.float64)
    lib().orc_margins(_p(out), int(reset))
    return out


# ---------------------------------------------------------------- model + state

class Oracle:
    """One model instance plus decoding state, mirroring the HIP library's call list."""

    def __init__(self, blob: np.ndarray, *, batch: int = 1, use_cfg: bool = False, max_cond: int,
                 grid_h: int, grid_w: int, k_max: int, samp_lo: int = 0, samp_n: int = 0,
                 rms_eps: float = 1e-5, rope_theta: float = 10000.0):
        self._blob = np.ascontiguousarray(blob, dtype=np.uint8)  # borrowed by the C side
        L = lib()
        self._m = L.orc_load(_p(self._blob), self._blob.nbytes, samp_lo, samp_n, rms_eps, rope_theta)
        if not self._m:
            raise ValueError("oracle: bad weight blob or sampling slice")
        self._s = L.orc_new_state(self._m, batch, int(use_cfg), max_cond, grid_h, grid_w, k_max)
        if not self._s:
            L.orc_free_model(self._m)
            raise ValueError("oracle: bad state arguments")
        hdr = self._blob[:64].view(np.int32)
        self.d, self.vocab = int(hdr[4]), int(hdr[7])
        self.v_s = samp_n if samp_n else self.vocab
        self.batch, self.use_cfg = batch, use_cfg
        self.n_seq = batch * (2 if use_cfg else 1)
        self.n_img, self.k_max = grid_h * grid_w, k_max
        self.k_last = 0

    @classmethod
    def from_shape(cls, shape, blob, *, batch=None, k_max=None):
        return cls(blob, batch=shape.batch if batch is None else batch, use_cfg=shape.use_cfg,
                   max_cond=shape.n_cond, grid_h=shape.grid_h, grid_w=shape.grid_w,
                   k_max=shape.k if k_max is None else k_max, samp_lo=shape.samp_lo,
                   samp_n=shape.samp_n, rms_eps=shape.rms_eps, rope_theta=shape.rope_theta)

    def close(self):
        if getattr(self, "_s", None):
            lib().orc_free_state(self._s)
            self._s = None
        if getattr(self, "_m", None):
            lib().orc_free_model(self._m)
            self._m = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, cond, uncond, temperature, top_k, cfg_scale, u_first):
        cond = _f32(cond)
        unc = None if uncond is None else _f32(uncond)
        _chk(lib().orc_prefill(self._s, _p(cond), _p(unc), cond.shape[1], temperature, top_k,
                               cfg_scale, _p(_f32(u_first))), "prefill")

    def draft(self, k, u_draft):
        out = np.full((self.batch, max(k, 1)), -1, dtype=np.int32)
        u = _f32(u_draft) if k > 0 else None
        _chk(lib().orc_draft(self._s, k, _p(u), _p(out) if k > 0 else None), "draft")
        self.k_last = k
        return out[:, :k]

    def draft_forced(self, k, tokens, point_mass):
        t = _i32(tokens) if k > 0 else None
        _chk(lib().orc_draft_forced(self._s, k, _p(t), int(point_mass)), "draft_forced")
        self.k_last = k

    def verify(self, k, u_acc, u_final):
        na = np.zeros(self.batch, dtype=np.int32)
        toks = np.zeros((self.batch, k + 1), dtype=np.int32)
        ua = _f32(u_acc) if k > 0 else None
        _chk(lib().orc_verify(self._s, k, _p(ua), _p(_f32(u_final)), _p(na), _p(toks)), "verify")
        return na, toks

    def force(self, n_from, tokens):
        t = _i32(tokens).reshape(self.batch, -1)
        _chk(lib().orc_force(self._s, _p(_i32(n_from)), _p(t), t.shape[1]), "force")

    def generate(self, cond, uncond, k, temperature, top_k, cfg_scale, seed):
        cond = _f32(cond)
        unc = None if uncond is None else _f32(uncond)
        grid = np.zeros((self.batch, self.n_img), dtype=np.int32)
        stats = np.zeros(4, dtype=np.int64)
        _chk(lib().orc_generate(self._s, _p(cond), _p(unc), cond.shape[1], k, temperature, top_k,
                                cfg_scale, seed, _p(grid), _p(stats)), "generate")
        self.k_last = k
        return grid, dict(steps=int(stats[0]), accepted=int(stats[1]), tokens=int(stats[2]),
                          iters=int(stats[3]))

    def n(self):
        out = np.zeros(self.batch, dtype=np.int32)
        _chk(lib().orc_get_n(self._s, _p(out)), "get_n")
        return out

    def grid(self):
        out = np.zeros((self.batch, self.n_img), dtype=np.int32)
        _chk(lib().orc_get_grid(self._s, _p(out)), "get_grid")
        return out

    def logits(self):
        out = np.zeros((self.batch, self.k_last + 1, self.v_s), dtype=np.float32)
        _chk(lib().orc_get_logits(self._s, _p(out)), "get_logits")
        return out

    def draft_logits(self):
        out = np.zeros((self.batch, max(self.k_last, 1), self.v_s), dtype=np.float32)
        _chk(lib().orc_get_draft_logits(self._s, _p(out)), "get_draft_logits")
        return out[:, : self.k_last]

    def h_prev(self):
        out = np.zeros((self.n_seq, self.d), dtype=np.float64)
        _chk(lib().orc_get_hprev(self._s, _p(out)), "get_hprev")
        return out

    def forward_row(self, seq, pos, x, want_logits=True):
        x = np.array(x, dtype=np.float64)
        lg = np.zeros(self.v_s, dtype=np.float32) if want_logits else None
        _chk(lib().orc_forward_row(self._s, seq, pos, _p(x), _p(lg)), "forward_row")
        return x, lg

    def draft_head(self, g_prev, left, up, want_logits=True):
        g = np.ascontiguousarray(g_prev, dtype=np.float64)
        out = np.zeros(self.d, dtype=np.float64)
        lg = np.zeros(self.v_s, dtype=np.float32) if want_logits else None
        _chk(lib().orc_draft_head(self._s, _p(g), left, up, _p(out), _p(lg)), "draft_head")
        return out, lg
