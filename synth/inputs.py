"""Synthetic model shapes, weight blobs, condition vectors and uniform tables.

Stand-ins for the trained target model, trained draft head and text prompts the paper's
experiments use (Experiment section, "Model and Benchmark"): none of those can be obtained
here, so every input is a seeded random draw with the shapes of the named model families.

Weight-blob container (little endian), read independently by the CPU oracle and by the HIP
library:

    header, 64 bytes = 16 x int32:
        [0] magic 'HAWK'  [1] version = 1  [2] dtype (0 = fp32, 1 = bf16)
        [3] n_layers  [4] d_model  [5] n_heads  [6] d_mlp  [7] vocab  [8..15] zero
    then the tensors, contiguous, row-major [out, in], all in `dtype`:
        E[vocab, d]
        per layer: g1[d] Wq[d,d] Wk[d,d] Wv[d,d] Wo[d,d] g2[d] W1[m,d] W3[m,d] W2[d,m]
        g_f[d]  W_out[vocab, d]  W_d[d, 3d]
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Iterator, Tuple

import numpy as np

BLOB_MAGIC = 0x4B574148  # b"HAWK" as little-endian int32
BLOB_HEADER_BYTES = 64


@dataclass(frozen=True)
class HawkShape:
    """One workload: target-model shape, image grid and decoding parameters."""

    name: str
    n_layers: int
    d_model: int
    n_heads: int
    d_mlp: int
    vocab: int
    n_cond: int
    grid_h: int
    grid_w: int
    k: int
    dtype: str = "bf16"  # "fp32" or "bf16": storage type of every tensor in the blob
    batch: int = 1
    cfg_scale: float = 1.0
    temperature: float = 1.0
    top_k: int = 1000
    samp_lo: int = 0  # first vocabulary id of the sampled (image-code) slice
    samp_n: int = 0  # size of the sampled slice; 0 means the whole vocabulary
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def v_s(self) -> int:
        return self.samp_n if self.samp_n else self.vocab

    @property
    def n_img(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def use_cfg(self) -> bool:
        return self.cfg_scale != 1.0

    @property
    def n_seq(self) -> int:
        return self.batch * (2 if self.use_cfg else 1)

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    def n_params(self) -> int:
        d, m, v = self.d_model, self.d_mlp, self.vocab
        return v * d + self.n_layers * (2 * d + 4 * d * d + 3 * d * m) + d + v * d + 3 * d * d

    def replace(self, **kw) -> "HawkShape":
        return dataclasses.replace(self, **kw)


# The five workloads: a tiny fp32 model for exact parity, LlamaGen-B- and -XL-shaped
# bf16 models, the XL shape under classifier-free guidance with 16 prompts, and a
# Chameleon / Lumina-mGPT-7B-shaped model that samples an 8192-entry image-code slice.
CONFIGS: Dict[int, HawkShape] = {
    0: HawkShape("tiny-fp32", 2, 256, 4, 1024, 4096, 16, 8, 8, 4, dtype="fp32"),
    1: HawkShape("B-bf16", 12, 768, 12, 2048, 16384, 120, 16, 16, 5),
    2: HawkShape("XL-bf16", 36, 1280, 20, 3456, 16384, 120, 24, 24, 5),
    3: HawkShape("XL-bf16-cfg4-b16", 36, 1280, 20, 3456, 16384, 120, 24, 24, 5,
                 batch=16, cfg_scale=4.0),
    4: HawkShape("7B-bf16-cfg3", 32, 4096, 32, 11008, 65536, 64, 32, 32, 5,
                 cfg_scale=3.0, top_k=2000, samp_lo=4, samp_n=8192),
}


def _tensor_list(s: HawkShape) -> Iterator[Tuple[str, Tuple[int, ...], bool]]:
    """(name, shape, is_gain) in blob order."""
    d, m, v = s.d_model, s.d_mlp, s.vocab
    yield "E", (v, d), False
    for l in range(s.n_layers):
        yield f"l{l}.g1", (d,), True
        yield f"l{l}.Wq", (d, d), False
        yield f"l{l}.Wk", (d, d), False
        yield f"l{l}.Wv", (d, d), False
        yield f"l{l}.Wo", (d, d), False
        yield f"l{l}.g2", (d,), True
        yield f"l{l}.W1", (m, d), False
        yield f"l{l}.W3", (m, d), False
        yield f"l{l}.W2", (d, m), False
    yield "g_f", (d,), True
    yield "W_out", (v, d), False
    yield "W_d", (d, 3 * d), False


def blob_layout(s: HawkShape) -> Dict[str, Tuple[int, Tuple[int, ...]]]:
    """name -> (byte offset in the blob, tensor shape)."""
    out = {}
    off = BLOB_HEADER_BYTES
    for name, shp, _ in _tensor_list(s):
        out[name] = (off, shp)
        off += int(np.prod(shp)) * s.itemsize
    out["__end__"] = (off, ())
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of finite fp32 values to bf16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_weights(s: HawkShape, seed: int = 0, std: float = 0.02, repeat_layer0: bool = False) -> np.ndarray:
    """The weight blob (uint8 array): every matrix N(0, std^2) drawn in fp32 in blob
    order from one PCG64 stream, norm gains exactly 1; bf16 blobs hold the
    round-to-nearest-even bf16 of the fp32 draw.  repeat_layer0: only the embedding, layer 0 and
    the tensors behind the layers are drawn and layer 0's bytes are copied into the other layers
    (timing runs of the largest shape: same sizes and value distribution in a tenth of the time;
    not for parity tests, whose blobs are drawn in full)."""
    if repeat_layer0 and s.n_layers > 1:
        one = make_weights(s.replace(n_layers=1), seed=seed, std=std)
        lay1, lay = blob_layout(s.replace(n_layers=1)), blob_layout(s)
        blob = np.zeros(lay["__end__"][0], dtype=np.uint8)
        a, b = lay1["l0.g1"][0], lay1["g_f"][0]            # layer 0's bytes in the one-layer blob
        blob[:b] = one[:b]
        for l in range(1, s.n_layers):
            o = lay[f"l{l}.g1"][0]
            blob[o:o + (b - a)] = one[a:b]
        tail = lay["g_f"][0]
        blob[tail:] = one[b:]
        blob[:BLOB_HEADER_BYTES].view(np.int32)[3] = s.n_layers
        return blob
    lay = blob_layout(s)
    blob = np.zeros(lay["__end__"][0], dtype=np.uint8)
    hdr = blob[:BLOB_HEADER_BYTES].view(np.int32)
    hdr[0] = BLOB_MAGIC
    hdr[1] = 1
    hdr[2] = 0 if s.dtype == "fp32" else 1
    hdr[3:8] = [s.n_layers, s.d_model, s.n_heads, s.d_mlp, s.vocab]
    rng = np.random.Generator(np.random.PCG64(seed))
    for name, shp, is_gain in _tensor_list(s):
        off, _ = lay[name]
        n = int(np.prod(shp))
        if is_gain:
            t = np.ones(n, dtype=np.float32)
        else:
            t = rng.standard_normal(n, dtype=np.float32)
            t *= np.float32(std)
        dst = blob[off:off + n * s.itemsize]
        if s.dtype == "fp32":
            dst.view(np.float32)[:] = t
        else:
            dst.view(np.uint16)[:] = f32_to_bf16_bits(t)
    return blob


def blob_tensor(s: HawkShape, blob: np.ndarray, name: str) -> np.ndarray:
    """One tensor of the blob as an fp32 array (bf16 upcast exactly)."""
    off, shp = blob_layout(s)[name]
    n = int(np.prod(shp))
    raw = blob[off:off + n * s.itemsize]
    if s.dtype == "fp32":
        return raw.view(np.float32).reshape(shp).copy()
    return bf16_bits_to_f32(raw.view(np.uint16)).reshape(shp)


def make_cond(s: HawkShape, seed: int = 2, batch: int | None = None) -> np.ndarray:
    """Condition vectors N(0,1), fp32 [batch, n_cond, d] (seed 2: conditional stream,
    seed 3 by convention: the unconditional stream of classifier-free guidance)."""
    b = s.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((b, s.n_cond, s.d_model), dtype=np.float32)


def make_uniforms(seed: int, shape) -> np.ndarray:
    """Uniforms in [0,1) carrying 24 random bits each (j / 2^24), fp32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    bits = rng.integers(0, 1 << 24, size=shape, dtype=np.uint32)
    return (bits.astype(np.float32) / np.float32(1 << 24)).astype(np.float32)


def make_spatial_heads(seed: int, rows: int, n_heads: int, d: int, v_s: int, std_head: float = 0.02,
                       std_out: float = 0.04):
    """Inputs of the dual-direction draft heads: hidden states N(0,1) fp32 [rows, d], head
    matrices N(0, std_head^2) [n_heads, d, d] and the output layer's sampled rows
    N(0, std_out^2) [v_s, d], both as bf16 bit patterns (round to nearest even)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    h = rng.standard_normal((rows, d), dtype=np.float32)
    w_heads = rng.standard_normal((n_heads, d, d), dtype=np.float32) * np.float32(std_head)
    w_out = rng.standard_normal((v_s, d), dtype=np.float32) * np.float32(std_out)
    return h, f32_to_bf16_bits(w_heads), f32_to_bf16_bits(w_out)


def make_logit_rows(seed: int, shape, std: float = 1.5) -> np.ndarray:
    """Logit rows N(0, std^2), fp32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)
