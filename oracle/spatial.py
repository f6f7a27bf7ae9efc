"""CPU oracle of the spatial drafting structures: dual-direction draft heads, the speculation
cache and the spatial sampling pool (Method, "Dual Direction Drafting Heads" and "Spatial Sampling
Pool"; appendix "Draft Heads Structure and Memory Overhead").

TEST INFRASTRUCTURE ONLY, like the rest of this package: plain numpy in fp64 and a dictionary; no
blocking, no ring buffers, nothing shared with the HIP path.

Conventions (T is the position the hidden state at hand predicts through the model's own output
layer, positions count in raster order, position = row * IW + column):
  * horizontal head j (1 <= j <= HD) proposes the token at T + j, vertical head d (1 <= d <= VSD)
    the token at T + d * IW;
  * one head is a linear layer of the hidden size followed by SiLU, added back to its input as in
    the Medusa block the appendix names, and the model's output layer is shared by all heads:
        g = h + silu(W h),   logits = W_out g;
  * the cache holds a vertical prediction from the moment the position it was made from is
    committed until the position it points to is committed;
  * VertSpec(t) = { the prediction made from t - delta * IW with depth delta, delta = 1 .. VSD },
    the pool at t = VertSpec(t) followed by the horizontal proposal for t (the appendix verifies the
    vertical candidate first), vertical members in ascending delta.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def spatial_heads(h: np.ndarray, W_heads: np.ndarray, W_out: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """h [rows, d]; W_heads [n_heads, d, d] (out, in); W_out [V_s, d].
    Returns g [rows, n_heads, d] (fp64) and logits [rows, n_heads, V_s] (rounded to fp32 once)."""
    h = np.asarray(h, np.float64)
    W_heads = np.asarray(W_heads, np.float64)
    W_out = np.asarray(W_out, np.float64)
    rows, d = h.shape
    n_heads = W_heads.shape[0]
    g = np.empty((rows, n_heads, d))
    for j in range(n_heads):
        g[:, j, :] = h + silu(h @ W_heads[j].T)
    logits = g.reshape(rows * n_heads, d) @ W_out.T
    return g, logits.reshape(rows, n_heads, -1).astype(np.float32)


def cache_entries(IW: int, VSD: int) -> int:
    """Entries the cache needs (Method, the equation after "we maintain a cache of size")."""
    return IW * (VSD * (VSD + 1)) // 2


class SpecCache:
    """The speculation cache by its definition: a map from (position pointed to, depth) to the
    prediction, filled when the source position is committed, emptied when the target is."""

    def __init__(self, IW: int, IH: int, VSD: int):
        self.IW, self.IH, self.VSD = IW, IH, VSD
        self.store: Dict[Tuple[int, int], object] = {}
        self.peak = 0

    def push(self, T: int, vertical: Sequence[object]) -> None:
        """The hidden state that predicted position T gave vertical[d - 1] for T + d * IW; T is
        committed now, so what pointed to T is done with."""
        assert len(vertical) == self.VSD
        for d in range(1, self.VSD + 1):
            self.store.pop((T, d), None)
        for d in range(1, self.VSD + 1):
            t = T + d * self.IW
            if t < self.IW * self.IH:
                self.store[(t, d)] = vertical[d - 1]
        self.peak = max(self.peak, len(self.store))

    def vert_spec(self, t: int) -> List[Tuple[int, object]]:
        """VertSpec(t) as (delta, prediction) in ascending delta; members never made are absent."""
        return [(dv, self.store[(t, dv)]) for dv in range(1, self.VSD + 1) if (t, dv) in self.store]

    def pool(self, t: int, horizontal: object) -> List[Tuple[int, object]]:
        """Spatial sampling pool at t: the vertical members, then the horizontal one (delta 0)."""
        return self.vert_spec(t) + [(0, horizontal)]
