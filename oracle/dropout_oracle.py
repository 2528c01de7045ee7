"""Dropout masks of the stage oracle: a counter-based generator, so that a recompute pass
regenerates exactly the masks of the forward pass it repeats.

TEST INFRASTRUCTURE (see stage_oracle.py).  The paper's implementation saves and restores
the GPU's random-number state around recomputation so that the recomputed activations equal
the forward ones (Implementation, the list of library functions); it names no generator.
This build's reading: masks are a pure function of (seed, micro-batch, layer, site, element),
drawn with Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
1, 2, 3", SC'11), which both this oracle and the HIP path implement independently.

Format (shared by definition, not by code):
  * key     = (seed mod 2^32, seed div 2^32)
  * counter = (R div 4, C div 4, site + 256*layer, micro-batch) for element (row R, column C)
    of a site's matrix: one call covers a 4x4 patch of elements;
  * the element's byte is byte (C mod 4) (little end first) of output word (R mod 4);
  * thr = round(256 p); the element is kept iff byte >= thr and kept values are multiplied
    by 256 / (256 - thr)  (the drop probability is thr/256, p rounded to 8 bits).
Sites: 0 = attention probabilities (row = (batch*heads + head)*s + query, column = key),
1 = attention-output projection (+bias) before the residual add, 2 = MLP output (+bias)
before the residual add (row = token, column = hidden index).
"""
from __future__ import annotations

import numpy as np

SITE_ATTN, SITE_PROJ, SITE_MLP = 0, 1, 2
_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
_LOW = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds.  counter: 4 arrays (or ints) of 32-bit values, key: 2 ints.
    Returns 4 uint64 arrays holding 32-bit words."""
    c = [np.asarray(x, dtype=np.uint64) & _LOW for x in counter]
    k0, k1 = np.uint64(key[0]) & _LOW, np.uint64(key[1]) & _LOW
    for _ in range(10):
        p0 = _M0 * c[0]
        p1 = _M1 * c[2]
        c = [(p1 >> _S32) ^ c[1] ^ k0, p1 & _LOW, (p0 >> _S32) ^ c[3] ^ k1, p0 & _LOW]
        k0 = (k0 + _W0) & _LOW
        k1 = (k1 + _W1) & _LOW
    return c


class Dropout:
    def __init__(self, p: float, seed: int):
        self.thr = int(round(256.0 * p))
        if not 0 <= self.thr <= 255:
            raise ValueError("dropout probability must round to 0..255 / 256")
        self.seed = int(seed)
        self.scale = 256.0 / (256.0 - self.thr)

    def bytes(self, site: int, layer: int, mb: int, row0: int, n_rows: int, n_cols: int) -> np.ndarray:
        """The random byte of every element of rows row0..row0+n_rows-1, columns 0..n_cols-1."""
        R, C = np.meshgrid(np.arange(row0, row0 + n_rows, dtype=np.uint64), np.arange(n_cols, dtype=np.uint64), indexing="ij")
        four = np.uint64(4)
        words = philox4x32_10((R // four, C // four, np.uint64(site + 256 * layer), np.uint64(mb)),
                              (self.seed & 0xFFFFFFFF, self.seed >> 32))
        w = np.choose((R % four).astype(np.int64), words)
        return ((w >> (np.uint64(8) * (C % four))) & np.uint64(0xFF)).astype(np.int64)

    def keep_scale(self, site: int, layer: int, mb: int, row0: int, n_rows: int, n_cols: int) -> np.ndarray:
        """scale where the element is kept, 0 where it is dropped (float64)."""
        if self.thr == 0:
            return np.ones((n_rows, n_cols))
        return np.where(self.bytes(site, layer, mb, row0, n_rows, n_cols) >= self.thr, self.scale, 0.0)
