"""Weights of a 7B-13B-shaped model held as bf16 bit patterns and widened on access.

`make_weights(cfg, bits=True)` keeps a bf16 model as uint16 arrays (2 bytes per value: 13 GB at the
LLaVA-1.5-7B shapes).  A consumer that computes in float64 cannot hold the whole model widened (53 GB),
so `LazyWeights` presents the same dict-of-arrays structure and widens one tensor at a time, when it is
read: `w["layers"][i]["wq"]`, `w["lm_head"]`, ... each return a fresh float64 array with exactly the
values the bit patterns encode.  Pure data plumbing: no arithmetic of the method lives here.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_POOL = None


def _pool():
    global _POOL
    if _POOL is None:
        _POOL = ThreadPoolExecutor(max(1, min(16, os.cpu_count() or 1)))
    return _POOL


def widen_bf16_bits(bits, dtype=np.float64):
    """uint16 bf16 bit patterns -> array of `dtype` with the same values (exact), row chunks in parallel."""
    bits = np.ascontiguousarray(bits)
    assert bits.dtype == np.uint16
    out = np.empty(bits.shape, dtype)
    flat_in, flat_out = bits.reshape(-1), out.reshape(-1)
    n = flat_in.shape[0]
    step = max(1 << 20, (n + 15) // 16)

    def work(a):
        b = min(n, a + step)
        flat_out[a:b] = (flat_in[a:b].astype(np.uint32) << np.uint32(16)).view(np.float32)

    list(_pool().map(work, range(0, n, step)))
    return out


class _LazyDict:
    """Read-only mapping name -> widened tensor over a dict of uint16 arrays."""

    def __init__(self, bits):
        self._bits = bits

    def __getitem__(self, name):
        return widen_bf16_bits(self._bits[name])

    def __contains__(self, name):
        return name in self._bits

    def keys(self):
        return self._bits.keys()


class LazyWeights(_LazyDict):
    """The structure `make_weights` returns (embed, lm_head, final_norm, layers [N]{...}, draft_layer {...},
    fuse_w, resid_rho), over its bits=True form; every tensor read is widened to float64 on the spot."""

    def __init__(self, bits):
        super().__init__(bits)
        self._layers = [_LazyDict(l) for l in bits["layers"]]
        self._draft = _LazyDict(bits["draft_layer"])

    def __getitem__(self, name):
        if name == "layers":
            return self._layers
        if name == "draft_layer":
            return self._draft
        return super().__getitem__(name)
