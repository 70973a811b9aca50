"""Seeded random draws and bf16 <-> fp32 bit conversion for synthetic inputs.

Every tensor is drawn block by block from its own Philox stream keyed by
(seed, tensor uid, block index), so the result does not depend on how many
threads draw it and any block can be regenerated on its own.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_BLOCK = 1 << 22   # elements per independently keyed block


def _draw_block(seed, uid, blk, count):
    ss = np.random.SeedSequence([int(seed), int(uid), int(blk)])
    gen = np.random.Generator(np.random.Philox(ss))
    return gen.standard_normal(count, dtype=np.float32)


def normal_f32(seed, uid, shape, std=1.0, threads=None):
    """N(0, std) samples as float32, shape `shape`, deterministic in (seed, uid)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    nblk = (n + _BLOCK - 1) // _BLOCK
    if threads is None:
        threads = min(16, os.cpu_count() or 1)

    def work(b):
        lo = b * _BLOCK
        hi = min(n, lo + _BLOCK)
        out[lo:hi] = _draw_block(seed, uid, b, hi - lo)

    if nblk > 1 and threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, range(nblk)))
    else:
        for b in range(nblk):
            work(b)
    if std != 1.0:
        out *= np.float32(std)
    return out.reshape(shape)


def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (nearest even); returns the 16-bit patterns."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(u):
    """Exact widening of bfloat16 bit patterns to float32."""
    u = np.ascontiguousarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << np.uint32(16)).view(np.float32)
