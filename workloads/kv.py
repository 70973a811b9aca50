"""Synthetic context K/V: N(0,1) entries in the model's storage dtype.

Stands in for the K/V a real prefill of the context would have produced at
shapes where a CPU prefill is out of reach.  Layout [layer][position][kv_head][head_dim].
"""
import numpy as np

from .configs import DTYPE_BF16
from .rng import normal_f32, f32_to_bf16_bits


def gen_context_kv(cfg, n_pos, seed=2345, layers=None):
    """Returns (K, V), each [L][n_pos][Hkv][hd]; uint16 bf16 bits or float32."""
    L = cfg.n_layers if layers is None else layers
    shape = (n_pos, cfg.n_kv_heads, cfg.head_dim)
    dt = np.uint16 if cfg.dtype == DTYPE_BF16 else np.float32
    K = np.empty((L,) + shape, dtype=dt)
    V = np.empty((L,) + shape, dtype=dt)
    for l in range(L):
        k = normal_f32(seed, 2 * l, shape)
        v = normal_f32(seed, 2 * l + 1, shape)
        if cfg.dtype == DTYPE_BF16:
            K[l] = f32_to_bf16_bits(k)
            V[l] = f32_to_bf16_bits(v)
        else:
            K[l] = k
            V[l] = v
    return K, V
