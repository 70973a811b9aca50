"""Random-init weights: every matrix N(0, 0.02) from a seed, row-major [out][in].

For bf16 models the float32 draw is rounded once to bfloat16 and those rounded
values *are* the model; arrays are returned as uint16 bit patterns.  For fp32
models arrays are float32.  Norm gains are ones (or 1 + 0.1 N(0,1) when the
config asks for random gains, so tests notice a missing or swapped gain).
"""
import numpy as np

from .configs import DTYPE_BF16
from .rng import normal_f32, f32_to_bf16_bits

# kind -> small integer used in the tensor uid
TENSOR_KINDS = {"embed": 0, "lm_head": 1, "norm_f": 2,
                "wq": 3, "wk": 4, "wv": 5, "wo": 6, "wg": 7, "wu": 8, "wd": 9,
                "norm1": 10, "norm2": 11}
LAYER_KINDS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "norm1", "norm2")
GLOBAL_KINDS = ("embed", "lm_head", "norm_f")


def tensor_shapes(cfg):
    """kind -> shape ([out][in] for matrices)."""
    d, F, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    return {"embed": (V, d), "lm_head": (V, d), "norm_f": (d,),
            "wq": (cfg.q_dim, d), "wk": (cfg.kv_dim, d), "wv": (cfg.kv_dim, d),
            "wo": (d, cfg.q_dim), "wg": (F, d), "wu": (F, d), "wd": (d, F),
            "norm1": (d,), "norm2": (d,)}


def _uid(kind, layer):
    return TENSOR_KINDS[kind] + 16 * (layer + 1)


def gen_tensor(cfg, seed, kind, layer=-1, std=0.02):
    """One tensor.  `layer` is -1 for the three global tensors."""
    shape = tensor_shapes(cfg)[kind]
    if kind.startswith("norm"):
        if cfg.norm_init == "ones":
            x = np.ones(shape, dtype=np.float32)
        else:
            x = (1.0 + 0.1 * normal_f32(seed, _uid(kind, layer), shape)).astype(np.float32)
    else:
        x = normal_f32(seed, _uid(kind, layer), shape, std=std)
    if cfg.dtype == DTYPE_BF16:
        return f32_to_bf16_bits(x)
    return x


def gen_layer(cfg, seed, layer):
    return {k: gen_tensor(cfg, seed, k, layer) for k in LAYER_KINDS}


def gen_weights(cfg, seed=1234):
    """All tensors: {"embed", "lm_head", "norm_f", "layers": [ {kind: arr}, ... ]}."""
    w = {k: gen_tensor(cfg, seed, k) for k in GLOBAL_KINDS}
    w["layers"] = [gen_layer(cfg, seed, l) for l in range(cfg.n_layers)]
    return w
