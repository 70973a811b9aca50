"""Textbook causal decoder over a whole token sequence.  TEST INFRASTRUCTURE ONLY.

An independently written second reference: no K/V cache, no tree, no mask
bookkeeping - a token sequence goes in, every position attends to itself and
everything before it, logits for every position come out.  It exists to
brute-force the defining property of tree verification (paper App. A.1, Sec.
4.1): the scores a tree node gets in the single masked pass must equal the
scores it would get if context + root + its root-to-node path were decoded as
an ordinary sequence.  It also serves as the real prefill that produces K/V
for small models.

Written with PyTorch CPU library routines in float64 (linear, rms_norm,
scaled_dot_product_attention with is_causal=True, silu) and a complex-number
formulation of the rotary embedding, so that it shares neither code nor
formulation with toolspec_oracle.py.
"""
import numpy as np
import torch
import torch.nn.functional as F


def _t(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:                      # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64)
    return torch.from_numpy(a.astype(np.float64))


def _rotary(x, positions, theta):
    """x: [T][H][hd].  Treat (x_j, x_{j+hd/2}) as a complex number and multiply it
    by exp(i * pos * theta^(-2j/hd))."""
    hd = x.shape[-1]
    half = hd // 2
    freqs = torch.pow(torch.tensor(theta, dtype=torch.float64),
                      -torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = torch.outer(positions.to(torch.float64), freqs)             # [T][half]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    z = torch.complex(x[..., :half], x[..., half:]) * rot
    return torch.cat([z.real, z.imag], dim=-1)


@torch.no_grad()
def causal_forward(cfg, weights, tokens, return_kv=False):
    """Logits [T][V] (float64 numpy) for a token sequence; optionally the per-layer
    rotated K and V, each [L][T][Hkv][hd]."""
    tokens = torch.as_tensor(np.asarray(tokens, dtype=np.int64))
    T = tokens.shape[0]
    pos = torch.arange(T)
    Hq, Hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    x = _t(np.asarray(weights["embed"])[tokens.numpy()])
    Ks, Vs = [], []
    for lw in weights["layers"]:
        h = F.rms_norm(x, (cfg.d_model,), _t(lw["norm1"]), cfg.rms_eps)
        q = F.linear(h, _t(lw["wq"])).view(T, Hq, hd)
        k = F.linear(h, _t(lw["wk"])).view(T, Hkv, hd)
        v = F.linear(h, _t(lw["wv"])).view(T, Hkv, hd)
        q, k = _rotary(q, pos, cfg.rope_theta), _rotary(k, pos, cfg.rope_theta)
        Ks.append(k.numpy().copy())
        Vs.append(v.numpy().copy())
        ke = k.repeat_interleave(Hq // Hkv, dim=1)
        ve = v.repeat_interleave(Hq // Hkv, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), ke.transpose(0, 1),
                                           ve.transpose(0, 1), is_causal=True)
        x = x + F.linear(a.transpose(0, 1).reshape(T, Hq * hd), _t(lw["wo"]))
        h = F.rms_norm(x, (cfg.d_model,), _t(lw["norm2"]), cfg.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, _t(lw["wg"]))) * F.linear(h, _t(lw["wu"])),
                         _t(lw["wd"]))
    h = F.rms_norm(x, (cfg.d_model,), _t(weights["norm_f"]), cfg.rms_eps)
    logits = F.linear(h, _t(weights["lm_head"])).numpy()
    if return_kv:
        return logits, np.stack(Ks), np.stack(Vs)
    return logits


def greedy_sequence(cfg, weights, prompt, n_tokens):
    """Plain greedy decoding by re-running the whole sequence each step."""
    seq = list(int(t) for t in prompt)
    out = []
    for _ in range(n_tokens):
        lg = causal_forward(cfg, weights, seq)
        nxt = int(np.argmax(lg[-1]))
        out.append(nxt)
        seq.append(nxt)
    return out
