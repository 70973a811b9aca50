"""Pins for WHERE the oracle's rounding mode "R" rounds (CPU only).

Mode R is the mode every integer decision of the bf16 path is compared in, so a rounding that
is misplaced, left out or of the wrong width must fail a test here.  The pins use a hand-sized
model (d_model 4, one head of dim 4, FFN 4, vocab 4, rms_eps 0) whose intermediate values are
chosen by hand:
  * every value dyadic and short  => no rounding point changes anything: mode R == mode E, bit
    for bit;
  * one value with a 2^-12 fraction planted at each projection input in turn (normalised
    activations of both norms and of the final norm, attention output, SwiGLU product): those
    inputs are carried as hi + lo halves (~22 bits), so mode R must follow mode E to 1e-6 where
    a single half would be 2.4e-4 off - and the same test fails when the pair rounding is
    swapped for a single half;
  * the coarse points must bite by exactly their step: new K/V entries are bfloat16 (library
    conversion of the exact values), the rotated Q is a single half (a planted quarter-ulp is
    dropped: mode R on the planted model equals mode E on the model without it), the soft-max
    probabilities are single halves relative to a power-of-two reference (a planted quarter-ulp
    in a probability is dropped);
  * the attention result does not depend on the order of the context keys.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import toolspec_oracle as O

I4 = np.eye(4)
E0 = np.array([1.0, 1.0, -1.0, 1.0])


def _cfg(theta=10000.0):
    return wl.ModelConfig("hand", 1, 4, 1, 1, 4, 4, 4, rope_theta=theta, rms_eps=0.0, dtype=wl.configs.DTYPE_BF16)


def _weights(**over):
    """Identity-like model: embedding rows +-E0, gains 1, Wv = Wo = I, everything else 0."""
    lay = dict(wq=np.zeros((4, 4)), wk=np.zeros((4, 4)), wv=I4.copy(), wo=I4.copy(),
               wg=np.zeros((4, 4)), wu=np.zeros((4, 4)), wd=np.zeros((4, 4)),
               norm1=np.ones(4), norm2=np.ones(4))
    w = dict(embed=np.stack([E0, -E0, E0, -E0]), lm_head=I4.copy(), norm_f=np.ones(4), layers=[lay])
    for k, v in over.items():
        if k in lay:
            lay[k] = np.asarray(v, np.float64)
        else:
            w[k] = np.asarray(v, np.float64)
    return w


def _kv(cfg, K=None, V=None, pending=0):
    P = 0 if K is None else K.shape[0]
    kv = O.OracleKV(cfg, P + 8)
    if P:
        kv.K[0, :P, 0, :] = K
        kv.V[0, :P, 0, :] = V
        kv.P = P
    kv.pending = pending
    return kv


def _run(w, kv, tok=(), par=(), mode="R", theta=10000.0):
    cfg = _cfg(theta)
    rows = O.tree_rows(kv.pending, np.asarray(tok, np.int32), np.asarray(par, np.int32))
    t, _, depth, vis = rows
    return O.forward_tree(O.OracleModel(cfg, w), kv, t, depth, vis, mode, return_hidden=True)


def test_all_dyadic_values_make_mode_R_equal_mode_E_bit_for_bit():
    # no context, root + star of children whose tokens repeat (or negate) the root's embedding:
    # every row sees 1 or 2 keys, all scores are 0 (K = 0), every norm's mean square is 1 or 4
    # (V = embedding, attention output = embedding or 0, residual = 2 x or x)
    w = _weights(wq=0.5 * I4, norm_f=[1.0, 0.25, 1.0, 4.0], lm_head=[[1, 2, 0, 0], [0, 1, 0, 0.5], [0, 0, 1, 0], [1, 1, 1, 1]])
    cfg = _cfg()
    outs = {m: _run(w, _kv(cfg), tok=[0, 1, 0], par=[-1, -1, -1], mode=m) for m in ("R", "E")}
    for a, b in zip(outs["R"], outs["E"]):
        assert np.array_equal(a, b)
    assert np.any(outs["R"][0] != 0) and np.any(outs["R"][2] != 0)      # logits and V rows are not trivially zero


def _planted_models():
    """(label, weights without the plant, weights with a 2^-12 fraction at one projection input)."""
    f = 1.0 + 2.0 ** -12
    out = []
    out.append(("pre-FFN norm", _weights(wg=64 * I4, wu=I4, wd=I4), _weights(wg=64 * I4, wu=I4, wd=I4, norm2=[f, 1, 1, 1])))
    out.append(("final norm", _weights(), _weights(norm_f=[f, 1, 1, 1])))
    # SwiGLU product: gate = 64 -> silu(64) = 64 exactly in float64, product = 64 * up
    out.append(("SwiGLU product", _weights(wg=64 * I4, wu=I4, wd=I4 / 16), _weights(wg=64 * I4, wu=I4 * f, wd=I4 / 16)))
    return out


@pytest.mark.parametrize("case", range(3))
def test_projection_inputs_keep_a_planted_2p12_fraction(case):
    label, w0, w1 = _planted_models()[case]
    cfg = _cfg()
    lE0 = _run(w0, _kv(cfg), mode="E")[0]
    lE1 = _run(w1, _kv(cfg), mode="E")[0]
    lR1 = _run(w1, _kv(cfg), mode="R")[0]
    signal = np.max(np.abs(lE1 - lE0)) / np.max(np.abs(lE0))
    assert signal > 5e-5, "%s: the plant does not reach the logits" % label
    err = np.max(np.abs(lR1 - lE1)) / np.max(np.abs(lE1))
    assert err < 1e-6, "%s: mode R lost the planted fraction (%.3g)" % (label, err)


def test_attention_output_keeps_a_planted_2p12_fraction():
    # 31 context keys with V = 1 and the root's own V = 1 + 2^-7 (a bfloat16 value): the uniform
    # soft-max over 32 keys gives an attention output of 1 + 2^-12 in dimension 0
    cfg = _cfg()
    Kc, Vc = np.zeros((31, 4)), np.ones((31, 4))
    w = _weights(wv=np.diag([1.0 + 2.0 ** -7, 1, 1, 1]), embed=np.ones((4, 4)))
    lE = _run(w, _kv(cfg, Kc, Vc), mode="E")[0]
    lR = _run(w, _kv(cfg, Kc, Vc), mode="R")[0]
    w_half = _weights(wv=I4, embed=np.ones((4, 4)))                       # what a single half would keep: 1.0
    lH = _run(w_half, _kv(cfg, Kc, Vc), mode="E")[0]
    assert np.max(np.abs(lE - lH)) / np.max(np.abs(lE)) > 5e-5
    assert np.max(np.abs(lR - lE)) / np.max(np.abs(lE)) < 1e-6


def test_pre_attention_activation_keeps_a_planted_2p12_fraction():
    # Behind this input sit only 16-bit roundings (Q, K, V), so the plant is read off the new V
    # entry: the activation 1 + 2^-8 + 2^-12 lies just above the bfloat16 tie 1 + 2^-8 and must
    # round UP to 1 + 2^-7; a single half would have dropped the 2^-12, hit the tie and gone to 1.
    cfg = _cfg()
    w = _weights(norm1=[1.0 + 2.0 ** -8 + 2.0 ** -12, 1, 1, 1])
    newV = _run(w, _kv(cfg), mode="R")[2]
    assert newV[0, 0, 0, 0] == 1.0 + 2.0 ** -7
    assert np.array_equal(newV[0, 0, 0, 1:], E0[1:])


def test_the_pins_above_fail_when_projection_inputs_are_single_halves(monkeypatch):
    monkeypatch.setattr(O, "fp16_pair_round", O.fp16_act_round)
    for case in range(3):
        with pytest.raises(AssertionError):
            test_projection_inputs_keep_a_planted_2p12_fraction(case)
    with pytest.raises(AssertionError):
        test_attention_output_keeps_a_planted_2p12_fraction()
    with pytest.raises(AssertionError):
        test_pre_attention_activation_keeps_a_planted_2p12_fraction()


def test_pair_rounding_is_hi_plus_lo_of_library_halves():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 5, 4000), [0.0, 65504.0, 7.0e4, -1.0e6, 1028.25 + 2.0 ** -13]])
    xs = torch.from_numpy(np.clip(x, -65504.0, 65504.0))
    hi = xs.to(torch.float32).to(torch.float16).to(torch.float64)
    lo = (xs - hi).to(torch.float32).to(torch.float16).to(torch.float64)
    assert np.array_equal(O.fp16_pair_round(x), (hi + lo).numpy())
    # 11 + 11 bits: a 24-bit value loses its last bit, a 22-bit value none
    assert O.fp16_pair_round(np.array([1028.25 + 2.0 ** -13]))[0] == 1028.25
    assert O.fp16_pair_round(np.array([1028.25 + 2.0 ** -11]))[0] == 1028.25 + 2.0 ** -11
    assert np.array_equal(O.fp16_pair_round(np.array([7.0e4, -1.0e6])), [65504.0, -65504.0])


def test_new_kv_entries_are_bfloat16_of_the_exact_values():
    # layer 0 of a random small model: upstream of K and V only the pair-rounded normalised
    # activation differs between the modes (2^-22), so mode R's new K/V must be the library's
    # bfloat16 conversion of mode E's
    cfg = wl.get_config("small_bf16_hd64")
    w = wl.gen_weights(cfg, 77)
    K, V = wl.gen_context_kv(cfg, 9, seed=5)
    rng = np.random.default_rng(2)
    tokd, par = wl.bfs_tree([], 12, cfg.vocab, rng)
    out = {}
    for mode in ("R", "E"):
        kv = O.OracleKV(cfg, 40)
        kv.import_context(K, V)
        kv.pending = 5
        tok, _, depth, vis = O.tree_rows(5, tokd, par)
        out[mode] = O.forward_tree(O.OracleModel(cfg, w), kv, tok, depth, vis, mode)
    for i in (1, 2):
        ref = torch.from_numpy(out["E"][i][0]).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
        got = out["R"][i][0]
        assert np.mean(got != ref) < 2e-3                    # a value within 2^-22 of a bf16 tie may land on the other side
        assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-30)) <= 2.0 ** -7
        assert np.any(out["E"][i][0] != ref)                 # mode E does not round them


def _two_key_case(q1, k1, k3=0.0):
    """One context key and the root (whose own key is 0, so its score is 0); RoPE switched off
    in effect (theta 1e30 and only the second rotation pair, whose angle is 1e-15 rad, carries q
    and k).  q = (0, q1, 0, 1), context key = (0, k1, 0, k3), context V = (3, 0, 0, 0), root V = 0.
    Returns weights, K, V."""
    wq = np.zeros((4, 4)); wq[1, 1] = q1; wq[3, 3] = 1.0     # xn = E0: xn1 = xn3 = 1
    Kc = np.zeros((1, 4)); Kc[0, 1] = k1; Kc[0, 3] = k3
    Vc = np.array([[3.0, 0.0, 0.0, 0.0]])
    return _weights(wq=wq, wv=I4 * 0.0), Kc, Vc


def test_rotated_q_is_a_single_half():
    # q = (q1, 1) with q1 = 1 + 2^-12 (a quarter of a half ulp) against the key (2^13, -2^13): the
    # score is (q1 - 1) * 2^13 / sqrt(4) = 1 unless Q is rounded to half first, which makes it 0.
    # Mode R on the planted model must equal mode E on the model with q1 = 1, and differ grossly
    # from mode E on the planted one.
    cfg = _cfg(1e30)
    wR, Kc, Vc = _two_key_case(1.0 + 2.0 ** -12, 2.0 ** 13, -2.0 ** 13)
    wE, _, _ = _two_key_case(1.0, 2.0 ** 13, -2.0 ** 13)
    run = lambda w, m: _run(w, _kv(cfg, Kc, Vc), mode=m, theta=1e30)[0]
    lR, lE_round, lE_plant = run(wR, "R"), run(wE, "E"), run(wR, "E")
    # (the probabilities themselves are rounded to half in mode R: 2^-11 relative)
    assert np.max(np.abs(lR - lE_round)) < 1e-3 * np.max(np.abs(lE_round))
    assert np.max(np.abs(lE_plant - lE_round)) > 0.05 * np.max(np.abs(lE_round))


def test_probabilities_are_single_halves_relative_to_a_power_of_two():
    # root key scores 0 (K = 0); one context key whose score in log2 units is log2(0.5 (1 + 2^-12)):
    # mode R rounds that probability to exactly 0.5, so the attention output is (1 * v_root +
    # 0.5 * v_ctx) / 1.5 with v_root = 0; mode E keeps 0.5 (1 + 2^-12)
    cfg = _cfg(1e30)
    t_target = np.log2(0.5 * (1.0 + 2.0 ** -12))
    scale = 0.5 * O.LOG2E                                    # 1/sqrt(hd) * log2(e)
    w, Kc, Vc = _two_key_case(1.0, t_target / scale)
    w["layers"][0]["wo"] = I4.copy()
    kvR, kvE = _kv(cfg, Kc, Vc), _kv(cfg, Kc, Vc)
    tok, _, depth, vis = O.tree_rows(0, np.zeros(0, np.int32), np.zeros(0, np.int32))
    m = O.OracleModel(cfg, w)
    xR = O.forward_tree(m, kvR, tok, depth, vis, "R", return_hidden=True)
    xE = O.forward_tree(m, kvE, tok, depth, vis, "E", return_hidden=True)
    # residual after the layer = embedding + attention output (FFN is off); undo the final norm
    # through the ratio of two coordinates: x0 / x1 = (e0 + a0) / e1 with e = E0, a0 = p/(1+p) * 3
    ratio = lambda out: out[3][0, 0] / out[3][0, 1]
    pR, pE = 0.5, 0.5 * (1.0 + 2.0 ** -12)
    assert abs(ratio(xR) - (1.0 + 3.0 * pR / (1.0 + pR))) < 1e-6
    assert abs(ratio(xE) - (1.0 + 3.0 * pE / (1.0 + pE))) < 1e-12
    assert abs(ratio(xR) - ratio(xE)) > 5e-5


def test_attention_does_not_depend_on_the_order_of_context_keys():
    cfg = wl.get_config("small_bf16_hd64")
    w = wl.gen_weights(cfg, 78)
    K, V = wl.gen_context_kv(cfg, 37, seed=6)
    perm = np.random.default_rng(4).permutation(37)
    outs = []
    for Kx, Vx in ((K, V), (K[:, perm], V[:, perm])):
        kv = O.OracleKV(cfg, 60)
        kv.import_context(Kx, Vx)
        kv.pending = 3
        tok, _, depth, vis = O.tree_rows(3, np.array([5, 6], np.int32), np.array([-1, 0], np.int32))
        outs.append(O.forward_tree(O.OracleModel(cfg, w), kv, tok, depth, vis, "R")[0])
    assert np.max(np.abs(outs[0] - outs[1])) < 1e-9 * np.max(np.abs(outs[0]))
