"""Shared helpers of the GPU parity tests: build the same model / cache / tree on the
HIP library and in the CPU oracle, and compare them under the stated rules.

Rules (floating point).  The CONTRACT: logits relative L2 <= 1e-5 on the fp32 path and
<= 2e-2 on the bf16 path, both against the oracle's exact float64 mode "E".  A CANARY on top of
it, self-imposed: <= 3e-3 against the rounding-emulating mode "R" (same 16-bit rounding points,
float64 accumulation) - most rows agree to ~1e-6 there; what remains are sparse one-step flips
of a 16-bit value (a new bf16 K/V entry, a half Q entry or probability within 1e-7 of a
rounding boundary lands on the other side in fp32).  It is tighter than the contract so that a
misplaced rounding on the device shows long before the contract breaks.  Integers (accept length, tokens,
node ids, bonus, cache layout) are bit-exact against mode "R" (fp32: mode "E"), except
that a row whose oracle top-2 logit margin is below 1e-2 may pick the runner-up; every
arg-max disagreement must be such a row and the walk must be exact given the arg-maxes.
"""
import numpy as np

import workloads as wl
from oracle import toolspec_oracle as O
from paper_2604_13519_amd import binding as B

MARGIN = 1e-2
TOL_F32 = 1e-5
TOL_BF16_E = 2e-2      # the contract (vs mode E)
TOL_BF16_R = 3e-3      # canary (vs mode R)

_models = {}


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def get_model(cfg_name, wseed=1234, weights=None):
    """(cfg, weights, device model handle, oracle model), cached per (config, seed)."""
    key = (cfg_name, wseed)
    if key not in _models:
        cfg = wl.get_config(cfg_name)
        w = weights if weights is not None else wl.gen_weights(cfg, wseed)
        print("[gpu_utils] loading %s (seed %d)" % (cfg_name, wseed), flush=True)
        m = B.ts_model_load(cfg, w)
        B.ts_model_keep_logits(m, True)
        _models[key] = (cfg, w, m, O.OracleModel(cfg, w, cache=True))
    return _models[key]


def drop_model(cfg_name, wseed=1234):
    key = (cfg_name, wseed)
    if key in _models:
        B.ts_model_free(_models[key][2])
        del _models[key]


def make_pair(cfg, model, K, V, pending, capacity=None, page_perm=None):
    """Device cache + oracle cache holding the same context K/V and pending token."""
    P = K.shape[1]
    cap = capacity or (P + 80)
    kv = B.ts_kv_alloc(model, cap)
    if page_perm is not None:
        B.ts_kv_set_page_table(kv, page_perm)
    if P > 0:
        B.ts_kv_import(kv, K, V)
    B.ts_set_pending(kv, pending)
    okv = O.OracleKV(cfg, cap)
    if P > 0:
        okv.import_context(K, V)
    okv.pending = int(pending)
    return kv, okv


def tolerances(cfg):
    return (TOL_F32, TOL_F32) if cfg.dtype == wl.configs.DTYPE_F32 else (TOL_BF16_E, TOL_BF16_R)


def check_verify(cfg, model, omodel, kv, okv, tok, par, check_kv=True, label=""):
    """One ts_verify against the oracle.  Returns (gpu result tuple, oracle result in
    the decision mode)."""
    fp32 = cfg.dtype == wl.configs.DTYPE_F32
    n = len(tok)
    M = n + 1
    P = B.ts_kv_len(kv)
    assert P == okv.P
    res = B.ts_verify(model, kv, tok, par)
    glog = B.ts_get_logits(model, 0, M, cfg.vocab).astype(np.float64)
    oR = O.verify(omodel, okv, tok, par, "E" if fp32 else "R")
    tolE, tolR = tolerances(cfg)
    errR = max(rel_l2(glog[r], oR.logits[r]) for r in range(M))
    print("%s: M=%d P=%d logits vs decision-mode oracle %.3g (min decisive margin %.3g)" % (label, M, P, errR, oR.decisive_margin))
    errE = None
    if not fp32:
        oE = O.verify(omodel, okv, tok, par, "E")
        errE = max(rel_l2(glog[r], oE.logits[r]) for r in range(M))
        print("%s: logits vs exact oracle %.3g; mode R vs mode E %.3g" % (
            label, errE, max(rel_l2(oR.logits[r], oE.logits[r]) for r in range(M))))
    assert errR <= tolR, "%s logits vs decision-mode oracle: rel L2 %.3g > %.3g" % (label, errR, tolR)
    if errE is not None:
        assert errE <= tolE, "%s logits vs exact oracle: rel L2 %.3g > %.3g" % (label, errE, tolE)
    # integer decisions: the tokens the fused lm_head epilogue decided on are the arg-max of the logits
    g_gpu = np.argmax(glog, axis=1)
    assert np.array_equal(B.ts_get_row_tokens(model, 0, M), g_gpu), "%s fused arg-max != arg-max of the stored logits" % label
    tokr, parr, depth, _ = oR.rows
    for r in np.nonzero(g_gpu != oR.greedy)[0]:
        assert oR.margin[r] < MARGIN, "%s row %d arg-max differs with oracle margin %.4g" % (label, r, oR.margin[r])
    best, path, _ = O.accept_walk(g_gpu, tokr, parr, depth)
    l, acc_t, acc_n, bonus = res
    assert l == len(path), "%s accept_len %d != walk over device arg-maxes %d" % (label, l, len(path))
    assert acc_n == [p - 1 for p in path] and acc_t == [int(tokr[p]) for p in path]
    assert bonus == int(g_gpu[best])
    if np.array_equal(g_gpu, oR.greedy):
        assert (l, acc_t, acc_n, bonus) == (oR.accept_len, oR.accepted_tokens, oR.accepted_nodes, oR.bonus_token)
    if check_kv:
        gk, gv = B.ts_kv_export(kv, P, M, cfg)
        if not fp32:
            gk, gv = wl.bf16_bits_to_f32(gk), wl.bf16_bits_to_f32(gv)
        tol = 1e-5 if fp32 else 3e-3      # bf16 entries: one-step flips of single elements allowed (canary, as above)
        assert rel_l2(gk, oR.newK) <= tol, "%s tree K rows: %.3g" % (label, rel_l2(gk, oR.newK))
        assert rel_l2(gv, oR.newV) <= tol, "%s tree V rows: %.3g" % (label, rel_l2(gv, oR.newV))
    return res, oR


def commit_both(cfg, kv, okv, res, oR):
    """Commit on both sides; the device's moved rows must be bitwise the rows it had in the
    tree slots, and the committed lengths must agree when the decisions agreed."""
    l, acc_t, acc_n, bonus = res
    P = B.ts_kv_len(kv)
    M = len(oR.rows[0])
    pre_k, pre_v = B.ts_kv_export(kv, P, M, cfg)
    B.ts_kv_commit(kv)
    assert B.ts_kv_len(kv) == P + l + 1
    post_k, post_v = B.ts_kv_export(kv, P, l + 1, cfg)
    rows = [0] + [a + 1 for a in acc_n]
    assert np.array_equal(post_k, pre_k[:, rows]) and np.array_equal(post_v, pre_v[:, rows])
    same = (l, acc_t, acc_n, bonus) == (oR.accept_len, oR.accepted_tokens, oR.accepted_nodes, oR.bonus_token)
    if same:
        O.commit(okv, oR)
    return same
