"""Context ingestion through the verification kernels (ts_prefill) against the oracle.

The plain definition of the context's K/V is a causal forward pass over the prompt; the dense
causal decoder (oracle/dense_causal.py) computes it directly.  The device ingests the same
prompt as causal chains of up to 65 rows.  Checked: the cache contents, a tree verification on
top of the ingested context, continuation of an ingestion in pieces, and a speculative decode
after it that must reproduce the plain greedy stream (the lossless invariant, paper Sec. 5.1).
"""
import numpy as np
import pytest

import workloads as wl
from oracle import toolspec_oracle as O
from oracle import dense_causal as D
from paper_2604_13519_amd import binding as B

import gpu_utils as U

pytestmark = pytest.mark.gpu


def _oracle_ingest(cfg, omodel, okv, seq, mode):
    """Oracle side of the ingestion: one tree-masked pass over the whole sequence as a chain
    (rows are independent of how a chain is cut into passes), all rows kept."""
    seq = [int(t) for t in seq]
    n = len(seq) - 1
    tok, par, depth, vis = O.tree_rows(seq[0], np.asarray(seq[1:n], np.int32), np.arange(-1, n - 2, dtype=np.int32))
    _, newK, newV = O.forward_tree(omodel, okv, tok, depth, vis, mode)
    okv.K[:, okv.P:okv.P + n] = newK
    okv.V[:, okv.P:okv.P + n] = newV
    okv.P += n
    okv.pending = seq[-1]


@pytest.mark.parametrize("cfg_name,n_prompt", [("small_fp32", 300), ("small_bf16", 300), ("small_bf16_hd64", 131),
                                                 ("small_bf16", 1100), ("small_fp32", 577), ("small_bf16", 2300)])
def test_prefill_cache_matches_causal_forward_and_supports_verify(cfg_name, n_prompt):
    cfg, w, model, omodel = U.get_model(cfg_name)
    fp32 = cfg.dtype == wl.configs.DTYPE_F32
    rng = np.random.default_rng([55, n_prompt])
    prompt = rng.integers(cfg.vocab, size=n_prompt).astype(np.int32)
    cap = n_prompt + 80
    kv = B.ts_kv_alloc(model, cap)
    try:
        # in two pieces: the second call continues from the pending token the first one left
        cut = 97
        B.ts_prefill(model, kv, prompt[:cut])
        assert B.ts_kv_len(kv) == cut - 1
        B.ts_prefill(model, kv, prompt[cut:])
        P = n_prompt - 1
        assert B.ts_kv_len(kv) == P
        gk, gv = B.ts_kv_export(kv, 0, P, cfg)
        if not fp32:
            gk, gv = wl.bf16_bits_to_f32(gk), wl.bf16_bits_to_f32(gv)
        _, K, V = D.causal_forward(cfg, w, prompt[:-1], return_kv=True)
        tol = 1e-5 if fp32 else 1e-2
        ek, ev = U.rel_l2(gk, K), U.rel_l2(gv, V)
        print("%s prefill %d tokens: K %.3g V %.3g vs dense causal forward" % (cfg_name, n_prompt, ek, ev))
        assert ek <= tol and ev <= tol, "prefilled K/V vs causal forward: %.3g %.3g" % (ek, ev)

        # a verification on top of it, against the oracle's own ingestion of the same prompt
        okv = O.OracleKV(cfg, cap)
        _oracle_ingest(cfg, omodel, okv, prompt, "E" if fp32 else "R")
        greedy = D.greedy_sequence(cfg, w, prompt, 12)
        tok, par = wl.bfs_tree(greedy, 40, cfg.vocab, rng)
        res, oR = U.check_verify(cfg, model, omodel, kv, okv, tok, par, check_kv=False, label=cfg_name + " after prefill")
        U.commit_both(cfg, kv, okv, res, oR)
    finally:
        B.ts_kv_free(kv)


@pytest.mark.parametrize("cfg_name", ["small_fp32", "small_bf16"])
def test_prefill_then_speculative_decode_is_lossless(cfg_name):
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(77)
    prompt = rng.integers(cfg.vocab, size=150).astype(np.int32)
    n_new = 40
    plain = D.greedy_sequence(cfg, w, prompt, n_new)      # the target's own greedy continuation
    # steps whose top-2 margin is tiny may legitimately differ: compare up to the first one
    logits = D.causal_forward(cfg, w, np.concatenate([prompt, np.asarray(plain[:-1], np.int32)]))
    top2 = np.sort(np.asarray(logits)[len(prompt) - 1:], axis=1)[:, -2:]
    safe = n_new
    for i in range(n_new):
        if top2[i, 1] - top2[i, 0] < U.MARGIN:
            safe = i
            break
    if safe < 8:
        pytest.skip("greedy stream has a near-tie within the first 8 tokens")
    kv = B.ts_kv_alloc(model, len(prompt) + n_new + 80)
    try:
        B.ts_prefill(model, kv, prompt)
        out = []
        while len(out) < n_new:
            k = len(out)
            tok, par = wl.chain_tree(plain[k:] + [0] * 16, 12, 0.25, cfg.vocab, rng)
            l, acc, _, bonus = B.ts_verify(model, kv, tok, par)
            B.ts_kv_commit(kv)
            out += acc + [bonus]
        assert out[:safe] == plain[:safe], "speculative stream %r != greedy %r" % (out[:safe], plain[:safe])
        assert B.ts_kv_len(kv) == len(prompt) - 1 + len(out)
    finally:
        B.ts_kv_free(kv)


def test_prefill_error_paths_leave_state_untouched():
    cfg, w, model, omodel = U.get_model("small_fp32")
    kv = B.ts_kv_alloc(model, 64)
    try:
        with pytest.raises(B.TsError) as e:
            B.ts_prefill(model, kv, np.arange(70, dtype=np.int32))          # 69 rows + 1 > 64
        assert e.value.status == B.TS_ERR_KV_CAPACITY
        with pytest.raises(B.TsError) as e:
            B.ts_prefill(model, kv, np.asarray([1, cfg.vocab], np.int32))
        assert e.value.status == B.TS_ERR_TOKEN_RANGE
        assert B.ts_kv_len(kv) == 0
        B.ts_prefill(model, kv, np.asarray([5], np.int32))                  # a single token only becomes pending
        assert B.ts_kv_len(kv) == 0
        l, acc, nodes, bonus = B.ts_verify(model, kv, [], [])
        assert l == 0 and 0 <= bonus < cfg.vocab
    finally:
        B.ts_kv_free(kv)


@pytest.mark.parametrize("cfg_name", ["small_fp32", "small_bf16"])
def test_last_token_hidden_state_for_retrieval(cfg_name):
    """h_x of Sec. 4.3: the final hidden state at the question's last token = row 0 of the first pass
    after the question was ingested; also every other row of a tree pass."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    fp32 = cfg.dtype == wl.configs.DTYPE_F32
    rng = np.random.default_rng(31)
    prompt = rng.integers(cfg.vocab, size=90).astype(np.int32)
    kv = B.ts_kv_alloc(model, 200)
    try:
        with pytest.raises(B.TsError):
            B.ts_prefill(model, kv, prompt)
            B.ts_get_hidden(model, 0, cfg.d_model)            # no verify yet: nothing to export
        okv = O.OracleKV(cfg, 200)
        mode = "E" if fp32 else "R"
        _oracle_ingest(cfg, omodel, okv, prompt, mode)
        tok, par = wl.bfs_tree([], 20, cfg.vocab, rng)
        B.ts_verify(model, kv, tok, par)
        rows = O.tree_rows(okv.pending, tok, par)
        _, _, _, hid = O.forward_tree(omodel, okv, rows[0], rows[2], rows[3], mode, return_hidden=True)
        tol = 1e-5 if fp32 else 1e-2
        errs = [U.rel_l2(B.ts_get_hidden(model, r, cfg.d_model), hid[r]) for r in range(len(tok) + 1)]
        print("%s hidden-state export: max rel L2 %.3g" % (cfg_name, max(errs)))
        assert max(errs) <= tol
        with pytest.raises(B.TsError) as e:
            B.ts_get_hidden(model, len(tok) + 1, cfg.d_model)
        assert e.value.status == B.TS_ERR_STATE
    finally:
        B.ts_kv_free(kv)
