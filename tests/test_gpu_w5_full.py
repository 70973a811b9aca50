"""Workload 5 at FULL depth: the 32B-class decoder (64 layers, d_model 5120, 64 query / 8 KV
heads, FFN 25600, vocab 151936; 64 GB of weights on the device), 4 requests over 32768-token
contexts with shuffled page tables, a 64-node schema tree each, one batched pass of 260 rows.

The CPU oracle needs minutes per pass at this size, so its results for one request are stored in
tests/golden/w5_expected.txt by tests/golden/make_w5_expected.py (which calls only the oracle
and the seeded generators): a short greedy continuation the request's tree is built from (so
part of the tree is accepted and the commit moves rows), and for all 65 rows the arg-max token,
the top-2 margin and the logits at a fixed sample of vocabulary ids, in the decision mode R and
in the exact mode E.  Checked here, for that request: logits on the sample (contract 2e-2 vs
mode E, canary vs mode R), every row's fused arg-max (differences only at oracle margins below
1e-2), the accepted path, bonus token and the compaction; for all four requests: the batched
pass decides exactly what a single-sequence pass over the same cache decides.
"""
import os
import time

import numpy as np
import pytest

import workloads as wl
from oracle import toolspec_oracle as O
from paper_2604_13519_amd import binding as B

import gpu_utils as U

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "w5_expected.txt")
REQ, P = 1, 32768


def _load_golden():
    g = {"rows": {}}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(" ", 1)
        if key in ("greedy", "tree_tokens", "tree_parents"):
            g[key] = [int(x) for x in rest.split()]
        elif key in ("result_R", "result_E"):
            l, bonus, nodes, toks = rest.split()
            g[key] = (int(l), [int(x) for x in toks.split(",")] if toks != "-" else [],
                      [int(x) for x in nodes.split(",")] if nodes != "-" else [], int(bonus))
        elif key == "row":
            head, ids, lr, le = rest.split(" | ")
            r, gR, mR, gE, mE = head.split()
            g["rows"][int(r)] = (int(gR), float(mR), int(gE), float(mE), np.array(ids.split(), np.int64),
                                 np.array(lr.split(), np.float64), np.array(le.split(), np.float64))
    return g


def test_qwen32b_full_depth_batch4_ctx32768_against_stored_oracle_results():
    assert os.path.exists(GOLDEN), "stored oracle results missing: run tests/golden/make_w5_expected.py"
    gold = _load_golden()
    cfg = wl.get_config("qwen32b")
    t0 = time.time()
    tok_g, par_g = wl.schema_retrieval_tree(gold["greedy"], cfg.vocab, np.random.default_rng([3456, 5, REQ]))
    assert tok_g.tolist() == gold["tree_tokens"] and par_g.tolist() == gold["tree_parents"], "tree recipe drifted from the stored one"
    model = B.ts_model_load(cfg, wl.gen_weights(cfg, 1234))
    B.ts_model_keep_logits(model, True)
    print("w5 full depth: model resident (%.0f s)" % (time.time() - t0), flush=True)
    kvs, trees = [], []
    try:
        for b in range(4):
            K, V = wl.gen_context_kv(cfg, P, seed=2345 + b)
            kv = B.ts_kv_alloc(model, P + 80)
            B.ts_kv_set_page_table(kv, np.random.default_rng([777, b]).permutation((P + 80 + 15) // 16).astype(np.int32))
            B.ts_kv_import(kv, K, V)
            del K, V
            B.ts_set_pending(kv, wl.root_token(cfg.vocab, P, seed=3456 + b))
            kvs.append(kv)
            trees.append((tok_g, par_g) if b == REQ else
                         wl.schema_retrieval_tree([], cfg.vocab, np.random.default_rng([3456, 5, b])))
            print("w5 full depth: request %d resident (%.0f s)" % (b, time.time() - t0), flush=True)

        batch = B.ts_verify_batch(model, kvs, trees)
        row0 = sum(len(t[0]) + 1 for t in trees[:REQ])
        M = len(tok_g) + 1
        blog = B.ts_get_logits(model, row0, M, cfg.vocab).astype(np.float64)
        brow = B.ts_get_row_tokens(model, row0, M)
        all_rows = B.ts_get_row_tokens(model, 0, sum(len(t[0]) + 1 for t in trees))
        print("w5 full depth: batched pass done (%.0f s)" % (time.time() - t0), flush=True)

        # ---- the stored request: logits on the sample, every row's decision --------------------
        errR = errE = 0.0
        worst_margin = 0.0
        for r in range(M):
            gR, mR, gE, mE, ids, lR, lE = gold["rows"][r]
            errR = max(errR, U.rel_l2(blog[r, ids], lR))
            errE = max(errE, U.rel_l2(blog[r, ids], lE))
            assert brow[r] == int(np.argmax(blog[r]))
            if brow[r] != gR:
                worst_margin = max(worst_margin, mR)
        print("w5 full depth: sampled logits vs mode R %.3g, vs mode E %.3g; largest margin of a differing row %.3g" % (
            errR, errE, worst_margin), flush=True)
        assert errE <= U.TOL_BF16_E and errR <= U.TOL_BF16_R
        assert worst_margin < U.MARGIN
        rows_tok, rows_par, depth, _ = O.tree_rows(wl.root_token(cfg.vocab, P, seed=3456 + REQ), tok_g, par_g)
        best, path, _ = O.accept_walk(brow, rows_tok, rows_par, depth)
        l, acc_t, acc_n, bonus = batch[REQ]
        assert (l, acc_n, acc_t, bonus) == (len(path), [p - 1 for p in path], [int(rows_tok[p]) for p in path], int(brow[best]))
        if all(brow[r] == gold["rows"][r][0] for r in range(M)):
            assert (l, acc_t, acc_n, bonus) == gold["result_R"]
        assert l >= 1, "the stored tree follows the greedy continuation: something must be accepted"

        # ---- batched == single for every request --------------------------------------------------
        r0 = 0
        for b, kv in enumerate(kvs):
            single = B.ts_verify(model, kv, trees[b][0], trees[b][1])
            srow = B.ts_get_row_tokens(model, 0, len(trees[b][0]) + 1)
            brows = all_rows[r0:r0 + len(srow)]
            if single != batch[b] or not np.array_equal(srow, brows):
                slog = B.ts_get_logits(model, 0, len(srow), cfg.vocab)
                top2 = np.sort(slog, axis=1)[:, -2:]
                differ = np.nonzero(srow != brows)[0]
                assert len(differ) and all(top2[r, 1] - top2[r, 0] < U.MARGIN for r in differ), \
                    "request %d: batched %r != single %r without a near-tie" % (b, batch[b], single)
            r0 += len(srow)
        print("w5 full depth: batched == single for all requests (%.0f s)" % (time.time() - t0), flush=True)

        # ---- compaction of the stored request (its last verify was the single pass) -----------------
        l, acc_t, acc_n, bonus = B.ts_verify(model, kvs[REQ], tok_g, par_g)
        pre_k, pre_v = B.ts_kv_export(kvs[REQ], P, M, cfg)
        B.ts_kv_commit(kvs[REQ])
        assert B.ts_kv_len(kvs[REQ]) == P + l + 1
        post_k, post_v = B.ts_kv_export(kvs[REQ], P, l + 1, cfg)
        rows = [0] + [a + 1 for a in acc_n]
        assert np.array_equal(post_k, pre_k[:, rows]) and np.array_equal(post_v, pre_v[:, rows])
    finally:
        for kv in kvs:
            B.ts_kv_free(kv)
        B.ts_model_free(model)
