"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Run with `pytest -m gpu` on an MI355X.

Sizes: small shapes the oracle finishes in seconds but that span several MFMA tiles,
ragged vocabularies and partial key blocks; the exact tiny fp32 workload (2 layers,
d 256, ctx 512, chain of 8); and the 8B layer shape.  Comparison rules are in gpu_utils.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import toolspec_oracle as O
from oracle import dense_causal as D
from paper_2604_13519_amd import binding as B

import gpu_utils as U

pytestmark = pytest.mark.gpu


def _random_tree(rng, n, vocab, dup_prob=0.3):
    par = np.array([rng.integers(-1, i) for i in range(n)], dtype=np.int32)
    tok = rng.integers(vocab, size=n).astype(np.int32)
    for i in range(1, n):
        if rng.random() < dup_prob:
            sib = [j for j in range(i) if par[j] == par[i]]
            if sib:
                tok[i] = tok[sib[0]]
    return tok, par


def _greedy_from_oracle(omodel, okv_template_args, n):
    cfg, K, V, pending, cap = okv_template_args
    okv = O.OracleKV(cfg, cap)
    if K.shape[1]:
        okv.import_context(K, V)
    okv.pending = int(pending)
    mode = "E" if cfg.dtype == wl.configs.DTYPE_F32 else "R"
    return O.greedy_decode(omodel, okv, n, mode)


# ------------------------------------------------------------------------------------
# the shipped configuration stores no logits: same decisions as with logits kept
# ------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg_name,P", [("small_bf16", 200), ("small_bf16_hd64", 70), ("llama8b_2l", 600)])
def test_results_without_stored_logits_equal_results_with_them(cfg_name, P):
    """Every other parity test keeps the logits (it compares them); the product default does not.
    Same trees both ways - single and batched, greedy-heavy and random - must give identical
    (accept_len, tokens, nodes, bonus) and identical per-row tokens; with the logits off
    ts_get_logits must refuse."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(4242)
    K, V = wl.gen_context_kv(cfg, P, seed=79)
    pending = int(rng.integers(cfg.vocab))
    greedy = _greedy_from_oracle(omodel, (cfg, K, V, pending, P + 80), 6)
    trees = [wl.chain_tree(greedy, 6, 0.0, cfg.vocab, rng), wl.bfs_tree(greedy, 40, cfg.vocab, rng),
             _random_tree(rng, 64, cfg.vocab), (np.zeros(0, np.int32), np.zeros(0, np.int32))]
    kvs = []
    try:
        for _ in trees:
            kv = B.ts_kv_alloc(model, P + 80)
            B.ts_kv_import(kv, K, V)
            B.ts_set_pending(kv, pending)
            kvs.append(kv)
        out = {}
        for keep in (True, False, True):
            B.ts_model_keep_logits(model, keep)
            single = []
            for kv, (tok, par) in zip(kvs, trees):
                res = B.ts_verify(model, kv, tok, par)
                single.append((res, B.ts_get_row_tokens(model, 0, len(tok) + 1).tolist()))
            batch = B.ts_verify_batch(model, kvs, trees)
            rows = B.ts_get_row_tokens(model, 0, sum(len(t[0]) + 1 for t in trees)).tolist()
            if not keep:
                with pytest.raises(B.TsError):
                    B.ts_get_logits(model, 0, 1, cfg.vocab)
            out.setdefault(keep, []).append((single, batch, rows))
        assert out[True][0] == out[False][0] == out[True][1]
        assert out[False][0][0][0][0][0] >= 1              # the walk accepts part of the greedy chain: not a trivial case
    finally:
        B.ts_model_keep_logits(model, True)
        for kv in kvs:
            B.ts_kv_free(kv)


# ------------------------------------------------------------------------------------
# single verify: logits, decisions, tree K/V rows
# ------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg_name,P,n_nodes", [
    ("micro_fp32", 0, 5), ("micro_fp32", 37, 13), ("small_fp32", 100, 64), ("small_fp32", 15, 0),
    ("small_bf16_hd64", 0, 7), ("small_bf16_hd64", 70, 33), ("small_bf16", 200, 64),
    ("small_bf16", 63, 16), ("small_bf16", 1000, 40), ("small_bf16", 129, 0),
])
def test_verify_matches_oracle_random_trees(cfg_name, P, n_nodes):
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(1000 + P + n_nodes)
    K, V = wl.gen_context_kv(cfg, P, seed=77)
    pending = int(rng.integers(cfg.vocab))
    kv, okv = U.make_pair(cfg, model, K, V, pending)
    try:
        tok, par = _random_tree(rng, n_nodes, cfg.vocab)
        U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="%s P=%d n=%d" % (cfg_name, P, n_nodes))
        # verify is pure: a second call gives the same answer
        r1 = B.ts_verify(model, kv, tok, par)
        r2 = B.ts_verify(model, kv, tok, par)
        assert r1 == r2
    finally:
        B.ts_kv_free(kv)


@pytest.mark.parametrize("cfg_name,n_nodes", [("small_bf16", 64), ("small_bf16", 20), ("small_bf16_hd64", 40)])
def test_softmax_reference_moving_late_in_the_context(cfg_name, n_nodes):
    """The attention kernel moves a row's soft-max reference only when the running maximum exceeds
    it by more than 2^8.  Random contexts settle the reference in the first key block; here the
    keys grow along the context (x 1/4, 1/2, 1, 4, 16 by segment, exact in bf16), so the maximum
    keeps climbing - by less than the slack inside a segment, by much more across segments - and
    both the stale-reference path and the late rescale are compared with the oracle."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(4242 + n_nodes)
    P = 1100
    K, V = wl.gen_context_kv(cfg, P, seed=91)
    Kf = wl.bf16_bits_to_f32(K)
    for seg, scale in enumerate((0.25, 0.5, 1.0, 4.0, 16.0)):
        Kf[:, seg * 220:(seg + 1) * 220] *= scale
    K = wl.f32_to_bf16_bits(Kf)
    kv, okv = U.make_pair(cfg, model, K, V, int(rng.integers(cfg.vocab)))
    try:
        tok, par = _random_tree(rng, n_nodes, cfg.vocab)
        U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="%s growing keys n=%d" % (cfg_name, n_nodes))
    finally:
        B.ts_kv_free(kv)


@pytest.mark.parametrize("cfg_name", ["small_fp32", "small_bf16"])
def test_tree_shapes_of_the_workloads(cfg_name):
    """Chain, schema+alternatives+retrieved tree, BFS tree, retrieved continuations (32,16,8,8),
    star, deepest-possible chain of 64 - built from the oracle's greedy continuation."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(5)
    P = 150
    K, V = wl.gen_context_kv(cfg, P, seed=78)
    pending = 11
    greedy = _greedy_from_oracle(omodel, (cfg, K, V, pending, P + 80), 34)
    trees = {
        "chain16": wl.chain_tree(greedy, 16, 0.2, cfg.vocab, rng),
        "schema": wl.schema_retrieval_tree(greedy, cfg.vocab, rng),
        "bfs32": wl.bfs_tree(greedy, 32, cfg.vocab, rng),
        "retrieved": wl.retrieval_tree(greedy, cfg.vocab, rng),
        "star": (rng.integers(cfg.vocab, size=64).astype(np.int32), np.full(64, -1, np.int32)),
        "chain64_exact": wl.chain_tree(greedy + list(rng.integers(cfg.vocab, size=64)), 64, 0.0, cfg.vocab, rng),
    }
    kv, okv = U.make_pair(cfg, model, K, V, pending)
    try:
        for name, (tok, par) in trees.items():
            res, oR = U.check_verify(cfg, model, omodel, kv, okv, tok, par, label=cfg_name + " " + name)
            if name == "chain64_exact" and oR.decisive_margin >= U.MARGIN:
                assert res[0] >= 34          # the whole known greedy prefix is accepted
    finally:
        B.ts_kv_free(kv)


def test_tiny_fp32_workload_chain8_ctx512_real_prefill():
    """Workload 1: 2 layers, d 256, 4 heads x 64, FFN 1024, vocab 4096, fp32; 512-token context
    prefilled for real (dense causal decoder), chain of 8 = greedy continuation mutated with
    p = 0.3."""
    cfg, w, model, omodel = U.get_model("tiny_fp32")
    rng = np.random.default_rng(42)
    prompt = rng.integers(cfg.vocab, size=512)
    _, K, V = D.causal_forward(cfg, w, prompt[:-1], return_kv=True)
    K32, V32 = K.astype(np.float32), V.astype(np.float32)
    kv, okv = U.make_pair(cfg, model, K32, V32, int(prompt[-1]), capacity=640)
    try:
        greedy = D.greedy_sequence(cfg, w, prompt, 9)
        for trial in range(4):
            tok, par = wl.chain_tree(greedy, 8, 0.3, cfg.vocab, rng)
            res, oR = U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="tiny chain8 #%d" % trial)
            if oR.decisive_margin >= U.MARGIN:
                assert res[1] == greedy[:res[0]] and res[3] == greedy[res[0]]
    finally:
        B.ts_kv_free(kv)


def test_8b_layer_shape_two_layers_schema_tree_ctx4096():
    """Two layers of the exact Llama-3-8B layer shape (d 4096, 32/8 heads x 128, FFN 14336),
    vocabulary cut to 32000: the production tile shapes, K splits and key splits, with the
    64-node schema + alternatives + retrieved-branches tree over a 4096-token context."""
    cfg, w, model, omodel = U.get_model("llama8b_2l")
    rng = np.random.default_rng(17)
    P = 4096
    K, V = wl.gen_context_kv(cfg, P, seed=2345)
    pending = 100
    greedy = _greedy_from_oracle(omodel, (cfg, K, V, pending, P + 80), 26)
    kv, okv = U.make_pair(cfg, model, K, V, pending)
    try:
        for name, (tok, par) in (("schema", wl.schema_retrieval_tree(greedy, cfg.vocab, rng)),
                                 ("chain16", wl.chain_tree(greedy, 16, 0.2, cfg.vocab, rng)),
                                 ("empty", (np.zeros(0, np.int32), np.zeros(0, np.int32)))):
            U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="llama8b_2l " + name)
    finally:
        B.ts_kv_free(kv)
        U.drop_model("llama8b_2l")


# ------------------------------------------------------------------------------------
# multi-step: losslessness, commit / compaction, pending-token hand-off
# ------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg_name,P0", [("small_fp32", 32), ("small_fp32", 33), ("small_bf16", 15), ("small_bf16_hd64", 251),
                                         ("small_bf16_hd64", 252)])
def test_speculative_stream_equals_plain_greedy_stream(cfg_name, P0):
    """Lossless property: K steps of verify + commit with mutated-greedy trees emit exactly the
    plain greedy stream (n_nodes = 0 decoding), on the device and against the oracle.  Streams
    are compared up to the first step whose oracle top-2 margin is below 1e-2."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(9)
    pending = 3
    n_out = 40
    cap = P0 + n_out + 80
    mode = "E" if cfg.dtype == wl.configs.DTYPE_F32 else "R"
    empty = np.zeros(0, np.int32)
    # random-init models have near-ties every few dozen tokens: take, among a few context seeds, the
    # one whose greedy stream stays clear of them longest
    best = None
    for seed in range(79, 85):
        K, V = wl.gen_context_kv(cfg, P0, seed=seed)
        okv = O.OracleKV(cfg, cap)
        okv.import_context(K, V)
        okv.pending = pending
        ref, safe = [], n_out
        for i in range(n_out):
            r = O.verify(omodel, okv, empty, empty, mode)
            O.commit(okv, r)
            ref.append(r.bonus_token)
            if r.margin[0] < U.MARGIN and safe == n_out:
                safe = i
        if best is None or safe > best[0]:
            best = (safe, K, V, ref)
        if safe >= 24:
            break
    safe, K, V, ref = best
    if safe < 8:
        pytest.skip("no context seed whose greedy stream is free of near-ties for 8 steps")
    # device, plain autoregressive (n_nodes = 0)
    kv, _ = U.make_pair(cfg, model, K, V, pending, capacity=cap)
    ar = []
    for _ in range(n_out):
        l, t, nn, b = B.ts_verify(model, kv, [], [])
        assert l == 0 and t == []
        B.ts_kv_commit(kv)
        ar.append(b)
    B.ts_kv_free(kv)
    assert ar[:safe] == ref[:safe]
    # device, speculative with mutated-greedy trees, checked step by step against the oracle
    kv, okv = U.make_pair(cfg, model, K, V, pending, capacity=cap)
    spec, steps, in_sync = [], 0, True
    try:
        while len(spec) < n_out:
            future = ref[len(spec):] if in_sync else []
            shape = steps % 3
            if shape == 0:
                tok, par = wl.chain_tree(future, 8, 0.25, cfg.vocab, rng)
            elif shape == 1:
                tok, par = wl.bfs_tree(future, 24, cfg.vocab, rng)
            else:
                tok, par = wl.retrieval_tree(future, cfg.vocab, rng, lengths=(12, 6, 3, 3))
            if in_sync:
                res, oR = U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="%s step %d" % (cfg_name, steps))
                in_sync = U.commit_both(cfg, kv, okv, res, oR)
            else:                      # a sub-margin pick diverged from the oracle: device-only from here
                res = B.ts_verify(model, kv, tok, par)
                B.ts_kv_commit(kv)
            assert B.ts_kv_len(kv) == P0 + len(spec) + res[0] + 1
            spec += res[1] + [res[3]]
            steps += 1
        assert spec[:safe] == ref[:safe] and spec[:safe] == ar[:safe]
        assert steps < n_out
    finally:
        B.ts_kv_free(kv)


@pytest.mark.parametrize("cfg_name", ["micro_fp32", "small_bf16"])
@pytest.mark.parametrize("P0", [0, 15, 16, 31])
def test_commit_adversarial_paths_and_page_straddles(cfg_name, P0):
    """Accepted rows r_d = d+1 (every target slot is another depth's source), last-sibling
    paths, and tree slots straddling page boundaries; after commit an empty-tree verify must
    reproduce the logits the accepted leaf had."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(3 + P0)
    K, V = wl.gen_context_kv(cfg, P0, seed=80)
    pending = 5
    greedy = _greedy_from_oracle(omodel, (cfg, K, V, pending, P0 + 200), 20)
    junk = lambda: int(rng.integers(cfg.vocab))
    # tree A: node 0 junk, then the greedy chain -> accepted rows are 2,3,4,... (r_d = d+1)
    tokA = [junk()] + greedy[:18]
    parA = [-1, -1] + list(range(1, 18))
    # tree B: at each depth three siblings, the greedy one LAST and the chain continues under it
    tokB, parB, parent = [], [], -1
    for d in range(12):
        tokB += [junk(), junk(), greedy[d]]
        parB += [parent, parent, parent]
        parent = len(tokB) - 1
    for tok, par, name in ((tokA, parA, "shifted"), (tokB, parB, "last-sibling")):
        kv, okv = U.make_pair(cfg, model, K, V, pending, capacity=P0 + 200)
        try:
            tok, par = np.asarray(tok, np.int32), np.asarray(par, np.int32)
            res, oR = U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="%s %s P0=%d" % (cfg_name, name, P0))
            leaf_row = (res[2][-1] + 1) if res[0] else 0
            leaf_logits = B.ts_get_logits(model, leaf_row, 1, cfg.vocab)[0]
            in_sync = U.commit_both(cfg, kv, okv, res, oR)
            if oR.decisive_margin >= U.MARGIN:
                assert res[0] >= 12 and in_sync
            # the committed cache must behave like the tree pass did: decode the bonus token's
            # predecessor state again = logits at the leaf; here: verify [] after truncating one
            B.ts_kv_truncate(kv, B.ts_kv_len(kv) - 1)
            last_tok = res[1][-1] if res[0] else pending
            B.ts_set_pending(kv, last_tok)
            B.ts_verify(model, kv, [], [])
            again = B.ts_get_logits(model, 0, 1, cfg.vocab)[0]
            tol = 1e-5 if cfg.dtype == wl.configs.DTYPE_F32 else 1e-2
            assert U.rel_l2(again, leaf_logits) <= tol
        finally:
            B.ts_kv_free(kv)


# ------------------------------------------------------------------------------------
# paging and batching
# ------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg_name", ["small_fp32", "small_bf16"])
def test_shuffled_page_table_gives_identical_results(cfg_name):
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(21)
    P = 203
    K, V = wl.gen_context_kv(cfg, P, seed=81)
    tok, par = _random_tree(rng, 30, cfg.vocab)
    cap = P + 80
    n_pages = (cap + 15) // 16
    outs = []
    for perm in (None, rng.permutation(n_pages).astype(np.int32)):
        kv, okv = U.make_pair(cfg, model, K, V, 9, capacity=cap, page_perm=perm)
        try:
            res, oR = U.check_verify(cfg, model, omodel, kv, okv, tok, par, label=cfg_name + " paged")
            outs.append((res, B.ts_get_logits(model, 0, 31, cfg.vocab)))
            k2, v2 = B.ts_kv_export(kv, 0, P, cfg)
            assert np.array_equal(k2, K) and np.array_equal(v2, V)       # import/export round trip
        finally:
            B.ts_kv_free(kv)
    assert outs[0][0] == outs[1][0]
    assert np.array_equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("cfg_name,n_seqs", [("small_fp32", 3), ("small_bf16", 5), ("small_bf16_hd64", 16)])
def test_batched_verify_equals_per_sequence_verify(cfg_name, n_seqs):
    """Ragged contexts, a different tree per sequence (one of them empty), shuffled page tables:
    the batched call must return exactly what one call per sequence returns."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(33)
    kvs, trees, singles = [], [], []
    try:
        for s in range(n_seqs):
            P = int(rng.integers(5, 400))
            K, V = wl.gen_context_kv(cfg, P, seed=90 + s)
            cap = P + 70
            perm = rng.permutation((cap + 15) // 16).astype(np.int32)
            kv, okv = U.make_pair(cfg, model, K, V, int(rng.integers(cfg.vocab)), capacity=cap, page_perm=perm)
            n = 0 if s == 1 else int(rng.integers(1, 33))
            tok, par = _random_tree(rng, n, cfg.vocab)
            kvs.append(kv)
            trees.append((tok, par))
            if s < 3:       # the oracle checks the first few, the rest are checked batch vs single
                res, _ = U.check_verify(cfg, model, omodel, kv, okv, tok, par, check_kv=False,
                                        label="%s seq %d" % (cfg_name, s))
            else:
                res = B.ts_verify(model, kv, tok, par)
            singles.append((res, B.ts_get_logits(model, 0, n + 1, cfg.vocab)))
        batch = B.ts_verify_batch(model, kvs, trees)
        row = 0
        for s in range(n_seqs):
            assert batch[s] == singles[s][0], "sequence %d" % s
            n = len(trees[s][0])
            lg = B.ts_get_logits(model, row, n + 1, cfg.vocab)
            tol = 1e-5 if cfg.dtype == wl.configs.DTYPE_F32 else 1e-2
            assert U.rel_l2(lg, singles[s][1]) <= tol       # same values up to split/accumulation order
            row += n + 1
        for kv in kvs:                                       # every sequence can commit its own result
            B.ts_kv_commit(kv)
    finally:
        for kv in kvs:
            B.ts_kv_free(kv)


@pytest.mark.parametrize("cfg_name,total_rows", [("small_bf16", 81), ("small_bf16", 112), ("small_bf16", 128),
                                                 ("small_bf16", 129), ("small_bf16_hd64", 209), ("small_bf16", 400)])
def test_many_row_projection_row_counts(cfg_name, total_rows):
    """Passes of more than 80 rows take the many-row projection kernel.  Row totals on both sides
    of its tile and block edges (81 = 6 row tiles with 15 idle rows, 128 = 8 full tiles, 129, ...):
    every sequence must get what its own single pass (skinny kernel) gets, and the first two are
    checked against the oracle."""
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(1000 + total_rows)
    n_seqs = (total_rows + 64) // 65
    rows = [total_rows // n_seqs + (1 if s < total_rows % n_seqs else 0) for s in range(n_seqs)]
    assert sum(rows) == total_rows and max(rows) <= 65
    kvs, trees, singles = [], [], []
    try:
        for s in range(n_seqs):
            P = int(rng.integers(20, 300))
            K, V = wl.gen_context_kv(cfg, P, seed=500 + s)
            kv, okv = U.make_pair(cfg, model, K, V, int(rng.integers(cfg.vocab)), capacity=P + 70)
            tok, par = _random_tree(rng, rows[s] - 1, cfg.vocab)
            kvs.append(kv)
            trees.append((tok, par))
            if s < 2:
                res, _ = U.check_verify(cfg, model, omodel, kv, okv, tok, par, check_kv=False,
                                        label="%s rows %d seq %d" % (cfg_name, total_rows, s))
            else:
                res = B.ts_verify(model, kv, tok, par)
            singles.append((res, B.ts_get_logits(model, 0, rows[s], cfg.vocab)))
        batch = B.ts_verify_batch(model, kvs, trees)
        row = 0
        for s in range(n_seqs):
            lg = B.ts_get_logits(model, row, rows[s], cfg.vocab)
            assert U.rel_l2(lg, singles[s][1]) <= 2e-3, "sequence %d" % s   # accumulation order only
            assert batch[s] == singles[s][0], "sequence %d" % s
            row += rows[s]
    finally:
        for kv in kvs:
            B.ts_kv_free(kv)


# ------------------------------------------------------------------------------------
# boundary: error paths (forced from the host; every kernel still exits normally)
# ------------------------------------------------------------------------------------
def test_saturated_projection_inputs_are_counted_not_hidden():
    """Activations beyond the largest finite half are clamped AND counted: an ordinary model
    reports 0 after a pass, a model whose first norm gain is blown up reports many."""
    cfg = wl.get_config("small_bf16")
    w = wl.gen_weights(cfg, 1234)
    rng = np.random.default_rng(8)
    K, V = wl.gen_context_kv(cfg, 40, seed=3)
    tok, par = _random_tree(rng, 20, cfg.vocab)
    counts = []
    for gain in (None, 3.0e5):
        ww = dict(w)
        ww["layers"] = [dict(l) for l in w["layers"]]
        if gain is not None:
            ww["layers"][0]["norm1"] = wl.f32_to_bf16_bits(np.full(cfg.d_model, gain, np.float32))
        model = B.ts_model_load(cfg, ww)
        kv = B.ts_kv_alloc(model, 120)
        try:
            B.ts_kv_import(kv, K, V)
            B.ts_set_pending(kv, 5)
            assert B.ts_model_saturations(model) == 0
            B.ts_verify(model, kv, tok, par)
            counts.append(B.ts_model_saturations(model))
        finally:
            B.ts_kv_free(kv)
            B.ts_model_free(model)
    assert counts[0] == 0 and counts[1] > 100, counts


def test_weight_beyond_half_range_fails_the_load():
    """bf16 models multiply in IEEE half: a finite weight that half cannot hold (|w| > 65504) must
    make ts_model_load fail instead of becoming an infinity; the largest finite half still loads."""
    cfg = wl.get_config("small_bf16_hd64")
    w = wl.gen_weights(cfg, 77)
    w["layers"][1]["wo"] = w["layers"][1]["wo"].copy()
    w["layers"][1]["wo"][3, 5] = 0x4780            # bf16 bits of 65536.0
    with pytest.raises(B.TsError) as e:
        B.ts_model_load(cfg, w)
    assert e.value.status == B.TS_ERR_INVALID_ARG, str(e.value)
    w["layers"][1]["wo"][3, 5] = 0x477F            # 65280.0, representable
    model = B.ts_model_load(cfg, w)
    B.ts_model_free(model)


def test_plain_read_reference_is_bracketed_and_leaves_results_alone():
    """The read-only reference kernel of the measurement interface: records appear under its own
    name with the tensor's size, nothing of the model changes (the next verify equals the previous)."""
    cfg = wl.get_config("small_bf16")
    model = B.ts_model_load(cfg, wl.gen_weights(cfg, 5))
    kv = B.ts_kv_alloc(model, 128)
    K, V = wl.gen_context_kv(cfg, 40, seed=6)
    B.ts_kv_import(kv, K, V)
    B.ts_set_pending(kv, 3)
    tok, par = _random_tree(np.random.default_rng(8), 12, cfg.vocab)
    before = B.ts_verify(model, kv, tok, par)
    B.ts_profile_filter(model, "plain_read")
    B.ts_profile_enable(model, True)
    nbytes = B.ts_profile_plain_read(model, 2 * cfg.n_layers + 1)
    rec = B.ts_profile_read(model)
    B.ts_profile_enable(model, False)
    B.ts_profile_filter(model, None)
    assert nbytes == 2 * cfg.d_ffn * cfg.d_model * 2
    assert list(rec) == ["plain_read"] and rec["plain_read"][0] == 2 * cfg.n_layers + 1 and rec["plain_read"][1] > 0
    assert B.ts_verify(model, kv, tok, par) == before
    B.ts_kv_free(kv)
    B.ts_model_free(model)


def test_error_paths_leave_state_untouched():
    cfg, w, model, omodel = U.get_model("micro_fp32")
    kv = B.ts_kv_alloc(model, 40)
    try:
        def expect(status, fn, *a):
            with pytest.raises(B.TsError) as e:
                fn(*a)
            assert e.value.status == status, str(e.value)

        expect(B.TS_ERR_STATE, B.ts_verify, model, kv, [], [])               # no pending token
        expect(B.TS_ERR_STATE, B.ts_kv_commit, kv)                           # nothing to commit
        expect(B.TS_ERR_TOKEN_RANGE, B.ts_set_pending, kv, cfg.vocab)
        B.ts_set_pending(kv, 1)
        expect(B.TS_ERR_INVALID_TREE, B.ts_verify, model, kv, [1, 2], [-1, 1])     # forward edge
        expect(B.TS_ERR_INVALID_TREE, B.ts_verify, model, kv, [1, 2], [-1, 2])     # beyond
        expect(B.TS_ERR_INVALID_TREE, B.ts_verify, model, kv, [1], [-2])
        expect(B.TS_ERR_INVALID_TREE, B.ts_verify, model, kv, [0] * 65, [-1] * 65)  # too many nodes
        expect(B.TS_ERR_TOKEN_RANGE, B.ts_verify, model, kv, [cfg.vocab], [-1])
        expect(B.TS_ERR_TOKEN_RANGE, B.ts_verify, model, kv, [-1], [-1])
        expect(B.TS_ERR_KV_CAPACITY, B.ts_verify, model, kv, [0] * 40, [-1] * 40)  # 41 rows > 40
        assert B.ts_kv_len(kv) == 0
        expect(B.TS_ERR_INVALID_ARG, B.ts_kv_alloc, model, 64, 32)           # unsupported page size
        expect(B.TS_ERR_INVALID_ARG, B.ts_kv_alloc, model, 0)
        # still usable after all of that; n_nodes = 0 and n_nodes = 39 (fills the capacity) are legal
        l, t, nn, b = B.ts_verify(model, kv, [], [])
        assert l == 0 and 0 <= b < cfg.vocab
        l2, _, _, _ = B.ts_verify(model, kv, [0] * 39, list(range(-1, 38)))
        B.ts_kv_commit(kv)
        expect(B.TS_ERR_STATE, B.ts_kv_commit, kv)                           # commit twice
        assert B.ts_kv_len(kv) == l2 + 1
        expect(B.TS_ERR_INVALID_ARG, B.ts_kv_truncate, kv, l2 + 2)
        expect(B.TS_ERR_STATE, B.ts_kv_set_page_table, kv, np.arange(3, dtype=np.int32))
    finally:
        B.ts_kv_free(kv)
    bad = wl.get_config("small_bf16").with_(d_model=500)
    with pytest.raises(B.TsError) as e:
        B.ts_model_load(bad, wl.gen_weights(wl.get_config("small_bf16"), 1))
    assert e.value.status == B.TS_ERR_INVALID_ARG


def test_max_size_tree_fills_exactly_the_capacity():
    cfg, w, model, omodel = U.get_model("small_bf16")
    rng = np.random.default_rng(8)
    P = 47
    K, V = wl.gen_context_kv(cfg, P, seed=83)
    kv, okv = U.make_pair(cfg, model, K, V, 2, capacity=P + 65)
    try:
        tok, par = _random_tree(rng, 64, cfg.vocab)
        U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="cap-exact")
    finally:
        B.ts_kv_free(kv)
