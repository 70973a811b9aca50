"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle (oracle/toolspec_oracle.py) is checked against things other than
itself: an independently written dense causal decoder (brute force over every
root-to-node path, paper App. A.1: each draft is verified as if it were an
ordinary sequential continuation), closed forms, library routines, and the
lossless property (Sec. 5.1 / App. B.3: output equals plain greedy decoding).
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import toolspec_oracle as O
from oracle import dense_causal as D


# --------------------------------------------------------------------------- #
# helpers
# --------------------------------------------------------------------------- #
def _setup(cfg_name, prompt_len, seed=7, wseed=1234):
    """Model + KV filled by a REAL prefill of a random prompt (dense decoder)."""
    cfg = wl.get_config(cfg_name)
    w = wl.gen_weights(cfg, wseed)
    rng = np.random.default_rng(seed)
    prompt = rng.integers(cfg.vocab, size=prompt_len)
    _, K, V = D.causal_forward(cfg, w, prompt[:-1], return_kv=True)
    kv = O.OracleKV(cfg, prompt_len + 80)
    kv.K[:, :prompt_len - 1] = K
    kv.V[:, :prompt_len - 1] = V
    kv.P = prompt_len - 1
    kv.pending = int(prompt[-1])
    return cfg, w, O.OracleModel(cfg, w), kv, prompt, rng


def _path_tokens(draft_tokens, parent_idx, node):
    toks = []
    while node >= 0:
        toks.append(int(draft_tokens[node]))
        node = int(parent_idx[node])
    return toks[::-1]


def _random_tree(rng, n, vocab, dup_prob=0.3):
    par = np.array([rng.integers(-1, i) for i in range(n)], dtype=np.int32)
    tok = rng.integers(vocab, size=n).astype(np.int32)
    for i in range(1, n):                    # duplicate sibling tokens are legal
        if rng.random() < dup_prob:
            sib = [j for j in range(i) if par[j] == par[i]]
            if sib:
                tok[i] = tok[sib[0]]
    return tok, par


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# --------------------------------------------------------------------------- #
# P1: brute force - tree pass == sequential decoding of every path
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("cfg_name,n_nodes", [("micro_fp32", 13), ("small_fp32", 9)])
def test_tree_pass_equals_sequential_decoding_of_every_path(cfg_name, n_nodes):
    cfg, w, model, kv, prompt, rng = _setup(cfg_name, 21)
    for trial in range(3):
        tok, par = _random_tree(rng, n_nodes, cfg.vocab)
        if trial == 2:
            par[:] = -1                       # depth-1-only tree
        rows = O.tree_rows(kv.pending, tok, par)
        logits, newK, newV = O.forward_tree(model, kv, rows[0], rows[2], rows[3])
        for node in range(-1, n_nodes):
            seq = list(prompt) + _path_tokens(tok, par, node)
            ref, K, V = D.causal_forward(cfg, w, seq, return_kv=True)
            assert _rel(logits[node + 1], ref[-1]) < 1e-10
            assert _rel(newK[:, node + 1], K[:, -1]) < 1e-10
            assert _rel(newV[:, node + 1], V[:, -1]) < 1e-10


def test_chain_equals_causal_chunk():
    cfg, w, model, kv, prompt, rng = _setup("micro_fp32", 17)
    n = 10
    tok = rng.integers(cfg.vocab, size=n).astype(np.int32)
    par = np.arange(-1, n - 1, dtype=np.int32)
    rows = O.tree_rows(kv.pending, tok, par)
    assert np.array_equal(rows[3], np.tril(np.ones((n + 1, n + 1), bool)))
    logits, _, _ = O.forward_tree(model, kv, rows[0], rows[2], rows[3])
    ref = D.causal_forward(cfg, w, list(prompt) + list(tok))
    assert _rel(logits, ref[len(prompt) - 1:]) < 1e-10


def test_star_tree_rows_depend_only_on_own_token():
    cfg, w, model, kv, prompt, rng = _setup("micro_fp32", 9)
    tok = np.array([5, 9, 5, 77, 9], dtype=np.int32)
    par = np.full(5, -1, dtype=np.int32)
    rows = O.tree_rows(kv.pending, tok, par)
    logits, _, _ = O.forward_tree(model, kv, rows[0], rows[2], rows[3])
    assert _rel(logits[1], logits[3]) < 1e-13
    assert _rel(logits[2], logits[5]) < 1e-13
    assert _rel(logits[1], logits[4]) > 1e-3


def test_empty_tree_is_single_token_decode():
    cfg, w, model, kv, prompt, rng = _setup("small_fp32", 12)
    e = np.zeros(0, np.int32)
    r = O.verify(model, kv, e, e)
    ref = D.causal_forward(cfg, w, prompt)
    assert r.accept_len == 0 and r.accepted_tokens == []
    assert r.bonus_token == int(np.argmax(ref[-1]))
    assert _rel(r.logits[0], ref[-1]) < 1e-10


def test_gqa_equals_mha_with_replicated_kv_heads():
    cfg = wl.get_config("micro_fp32")                     # 4 q heads, 2 kv heads
    w = wl.gen_weights(cfg, 99)
    mha = cfg.with_(n_kv_heads=cfg.n_q_heads)
    G, hd = cfg.group, cfg.head_dim
    w2 = {k: v for k, v in w.items() if k != "layers"}
    w2["layers"] = []
    for lw in w["layers"]:
        lw2 = dict(lw)
        for k in ("wk", "wv"):
            m = lw[k].reshape(cfg.n_kv_heads, hd, cfg.d_model)
            lw2[k] = np.repeat(m, G, axis=0).reshape(cfg.n_q_heads * hd, cfg.d_model)
        w2["layers"].append(lw2)
    rng = np.random.default_rng(3)
    ctxK, ctxV = wl.gen_context_kv(cfg, 11, seed=5)
    tok, par = _random_tree(rng, 7, cfg.vocab)
    out = []
    for c, ww, rep in ((cfg, w, 1), (mha, w2, G)):
        kv = O.OracleKV(c, 32)
        kv.import_context(np.repeat(ctxK, rep, axis=2), np.repeat(ctxV, rep, axis=2))
        kv.pending = 3
        out.append(O.verify(O.OracleModel(c, ww), kv, tok, par).logits)
    assert _rel(out[0], out[1]) < 1e-12


# --------------------------------------------------------------------------- #
# P4: closed forms and library routines
# --------------------------------------------------------------------------- #
def test_rmsnorm_closed_form_and_library():
    x = np.full((2, 8), 3.0)
    g = np.arange(1, 9, dtype=np.float64)
    assert np.allclose(O.rmsnorm(x, g, 1e-5), 3.0 / np.sqrt(9.0 + 1e-5) * g, rtol=1e-14)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    g = rng.standard_normal(64)
    ref = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-5).numpy()
    assert np.allclose(O.rmsnorm(x, g, 1e-5), ref, rtol=1e-13, atol=1e-15)


def test_silu_library():
    x = np.linspace(-20, 20, 401)
    assert np.allclose(O.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-300)


def test_rope_identity_norm_and_relative_position():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, 3, 32))
    k = rng.standard_normal((1, 3, 32))
    assert np.array_equal(O.rope(q, [0], 10000.0), q)
    for a, b in ((5, 2), (100, 97), (1003, 1000)):
        qa, kb = O.rope(q, [a], 10000.0), O.rope(k, [b], 10000.0)
        q3, k0 = O.rope(q, [3], 10000.0), O.rope(k, [0], 10000.0)
        assert np.allclose(np.sum(qa * kb, -1), np.sum(q3 * k0, -1), rtol=1e-9, atol=1e-11)
        assert np.allclose(np.linalg.norm(qa, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    # first pair rotates by exactly `pos` radians (inv_freq_0 = 1), last pair slowest
    e = np.zeros((1, 1, 32)); e[0, 0, 0] = 1.0
    r = O.rope(e, [2], 10000.0)
    assert np.isclose(r[0, 0, 0], np.cos(2.0)) and np.isclose(r[0, 0, 16], np.sin(2.0))
    e = np.zeros((1, 1, 32)); e[0, 0, 15] = 1.0
    r = O.rope(e, [2], 10000.0)
    ang = 2.0 * 10000.0 ** (-30.0 / 32.0)
    assert np.isclose(r[0, 0, 15], np.cos(ang)) and np.isclose(r[0, 0, 31], np.sin(ang))


def test_uniform_scores_give_masked_mean_of_values():
    """wq = 0 makes all scores equal; wv = 0 makes tree V rows zero; a constant
    context V then gives attention = c * P / (P + #visible tree rows): this pins
    the size of each row's visible set = depth + 1."""
    cfg = wl.get_config("micro_fp32").with_(n_layers=1, norm_init="ones")
    w = wl.gen_weights(cfg, 5)
    lw = w["layers"][0]
    lw["wq"][:] = 0
    lw["wv"][:] = 0
    lw["wd"][:] = 0
    lw["wo"][:] = np.eye(cfg.d_model, dtype=np.float32)       # q_dim == d_model here
    assert cfg.q_dim == cfg.d_model
    P = 6
    kv = O.OracleKV(cfg, 32)
    c = np.random.default_rng(2).standard_normal((cfg.n_kv_heads, cfg.head_dim))
    kv.V[0, :P] = c
    kv.K[0, :P] = 1.0
    kv.P, kv.pending = P, 1
    tok = np.array([4, 5, 6, 7, 8], np.int32)
    par = np.array([-1, 0, 0, 2, -1], np.int32)          # depths 1,2,2,3,1
    rows = O.tree_rows(1, tok, par)
    logits, _, _ = O.forward_tree(O.OracleModel(cfg, w), kv, rows[0], rows[2], rows[3])
    depth = np.array([0, 1, 2, 2, 3, 1])
    emb = w["embed"][np.concatenate([[1], tok])].astype(np.float64)
    cq = np.repeat(c, cfg.group, axis=0).reshape(-1)         # per query head
    X = emb + cq[None, :] * (P / (P + depth + 1.0))[:, None]
    h = F.rms_norm(torch.from_numpy(X), (cfg.d_model,), None, cfg.rms_eps)
    ref = F.linear(h, torch.from_numpy(w["lm_head"].astype(np.float64))).numpy()
    assert _rel(logits, ref) < 1e-12


def test_zero_output_projections_reduce_to_head_of_embedding():
    cfg = wl.get_config("small_fp32")
    w = wl.gen_weights(cfg, 8)
    for lw in w["layers"]:
        lw["wo"][:] = 0
        lw["wd"][:] = 0
    kv = O.OracleKV(cfg, 16)
    kv.pending = 17
    tok = np.array([1, 2, 3], np.int32)
    par = np.array([-1, 0, -1], np.int32)
    r = O.verify(O.OracleModel(cfg, w), kv, tok, par)
    emb = torch.from_numpy(w["embed"][[17, 1, 2, 3]].astype(np.float64))
    h = F.rms_norm(emb, (cfg.d_model,), torch.from_numpy(w["norm_f"].astype(np.float64)), cfg.rms_eps)
    ref = F.linear(h, torch.from_numpy(w["lm_head"].astype(np.float64))).numpy()
    assert _rel(r.logits, ref) < 1e-13


def test_bf16_round_matches_library_conversion():
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 6, 5000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895e38 / 2]])
    ref = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.bf16_round(x), ref)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.bf16_round(np.array([1.00390625]))[0] == 1.0
    assert O.bf16_round(np.array([1.01171875]))[0] == 1.015625


def test_half_rounding_matches_library_conversion_and_saturates():
    """Projection inputs of the decision mode: IEEE half, nearest even, saturating at 65504."""
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-7, 4, 5000),
                        [0.0, -0.0, 1.0, 1.00048828125, 1.00146484375, 65504.0, 6.0e-8, 3.0e-8]])
    ref = torch.from_numpy(x).to(torch.float32).to(torch.float16).to(torch.float64).numpy()
    assert np.array_equal(O.fp16_round(x), ref)
    assert np.array_equal(O.fp16_act_round(x), ref)             # nothing here is out of range
    # ties go to even: 1 + 2^-11 is halfway between 1 and 1 + 2^-10
    assert O.fp16_round(np.array([1.00048828125]))[0] == 1.0
    assert O.fp16_round(np.array([1.00146484375]))[0] == 1.001953125
    # half's subnormal grid has steps of 2^-24
    assert O.fp16_round(np.array([6.0e-8]))[0] == 2.0 ** -24 and O.fp16_round(np.array([2.9e-8]))[0] == 0.0
    # beyond the largest finite half: the activation rounding saturates, the plain rounding overflows
    big = np.array([65520.0, 1.0e6, -7.0e4])
    assert np.array_equal(O.fp16_act_round(big), [65504.0, 65504.0, -65504.0])
    assert np.all(np.isinf(O.fp16_round(big)))


# --------------------------------------------------------------------------- #
# acceptance walk against exhaustive enumeration of the definition
# --------------------------------------------------------------------------- #
def test_accept_walk_matches_exhaustive_definition():
    rng = np.random.default_rng(11)
    for trial in range(300):
        n = int(rng.integers(0, 12))
        V = 3                                        # tiny vocab -> many matches
        tok_d, par_d = _random_tree(rng, n, V, dup_prob=0.5)
        tok, par, depth, vis = O.tree_rows(int(rng.integers(V)), tok_d, par_d)
        g = rng.integers(V, size=n + 1)
        best, path, valid = O.accept_walk(g, tok, par, depth)
        # definition: node valid iff every token on its path equals the greedy token
        # of the row before it; answer = deepest valid node, lowest index on ties
        exp_best, exp_depth = 0, 0
        for r in range(1, n + 1):
            chain, q = [], r
            while q > 0:
                chain.append(q)
                q = par[q]
            chain = [0] + chain[::-1]
            ok = all(tok[chain[i + 1]] == g[chain[i]] for i in range(len(chain) - 1))
            assert ok == bool(valid[r])
            if ok and len(chain) - 1 > exp_depth:
                exp_best, exp_depth = r, len(chain) - 1
        assert best == exp_best and len(path) == exp_depth
        assert all(depth[p] == i + 1 for i, p in enumerate(path))


# --------------------------------------------------------------------------- #
# P2: losslessness - speculative output == plain greedy output, token for token
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("cfg_name", ["micro_fp32", "small_fp32"])
def test_lossless_against_independent_greedy_decoder(cfg_name):
    cfg, w, model, kv, prompt, rng = _setup(cfg_name, 10)
    n_out = 30
    ref = D.greedy_sequence(cfg, w, prompt, n_out)        # independent decoder
    out, steps = [], 0
    while len(out) < n_out:
        future = ref[len(out):]                           # oracle-side draft source
        shape = steps % 3
        if shape == 0:
            tok, par = wl.chain_tree(future, 6, 0.3, cfg.vocab, rng)
        elif shape == 1:
            tok, par = wl.bfs_tree(future, 12, cfg.vocab, rng)
        else:
            tok, par = wl.retrieval_tree(future, cfg.vocab, rng, lengths=(6, 4, 3, 3))
        r = O.verify(model, kv, tok, par)
        P0 = kv.P
        O.commit(kv, r)
        assert kv.P == P0 + r.accept_len + 1
        out += r.accepted_tokens + [r.bonus_token]
        steps += 1
    assert out[:n_out] == ref
    assert steps < n_out                                   # some drafts were accepted


@pytest.mark.parametrize("cfg_name", ["micro_fp32", "small_fp32"])
def test_greedy_decode_equals_the_independent_decoder(cfg_name):
    """greedy_decode (verify with an empty tree + commit, repeated) against the dense causal decoder's
    own greedy continuation: same tokens, cache length advanced by one per token, and the cache equal
    to a real prefill of the emitted sequence."""
    cfg, w, model, kv, prompt, rng = _setup(cfg_name, 9)
    n = 12
    ref = D.greedy_sequence(cfg, w, prompt, n)
    P0 = kv.P
    out = O.greedy_decode(model, kv, n)
    assert out == ref
    assert kv.P == P0 + n and kv.pending == ref[-1]
    _, K, V = D.causal_forward(cfg, w, list(prompt) + ref[:-1], return_kv=True)
    assert _rel(kv.K[:, :kv.P], K) < 1e-10 and _rel(kv.V[:, :kv.P], V) < 1e-10


def test_commit_moves_accepted_rows_and_requires_nothing_else():
    """After commit the cache must equal what a real prefill of the emitted sequence
    would hold (rows moved to positions P+1..P+l, root at P)."""
    cfg, w, model, kv, prompt, rng = _setup("micro_fp32", 10)
    ref = D.greedy_sequence(cfg, w, prompt, 8)
    tok, par = wl.retrieval_tree(ref, cfg.vocab, rng, lengths=(2, 6, 3, 1), p=(1.0, 0.0, 0.0, 0.0))
    r = O.verify(model, kv, tok, par)
    assert r.accept_len == 6 and r.accepted_nodes == [2, 3, 4, 5, 6, 7]
    assert r.accepted_tokens == ref[:6] and r.bonus_token == ref[6]
    O.commit(kv, r)
    _, K, V = D.causal_forward(cfg, w, list(prompt) + ref[:6], return_kv=True)
    assert kv.P == len(prompt) + 6
    assert _rel(kv.K[:, :kv.P], K) < 1e-10 and _rel(kv.V[:, :kv.P], V) < 1e-10


# --------------------------------------------------------------------------- #
# P5: acceptance statistics of a mutated chain, closed form (1-p)^k
# --------------------------------------------------------------------------- #
def test_chain_acceptance_follows_geometric_law():
    cfg, w, model, kv, prompt, rng = _setup("micro_fp32", 8)
    n, p, trials = 6, 0.3, 300
    ref = D.greedy_sequence(cfg, w, prompt, n + 1)
    counts = np.zeros(n + 1)
    for _ in range(trials):
        tok, par = wl.chain_tree(ref, n, p, cfg.vocab, rng)
        r = O.verify(model, kv, tok, par)
        counts[:r.accept_len + 1] += 1
        assert r.accepted_tokens == ref[:r.accept_len]
    q = 1 - p + p / cfg.vocab
    for k in range(1, n + 1):
        e = q ** k
        sd = np.sqrt(e * (1 - e) / trials)
        assert abs(counts[k] / trials - e) < 4.5 * sd + 1e-9


# --------------------------------------------------------------------------- #
# P6: rounding-emulating mode stays within the bf16 budget of the exact mode
# --------------------------------------------------------------------------- #
def test_mode_R_close_to_mode_E_on_bf16_model():
    cfg = wl.get_config("small_bf16_hd64")
    w = wl.gen_weights(cfg, 21)
    K, V = wl.gen_context_kv(cfg, 40, seed=3)
    rng = np.random.default_rng(5)
    tok, par = _random_tree(rng, 10, cfg.vocab)
    res = {}
    for mode in ("E", "R"):
        kv = O.OracleKV(cfg, 64)
        kv.import_context(K, V)
        kv.pending = 11
        res[mode] = O.verify(O.OracleModel(cfg, w), kv, tok, par, mode).logits
    rel = _rel(res["R"], res["E"])
    assert 1e-5 < rel < 2e-2
