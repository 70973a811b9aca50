"""The C++ host drafter (include/toolspec_draft.h), called through its C ABI, against the
drafting oracle on the same seeded inputs.  Host-only code: runs without a GPU.  Trees, FSM
states and retrieved indices are integers: compared exactly."""
import json
import os
import time

import numpy as np
import pytest

from oracle import drafting_oracle as DO
from paper_2604_13519_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "drafting_worked_examples.json")


def _random_schema(rng, vocab, n_tools):
    """Random token-level schema; short alphabets make shared prefixes and ambiguous names common."""
    seq = lambda lo, hi: [int(t) for t in rng.integers(0, vocab, size=int(rng.integers(lo, hi + 1)))]
    s = {"call_open": seq(1, 2), "name_prefix": seq(0, 3), "name_suffix": seq(0, 3), "param_prefix": seq(0, 2),
         "param_suffix": seq(0, 2), "value_end": seq(1, 2), "call_close": seq(1, 2)}
    s["tools"] = [seq(1, 4) for _ in range(n_tools)]
    s["params"] = [[seq(1, 3) for _ in range(int(rng.integers(0, 4)))] for _ in range(n_tools)]
    return s


def _schema_stream(rng, s, vocab, n_calls):
    """A token stream that mostly follows the schema (so that every state is visited), with noise."""
    y = []
    for _ in range(n_calls):
        y += [int(t) for t in rng.integers(0, vocab, size=int(rng.integers(0, 4)))]
        y += s["call_open"]
        if rng.random() < 0.15:
            continue
        i = int(rng.integers(len(s["tools"])))
        y += s["name_prefix"] + s["tools"][i] + s["name_suffix"]
        for p in s["params"][i]:
            if rng.random() < 0.2:
                break
            y += s["param_prefix"] + p + s["param_suffix"]
            y += [int(t) for t in rng.integers(0, vocab, size=int(rng.integers(0, 5)))]
            y += s["value_end"] if rng.random() < 0.7 else s["call_close"]
        y += s["call_close"]
    return y


@pytest.mark.parametrize("vocab,seed", [(3, 1), (6, 2), (50, 3), (6, 4)])
def test_fsm_and_draft_trees_match_the_oracle_token_by_token(vocab, seed):
    rng = np.random.default_rng([404, seed])
    for trial in range(25):
        s = _random_schema(rng, vocab, int(rng.integers(1, 6)))
        stream = _schema_stream(rng, s, vocab, 4)
        calls = [_schema_stream(rng, s, vocab, 2) for _ in range(int(rng.integers(0, 4)))]
        d = B.ts_drafter_create(s)
        try:
            if calls:      # all historical calls retrieved, in datastore order (identical embeddings)
                B.ts_drafter_retrieve(d, np.ones(4), np.ones((len(calls), 4)), calls, k=len(calls))
            B.ts_drafter_reset(d)
            y = []
            i = 0
            while i < len(stream):
                step = int(rng.integers(1, 5))                    # append in steps of 1..4 tokens
                B.ts_drafter_append(d, stream[i:i + step])
                y += stream[i:i + step]
                i += step
                st, tool, ylen = B.ts_drafter_state(d)
                ost, otool, _ = DO.fsm_replay(s, y)
                assert (st, tool, ylen) == (ost, otool, len(y)), (s, y)
                max_nodes = int(rng.choice([64, 64, 7, 1]))
                toks, par, src = B.ts_drafter_draft(d, max_nodes)
                otoks, opar, osrc = DO.draft(s, calls, y, max_nodes)
                assert toks.tolist() == otoks and par.tolist() == opar and src == osrc, (s, calls, y)
        finally:
            B.ts_drafter_free(d)


def test_worked_examples_through_the_c_abi():
    g = json.load(open(GOLDEN))
    idx = {w: i for i, w in enumerate(g["vocab"])}
    enc = lambda ws: [idx[w] for w in ws]
    sc = g["schema"]
    s = {k: enc(sc[k]) for k in ("call_open", "name_prefix", "name_suffix", "param_prefix", "param_suffix", "value_end", "call_close")}
    s["tools"] = [enc(t) for t in sc["tools"]]
    s["params"] = [[enc(p) for p in ps] for ps in sc["params"]]
    d = B.ts_drafter_create(s)
    try:
        trees = {c["n_generated"]: c for c in g["tree_after"]}
        for n, (word, state, tool) in enumerate(g["fsm_trace"], start=1):
            B.ts_drafter_append(d, enc([word]))
            assert B.ts_drafter_state(d)[:2] == (state, tool)
            if n in trees:
                toks, par, src = B.ts_drafter_draft(d)
                assert toks.tolist() == enc(trees[n]["tokens"]) and par.tolist() == trees[n]["parents"] and src == trees[n]["source"]
        sm = g["suffix_match"]
        B.ts_drafter_retrieve(d, np.ones(2), np.ones((2, 2)), sm["calls"], k=10)
        B.ts_drafter_reset(d)
        B.ts_drafter_append(d, sm["y"])
        toks, par, src = B.ts_drafter_draft(d)
        want = DO.pack_tree(sm["drafts"])
        assert src == B_RETRIEVAL and toks.tolist() == want[0] and par.tolist() == want[1]
        assert len(toks) == 32 + 10                                # the two continuations share no prefix
    finally:
        B.ts_drafter_free(d)


B_RETRIEVAL = 1


def test_topk_retrieval_matches_the_oracle():
    rng = np.random.default_rng(12)
    s = _random_schema(rng, 10, 2)
    d = B.ts_drafter_create(s)
    try:
        for n_entries, dim, k in ((597, 64, 10), (5, 8, 10), (40, 16, 1), (0, 4, 10)):
            H = rng.standard_normal((n_entries, dim)).astype(np.float32)
            if n_entries > 6:
                H[3] = H[1]                                       # equal similarity: lower index first
                H[5] = 0.0                                        # zero vector: similarity 0
            h = rng.standard_normal(dim).astype(np.float32)
            calls = [[int(t) for t in rng.integers(0, 10, size=6)] for _ in range(n_entries)]
            top = B.ts_drafter_retrieve(d, h, H, calls, k=k)
            assert top == DO.topk_cosine(h, H, k)[0]
    finally:
        B.ts_drafter_free(d)


def test_error_paths():
    s = _random_schema(np.random.default_rng(1), 5, 2)
    bad = dict(s, value_end=[])
    with pytest.raises(B.TsError) as e:
        B.ts_drafter_create(bad)
    assert e.value.status == B.TS_ERR_INVALID_ARG
    bad = dict(s, tools=[[1], []])
    with pytest.raises(B.TsError):
        B.ts_drafter_create(bad)
    d = B.ts_drafter_create(s)
    try:
        with pytest.raises(B.TsError):
            B.ts_drafter_draft(d, 65)                              # more than TS_MAX_NODES
        toks, par, src = B.ts_drafter_draft(d, 0)
        assert len(toks) == 0 and src == 0
    finally:
        B.ts_drafter_free(d)


def test_drafting_latency_is_negligible_next_to_a_verify_step():
    """The paper attributes 5.7 % of the runtime to drafting and tree construction (Sec. 5.4); here a
    draft over 10 retrieved calls of 200 tokens must take far less than a millisecond."""
    rng = np.random.default_rng(8)
    s = _random_schema(rng, 1000, 20)
    calls = [[int(t) for t in rng.integers(0, 1000, size=200)] for _ in range(10)]
    d = B.ts_drafter_create(s)
    try:
        B.ts_drafter_retrieve(d, np.ones(8), np.ones((10, 8)), calls, k=10)
        B.ts_drafter_append(d, calls[3][:50])
        t0 = time.perf_counter()
        n = 2000
        for _ in range(n):
            toks, par, src = B.ts_drafter_draft(d)
        us = (time.perf_counter() - t0) / n * 1e6
        assert src == 1 and len(toks) > 0
        print("draft (suffix match over 10 x 200 tokens + tree packing, incl. ctypes): %.1f us" % us)
        assert us < 500
    finally:
        B.ts_drafter_free(d)
