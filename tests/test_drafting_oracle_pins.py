"""Pins of the drafting oracle (CPU only): hand-worked examples from the paper's rules,
library routines, closed forms and invariants - none of them produced by the oracle itself."""
import json
import os

import numpy as np
import pytest

from oracle import drafting_oracle as DO

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "drafting_worked_examples.json")


def _load():
    d = json.load(open(GOLDEN))
    idx = {w: i for i, w in enumerate(d["vocab"])}
    enc = lambda ws: [idx[w] for w in ws]
    s = d["schema"]
    schema = {k: enc(s[k]) for k in ("call_open", "name_prefix", "name_suffix", "param_prefix", "param_suffix", "value_end", "call_close")}
    schema["tools"] = [enc(t) for t in s["tools"]]
    schema["params"] = [[enc(p) for p in ps] for ps in s["params"]]
    return d, schema, enc


def test_fsm_follows_the_hand_worked_trace():
    """Sec. 4.2 / Fig. 2 walk-through: state and selected tool after every token."""
    d, schema, enc = _load()
    y = []
    for word, state, tool in d["fsm_trace"]:
        y += enc([word])
        got = DO.fsm_replay(schema, y)
        assert (got[0], got[1]) == (state, tool), "after %r: %r" % (word, got)
    off = d["off_schema"]
    st = DO.fsm_replay(schema, enc(off["y"]))
    assert (st[0], st[1]) == (off["state"], off["tool"])


def test_schema_draft_trees_match_the_hand_worked_ones():
    """Eq. 2 drafts packed as a tree (App. A.1), worked by hand at four points of the trace."""
    d, schema, enc = _load()
    y_all = enc([w for w, _, _ in d["fsm_trace"]])
    for case in d["tree_after"]:
        toks, par, src = DO.draft(schema, [], y_all[:case["n_generated"]])
        assert toks == enc(case["tokens"]) and par == case["parents"] and src == case["source"], case["n_generated"]


def test_eq2_paths_are_prefix_name_suffix():
    """In q_t with nothing generated yet the root-to-leaf paths are exactly prefix (+) name (+) suffix."""
    d, schema, enc = _load()
    toks, par, _ = DO.draft(schema, [], schema["call_open"])
    leaves = set(range(len(toks))) - set(par)
    paths = set()
    for leaf in leaves:
        p, n = [], leaf
        while n >= 0:
            p.append(toks[n])
            n = par[n]
        paths.add(tuple(p[::-1]))
    want = {tuple(schema["name_prefix"] + t + schema["name_suffix"]) for t in schema["tools"]}
    assert paths == want


def test_suffix_match_hand_worked_example():
    """Eq. 4 + App. B.2: longest suffix first, continuations 32 / 16 / 8 / 8 in order of occurrence."""
    d, _, _ = _load()
    sm = d["suffix_match"]
    assert DO.suffix_match_drafts(sm["y"], sm["calls"]) == sm["drafts"]
    assert DO.suffix_match_drafts(sm["y_short"], sm["calls"])[0] == sm["drafts_short_first"]
    assert DO.suffix_match_drafts([1, 2, 3, 4], sm["calls"]) == []          # shorter than the shortest suffix


def _find_all(hay, needle):
    """Occurrences of a token sequence, by the bytes.find library routine."""
    hb = np.asarray(hay, "<i4").tobytes()
    nb = np.asarray(needle, "<i4").tobytes()
    out, start = [], 0
    while True:
        i = hb.find(nb, start)
        if i < 0:
            return out
        if i % 4 == 0:
            out.append(i // 4)
        start = i + 1


def test_suffix_match_against_library_search_on_random_streams():
    rng = np.random.default_rng(5)
    hits = 0
    for trial in range(300):
        calls = [list(rng.integers(0, 3, size=int(rng.integers(5, 80)))) for _ in range(int(rng.integers(1, 5)))]
        y = list(rng.integers(0, 3, size=int(rng.integers(3, 30))))
        drafts = DO.suffix_match_drafts(y, calls)
        # the definition, through the library search: the longest L in {7,6,5} with any usable occurrence
        want = []
        for L in (7, 6, 5):
            if len(y) < L:
                continue
            occ = [(c, p + L) for c, call in enumerate(calls) for p in _find_all(call, y[-L:]) if p + L < len(call)]
            if occ:
                want = [calls[c][m:m + n] for (c, m), n in zip(occ, (32, 16, 8, 8))]
                break
        assert drafts == want
        hits += bool(drafts)
    assert hits > 50


def test_topk_cosine_against_library_routines():
    from sklearn.metrics.pairwise import cosine_similarity
    rng = np.random.default_rng(9)
    H = rng.standard_normal((597, 64))
    h = rng.standard_normal(64)
    idx, sims = DO.topk_cosine(h, H, 10)
    ref = cosine_similarity(h[None], H)[0]
    assert np.allclose(sims, ref, atol=1e-12)
    assert idx == list(np.argsort(-ref, kind="stable")[:10])
    assert DO.topk_cosine(3.0 * h, 0.5 * H, 10)[0] == idx                    # scale invariance of the cosine
    # equal similarities rank by index; zero vectors have similarity 0
    H2 = np.stack([h, np.zeros(64), 2 * h, -h])
    assert DO.topk_cosine(h, H2, 4)[0] == [0, 2, 1, 3]
    assert DO.topk_cosine(h, H2, 10)[0] == [0, 2, 1, 3]                      # k larger than the datastore


def test_pack_tree_is_the_trie_of_the_drafts():
    """Closed form: one node per distinct non-empty prefix; parents precede children; the set of
    root-to-node paths is the prefix closure of the drafts."""
    rng = np.random.default_rng(3)
    for trial in range(200):
        drafts = [list(rng.integers(0, 4, size=int(rng.integers(1, 9)))) for _ in range(int(rng.integers(1, 7)))]
        toks, par = DO.pack_tree(drafts, 64)
        prefixes = {tuple(d[:i]) for d in drafts for i in range(1, len(d) + 1)}
        assert len(toks) == len(prefixes)
        paths = set()
        for n in range(len(toks)):
            assert -1 <= par[n] < n
            p, m = [], n
            while m >= 0:
                p.append(toks[m])
                m = par[m]
            paths.add(tuple(p[::-1]))
        assert paths == prefixes
        # truncation keeps a prefix-closed part of the same numbering
        t2, p2 = DO.pack_tree(drafts, 5)
        assert len(t2) == min(5, len(toks))
        for n in range(len(t2)):
            assert -1 <= p2[n] < n


def test_alg1_prefers_retrieval_over_schema():
    d, schema, enc = _load()
    y = enc(["Sure", "<tool_call>"])
    calls = [[7, 7, 7] + y[-1:] * 0 + [40, 41, 42, 43, 44] + y + [77, 78, 79]]
    # y is only 2 tokens long: no suffix of length 5 exists, schema drafts are used
    assert DO.draft(schema, calls, y)[2] == DO.DRAFT_SCHEMA
    y5 = [40, 41, 42, 43, 44] + y
    toks, par, src = DO.draft(schema, calls, y5)
    assert src == DO.DRAFT_RETRIEVAL and toks == [77, 78, 79] and par == [-1, 0, 1]
