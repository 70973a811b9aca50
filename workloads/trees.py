"""Draft-tree shapes of the tool-calling workloads, as (draft_tokens, parent_idx).

`parent_idx[i]` is the index of node i's parent among the draft nodes, or -1
when node i hangs off the root (the pending token, which is not a draft node).
Parents always precede children.  Tokens come from a greedy continuation
`greedy = [g_1, g_2, ...]` (g_k = what plain greedy decoding would emit k steps
after the root) supplied by the caller, each replaced by a uniform random id
with a given mutation probability; where `greedy` is too short the missing
tokens are uniform random ids.

Shapes mirror the drafting sources of the method: a schema-fixed chain, sibling
alternatives for a constrained field such as the tool name, an argument chain,
and retrieved continuations of preset lengths (32, 16, 8, 8).
"""
import numpy as np


def _g(greedy, k, vocab, rng):
    """g_k (1-based depth) or a uniform id past the end of `greedy`."""
    if k - 1 < len(greedy):
        return int(greedy[k - 1])
    return int(rng.integers(vocab))


def _mut(tok, p, vocab, rng):
    if rng.random() < p:
        return int(rng.integers(vocab))
    return tok


def mutate_chain(greedy, n, p, vocab, rng, first_depth=1):
    return [_mut(_g(greedy, first_depth + i, vocab, rng), p, vocab, rng) for i in range(n)]


def chain_tree(greedy, n, p, vocab, rng):
    """Single linear chain of n nodes below the root."""
    toks = mutate_chain(greedy, n, p, vocab, rng)
    par = [-1] + list(range(n - 1))
    return np.asarray(toks, np.int32), np.asarray(par[:n], np.int32)


def _append_chain(toks, par, parent, chain):
    for t in chain:
        toks.append(t)
        par.append(parent)
        parent = len(toks) - 1
    return parent


def schema_retrieval_tree(greedy, vocab, rng, p_schema=0.05, p_args=0.2,
                          p_retrieved=(0.05, 0.2, 0.5, 0.8)):
    """64 nodes: 12-token schema chain, 8 sibling alternatives under its end (one of
    them the greedy token, at a random slot), a 12-token argument chain under that
    sibling, and four 8-token retrieved chains from the root."""
    toks, par = [], []
    end = _append_chain(toks, par, -1, mutate_chain(greedy, 12, p_schema, vocab, rng))
    slot = int(rng.integers(8))
    good = _mut(_g(greedy, 13, vocab, rng), p_schema, vocab, rng)
    others = set()
    while len(others) < 7:
        t = int(rng.integers(vocab))
        if t != good:
            others.add(t)
    others = sorted(others)
    rng.shuffle(others)
    good_node = -1
    for s in range(8):
        if s == slot:
            toks.append(good)
            good_node = len(toks)
        else:
            toks.append(int(others.pop()))
        par.append(end)
    good_node -= 1
    _append_chain(toks, par, good_node,
                  mutate_chain(greedy, 12, p_args, vocab, rng, first_depth=14))
    for p in p_retrieved:
        _append_chain(toks, par, -1, mutate_chain(greedy, 8, p, vocab, rng))
    assert len(toks) == 64
    return np.asarray(toks, np.int32), np.asarray(par, np.int32)


def retrieval_tree(greedy, vocab, rng, lengths=(32, 16, 8, 8), p=(0.05, 0.2, 0.5, 0.8)):
    """Retrieved continuations of the preset lengths, each a chain from the root."""
    toks, par = [], []
    for n, pp in zip(lengths, p):
        _append_chain(toks, par, -1, mutate_chain(greedy, n, pp, vocab, rng))
    return np.asarray(toks, np.int32), np.asarray(par, np.int32)


def bfs_tree(greedy, n_nodes, vocab, rng, max_branch=4, max_depth=12, p_keep=0.7):
    """Breadth-first growth: each expanded node gets 1..max_branch children until
    n_nodes exist; child 0 is the greedy token of its depth with probability p_keep,
    the other siblings are distinct uniform ids."""
    toks, par, depth = [], [], []
    queue = [(-1, 0)]
    while queue and len(toks) < n_nodes:
        node, d = queue.pop(0)
        if d + 1 > max_depth:
            continue
        b = int(rng.integers(1, max_branch + 1))
        b = min(b, n_nodes - len(toks))
        used = set()
        for c in range(b):
            if c == 0 and rng.random() < p_keep:
                t = _g(greedy, d + 1, vocab, rng)
            else:
                t = int(rng.integers(vocab))
                while t in used:
                    t = int(rng.integers(vocab))
            used.add(t)
            toks.append(t)
            par.append(node)
            depth.append(d + 1)
            queue.append((len(toks) - 1, d + 1))
    return np.asarray(toks, np.int32), np.asarray(par, np.int32)


def random_tree(n_nodes, vocab, rng):
    """Uniformly random shape and tokens: node i hangs off a uniform choice among the root and
    the nodes before it; every token is a uniform id.  Nothing in it follows the target's
    greedy choice, so almost every row's decision is between two arbitrary near-top tokens."""
    par = np.array([rng.integers(-1, i) for i in range(n_nodes)], dtype=np.int32)
    tok = rng.integers(vocab, size=n_nodes).astype(np.int32)
    return tok, par


def decision_sweep_case(cfg, t, P=512, n_nodes=64):
    """Case t of the arg-max decision sweep: (context K, V, root token, draft tokens, parents)."""
    from .kv import gen_context_kv
    rng = np.random.default_rng([777, t])
    K, V = gen_context_kv(cfg, P, seed=4000 + t)
    root = int(rng.integers(cfg.vocab))
    tok, par = random_tree(n_nodes, cfg.vocab, rng)
    return K, V, root, tok, par


def root_token(vocab, P, seed=3456):
    """Pending (root) token of the synthetic-context workloads: one seeded uniform id."""
    return int(np.random.default_rng([seed, P]).integers(vocab))


def load_greedy(path):
    """Token ids (first column) of a stored greedy-continuation file; [] if absent."""
    import os
    if not os.path.exists(path):
        return []
    out = []
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            out.append(int(line.split()[0]))
    return out


def tree_depths(parent_idx):
    """Depth of every draft node (children of the root have depth 1)."""
    d = np.zeros(len(parent_idx), np.int32)
    for i, p in enumerate(parent_idx):
        d[i] = 1 if p < 0 else d[p] + 1
    return d
