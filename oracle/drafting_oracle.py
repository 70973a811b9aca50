"""CPU oracle of the host-side drafting steps (test infrastructure only).

Plain, slow and stateless Python written from the paper: every function recomputes its
answer from the whole generated output y, so it shares neither code nor state handling with
the incremental C++ drafter it checks.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this module.

  topk_cosine          Sec. 4.3, Eq. 3: Top-K of cos(h_x, h_j); k = 10 in App. B.2
  suffix_match_drafts  Sec. 4.3, Eq. 4 + App. B.2: L in {7, 6, 5} longest first, continuations
                       of lengths 32, 16, 8, 8 taken in order of occurrence
  fsm_replay           Sec. 4.2, Fig. 2: delta folded over y from q0
  schema_drafts        Sec. 4.2, Eq. 2: prefix (+) tool_name (+) suffix (and the same for
                       parameter names), minus what has been generated already
  pack_tree            App. A.1: drafts compacted into one flattened sequence under a tree mask
  draft                Alg. 1: retrieval drafts if the suffix matches, else schema drafts

Readings where the paper is silent (the C++ header states the same ones): the schema is a set
of token sequences; a structural state ends when one candidate is fully generated and is left
for "others" when no candidate fits; delimiters are tested on the tokens generated inside the
value state, call_close before value_end; equal similarities rank by index; a match at the
very end of a historical call has no continuation and is skipped.
"""
import numpy as np

Q_OTHERS, Q_TOOL_NAME, Q_PARAM_NAME, Q_PARAM_VALUE = 0, 1, 2, 3
DRAFT_NONE, DRAFT_RETRIEVAL, DRAFT_SCHEMA = 0, 1, 2
SUFFIX_LENGTHS = (7, 6, 5)
CONTINUATION_LENGTHS = (32, 16, 8, 8)


def topk_cosine(h_x, H, k):
    """Indices of the k rows of H most similar to h_x (cosine), most similar first."""
    h = np.asarray(h_x, np.float64)
    H = np.asarray(H, np.float64).reshape(-1, h.shape[0])
    nh = np.sqrt(np.sum(h * h))
    sims = []
    for j in range(H.shape[0]):
        nj = np.sqrt(np.sum(H[j] * H[j]))
        sims.append(float(np.dot(H[j], h) / (nh * nj)) if nh > 0 and nj > 0 else 0.0)
    order = sorted(range(len(sims)), key=lambda j: (-sims[j], j))
    return order[:max(0, min(k, len(order)))], sims


def suffix_match_drafts(y, calls):
    """Continuations after occurrences of y's last L tokens in the retrieved calls."""
    y = [int(t) for t in y]
    for L in SUFFIX_LENGTHS:
        if len(y) < L:
            continue
        pat = y[len(y) - L:]
        drafts = []
        for call in calls:
            call = [int(t) for t in call]
            for m in range(L, len(call) + 1):
                if len(drafts) == len(CONTINUATION_LENGTHS):
                    break
                if call[m - L:m] == pat:
                    cont = call[m:m + CONTINUATION_LENGTHS[len(drafts)]]
                    if cont:
                        drafts.append(cont)
        if drafts:
            return drafts
    return []


def _candidates(schema, state, tool):
    if state == Q_TOOL_NAME:
        return [list(schema["name_prefix"]) + list(t) + list(schema["name_suffix"]) for t in schema["tools"]]
    if state == Q_PARAM_NAME:
        return [list(schema["param_prefix"]) + list(p) + list(schema["param_suffix"]) for p in schema["params"][tool]]
    return []


def fsm_replay(schema, y):
    """(state, tool, tokens generated since the structural state was entered)."""
    state, tool, since, in_value = Q_OTHERS, -1, [], 0
    out = []
    co, cc, ve = list(schema["call_open"]), list(schema["call_close"]), list(schema["value_end"])
    for x in y:
        x = int(x)
        out.append(x)
        if state in (Q_TOOL_NAME, Q_PARAM_NAME):
            since = since + [x]
            cands = _candidates(schema, state, tool)
            full = [i for i, c in enumerate(cands) if c == since]
            if full:
                if state == Q_TOOL_NAME:
                    state, tool = Q_PARAM_NAME, full[0]
                else:
                    state, in_value = Q_PARAM_VALUE, 0
                since = []
            elif not any(c[:len(since)] == since for c in cands):
                state, tool, since = Q_OTHERS, -1, []
        elif state == Q_PARAM_VALUE:
            in_value += 1
            if in_value >= len(cc) and out[len(out) - len(cc):] == cc:
                state, tool = Q_OTHERS, -1
            elif in_value >= len(ve) and out[len(out) - len(ve):] == ve:
                state, since = Q_PARAM_NAME, []
            continue
        if state == Q_OTHERS and len(out) >= len(co) and out[len(out) - len(co):] == co:
            state, since = Q_TOOL_NAME, []
    return state, tool, since


def schema_drafts(schema, y):
    state, tool, since = fsm_replay(schema, y)
    return [c[len(since):] for c in _candidates(schema, state, tool)
            if c[:len(since)] == since and len(c) > len(since)]


def pack_tree(drafts, max_nodes=64):
    """Trie of the drafts: (draft_tokens, parent_idx), nodes in creation order."""
    toks, par = [], []
    children = {}                      # (parent node or -1, token) -> node
    for dr in drafts:
        node = -1
        for t in dr:
            key = (node, int(t))
            if key not in children:
                if len(toks) >= max_nodes:
                    break
                children[key] = len(toks)
                toks.append(int(t))
                par.append(node)
            node = children[key]
    return toks, par


def draft(schema, calls, y, max_nodes=64):
    """(draft_tokens, parent_idx, source) of the next step."""
    drafts = suffix_match_drafts(y, calls)
    source = DRAFT_RETRIEVAL
    if not drafts:
        drafts = schema_drafts(schema, y)
        source = DRAFT_SCHEMA
    toks, par = pack_tree(drafts, max_nodes)
    return toks, par, (source if toks else DRAFT_NONE)
