"""CPU oracle for single-pass draft-tree verification.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain reference the HIP library is checked against.  It
is not part of the product: only tests, the smoke check and the benchmark's
cpu_baseline leg may import it, and it shares no code with the device path.

What it computes (paper: task formulation in Sec. 4.1; parallel verification in
App. A.1; the pack / verify / select-longest-accepted-prefix / append steps of
Alg. 1): the candidate drafts are flattened into one sequence of tree nodes,
the target decoder scores all of them in ONE forward pass in which a node
attends to the whole committed context, to its ancestors and to itself, and the
longest path whose every token equals the target's greedy choice is accepted,
followed by one bonus token.  By construction this equals plain greedy
decoding, only faster (the method preserves the target's output, Sec. 5.1
"Evaluation Metrics" and App. B.3).

Readings taken where the paper is silent (listed with reasons in the design
notes): acceptance is greedy (temperature-0 limit of speculative sampling);
the tree root is the pending token (last emitted token, K/V not yet cached)
and is row 0 of the pass; position of a node = committed length + depth; ties
between equally deep accepted paths go to the lowest node index, ties between
equal logits to the lowest token id; Llama-style block (RMSNorm, rotate-half
RoPE with inv_freq_j = theta^(-2j/hd), GQA, SwiGLU, no biases, untied head).

Arithmetic: float64 throughout.  Two modes for models stored in bfloat16:
  mode "E"  exact float64 math on the stored (bf16-valued) weights and context.
  mode "R"  same float64 math, but values are rounded (nearest even, via float32)
            at the points where the device path stores or feeds 16-bit values.
            bfloat16: new K/V cache entries.  IEEE half, the format of the paper's
            own runs (App. B, "Performance Comparison", Table 5: the one accuracy
            deviation is put down to fp16 precision): the rotated Q and the
            unnormalised softmax probabilities entering the P.V product (taken
            relative to the row maximum rounded up to a whole power of two, see
            forward_tree).  Every activation that enters a weight projection - the
            normalised activations, the attention output and the SwiGLU product -
            is carried as the sum of TWO halves, hi = half(x) (saturating at the
            largest finite half) and lo = half(x - hi), about 22 significant bits:
            a projection input as coarse as one half lets two correct
            implementations drift apart by whole half steps, more than the method's
            exactness (output identical to plain decoding, Sec. 5.1 "Evaluation
            Metrics", App. B.3) can absorb at near-tied logits.  bf16 K/V entries and bf16 weights widen to half
            exactly in half's normal range; the device re-encodes the projection
            weights as half once at load (magnitudes below 2^-14 move by less than
            3e-8; not modelled here).  The residual stream and the logits are never
            rounded.  Integer decisions (argmax, acceptance) are compared in this
            mode so both sides decide in the same precision.

Pins (tests/test_oracle_*.py): brute-force agreement with an independently
written dense causal decoder on every root-to-node path; chain == causal
chunk; star tree; MHA == GQA with replicated heads; closed forms for RMSNorm,
uniform softmax, RoPE; zeroed output projections; library routines (torch
rms_norm / scaled_dot_product_attention / silu); losslessness against plain
greedy decoding; acceptance walk against exhaustive path enumeration.
Absolute logit values of a random 8B-shaped model have no external pin
("parity unpinned" beyond the agreements above): the paper prints no numeric
example of a forward pass.
"""
import numpy as np

DTYPE_F32 = 0
DTYPE_BF16 = 1
LOG2E = 1.4426950408889634


# --------------------------------------------------------------------------- #
# number formats
# --------------------------------------------------------------------------- #
def bf16_round(x):
    """Round float64 -> float32 -> bfloat16 (nearest even), returned as float64."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    b = f.view(np.uint32).astype(np.uint64)
    lsb = (b >> np.uint64(16)) & np.uint64(1)
    r = ((b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    return r.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def fp16_round(x):
    """Round float64 -> float32 -> IEEE half (nearest even), returned as float64."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float16).astype(np.float64)


def fp16_act_round(x):
    """A single IEEE half, saturating at the largest finite half."""
    return fp16_round(np.clip(np.asarray(x, dtype=np.float64), -65504.0, 65504.0))


def fp16_pair_round(x):
    """Activation entering a projection: hi + lo with hi = half(x), saturating at the largest
    finite half, and lo = half(x - hi)."""
    xs = np.clip(np.asarray(x, dtype=np.float64), -65504.0, 65504.0)
    hi = fp16_round(xs)
    return hi + fp16_round(xs - hi)


def _widen(a):
    """Stored tensor (float32, or uint16 bf16 bit patterns) -> float64, exactly."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------- #
# model pieces
# --------------------------------------------------------------------------- #
def rmsnorm(x, g, eps):
    """x * rsqrt(mean(x^2) + eps) * g over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x, pos, theta):
    """Rotary embedding, rotate-half pairing.  x: [rows][heads][hd], pos: [rows].
    Pair (j, j + hd/2) is rotated by angle pos * theta^(-2j/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None, None] * inv_freq[None, None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


class OracleModel:
    """Weights as handed to the device loader; widened to float64 on use.

    `weights` is {"embed","lm_head","norm_f","layers":[{wq,wk,wv,wo,wg,wu,wd,
    norm1,norm2}]}, matrices row-major [out][in] (y = x W^T).  `layers` may also
    be a callable layer -> dict, so that big shapes are produced one layer at a
    time.  With cache=True widened float32 copies are kept between calls.
    """

    def __init__(self, cfg, weights, cache=False):
        self.cfg = cfg
        self.w = weights
        self._cache = {} if cache else None

    def tensor(self, kind, layer=-1):
        key = (kind, layer)
        if self._cache is not None and key in self._cache:
            return self._cache[key].astype(np.float64)
        if layer < 0:
            a = self.w[kind]
        else:
            lay = self.w["layers"]
            a = (lay(layer) if callable(lay) else lay[layer])[kind]
        if self._cache is not None:
            a32 = _widen(a).astype(np.float32)      # exact: stored values fit float32
            self._cache[key] = a32
            return a32.astype(np.float64)
        return _widen(a)

    def embed_rows(self, tokens):
        e = self.w["embed"]
        return _widen(np.asarray(e)[np.asarray(tokens, dtype=np.int64)])


class OracleKV:
    """Per-sequence K/V store: position-major, float64, [L][capacity][Hkv][hd]."""

    def __init__(self, cfg, capacity):
        shp = (cfg.n_layers, capacity, cfg.n_kv_heads, cfg.head_dim)
        self.K = np.zeros(shp, dtype=np.float64)
        self.V = np.zeros(shp, dtype=np.float64)
        self.P = 0                 # committed positions
        self.pending = None        # root token of the next verify
        self.capacity = capacity

    def import_context(self, K, V):
        n = K.shape[1]
        self.K[:, :n] = _widen(K)
        self.V[:, :n] = _widen(V)
        self.P = n


# --------------------------------------------------------------------------- #
# tree bookkeeping (Alg. 1: pack drafts as a flattened sequence + tree mask)
# --------------------------------------------------------------------------- #
def tree_rows(root_token, draft_tokens, parent_idx):
    """Rows of the pass: row 0 = root, row i+1 = draft node i.
    Returns tok[M], par[M] (row index of the parent, -1 for the root row),
    depth[M], vis[M][M] with vis[r][s] = 1 iff s is r or an ancestor row of r."""
    n = len(draft_tokens)
    M = n + 1
    tok = np.empty(M, dtype=np.int64)
    par = np.empty(M, dtype=np.int64)
    depth = np.zeros(M, dtype=np.int64)
    vis = np.zeros((M, M), dtype=bool)
    tok[0], par[0] = root_token, -1
    vis[0, 0] = True
    for i in range(n):
        p = int(parent_idx[i])
        if not (-1 <= p < i):
            raise ValueError("parent_idx must satisfy -1 <= parent_idx[i] < i")
        r = i + 1
        tok[r] = draft_tokens[i]
        par[r] = p + 1
        depth[r] = depth[par[r]] + 1
        vis[r] = vis[par[r]]
        vis[r, r] = True
    return tok, par, depth, vis


# --------------------------------------------------------------------------- #
# the single forward pass with the tree mask (App. A.1)
# --------------------------------------------------------------------------- #
def forward_tree(model, kv, tok, depth, vis, mode="E", layer_limit=None, return_hidden=False):
    """Scores all rows in one pass.  Returns (logits[M][V], newK, newV) with
    newK/newV [L][M][Hkv][hd] = the K/V rows of the pass (row r belongs at
    slot P + r until commit).  Does not modify `kv`.  With return_hidden also the
    final normalised hidden state [M][d] the logits were computed from (the last-token
    representation h_x of Sec. 4.3 when the row is a question's last token)."""
    cfg = model.cfg
    rounding = mode == "R" and cfg.dtype == DTYPE_BF16
    rb = bf16_round if rounding else (lambda a: a)               # single bf16 value
    ra = fp16_pair_round if rounding else (lambda a: a)          # projection inputs: hi + lo halves
    rh = fp16_round if rounding else (lambda a: a)               # half precision (attention operands)
    M = len(tok)
    P = kv.P
    Hq, Hkv, hd = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = Hq // Hkv
    L = cfg.n_layers if layer_limit is None else layer_limit
    pos = P + np.asarray(depth)
    scale = 1.0 / np.sqrt(float(hd))

    X = model.embed_rows(tok)                                   # [M][d]
    newK = np.zeros((cfg.n_layers, M, Hkv, hd))
    newV = np.zeros((cfg.n_layers, M, Hkv, hd))
    for l in range(L):
        Xn = ra(rmsnorm(X, model.tensor("norm1", l), cfg.rms_eps))
        Q = (Xn @ model.tensor("wq", l).T).reshape(M, Hq, hd)
        K = (Xn @ model.tensor("wk", l).T).reshape(M, Hkv, hd)
        V = (Xn @ model.tensor("wv", l).T).reshape(M, Hkv, hd)
        Q = rh(rope(Q, pos, cfg.rope_theta))
        K = rb(rope(K, pos, cfg.rope_theta))
        V = rb(V)
        newK[l], newV[l] = K, V

        A = np.zeros((M, Hq, hd))
        for h in range(Hq):
            g = h // G
            Kc, Vc = kv.K[l, :P, g, :], kv.V[l, :P, g, :]          # committed context
            s_ctx = (Q[:, h, :] @ Kc.T) * scale                     # [M][P]  all visible
            s_tree = (Q[:, h, :] @ K[:, g, :].T) * scale            # [M][M]  masked
            s_tree = np.where(vis, s_tree, -np.inf)
            s = np.concatenate([s_ctx, s_tree], axis=1)
            if rounding:
                # half-precision probabilities: exponentials relative to the row maximum
                # rounded UP to a whole power of two.  Rounding commutes with scaling by
                # powers of two (above the subnormal range), so this is independent of the
                # order in which keys are visited.
                t = s * LOG2E
                m = np.ceil(np.max(t, axis=1, keepdims=True))
                p = rh(np.exp2(t - m))                              # masked entries -> 0
            else:
                m = np.max(s, axis=1, keepdims=True)
                p = np.exp(s - m)                                   # masked entries -> 0
            denom = np.sum(p, axis=1, keepdims=True)
            vals = np.concatenate([Vc, V[:, g, :]], axis=0)         # [P+M][hd]
            A[:, h, :] = (p @ vals) / denom
        A = ra(A.reshape(M, Hq * hd))
        X = X + A @ model.tensor("wo", l).T

        Xn = ra(rmsnorm(X, model.tensor("norm2", l), cfg.rms_eps))
        gate = Xn @ model.tensor("wg", l).T
        up = Xn @ model.tensor("wu", l).T
        act = ra(silu(gate) * up)
        X = X + act @ model.tensor("wd", l).T

    Xf = ra(rmsnorm(X, model.tensor("norm_f"), cfg.rms_eps))
    logits = Xf @ model.tensor("lm_head").T
    if return_hidden:
        return logits, newK, newV, Xf
    return logits, newK, newV


# --------------------------------------------------------------------------- #
# greedy acceptance (Alg. 1: select the longest accepted prefix)
# --------------------------------------------------------------------------- #
def accept_walk(g, tok, par, depth):
    """g[r] = the target's greedy token after row r.  A row is valid iff its parent
    is valid and its token equals the parent's greedy token; the root is valid.
    Returns (best_row, path_rows root-exclusive, valid[M])."""
    M = len(tok)
    valid = np.zeros(M, dtype=bool)
    valid[0] = True
    best = 0
    for r in range(1, M):
        valid[r] = valid[par[r]] and (tok[r] == g[par[r]])
        if valid[r] and depth[r] > depth[best]:
            best = r
    path = []
    r = best
    while r > 0:
        path.append(r)
        r = par[r]
    return best, path[::-1], valid


class VerifyResult:
    pass


def verify(model, kv, draft_tokens, parent_idx, mode="E"):
    """One verification step; `kv` is left untouched (commit applies the result)."""
    if kv.pending is None:
        raise ValueError("no pending root token")
    n = len(draft_tokens)
    if kv.P + n + 1 > kv.capacity:
        raise ValueError("KV capacity exceeded")
    tok, par, depth, vis = tree_rows(kv.pending, draft_tokens, parent_idx)
    logits, newK, newV = forward_tree(model, kv, tok, depth, vis, mode)
    g = np.argmax(logits, axis=1)                  # first maximum = lowest id
    best, path, valid = accept_walk(g, tok, par, depth)
    top2 = np.partition(logits, -2, axis=1)[:, -2:]
    margin = top2[:, 1] - top2[:, 0]
    r = VerifyResult()
    r.accept_len = len(path)
    r.accepted_nodes = [p - 1 for p in path]
    r.accepted_tokens = [int(tok[p]) for p in path]
    r.bonus_token = int(g[best])
    r.logits, r.greedy, r.valid, r.margin = logits, g, valid, margin
    r.rows = (tok, par, depth, vis)
    r.path_rows, r.best_row = path, best
    r.newK, r.newV = newK, newV
    # the smallest top-2 margin among rows whose argmax steered the walk
    r.decisive_margin = float(np.min(margin[valid]))
    return r


def commit(kv, res):
    """Root K/V -> slot P; accepted row of depth d -> slot P+d; P += accept_len+1;
    the bonus token becomes the pending root of the next step."""
    P = kv.P
    kv.K[:, P] = res.newK[:, 0]
    kv.V[:, P] = res.newV[:, 0]
    for d, row in enumerate(res.path_rows, start=1):
        kv.K[:, P + d] = res.newK[:, row]
        kv.V[:, P + d] = res.newV[:, row]
    kv.P = P + res.accept_len + 1
    kv.pending = res.bonus_token


def greedy_decode(model, kv, n_tokens, mode="E"):
    """Plain autoregressive greedy decoding = verify with an empty tree, n_tokens
    times.  Returns the emitted tokens; advances `kv`."""
    out = []
    empty = np.zeros(0, dtype=np.int32)
    for _ in range(n_tokens):
        r = verify(model, kv, empty, empty, mode)
        commit(kv, r)
        out.append(r.bonus_token)
    return out
