"""CPU oracle of stochastic acceptance on a draft tree (test infrastructure only).

The paper accepts drafts by speculative sampling (Sec. 5.1 setup, App. B.2, citing Leviathan
et al. 2023) at batch 1.  With deterministic drafts every candidate's draft distribution is a
point mass, so the accept / resample rule of that scheme becomes, at a row with target
distribution p = softmax(logits / T) and children c_1, c_2, ... in node order:

    accept c_i with probability p(x_i) / (1 - sum of p over the rejected siblings' tokens);
    on rejection the token x_i is removed from the distribution (residual max(0, p - q),
    renormalised); a sibling repeating an already rejected token is rejected outright;
    if every child is rejected, the step's last token is a sample of the residual.

The emitted tokens are then distributed exactly as the target's own samples (lossless in
distribution).  Randomness: one uniform per draft node, passed in; the residual sample is the
arg-max of logits / T + Gumbel noise over the tokens that are not excluded (Gumbel-max), with
noise from a counter-based generator (one splitmix64 output per (seed, row, token)) that the
device implements as well.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.
"""
import numpy as np

_M64 = (1 << 64) - 1


def splitmix64(state):
    """Output function of the splitmix64 generator for a 64-bit state (one step)."""
    z = (int(state) + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def gumbel_noise(seed, row, n_vocab):
    """Gumbel(0,1) noise of one row: u = (top 23 bits + 0.5) / 2^23 (exact in single precision as
    well), g = -log(-log u)."""
    v = np.arange(n_vocab, dtype=np.uint64)
    s = (np.uint64(seed & _M64) + ((np.uint64(row) << np.uint64(32)) | v))
    z = s + np.uint64(0x9E3779B97F4A7C15)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    z = z ^ (z >> np.uint64(31))
    u = ((z >> np.uint64(41)).astype(np.float64) + 0.5) / float(1 << 23)
    return -np.log(-np.log(u))


class SampleResult:
    pass


def sample_walk(logits, tok, par, temperature, node_uniform, seed):
    """Stochastic acceptance over the rows of one pass.

    logits [M][V]; tok / par: row tokens and parent rows (row 0 = root, par[0] = -1);
    node_uniform[i] in [0,1) for draft node i (row i+1).  Returns accept_len,
    accepted_tokens, accepted_nodes, bonus_token and, for the tolerance rule of the tests,
    the smallest |u - acceptance probability| over the decisions taken and the top-2 gap of the
    perturbed scores the bonus token was chosen from."""
    logits = np.asarray(logits, np.float64)
    M, V = logits.shape
    with np.errstate(over="ignore"):
        seed = int(seed) & _M64
    inv_t = 1.0 / float(temperature)
    r = 0
    path = []
    decision_gap = np.inf
    while True:
        z = logits[r] * inv_t
        lse = np.max(z) + np.log(np.sum(np.exp(z - np.max(z))))
        rem = 1.0
        rejected = []
        nxt = -1
        for c in range(1, M):
            if par[c] != r:
                continue
            x = int(tok[c])
            if x in rejected:
                continue
            p = float(np.exp(z[x] - lse))
            q = p / rem
            decision_gap = min(decision_gap, abs(float(node_uniform[c - 1]) - q))
            if float(node_uniform[c - 1]) < q:
                nxt = c
                break
            rejected.append(x)
            rem -= p
        if nxt < 0:
            score = z + gumbel_noise(seed, r, V)
            score[rejected] = -np.inf
            bonus = int(np.argmax(score))
            top2 = np.partition(score, -2)[-2:]
            res = SampleResult()
            res.accept_len = len(path)
            res.accepted_nodes = [c - 1 for c in path]
            res.accepted_tokens = [int(tok[c]) for c in path]
            res.bonus_token = bonus
            res.stop_row = r
            res.decision_gap = float(decision_gap)
            res.bonus_gap = float(top2[1] - top2[0])
            return res
        path.append(nxt)
        r = nxt
