"""Pins of the stochastic-acceptance oracle (CPU only)."""
import numpy as np
from scipy import stats

from oracle import sampling_oracle as SO
from oracle import toolspec_oracle as O


def test_splitmix64_known_answers():
    """Published test vectors of splitmix64 seeded with 0 (first three outputs) and the single-step form
    used here: output(state) for state = 0, golden, 2 * golden."""
    g = 0x9E3779B97F4A7C15
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [SO.splitmix64((i * g) & ((1 << 64) - 1)) for i in range(3)] == want
    # the vectorised row generator is the same function of (seed, row, token)
    seed, row = 0x1234567890ABCDEF, 7
    gn = SO.gumbel_noise(seed, row, 5)
    for v in range(5):
        z = SO.splitmix64((seed + ((row << 32) | v)) & ((1 << 64) - 1))
        u = ((z >> 41) + 0.5) / (1 << 23)
        assert abs(gn[v] - (-np.log(-np.log(u)))) < 1e-12


def test_gumbel_max_samples_follow_the_softmax():
    """Gumbel-max with this generator: arg-max of z + g over many rows is distributed as softmax(z)."""
    z = np.array([0.3, -1.2, 2.0, 0.0, 1.1, -0.4])
    p = np.exp(z) / np.sum(np.exp(z))
    counts = np.zeros(6)
    n = 40000
    for row in range(n):
        counts[int(np.argmax(z + SO.gumbel_noise(99, row, 6)))] += 1
    chi2 = np.sum((counts - n * p) ** 2 / (n * p))
    assert chi2 < stats.chi2.ppf(0.999, df=5), (chi2, counts / n, p)


def _tree(kind):
    if kind == "siblings":            # three candidates for the first token, one continues
        return [7, 1, 2, 3, 4], [-1, 0, 0, 0, 2]       # rows: root, a, b, c, child of b
    if kind == "chain":
        return [7, 1, 2, 3], [-1, 0, 1, 2]
    return [7, 1, 1, 2], [-1, 0, 0, 0]                  # duplicate sibling token


def test_first_emitted_token_is_distributed_as_the_target():
    """The defining property (lossless in distribution): whatever the drafts, the first token of the
    step - accepted draft or residual sample - follows softmax(logits[root] / T)."""
    rng = np.random.default_rng(0)
    V, T = 6, 0.8
    for kind in ("siblings", "chain", "dup"):
        tok, par = _tree(kind)
        logits = rng.standard_normal((len(tok), V)) * 1.5
        p = np.exp(logits[0] / T) / np.sum(np.exp(logits[0] / T))
        counts = np.zeros(V)
        n = 30000
        for trial in range(n):
            u = rng.random(len(tok) - 1)
            r = SO.sample_walk(logits, tok, par, T, u, seed=trial)
            first = r.accepted_tokens[0] if r.accept_len else r.bonus_token
            counts[first] += 1
        chi2 = np.sum((counts - n * p) ** 2 / (n * p))
        assert chi2 < stats.chi2.ppf(0.999, df=V - 1), (kind, chi2, counts / n, p)


def test_second_token_given_an_accepted_first_follows_the_child_row():
    rng = np.random.default_rng(1)
    V, T = 5, 1.3
    tok, par = [0, 2, 3], [-1, 0, 1]
    logits = rng.standard_normal((3, V))
    p1 = np.exp(logits[1] / T) / np.sum(np.exp(logits[1] / T))
    counts, n_acc = np.zeros(V), 0
    for trial in range(60000):
        r = SO.sample_walk(logits, tok, par, T, rng.random(2), seed=trial)
        if r.accept_len >= 1:
            n_acc += 1
            counts[r.accepted_tokens[1] if r.accept_len > 1 else r.bonus_token] += 1
    chi2 = np.sum((counts - n_acc * p1) ** 2 / (n_acc * p1))
    assert n_acc > 3000 and chi2 < stats.chi2.ppf(0.999, df=V - 1)


def test_acceptance_probabilities_closed_form():
    """P(accept c1) = p(x1); P(accept c2) = (1 - p(x1)) * p(x2) / (1 - p(x1)) = p(x2): thresholds on u."""
    V, T = 4, 1.0
    logits = np.log(np.array([[0.1, 0.2, 0.3, 0.4]]).repeat(3, axis=0))
    tok, par = [0, 1, 3], [-1, 0, 0]                    # candidates: token 1 (p 0.2), then token 3 (p 0.4)
    acc = lambda u1, u2: SO.sample_walk(logits, tok, par, T, [u1, u2], 5)
    assert acc(0.1999, 0.9).accepted_nodes == [0] and acc(0.2001, 0.9).accept_len == 0
    # second candidate faces the residual 0.4 / 0.8 = 0.5
    assert acc(0.5, 0.4999).accepted_nodes == [1] and acc(0.5, 0.5001).accept_len == 0
    r = acc(0.9, 0.9)                                   # both rejected: bonus from {0, 2} only
    assert r.bonus_token in (0, 2)
    counts = np.zeros(4)
    for s in range(20000):
        counts[SO.sample_walk(logits, tok, par, T, [0.9, 0.9], s).bonus_token] += 1
    assert counts[1] == 0 and counts[3] == 0 and abs(counts[0] / 20000 - 0.25) < 0.012   # 0.1 / (0.1 + 0.3)


def test_low_temperature_limit_is_the_greedy_walk():
    rng = np.random.default_rng(2)
    for trial in range(50):
        n = 12
        par = np.array([-1] + [int(rng.integers(0, i + 1)) for i in range(n)])
        logits = rng.standard_normal((n + 1, 9))
        tok = [0]
        for i in range(1, n + 1):       # sibling tokens distinct, so at most one child of a row can be valid
            used = {tok[j] for j in range(1, i) if par[j] == par[i]}
            t = int(np.argmax(logits[par[i]])) if rng.random() < 0.6 else int(rng.integers(9))
            while t in used:
                t = int(rng.integers(9))
            tok.append(t)
        tok = np.asarray(tok)
        depth = np.zeros(n + 1, int)
        for i in range(1, n + 1):
            depth[i] = depth[par[i]] + 1
        r = SO.sample_walk(logits, tok, par, 1e-4, rng.random(n) * 0.98 + 0.01, seed=trial)
        g = np.argmax(logits, axis=1)
        best, path, _ = O.accept_walk(g, tok, par, depth)
        # at T -> 0 a child is accepted iff its token is the row's arg-max: the greedy path
        assert r.accepted_nodes == [p - 1 for p in path] and r.bonus_token == int(g[best])
