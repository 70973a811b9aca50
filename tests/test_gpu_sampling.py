"""Stochastic acceptance (ts_verify_sample) against the sampling oracle.

The oracle walks its own logits (exact mode for fp32 models, rounding mode for bf16 ones) with the
same uniforms and noise seed.  A decision of the walk is a comparison u < p / rest; the device takes
it in single precision on its own logits, so a case is compared exactly only when every decision
the oracle took is further than a gap from its threshold and the bonus token's perturbed score
leads by more than a gap (fp32 path 1e-4, bf16 path 1e-2, the margin of the greedy rule); most
cases must be such cases.  A second test checks the defining property on the device alone: the
first emitted token follows softmax(logits / T)."""
import numpy as np
import pytest
from scipy import stats

import workloads as wl
from oracle import toolspec_oracle as O
from oracle import sampling_oracle as SO
from paper_2604_13519_amd import binding as B

import gpu_utils as U

pytestmark = pytest.mark.gpu


def _setup(cfg_name, P, seed):
    cfg, w, model, omodel = U.get_model(cfg_name)
    K, V = wl.gen_context_kv(cfg, P, seed=seed)
    kv, okv = U.make_pair(cfg, model, K, V, 11)
    return cfg, model, omodel, kv, okv


@pytest.mark.parametrize("cfg_name", ["small_fp32", "small_bf16"])
def test_sampled_walk_matches_the_oracle(cfg_name):
    cfg, model, omodel, kv, okv = _setup(cfg_name, 150, 91)
    fp32 = cfg.dtype == wl.configs.DTYPE_F32
    gap = 1e-4 if fp32 else 1e-2
    rng = np.random.default_rng(6)
    try:
        exact, total = 0, 0
        for trial in range(6):
            n = int(rng.choice([0, 1, 8, 30, 64]))
            greedy = [int(t) for t in rng.integers(cfg.vocab, size=16)]
            tok, par = wl.bfs_tree(greedy, n, cfg.vocab, rng) if n else (np.zeros(0, np.int32), np.zeros(0, np.int32))
            rows = O.tree_rows(okv.pending, tok, par)
            ologits, _, _ = O.forward_tree(omodel, okv, rows[0], rows[2], rows[3], "E" if fp32 else "R")
            # make some drafts plausible: replace a few node tokens by likely tokens of their parents
            for i in range(len(tok)):
                if rng.random() < 0.5:
                    tok[i] = int(np.argsort(ologits[rows[1][i + 1]])[-1 - int(rng.integers(0, 3))])
            rows = O.tree_rows(okv.pending, tok, par)
            ologits, _, _ = O.forward_tree(omodel, okv, rows[0], rows[2], rows[3], "E" if fp32 else "R")
            for T in (0.7, 1.0, 3.0):
                for rep in range(4):
                    u = rng.random(len(tok)).astype(np.float32)
                    seed = int(rng.integers(1 << 62))
                    got = B.ts_verify_sample(model, kv, tok, par, T, u, seed)
                    want = SO.sample_walk(ologits, rows[0], rows[1], T, u, seed)
                    total += 1
                    if want.decision_gap > gap and want.bonus_gap > gap:
                        exact += 1
                        assert got == (want.accept_len, want.accepted_tokens, want.accepted_nodes, want.bonus_token), \
                            "n=%d T=%g: %r != oracle (gaps %.3g %.3g)" % (n, T, got, want.decision_gap, want.bonus_gap)
                    else:   # a decision within the gap: the device may fall on either side; its output is still a valid path
                        assert 0 <= got[0] <= len(tok) and 0 <= got[3] < cfg.vocab
                    if got[0]:
                        B.ts_kv_commit(kv)          # the result is committable like a greedy one
                        B.ts_kv_truncate(kv, 150)
                        B.ts_set_pending(kv, 11)
        print("%s sampling: %d of %d cases compared exactly" % (cfg_name, exact, total))
        assert exact >= 0.6 * total
    finally:
        B.ts_kv_free(kv)


def test_first_token_distribution_on_the_device():
    """Lossless in distribution: over many draws the first emitted token (accepted draft or residual
    sample) follows softmax(logits[root] / T) of the device's own logits."""
    cfg, model, omodel, kv, okv = _setup("small_fp32", 60, 92)
    rng = np.random.default_rng(10)
    try:
        T = 0.04                                   # the random-init logits are small: a low temperature gives a peaked distribution
        B.ts_verify(model, kv, [], [])
        z = B.ts_get_logits(model, 0, 1, cfg.vocab)[0].astype(np.float64) / T
        p = np.exp(z - z.max())
        p /= p.sum()
        top = np.argsort(p)[::-1][:6]
        # three sibling candidates (the 1st, 3rd and 5th most likely tokens), one with a child
        tok = np.asarray([top[0], top[2], top[4], 5], np.int32)
        par = np.asarray([-1, -1, -1, 0], np.int32)
        n = 6000
        counts = np.zeros(7)                     # six most likely tokens + everything else
        for i in range(n):
            l, acc, _, bonus = B.ts_verify_sample(model, kv, tok, par, T, rng.random(4).astype(np.float32), int(rng.integers(1 << 62)))
            first = acc[0] if l else bonus
            j = np.nonzero(top == first)[0]
            counts[j[0] if len(j) else 6] += 1
        expect = np.concatenate([p[top], [1.0 - p[top].sum()]]) * n
        chi2 = np.sum((counts - expect) ** 2 / expect)
        print("sampling first-token chi2 %.2f (df 6), p(top) %s" % (chi2, np.round(p[top], 4)))
        assert chi2 < stats.chi2.ppf(0.999, df=6), (chi2, counts, expect)
    finally:
        B.ts_kv_free(kv)


def test_sampling_error_paths():
    cfg, model, omodel, kv, okv = _setup("small_fp32", 20, 93)
    try:
        for bad_t in (0.0, -1.0, float("nan")):
            with pytest.raises(B.TsError) as e:
                B.ts_verify_sample(model, kv, [1], [-1], bad_t, [0.5], 1)
            assert e.value.status == B.TS_ERR_INVALID_ARG
        with pytest.raises(B.TsError):
            B.ts_verify_sample(model, kv, [1], [-1], 1.0, [1.0], 1)          # uniform outside [0,1)
        assert B.ts_kv_len(kv) == 20
    finally:
        B.ts_kv_free(kv)
