"""Shared K/V page pool: caches of different lengths draw their pages from one allocation.

The claim to test is that results do not depend on where a cache's pages lie: a pooled cache
whose pages are scattered between another request's pages gives bit for bit the logits,
decisions and committed K/V of a cache with its own allocation; the oracle is compared with
once (the own-allocation path is what every other parity test covers).  Plus the pool's
bookkeeping and error paths.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import toolspec_oracle as O
from paper_2604_13519_amd import binding as B

import gpu_utils as U

pytestmark = pytest.mark.gpu


def _fill(kv, K, V, pending):
    B.ts_kv_import(kv, K, V)
    B.ts_set_pending(kv, pending)


@pytest.mark.parametrize("cfg_name", ["small_fp32", "small_bf16"])
def test_pooled_caches_with_scattered_pages_equal_own_allocations(cfg_name):
    cfg, w, model, omodel = U.get_model(cfg_name)
    rng = np.random.default_rng(606)
    lens = [150, 37, 260]
    ctx = [wl.gen_context_kv(cfg, P, seed=300 + i) for i, P in enumerate(lens)]
    pend = [int(rng.integers(cfg.vocab)) for _ in lens]
    trees = [wl.bfs_tree([], 40, cfg.vocab, rng), wl.chain_tree([], 9, 1.0, cfg.vocab, rng), wl.bfs_tree([], 64, cfg.vocab, rng)]
    pages = lambda P: (P + 80 + 15) // 16
    pool = B.ts_kv_pool_create(model, sum(pages(P) for P in lens) + 9)
    own, pooled = [], []
    try:
        total = B.ts_kv_pool_pages_free(pool)
        # fragment the pool: allocate small fillers between the real caches and free them again, so
        # that later caches pick up pages lying between the pages of the earlier ones
        fillers = []
        for i, P in enumerate(lens):
            fillers.append(B.ts_kv_alloc_pooled(pool, 16 * (2 + i)))
            pooled.append(B.ts_kv_alloc_pooled(pool, (P + 80) // 2))       # half now ...
        for f in fillers:
            B.ts_kv_free(f)
        for kv in pooled:
            B.ts_kv_free(kv)                                              # ... all back, in a scrambled order
        assert B.ts_kv_pool_pages_free(pool) == total
        pooled = [B.ts_kv_alloc_pooled(pool, P + 80) for P in lens]
        assert B.ts_kv_pool_pages_free(pool) == total - sum(pages(P) for P in lens)
        for i, P in enumerate(lens):
            kv = B.ts_kv_alloc(model, P + 80)
            own.append(kv)
            _fill(kv, *ctx[i], pend[i])
            _fill(pooled[i], *ctx[i], pend[i])

        # single passes: bitwise equal logits and equal results
        for i in range(len(lens)):
            a = B.ts_verify(model, own[i], *trees[i])
            la = B.ts_get_logits(model, 0, len(trees[i][0]) + 1, cfg.vocab).copy()
            b = B.ts_verify(model, pooled[i], *trees[i])
            lb = B.ts_get_logits(model, 0, len(trees[i][0]) + 1, cfg.vocab)
            assert a == b and np.array_equal(la, lb), "request %d: pooled cache differs from its own-allocation twin" % i
        # one batched pass over the pooled caches equals the batched pass over the own allocations
        assert B.ts_verify_batch(model, pooled, trees) == B.ts_verify_batch(model, own, trees)

        # against the oracle, and through a commit: the compacted K/V equal the twin's bit for bit
        i = 2
        okv = O.OracleKV(cfg, lens[i] + 80)
        okv.import_context(*ctx[i])
        okv.pending = pend[i]
        greedy = O.greedy_decode(omodel, okv, 5, "E" if cfg.dtype == wl.configs.DTYPE_F32 else "R")
        okv = O.OracleKV(cfg, lens[i] + 80)
        okv.import_context(*ctx[i])
        okv.pending = pend[i]
        tok, par = wl.bfs_tree(greedy, 48, cfg.vocab, rng, p_keep=1.0)
        res, oR = U.check_verify(cfg, model, omodel, pooled[i], okv, tok, par, label=cfg_name + " pooled")
        assert res[0] >= 1
        U.commit_both(cfg, pooled[i], okv, res, oR)
        assert B.ts_verify(model, own[i], tok, par) == res
        B.ts_kv_commit(own[i])
        n = B.ts_kv_len(own[i])
        assert n == B.ts_kv_len(pooled[i]) == lens[i] + res[0] + 1
        ka, va = B.ts_kv_export(own[i], 0, n, cfg)
        kb, vb = B.ts_kv_export(pooled[i], 0, n, cfg)
        assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    finally:
        for kv in own + pooled:
            B.ts_kv_free(kv)
        B.ts_kv_pool_free(pool)


def test_pool_bookkeeping_and_error_paths():
    cfg, w, model, omodel = U.get_model("small_fp32")
    pool = B.ts_kv_pool_create(model, 10)
    kv = None
    try:
        assert B.ts_kv_pool_pages_free(pool) == 10
        kv = B.ts_kv_alloc_pooled(pool, 100)                 # 7 pages
        assert B.ts_kv_pool_pages_free(pool) == 3
        with pytest.raises(B.TsError) as e:
            B.ts_kv_alloc_pooled(pool, 49)                   # 4 pages: one too many
        assert e.value.status == B.TS_ERR_OOM and B.ts_kv_pool_pages_free(pool) == 3
        with pytest.raises(B.TsError) as e:
            B.ts_kv_set_page_table(kv, np.arange(7, dtype=np.int32))
        assert e.value.status == B.TS_ERR_STATE
        with pytest.raises(B.TsError) as e:
            B.ts_kv_pool_free(pool)                          # a cache is still alive
        assert e.value.status == B.TS_ERR_STATE
        with pytest.raises(B.TsError) as e:
            B.ts_kv_alloc_pooled(pool, 0)
        assert e.value.status == B.TS_ERR_INVALID_ARG
        small = B.ts_kv_alloc_pooled(pool, 48)               # exactly the 3 pages left
        assert B.ts_kv_pool_pages_free(pool) == 0
        B.ts_kv_free(small)
        B.ts_kv_free(kv)
        kv = None
        assert B.ts_kv_pool_pages_free(pool) == 10
    finally:
        if kv is not None:
            B.ts_kv_free(kv)
        B.ts_kv_pool_free(pool)
    with pytest.raises(B.TsError) as e:
        B.ts_kv_pool_create(model, 0)
    assert e.value.status == B.TS_ERR_INVALID_ARG
