"""The allocation-free export entry point against the allocating one: bitwise equal output on
two calls in a row (the second smaller, so stale contents of the shared staging area would
show), the size limit's error, and both storage types."""
import numpy as np
import pytest

import workloads as wl
from paper_2604_13519_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg_name", ["small_bf16", "small_fp32"])
def test_export_noalloc_matches_export_twice_second_smaller(cfg_name):
    cfg = wl.get_config(cfg_name)
    model = B.ts_model_load(cfg, wl.gen_weights(cfg, 1234))
    try:
        K, V = wl.gen_context_kv(cfg, 333, seed=91)
        kv = B.ts_kv_alloc(model, 400)
        B.ts_kv_set_page_table(kv, np.random.default_rng(3).permutation(25).astype(np.int32))
        B.ts_kv_import(kv, K, V)
        try:
            for pos0, n_pos in ((5, 300), (17, 41)):          # page-straddling ranges, the second smaller
                k_ref, v_ref = B.ts_kv_export(kv, pos0, n_pos, cfg)
                k_new, v_new = B.ts_kv_export_noalloc(kv, pos0, n_pos, cfg)
                assert np.array_equal(k_new, k_ref) and np.array_equal(v_new, v_ref)
                assert np.array_equal(k_new, K[:, pos0:pos0 + n_pos]) and np.array_equal(v_new, V[:, pos0:pos0 + n_pos])
            k0, v0 = B.ts_kv_export_noalloc(kv, 0, 0, cfg)
            assert k0.size == 0 and v0.size == 0
        finally:
            B.ts_kv_free(kv)
        # beyond the static staging area: a clear error, nothing copied
        per_pos = cfg.n_kv_heads * cfg.head_dim * (4 if cfg.dtype == wl.configs.DTYPE_F32 else 2)
        too_many = (1 << 20) // per_pos + 1
        big = B.ts_kv_alloc(model, too_many + 16)
        try:
            with pytest.raises(B.TsError) as ei:
                B.ts_kv_export_noalloc(big, 0, too_many, cfg)
            assert ei.value.status == B.TS_ERR_INVALID_ARG and "static staging area" in str(ei.value)
            k1, v1 = B.ts_kv_export_noalloc(big, 0, too_many - 1, cfg)     # the largest legal request works
            k2, v2 = B.ts_kv_export(big, 0, too_many - 1, cfg)
            assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
        finally:
            B.ts_kv_free(big)
    finally:
        B.ts_model_free(model)
