"""Full-size parity: the Llama-3-8B-shaped model (32 layers, bf16, vocab 128256) on the
benchmark workload - 8192-token synthetic context, 64-node schema + alternatives + retrieved
tree built from the stored oracle greedy continuation - in the launch configuration bench.py
times.  All 65 rows of logits are compared with the oracle (exact mode and rounding mode),
then the accepted path, bonus token, tree K/V rows and the compaction.  Also the 16-node
chain workload over 4096 tokens of context on the same model."""
import os
import time

import numpy as np
import pytest

import workloads as wl
from oracle import toolspec_oracle as O
from paper_2604_13519_amd import binding as B

import gpu_utils as U

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_llama8b_full_model_tree_verify_ctx8192_and_chain_ctx4096():
    cfg, w, model, omodel = U.get_model("llama8b")
    try:
        for P, kind in ((8192, "schema"), (4096, "chain16")):
            t0 = time.time()
            K, V = wl.gen_context_kv(cfg, P, seed=2345)
            greedy = wl.load_greedy(os.path.join(GOLDEN, "greedy_llama8b_ctx%d.txt" % P))
            assert len(greedy) >= 17, "stored greedy continuation missing"
            rng = np.random.default_rng([3456, 0])
            if kind == "schema":
                tok, par = wl.schema_retrieval_tree(greedy, cfg.vocab, rng)
            else:
                tok, par = wl.chain_tree(greedy, 16, 0.2, cfg.vocab, rng)
            kv, okv = U.make_pair(cfg, model, K, V, wl.root_token(cfg.vocab, P))
            try:
                res, oR = U.check_verify(cfg, model, omodel, kv, okv, tok, par, label="llama8b %s ctx%d" % (kind, P))
                print("llama8b %s ctx%d: accept_len %d, %.0f s" % (kind, P, res[0], time.time() - t0), flush=True)
                if oR.decisive_margin >= U.MARGIN:
                    # stored continuation = what the oracle decodes: the accepted tokens follow it
                    assert res[1] == greedy[:res[0]] and res[3] == greedy[res[0]]
                U.commit_both(cfg, kv, okv, res, oR)
            finally:
                B.ts_kv_free(kv)
            del K, V, okv
    finally:
        U.drop_model("llama8b")
