"""Writes tests/golden/greedy_<model>_ctx<P>.txt: the oracle's plain greedy
continuation after the synthetic context of the 8B-shaped workloads.

Draft trees for those workloads are "mutated greedy continuations"; the greedy
tokens themselves can only come from decoding one token at a time, which at the
8B shape takes the CPU oracle about 20 s per token.  This script does that once
and stores the token ids (and each step's top-2 logit margin).  It calls only
oracle/ and the seeded input generators in workloads/.

Recipe: weights seed 1234, context K/V seed 2345 (N(0,1) in bf16), root token =
workloads.root_token(vocab, P), oracle mode "R" (bf16 rounding points of
the device path, float64 accumulation).

Usage: python tests/golden/make_greedy_continuations.py [model] [P:n_tokens ...]
"""
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import workloads as wl                                    # noqa: E402
from workloads.weights import gen_layer, gen_tensor       # noqa: E402
from oracle import toolspec_oracle as O                   # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def root_token(cfg, P):
    return wl.root_token(cfg.vocab, P)


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "llama8b"
    jobs = sys.argv[2:] or ["4096:17", "8192:33"]
    cfg = wl.get_config(name)
    w = {k: gen_tensor(cfg, 1234, k) for k in ("embed", "lm_head", "norm_f")}
    w["layers"] = lambda l: gen_layer(cfg, 1234, l)
    model = O.OracleModel(cfg, w, cache=True)
    for job in jobs:
        P, n = (int(x) for x in job.split(":"))
        K, V = wl.gen_context_kv(cfg, P, seed=2345)
        kv = O.OracleKV(cfg, P + n + 1)
        kv.import_context(K, V)
        del K, V
        kv.pending = root_token(cfg, P)
        root = kv.pending
        empty = np.zeros(0, np.int32)
        lines = []
        for i in range(n):
            t0 = time.time()
            r = O.verify(model, kv, empty, empty, "R")
            O.commit(kv, r)
            lines.append("%d %.6f" % (r.bonus_token, r.margin[0]))
            print("P=%d step %d token %d margin %.4f (%.1fs)" %
                  (P, i + 1, r.bonus_token, r.margin[0], time.time() - t0), flush=True)
        path = os.path.join(HERE, "greedy_%s_ctx%d.txt" % (name, P))
        with open(path, "w") as f:
            f.write("# greedy continuation g_1..g_%d of the CPU oracle (mode R), model %s,\n" % (n, name))
            f.write("# weights seed 1234, context K/V seed 2345, P=%d, root token %d.\n" % (P, root))
            f.write("# columns: token id, top-2 logit margin of that step.\n")
            f.write("# written by tests/golden/make_greedy_continuations.py\n")
            f.write("\n".join(lines) + "\n")
        print("wrote", path, flush=True)


if __name__ == "__main__":
    main()
