"""Writes tests/golden/w4_expected.txt: what the CPU oracle computes for the requests of the batched
8B workload (16 requests, ragged contexts drawn from [2048, 16384], a 32-node breadth-first tree
each) that the GPU test does not run the oracle on live - all but the shortest and the longest.

Per request and row, in the decision mode R and the exact mode E: the arg-max token, the top-2
margin and the logits at a fixed sample of vocabulary ids (both modes' top two and 12 seeded ids).
The GPU test compares the batched pass of all 16 requests against these: sampled logits within
the tolerances, every arg-max difference on a row whose oracle margin is below 1e-2, the accepted
path recomputed from the stored decisions.

Calls only oracle/ and the seeded input generators in workloads/.  About half a minute per request
on 16 host threads; a run appends to an existing file and skips the requests it already holds.

Usage: python tests/golden/make_w4_expected.py [output file]
"""
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import workloads as wl                                    # noqa: E402
from workloads.weights import gen_tensor                  # noqa: E402
from oracle import toolspec_oracle as O                   # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
N_SAMPLE = 12


class LazyLayer:
    """layer -> tensors, each generated only when asked for."""

    def __init__(self, cfg, layer):
        self.cfg, self.layer = cfg, layer

    def __getitem__(self, kind):
        return gen_tensor(self.cfg, 1234, kind, self.layer)


def main():
    path = sys.argv[1] if len(sys.argv) > 1 else os.path.join(HERE, "w4_expected.txt")
    cfg = wl.get_config("llama8b")
    contexts = [int(x) for x in np.random.default_rng([2345, 4]).integers(2048, 16385, size=16)]
    live = {int(np.argmin(contexts)), int(np.argmax(contexts))}      # the GPU test runs the oracle on these itself
    done = set()
    if os.path.exists(path):
        done = {int(line.split()[1]) for line in open(path) if line.startswith("request ")}
    else:
        with open(path, "w") as f:
            f.write("# CPU oracle, batched 8B workload (config llama8b, weights seed 1234): request b has context\n")
            f.write("# contexts[b] (K/V seed 2345 + b), root token seed 3456 + b, tree wl.bfs_tree([], 32, vocab, rng([3456, 4, b])).\n")
            f.write("# row line: b row argmax_R margin_R argmax_E margin_E | sampled ids | logits_R at them | logits_E at them\n")
            f.write("# written by tests/golden/make_w4_expected.py\n")
    w = {k: gen_tensor(cfg, 1234, k) for k in ("embed", "lm_head", "norm_f")}
    w["layers"] = lambda l: LazyLayer(cfg, l)
    model = O.OracleModel(cfg, w, cache=True)
    for b, P in enumerate(contexts):
        if b in live or b in done:
            continue
        t0 = time.time()
        K, V = wl.gen_context_kv(cfg, P, seed=2345 + b)
        kv = O.OracleKV(cfg, P + 80)
        kv.import_context(K, V)
        kv.pending = int(wl.root_token(cfg.vocab, P, seed=3456 + b))
        del K, V
        tok, par = wl.bfs_tree([], 32, cfg.vocab, np.random.default_rng([3456, 4, b]))
        res = {m: O.verify(model, kv, tok, par, m) for m in ("R", "E")}
        extra = np.random.default_rng([98, b]).choice(cfg.vocab, size=N_SAMPLE, replace=False)
        with open(path, "a") as f:
            for row in range(len(tok) + 1):
                ids = []
                for m in ("R", "E"):
                    top2 = np.argsort(res[m].logits[row])[-2:]
                    ids += [int(top2[1]), int(top2[0])]
                ids = list(dict.fromkeys(ids + [int(x) for x in extra]))
                f.write("%d %d %d %.6e %d %.6e | %s | %s | %s\n" % (
                    b, row, res["R"].greedy[row], res["R"].margin[row], res["E"].greedy[row], res["E"].margin[row],
                    " ".join(str(i) for i in ids),
                    " ".join("%.9e" % res["R"].logits[row][i] for i in ids),
                    " ".join("%.9e" % res["E"].logits[row][i] for i in ids)))
            f.write("request %d context %d rows %d\n" % (b, P, len(tok) + 1))
        print("request %d (context %d) done (%.0f s)" % (b, P, time.time() - t0), flush=True)


if __name__ == "__main__":
    main()
