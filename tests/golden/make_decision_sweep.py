"""Writes tests/golden/decisions_<model>.txt: the CPU oracle's per-row decisions on the arg-max
decision sweep - random 64-node trees with uniform random tokens over 512-token synthetic
contexts (workloads.decision_sweep_case) - at a model size where the oracle needs about half a
minute per pass, so that the GPU test can compare thousands of full-size rows in seconds.

Per row, in both oracle modes (R: rounding points of the device path, the mode decisions are
compared in; E: exact float64): the arg-max token and the top-2 logit margin.  The GPU test
requires every device / oracle arg-max difference to sit on a row whose oracle margin is below
1e-2 (the method's output must equal plain greedy decoding, Sec. 5.1 "Evaluation Metrics",
App. B.3; near-tied logits are exempt).

Calls only oracle/ and the seeded input generators in workloads/.

Usage: python tests/golden/make_decision_sweep.py [model] [n_trees] [first_tree] [output file]
       (appends to an existing file when first_tree > 0; the default output is
       tests/golden/decisions_<model>.txt)
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
P = 512


class LazyLayer:
    """layer -> tensors, each generated only when asked for."""

    def __init__(self, cfg, layer):
        self.cfg, self.layer = cfg, layer

    def __getitem__(self, kind):
        return gen_tensor(self.cfg, 1234, kind, self.layer)


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "llama8b"
    n_trees = int(sys.argv[2]) if len(sys.argv) > 2 else 40
    first = int(sys.argv[3]) if len(sys.argv) > 3 else 0
    cfg = wl.get_config(name)
    w = {k: gen_tensor(cfg, 1234, k) for k in ("embed", "lm_head", "norm_f")}
    w["layers"] = lambda l: LazyLayer(cfg, l)
    model = O.OracleModel(cfg, w, cache=True)
    path = sys.argv[4] if len(sys.argv) > 4 else os.path.join(HERE, "decisions_%s.txt" % name)
    if first == 0 or not os.path.exists(path):
        with open(path, "w") as f:
            f.write("# CPU oracle decisions on the arg-max decision sweep, model %s, weights seed 1234,\n" % name)
            f.write("# case t = workloads.decision_sweep_case(cfg, t, P=%d, n_nodes=64); 65 rows per case.\n" % P)
            f.write("# line: case row argmax_R margin_R argmax_E margin_E\n")
            f.write("# written by tests/golden/make_decision_sweep.py\n")
    for t in range(first, first + n_trees):
        t0 = time.time()
        K, V, root, tok, par = wl.decision_sweep_case(cfg, t, P=P)
        kv = O.OracleKV(cfg, P + 80)
        kv.import_context(K, V)
        kv.pending = root
        res = {m: O.verify(model, kv, tok, par, m) for m in ("R", "E")}
        with open(path, "a") as f:
            for r in range(len(tok) + 1):
                f.write("%d %d %d %.6e %d %.6e\n" % (t, r, res["R"].greedy[r], res["R"].margin[r],
                                                    res["E"].greedy[r], res["E"].margin[r]))
        print("case %d done (%.0f s)" % (t, time.time() - t0), flush=True)


if __name__ == "__main__":
    main()
