"""Writes tests/golden/w5_expected.txt: what the CPU oracle computes for one request of the
32B-class workload at FULL depth (64 layers, d_model 5120, 64 query / 8 KV heads, FFN 25600,
vocab 151936; context of 32768 synthetic positions, 64-node schema tree).

The oracle needs several minutes per pass at this size (64 GB of weights are generated layer by
layer, the context K/V are held as bfloat16 bit patterns and widened one layer at a time), so
the GPU test cannot run it live.  This script runs, for request `REQ` of the batch:
  1. GREEDY plain decoding steps (mode R) from the request's context, to get a short greedy
     continuation; the request's tree is the workload's 64-node schema tree built from it, so a
     part of the tree is accepted and the compaction moves rows;
  2. the tree pass in mode R (the mode decisions are compared in) and in mode E (exact float64);
and stores: the greedy tokens, the tree, and per row the arg-max token and top-2 margin in both
modes plus the logits at a fixed sample of vocabulary ids (the arg-max ids of both modes, their
runners-up, and 28 seeded ids) - enough for a relative-L2 comparison on the sample and an exact
comparison of the accepted path.

Calls only oracle/ and the seeded input generators in workloads/.

Usage: python tests/golden/make_w5_expected.py [greedy_steps] [output file] [greedy side file]
       (the greedy continuation is appended to the side file, tests/golden/w5_greedy.txt by default,
       step by step; a run that finds it complete goes straight to the tree passes)
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
CFG = "qwen32b"
REQ = 1                     # request of the batch that is compared with the oracle
P = 32768
N_SAMPLE = 28


class LazyLayer:
    """layer -> tensors, each generated only when asked for."""

    def __init__(self, cfg, layer):
        self.cfg, self.layer = cfg, layer

    def __getitem__(self, kind):
        if kind == "norm1" and self.layer % 8 == 0:
            print("  layer %d" % self.layer, flush=True)
        return gen_tensor(self.cfg, 1234, kind, self.layer)


class _Store:
    """K or V of one sequence: the imported context as bfloat16 bit patterns (widened on read, one
    layer and KV head at a time) plus a float64 tail for the positions appended by commits."""

    def __init__(self, ctx16, tail_rows):
        self.ctx = ctx16                                            # [L][P][Hkv][hd] uint16
        L, self.P0, Hkv, hd = ctx16.shape
        self.tail = np.zeros((L, tail_rows, Hkv, hd))

    def __getitem__(self, idx):
        l, pos, g, dd = idx                                         # the oracle reads [l, :P, g, :]
        assert isinstance(pos, slice) and pos.start is None and dd == slice(None)
        stop = pos.stop
        head = O._widen(self.ctx[l, :min(stop, self.P0), g, :])
        if stop <= self.P0:
            return head
        return np.concatenate([head, self.tail[l, :stop - self.P0, g, :]], axis=0)

    def __setitem__(self, idx, val):
        sl, pos = idx                                               # commit writes [:, position]
        assert sl == slice(None) and pos >= self.P0
        self.tail[:, pos - self.P0] = val


class LazyKV:
    def __init__(self, cfg, K16, V16, pending, tail_rows=80):
        self.K, self.V = _Store(K16, tail_rows), _Store(V16, tail_rows)
        self.P = K16.shape[1]
        self.pending = int(pending)
        self.capacity = self.P + tail_rows


def main():
    greedy_steps = int(sys.argv[1]) if len(sys.argv) > 1 else 4
    cfg = wl.get_config(CFG)
    w = {k: gen_tensor(cfg, 1234, k) for k in ("embed", "lm_head", "norm_f")}
    w["layers"] = lambda l: LazyLayer(cfg, l)
    model = O.OracleModel(cfg, w)                       # nothing cached: 64 GB would not fit
    t0 = time.time()
    K16, V16 = wl.gen_context_kv(cfg, P, seed=2345 + REQ)
    root = wl.root_token(cfg.vocab, P, seed=3456 + REQ)
    print("context generated (%.0f s)" % (time.time() - t0), flush=True)

    # the greedy continuation is kept in a side file as it grows, so that an interrupted run resumes
    path = sys.argv[2] if len(sys.argv) > 2 else os.path.join(HERE, "w5_expected.txt")
    side = sys.argv[3] if len(sys.argv) > 3 else os.path.join(HERE, "w5_greedy.txt")
    greedy, gmargin = [], []
    if os.path.exists(side):
        for line in open(side):
            t, mg = line.split()
            greedy.append(int(t))
            gmargin.append(float(mg))
        print("resuming after %d stored greedy steps" % len(greedy), flush=True)
    kv = LazyKV(cfg, K16, V16, root)
    empty = np.zeros(0, np.int32)
    for i in range(greedy_steps if len(greedy) < greedy_steps else 0):   # all steps stored: nothing to replay
        if i < len(greedy):
            # replay a stored step: the pass is needed anyway for the K/V of the committed token
            r = O.verify(model, kv, np.zeros(0, np.int32), np.zeros(0, np.int32), "R")
            assert r.bonus_token == greedy[i]
            O.commit(kv, r)
            continue
        r = O.verify(model, kv, empty, empty, "R")
        O.commit(kv, r)
        greedy.append(r.bonus_token)
        gmargin.append(float(r.margin[0]))
        with open(side, "a") as f:
            f.write("%d %.6e\n" % (r.bonus_token, r.margin[0]))
        print("greedy step %d: token %d margin %.4f (%.0f s)" % (i + 1, r.bonus_token, r.margin[0], time.time() - t0), flush=True)

    greedy, gmargin = greedy[:greedy_steps], gmargin[:greedy_steps]
    tok, par = wl.schema_retrieval_tree(greedy, cfg.vocab, np.random.default_rng([3456, 5, REQ]))
    kv = LazyKV(cfg, K16, V16, root)
    res = {}
    for mode in ("R", "E"):
        res[mode] = O.verify(model, kv, tok, par, mode)
        print("tree pass mode %s: accept_len %d bonus %d (%.0f s)" % (mode, res[mode].accept_len, res[mode].bonus_token, time.time() - t0), flush=True)

    rng = np.random.default_rng([99, REQ])
    extra = rng.choice(cfg.vocab, size=N_SAMPLE, replace=False)
    with open(path, "w") as f:
        f.write("# CPU oracle, 32B-class shape at full depth (config %s, weights seed 1234), request %d of the batch:\n" % (CFG, REQ))
        f.write("# context K/V seed %d, P = %d, root token %d.  Written by tests/golden/make_w5_expected.py\n" % (2345 + REQ, P, root))
        f.write("greedy " + " ".join(str(t) for t in greedy) + "\n")
        f.write("greedy_margin " + " ".join("%.6e" % x for x in gmargin) + "\n")
        f.write("tree_tokens " + " ".join(str(int(t)) for t in tok) + "\n")
        f.write("tree_parents " + " ".join(str(int(t)) for t in par) + "\n")
        for mode in ("R", "E"):
            r = res[mode]
            f.write("result_%s %d %d %s %s\n" % (mode, r.accept_len, r.bonus_token,
                                                 ",".join(str(x) for x in r.accepted_nodes) or "-",
                                                 ",".join(str(x) for x in r.accepted_tokens) or "-"))
        f.write("# row: row argmax_R margin_R argmax_E margin_E | sampled ids | logits_R at them | logits_E at them\n")
        for row in range(len(tok) + 1):
            ids = []
            for mode in ("R", "E"):
                top2 = np.argsort(res[mode].logits[row])[-2:]
                ids += [int(top2[1]), int(top2[0])]
            ids = list(dict.fromkeys(ids + [int(x) for x in extra]))
            f.write("row %d %d %.6e %d %.6e | %s | %s | %s\n" % (
                row, res["R"].greedy[row], res["R"].margin[row], res["E"].greedy[row], res["E"].margin[row],
                " ".join(str(i) for i in ids),
                " ".join("%.9e" % res["R"].logits[row][i] for i in ids),
                " ".join("%.9e" % res["E"].logits[row][i] for i in ids)))
    print("wrote %s (%.0f s)" % (path, time.time() - t0), flush=True)


if __name__ == "__main__":
    main()
