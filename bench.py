#!/usr/bin/env python3
"""Benchmark of the tree-verify step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload w3|w2|w4|w5|dev]

A step is one pass of the whole hot path over one draft tree: ts_verify (tree ingest,
32-layer masked forward pass, fused vocab arg-max, acceptance walk, result to host) followed
by ts_kv_commit (K/V compaction of the accepted path), then a host-side roll-back to the
same context so every step sees the same cache length.  Inputs (weights, context K/V,
trees) are resident in HBM before the timed region; trees cycle over 32 seeds.

Default workload w3: Llama-3-8B-shaped decoder, bf16, random-init, batch 1, synthetic
8192-token context, 64-node tree (12-token schema chain, 8 sibling alternatives, 12-token
argument chain, four 8-token retrieved branches), mutated greedy continuation.

`dtype` is "f16": the model is stored in bf16 (weights, K/V cache) and every matrix product
runs in IEEE half with fp32 accumulation (bf16 values widen to half exactly).

Prints ONE JSON line.  `value` = accepted tokens per second (tokens emitted per step =
accepted draft tokens + bonus token, divided by the step time).  `roofline` is for the
dominant kernel (the fused gate/up projection): algorithmic weight bytes per launch over
its mean duration between HIP events on the library's stream, measured in a second,
event-bracketed repeat of the same steps right after the timed region (bracketing every
launch inside the timed region itself would slow the step).  `roofline.plain_read` is a
reference point from the same run: a kernel that only reads, over the same weight tensors,
between the same events; `step_frac_of_plain_read` relates the whole step's algorithmic
bytes per second to it.  `cpu_baseline` is the CPU oracle, as it stands, on a bounded sample
of the same workload.

--workload w4 times the batched pass instead (16 paged requests, contexts U[2048, 16384], a
32-node tree each: 528 rows through ts_verify_batch, then one commit per request).  Its
projections are bound by the matrix cores, so its `roofline` is for the gate/up launch against
the dense 16-bit MFMA peak (2 x R x N x K flop);
`step_hbm_frac` is the whole step against HBM as for the other workloads.  --workload w5 does the
same for the 32B-class shape at full depth (64 layers, 4 requests x 32768-token contexts, 64-node
trees: 64 GB of weights and 34 GB of cache on the device; about a minute of set-up).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="w3", choices=["w3", "w2", "w4", "w5", "dev"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def workload(name):
    """(config name, context length, tree builder name, description)."""
    if name == "w3":
        return "llama8b", 8192, "schema", "llama3-8b-shape bf16, batch 1, ctx 8192, 64-node schema+alternatives+retrieved tree"
    if name == "w2":
        return "llama8b", 4096, "chain16", "llama3-8b-shape bf16, batch 1, ctx 4096, chain of 16 (p=0.2)"
    return "llama8b_2l", 4096, "schema", "DEV ONLY: 2 layers of the 8b layer shape, ctx 4096, 64-node tree"


def build_trees(wl, cfg, kind, greedy, n_trees=32):
    trees = []
    for s in range(n_trees):
        rng = np.random.default_rng([3456, s])
        if kind == "schema":
            trees.append(wl.schema_retrieval_tree(greedy, cfg.vocab, rng))
        else:
            trees.append(wl.chain_tree(greedy, 16, 0.2, cfg.vocab, rng))
    return trees


def algorithmic_bytes(cfg, P):
    return 2 * cfg.streamed_params() + P * cfg.kv_bytes_per_token()


def cpu_baseline(wl, cfg, weights, K, V, root, tree, mean_tokens):
    """Oracle forward pass of the same tree on a bounded sample: the first 2 and the first 4
    layers (plus final norm and lm_head each time); per-layer and head times are separated by
    differencing and scaled to all layers."""
    from oracle import toolspec_oracle as O
    om = O.OracleModel(cfg, weights)
    okv = O.OracleKV(cfg, K.shape[1] + len(tree[0]) + 1)
    okv.K[:4, :K.shape[1]] = O._widen(K[:4])
    okv.V[:4, :K.shape[1]] = O._widen(V[:4])
    okv.P = K.shape[1]
    rows = O.tree_rows(root, tree[0], tree[1])
    t = {}
    for nl in (2, 4):
        t0 = time.time()
        O.forward_tree(om, okv, rows[0], rows[2], rows[3], mode="R", layer_limit=min(nl, cfg.n_layers))
        t[nl] = time.time() - t0
    per_layer = max((t[4] - t[2]) / 2.0, 1e-9)
    head = max(t[2] - 2 * per_layer, 0.0)
    full = head + cfg.n_layers * per_layer
    try:
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": mean_tokens / full, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "oracle forward_tree (mode R, float64) of one %d-row tree timed on layers 0-1 (%.1f s) and "
                      "0-3 (%.1f s) incl. lm_head; per-layer %.2f s and head %.2f s scaled to %d layers = %.1f s per "
                      "verify step" % (len(rows[0]), t[2], t[4], per_layer, head, cfg.n_layers, full),
            "est_step_s": full}


def main_batched(a, wl, B, torch):
    """w4 / w5: one step = ts_verify_batch over all requests + one commit each + host roll-back."""
    if a.workload == "w4":
        cfg = wl.get_config("llama8b")
        contexts = [int(x) for x in np.random.default_rng([2345, 4]).integers(2048, 16385, size=16)]
        desc = "llama3-8b-shape bf16, batch 16, paged contexts U[2048,16384], 32-node BFS trees"
        make_tree = lambda b: wl.bfs_tree([], 32, cfg.vocab, np.random.default_rng([3456, 4, b]))
    else:
        cfg = wl.get_config("qwen32b")
        contexts = [32768] * 4
        desc = "32b-class shape (64 layers, d 5120, 64/8 heads, ffn 25600) bf16, batch 4, ctx 32768, 64-node trees"
        make_tree = lambda b: wl.schema_retrieval_tree([], cfg.vocab, np.random.default_rng([3456, 5, b]))
    weights = wl.gen_weights(cfg, 1234)
    model = B.ts_model_load(cfg, weights)
    del weights
    kvs, trees, roots = [], [], []
    for b, P in enumerate(contexts):
        K, V = wl.gen_context_kv(cfg, P, seed=2345 + b)
        kv = B.ts_kv_alloc(model, P + 80)
        B.ts_kv_import(kv, K, V)
        del K, V
        roots.append(wl.root_token(cfg.vocab, P, seed=3456 + b))
        B.ts_set_pending(kv, roots[-1])
        kvs.append(kv)
        trees.append(make_tree(b))
        print("[bench] request %d: context %d resident" % (b, P), file=sys.stderr, flush=True)
    R = sum(len(t[0]) + 1 for t in trees)

    def step():
        res = B.ts_verify_batch(model, kvs, trees)
        for kv, P, root in zip(kvs, contexts, roots):
            B.ts_kv_commit(kv)
            B.ts_kv_truncate(kv, P)
            B.ts_set_pending(kv, root)
        return sum(r[0] + 1 for r in res)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    emitted = 0
    for _ in range(a.steps):
        emitted += step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    t0 = time.perf_counter()
    for _ in range(a.steps):
        B.ts_verify_batch(model, kvs, trees)
    verify_ms = (time.perf_counter() - t0) / a.steps * 1e3
    B.ts_profile_enable(model, True)
    B.ts_verify_batch(model, kvs, trees)
    kernels = {k: {"launches_per_step": n, "avg_us": ms / n * 1e3, "ms_per_step": ms}
               for k, (n, ms) in B.ts_profile_read(model).items()}
    B.ts_profile_enable(model, False)
    dom = "gemm_gate_up"
    flop = 2.0 * R * (2 * cfg.d_ffn) * cfg.d_model
    achieved = flop / (kernels[dom]["avg_us"] * 1e-6) / 1e12
    total_bytes = 2 * cfg.streamed_params() + sum(contexts) * cfg.kv_bytes_per_token()
    out = {
        "metric": "accepted tokens/s of single-pass tree verification (verify + commit), batched; "
                  "with verify-step latency and % of HBM roofline",
        "value": emitted / dt, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt / a.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": desc, "batch": len(contexts), "rows": R, "context_total": int(sum(contexts)),
                   "storage": "bf16 weights and K/V cache; products in IEEE half, fp32 accumulation"},
        "verify_ms": verify_ms, "mean_tokens_per_step": emitted / a.steps,
        "step_algorithmic_gb": total_bytes / 1e9,
        "step_hbm_frac": total_bytes / (verify_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": achieved / 2500.0, "traffic": None, "flop_per_launch": flop,
                     "avg_us": kernels[dom]["avg_us"]},
        "kernels": kernels,
    }
    for kv in kvs:
        B.ts_kv_free(kv)
    B.ts_model_free(model)
    print(json.dumps(out))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding "
              "are part of it)" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    import workloads as wl
    from paper_2604_13519_amd import binding as B
    B.load_library()

    if a.workload in ("w4", "w5"):
        return main_batched(a, wl, B, torch)
    cfg_name, P, tree_kind, desc = workload(a.workload)
    cfg = wl.get_config(cfg_name)
    t0 = time.time()
    weights = wl.gen_weights(cfg, 1234)
    K, V = wl.gen_context_kv(cfg, P, seed=2345)
    print("[bench] inputs generated in %.1f s" % (time.time() - t0), file=sys.stderr, flush=True)
    t0 = time.time()
    model = B.ts_model_load(cfg, weights)
    kv = B.ts_kv_alloc(model, P + 80)
    B.ts_kv_import(kv, K, V)
    root = wl.root_token(cfg.vocab, P)
    B.ts_set_pending(kv, root)
    print("[bench] model + cache resident in %.1f s" % (time.time() - t0), file=sys.stderr, flush=True)
    greedy = wl.load_greedy(os.path.join(ROOT, "tests", "golden", "greedy_llama8b_ctx%d.txt" % P)) \
        if cfg_name == "llama8b" else []
    trees = build_trees(wl, cfg, tree_kind, greedy)

    def step(i):
        tok, par = trees[i % len(trees)]
        l, _, _, _ = B.ts_verify(model, kv, tok, par)
        B.ts_kv_commit(kv)
        B.ts_kv_truncate(kv, P)
        B.ts_set_pending(kv, root)
        return l + 1

    if os.environ.get("TS_BENCH_CALIB"):
        # counter calibration for profiling runs: a plain device copy of known size (1 GiB read, 1 GiB written)
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    emitted = 0
    for i in range(a.steps):
        emitted += step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / a.steps * 1e3

    # verify-only latency (no commit), same trees
    t0 = time.perf_counter()
    for i in range(a.steps):
        tok, par = trees[i % len(trees)]
        B.ts_verify(model, kv, tok, par)
    verify_ms = (time.perf_counter() - t0) / a.steps * 1e3

    # event-bracketed repeats: first the dominant kernel alone (its launches only, so the other
    # ~290 launches of a step run undisturbed), then every kernel kind for the breakdown table
    def bracketed(kind, n_rep):
        B.ts_profile_filter(model, kind)
        B.ts_profile_enable(model, True)
        agg = {}
        for i in range(n_rep):
            tok, par = trees[i % len(trees)]
            B.ts_verify(model, kv, tok, par)
            for k, (n, ms) in B.ts_profile_read(model).items():
                c = agg.setdefault(k, [0, 0.0])
                c[0] += n
                c[1] += ms
        B.ts_profile_enable(model, False)
        B.ts_profile_filter(model, None)
        return {k: {"launches_per_step": v[0] / n_rep, "avg_us": v[1] / v[0] * 1e3, "ms_per_step": v[1] / n_rep}
                for k, v in agg.items()}

    n_prof = min(a.steps, 16)
    dom_only = bracketed("gemm_gate_up", n_prof)
    kernels = bracketed(None, n_prof)
    kernels["gemm_gate_up"] = dom_only["gemm_gate_up"]
    # the same brackets around a kernel that only reads the gate/up weight tensors (one layer's per
    # launch, layers cycled): what the memory system gives a plain streaming read of those bytes
    B.ts_profile_filter(model, "plain_read")
    B.ts_profile_enable(model, True)
    plain_bytes = B.ts_profile_plain_read(model, 5 * cfg.n_layers)
    pn, pms = B.ts_profile_read(model)["plain_read"]
    B.ts_profile_enable(model, False)
    B.ts_profile_filter(model, None)
    plain_us = pms / pn * 1e3
    dom = "gemm_gate_up"
    dom_bytes = 2 * cfg.d_ffn * cfg.d_model * 2            # gate + up weights, bf16, per launch
    dom_us = kernels[dom]["avg_us"]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(dom, {}).get("bytes")   # rocprofv3 counter passes, see profiles/
        except Exception:
            traffic = None
    total_bytes = algorithmic_bytes(cfg, P)
    out = {
        "metric": "accepted tokens/s of single-pass tree verification (verify + commit), 8B bf16; "
                  "with verify-step latency and % of HBM roofline",
        "value": emitted / dt, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": desc, "context": P, "tree_nodes": int(len(trees[0][0])), "batch": 1,
                   "trees": "%d seeded trees cycled" % len(trees),
                   "storage": "bf16 weights and K/V cache; products in IEEE half, fp32 accumulation"},
        "verify_ms": verify_ms, "commit_ms": ms_per_step - verify_ms,
        "mean_tokens_per_step": emitted / a.steps,
        "step_algorithmic_gb": total_bytes / 1e9,
        "step_hbm_frac": total_bytes / (verify_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "step_frac_of_plain_read": total_bytes / (verify_ms * 1e-3) / (plain_bytes / (plain_us * 1e-6)),
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "bytes_per_launch": dom_bytes,
                     "avg_us": dom_us,
                     "plain_read": {"avg_us": plain_us, "GB/s": plain_bytes / (plain_us * 1e-6) / 1e9,
                                    "bytes_per_launch": plain_bytes, "launches": pn,
                                    "kernel_frac_of_plain_read": plain_us / dom_us,
                                    "what": "read-only kernel over the same weight tensors, same event brackets"}},
        "kernels": kernels,
    }
    if not a.no_cpu_baseline:
        print("[bench] timing the CPU oracle sample ...", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(wl, cfg, weights, K, V, root, trees[0], emitted / a.steps)
    B.ts_kv_free(kv)
    B.ts_model_free(model)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
