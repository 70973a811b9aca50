"""Summaries of rocprofv3 runs over bench.py, written under profiles/.

    python -m paper_2604_13519_amd.counters trace <kernel_trace.db> [--workload w3] [--command "..."] [--bench line.json]

writes profiles/verify_<workload>_kernel_trace.md: per kernel (the split projections told apart by
their grids) calls, total and average duration, and the launches, span and gaps of one timed step.

    python -m paper_2604_13519_amd.counters sq <w3_pass.db> <w4_pass.db> [--out file] [--commit hash]

writes profiles/verify_mfma_lds_counters.md (or --out): matrix-pipe and LDS utilisation per kernel from one
pass per workload of

    rocprofv3 --pmc SQ_ACTIVE_INST_ANY SQ_BUSY_CU_CYCLES SQ_INSTS_MFMA SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE \\
              SQ_VALU_MFMA_BUSY_CYCLES SQ_WAIT_ANY SQ_WAVE_CYCLES -d <dir> -o p -- python3 bench.py [--workload w4] --steps 1 --warmup 1 --no-cpu-baseline

HBM traffic per kernel launch from two rocprofv3 counter passes over bench.py:

    python -m paper_2604_13519_amd.counters <read_pass.db> <write_pass.db> [--workload w3]

writes profiles/traffic.json (what bench.py reports as roofline.traffic) and
profiles/verify_<workload>_hbm_traffic.md (the summary table), both stamped with the commit of the
tree they were measured on.  The two passes are (run from /tmp with TMPDIR=/tmp, one MI355X;
TS_BENCH_CALIB=1 makes bench.py add three plain 1 GiB device copies to the same process):

    rocprofv3 --pmc TCC_EA0_RDREQ_sum TCC_EA0_RDREQ_32B_sum TCC_EA0_RDREQ_64B_sum TCC_EA0_RDREQ_128B_sum \\
              -d <dir_rd> -o p -- python3 bench.py --steps 1 --warmup 1 --no-cpu-baseline
    rocprofv3 --pmc WRITE_SIZE TCC_EA0_WRREQ_sum TCC_EA0_WRREQ_64B_sum \\
              -d <dir_wr> -o p -- python3 bench.py --steps 1 --warmup 1 --no-cpu-baseline

Reads = 128 B x RDREQ_128B + 64 B x RDREQ_64B + 32 B x RDREQ_32B (the derived FETCH_SIZE counter
of this ROCm release reads 21 KiB for a 1 GiB copy on gfx950, so the request counters it is built
from are used directly); writes = WRITE_SIZE KiB.  Both are scaled by what the same counters read
for the 1 GiB copy kernel of the same process.
"""
import collections
import json
import os
import re
import sqlite3
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GIB = 1 << 30


def _short(k):
    k = k.replace("(anonymous namespace)::", "").replace("void ", "")
    return re.sub(r"\((?!anon).*", "", k)


def _gemm_mode(name):
    m = re.match(r"k_gemm_bf16<(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+)>", name)
    return int(m.group(7)) if m else None


def _load(db):
    """{kernel (split projections: name + ' grid GxS'): {counter: [values]}}"""
    cur = sqlite3.connect(db).cursor()
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for k, c, v, gx, gy, wx in cur.execute(
            "select kernel_name, counter_name, value, grid_size_x, grid_size_y, workgroup_size_x from counters_collection"):
        k = _short(k)
        if _gemm_mode(k) == 0:
            k += " grid %dx%d" % (gx // wx, gy)
        agg[k][c].append(v)
    return agg


def kernel_kind(name):
    """Kernel name of the library -> the kind bench.py reports it under (None: not one of ours).
    The split projections share one kernel; on the 8B shape the QKV projection is the launch with
    48 column groups, the O and down projections both run 32 groups x 8 splits."""
    mode = _gemm_mode(name.split(" grid ")[0])
    if mode == 2:
        return "gemm_gate_up"
    if mode == 1:
        return "gemm_lm_head_argmax"
    if mode == 0:
        grid = name.split(" grid ")[1] if " grid " in name else ""
        return "gemm_qkv" if grid.startswith("48x") else "gemm_o+gemm_down"
    return {"k_attn_bf16": "attn_bf16", "k_attn_merge": "attn_merge", "k_norm": "residual_rmsnorm",
            "k_rope_kv": "rope_kv_write", "k_plain_read": "plain_read"}.get(name.split("<")[0])


def sq_summary(dbs, out_path, commit):
    """Matrix-pipe and LDS utilisation per kernel: means per launch of the SQ counters, summed over their dimensions."""
    with open(out_path, "w") as f:
        f.write("# rocprofv3 counters: matrix-pipe and LDS utilisation of the projections and the attention kernel\n\n")
        f.write("Measured on commit %s.  One counter pass per workload (run from /tmp with TMPDIR=/tmp on one MI355X), then\n"
                "`python -m paper_2604_13519_amd.counters sq <w3.db> <w4.db>`:\n\n" % commit)
        f.write("    rocprofv3 --pmc SQ_ACTIVE_INST_ANY SQ_BUSY_CU_CYCLES SQ_INSTS_MFMA SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES "
                "SQ_WAIT_ANY SQ_WAVE_CYCLES -d <dir> -o p -- python3 bench.py [--workload w4] --steps 1 --warmup 1 --no-cpu-baseline\n\n")
        f.write("Values are means per launch, each counter summed over its dimensions.  Matrix pipe busy = SQ_VALU_MFMA_BUSY_CYCLES / "
                "(4 x SQ_BUSY_CU_CYCLES)\n(four SIMDs per CU), LDS active = SQ_LDS_IDX_ACTIVE / SQ_BUSY_CU_CYCLES, LDS conflict = "
                "SQ_LDS_BANK_CONFLICT / SQ_BUSY_CU_CYCLES,\nwaves waiting = SQ_WAIT_ANY / SQ_WAVE_CYCLES.\n")
        for title, db in dbs:
            cur = sqlite3.connect(db).cursor()
            per = collections.defaultdict(lambda: collections.defaultdict(list))
            q = ("select kernel_name, grid_size_x, grid_size_y, workgroup_size_x, dispatch_id, counter_name, sum(value) "
                 "from counters_collection group by kernel_name, dispatch_id, counter_name")
            for k, gx, gy, wx, _, c, v in cur.execute(q):
                k = _short(k)
                if not (k.startswith("k_gemm") or k.startswith("k_attn_bf16")):
                    continue
                if _gemm_mode(k) == 0 or k.startswith("k_gemm_rows_bf16"):
                    k += " grid %dx%d" % (gx // wx, gy)
                per[k][c].append(v)
            f.write("\n## %s\n\n| kernel | launches | MFMAs / launch | matrix pipe busy | LDS active | LDS conflict | waves waiting |\n"
                    "|---|---:|---:|---:|---:|---:|---:|\n" % title)
            mean = lambda k, c: sum(per[k][c]) / max(len(per[k][c]), 1)
            for k in sorted(per, key=lambda k: -mean(k, "SQ_BUSY_CU_CYCLES") * len(per[k]["SQ_BUSY_CU_CYCLES"])):
                busy = max(mean(k, "SQ_BUSY_CU_CYCLES"), 1.0)
                f.write("| `%s` | %d | %.0f | %.1f %% | %.1f %% | %.1f %% | %.1f %% |\n" % (
                    k, len(per[k]["SQ_BUSY_CU_CYCLES"]), mean(k, "SQ_INSTS_MFMA"), 100 * mean(k, "SQ_VALU_MFMA_BUSY_CYCLES") / (4 * busy),
                    100 * mean(k, "SQ_LDS_IDX_ACTIVE") / busy, 100 * mean(k, "SQ_LDS_BANK_CONFLICT") / busy,
                    100 * mean(k, "SQ_WAIT_ANY") / max(mean(k, "SQ_WAVE_CYCLES"), 1.0)))
    print("wrote", out_path)
    return 0


def trace_summary(db, workload, command, bench_json=None):
    """profiles/verify_<workload>_kernel_trace.md from a --kernel-trace results database."""
    cur = sqlite3.connect(db).cursor()
    rows = list(cur.execute("select name, start, end, grid_x, grid_y, workgroup_x from kernels order by start"))
    agg = collections.OrderedDict()
    names = []
    for name, st, en, gx, gy, wx in rows:
        k = _short(name)
        if _gemm_mode(k) == 0 or k.startswith("k_gemm_rows_bf16"):
            k += " grid %dx%d" % (gx // wx, gy)
        names.append(k)
        a = agg.setdefault(k, [0, 0.0])
        a[0] += 1
        a[1] += (en - st) / 1e3
    total = sum(a[1] for a in agg.values())
    commit = _commit()
    path = os.path.join(ROOT, "profiles", "verify_%s_kernel_trace.md" % workload)
    with open(path, "w") as f:
        f.write("# rocprofv3 kernel trace: tree-verify step, workload %s\n\n" % workload)
        f.write("Measured on commit %s.  Command (run from /tmp with TMPDIR=/tmp on one MI355X), then\n" % commit)
        f.write("`python -m paper_2604_13519_amd.counters trace <results.db> --workload %s`:\n\n    %s\n\n" % (workload, command))
        f.write("Durations are kernel begin-to-end times from the trace; the run also holds model load (k_repack_tiles, k_kv_xfer)\n"
                "and bench.py's untimed passes.  Template arguments of `k_gemm_bf16`: row tiles, tiles per wave, column sets, k-waves,\n"
                "chunk, prefetch depth, mode (0 partial sums, 1 arg-max, 2 SwiGLU), LDS pad; `grid GxS` = column groups x K splits.\n\n")
        f.write("| kernel | calls | total us | avg us | % |\n|---|---:|---:|---:|---:|\n")
        for k, (n, t) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
            if t / total < 0.0005:
                continue
            f.write("| `%s` | %d | %.1f | %.2f | %.1f |\n" % (k, n, t, t / n, 100.0 * t / total))
        # one step in the middle of the run: from one row set-up kernel to the next
        starts = [i for i, k in enumerate(names) if k.startswith("k_embed")]
        if len(starts) >= 3:
            i0, i1 = starts[len(starts) // 2], starts[len(starts) // 2 + 1]
            step = rows[i0:i1]
            # the pass ends with the acceptance walk; what follows (commit, roll-back) belongs to the step too
            span = (step[-1][2] - step[0][1]) / 1e3
            busy = sum(r[2] - r[1] for r in step) / 1e3
            gaps = [(step[i + 1][1] - step[i][2]) / 1e3 for i in range(len(step) - 1)]
            f.write("\nOne step in the middle of the run (row set-up kernel to the last kernel before the next one): %d kernels, span %.1f us, "
                    "busy %.1f us, gaps %.1f us (largest %.2f us).\n" % (len(step), span, busy, sum(g for g in gaps if g > 0), max(gaps)))
        if bench_json:
            d = json.loads(open(bench_json).read().strip().splitlines()[-1])
            rf = d["roofline"]
            kname = [k for k in agg if _gemm_mode(k.split(" grid ")[0]) == (2 if rf["kernel"] == "gemm_gate_up" else -1) or
                     (rf["kernel"] == "gemm_gate_up" and k.startswith("k_gemm_rows_bf16") and k.split(",")[-1].startswith(" 2>"))]
            if kname:
                n, t = agg[kname[0]]
                f.write("\nRoofline kernel of bench.py's line for this build (`%s`): trace average %.2f us per launch; bench.py's HIP-event "
                        "bracket around the same launches reads %.2f us (each bracket carries 2 - 3 us of event overhead), i.e. %s %.0f from the "
                        "trace against %.0f reported.\n" % (rf["kernel"], t / n, rf["avg_us"], rf["unit"],
                                                          rf["achieved"] * rf["avg_us"] / (t / n), rf["achieved"]))
    print("wrote", path)
    return 0


_COMMIT_OVERRIDE = None      # --commit <hash>: the tree the profiler ran on, when that is not the checked-out one


def _commit():
    if _COMMIT_OVERRIDE:
        return _COMMIT_OVERRIDE
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], capture_output=True, text=True).stdout.strip()
    except Exception:
        return ""


def main(argv):
    if len(argv) < 2:
        print(__doc__)
        return 2
    workload = argv[argv.index("--workload") + 1] if "--workload" in argv else "w3"
    if "--commit" in argv:
        global _COMMIT_OVERRIDE
        _COMMIT_OVERRIDE = argv[argv.index("--commit") + 1]
    if argv[0] == "sq":
        out = argv[argv.index("--out") + 1] if "--out" in argv else os.path.join(ROOT, "profiles", "verify_mfma_lds_counters.md")
        commit = argv[argv.index("--commit") + 1] if "--commit" in argv else _commit()
        return sq_summary([("w3 (65 rows, context 8192): projections bound by HBM", argv[1]),
                           ("w4 (528 rows, 16 requests): projections bound by the matrix pipes", argv[2])], out, commit)
    if argv[0] == "trace":
        command = argv[argv.index("--command") + 1] if "--command" in argv else \
            "rocprofv3 --kernel-trace --stats -d <dir> -o t -- python3 bench.py --steps 8 --warmup 2 --no-cpu-baseline" + \
            ("" if workload == "w3" else " --workload " + workload)
        return trace_summary(argv[1], workload, command, argv[argv.index("--bench") + 1] if "--bench" in argv else None)
    rd, wr = argv[0], argv[1]
    R, W = _load(rd), _load(wr)
    copy_rd = max(R[[k for k in R if "copyBuffer" in k][0]]["TCC_EA0_RDREQ_128B_sum"]) * 128
    copy_wr = max(W[[k for k in W if "copyBuffer" in k][0]]["WRITE_SIZE"]) * 1024
    out, rows = {}, []
    for k in R:
        kd = kernel_kind(k)
        if not kd:
            continue
        mean = lambda d, c: sum(d[k][c]) / max(len(d[k][c]), 1)
        rb = 128 * mean(R, "TCC_EA0_RDREQ_128B_sum") + 64 * mean(R, "TCC_EA0_RDREQ_64B_sum") + 32 * mean(R, "TCC_EA0_RDREQ_32B_sum")
        wb = 1024 * mean(W, "WRITE_SIZE")
        rb *= GIB / copy_rd
        wb *= GIB / copy_wr
        out[kd] = {"read_bytes": rb, "write_bytes": wb, "bytes": rb + wb}
        rows.append((kd, k, len(R[k]["TCC_EA0_RDREQ_sum"]), rb, wb))
    commit = _commit()
    out["_measured_on"] = {"commit": commit, "workload": workload,
                           "scale_read": GIB / copy_rd, "scale_write": GIB / copy_wr}
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    json.dump(out, open(os.path.join(ROOT, "profiles", "traffic.json"), "w"), indent=1, sort_keys=True)
    with open(os.path.join(ROOT, "profiles", "verify_%s_hbm_traffic.md" % workload), "w") as f:
        f.write("# HBM traffic per launch: tree-verify step, workload %s\n\n" % workload)
        f.write("Measured on commit %s.  Command and method: see the docstring of `paper_2604_13519_amd/counters.py`\n" % commit)
        f.write("(two `rocprofv3 --pmc` passes over `python3 bench.py --steps 1 --warmup 1 --no-cpu-baseline` with\n")
        f.write("`TS_BENCH_CALIB=1`, then `python -m paper_2604_13519_amd.counters <read.db> <write.db>`).\n\n")
        f.write("Calibration on the 1 GiB copy (`__amd_rocclr_copyBuffer`): reads %.0f B, writes %.0f B per dispatch -> scale "
                "factors %.4f and %.4f.\n\n" % (copy_rd, copy_wr, GIB / copy_rd, GIB / copy_wr))
        f.write("| kernel kind | kernel | launches | read MB / launch | written MB / launch |\n|---|---|---:|---:|---:|\n")
        for kd, k, n, rb, wb in sorted(rows, key=lambda r: -r[3]):
            f.write("| %s | `%s` | %d | %.2f | %.2f |\n" % (kd, k, n, rb / 1e6, wb / 1e6))
    print(json.dumps(out, indent=1))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
