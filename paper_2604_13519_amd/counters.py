"""HBM traffic per kernel launch from two rocprofv3 counter passes over bench.py.

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


def _load(db):
    cur = sqlite3.connect(db).cursor()
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for k, c, v in cur.execute("select kernel_name, counter_name, value from counters_collection"):
        k = k.replace("(anonymous namespace)::", "").replace("void ", "")
        k = re.sub(r"\((?!anon).*", "", k)
        agg[k][c].append(v)
    return agg


def kernel_kind(name):
    """Kernel name of the library -> the kind bench.py reports it under (None: not one of ours)."""
    m = re.match(r"k_gemm_bf16<(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+)>", name)
    if m:
        mode, cs, kw = int(m.group(7)), int(m.group(3)), int(m.group(4))
        if mode == 2:
            return "gemm_gate_up"
        if mode == 1:
            return "gemm_lm_head_argmax"
        if kw == 1:
            return "gemm_down"
        return "gemm_qkv" if cs == 3 else "gemm_o+gemm_down"
    return {"k_attn_bf16": "attn_bf16", "k_attn_merge": "attn_merge", "k_norm": "residual_rmsnorm",
            "k_rope_kv": "rope_kv_write", "k_plain_read": "plain_read"}.get(name.split("<")[0])


def _commit():
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], capture_output=True, text=True).stdout.strip()
    except Exception:
        return ""


def main(argv):
    if len(argv) < 2:
        print(__doc__)
        return 2
    rd, wr = argv[0], argv[1]
    workload = argv[argv.index("--workload") + 1] if "--workload" in argv else "w3"
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
