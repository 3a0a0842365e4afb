#!/usr/bin/env python3
"""Turns rocprofv3 result databases of bench.py runs into the short text summaries under profiles/ and into
profiles/measured_counters.json, which bench.py reads back (HBM-side traffic per call, matrix-pipe utilisation).

rocprofv3 is run on the GPU machine (from /tmp with TMPDIR=/tmp; R = repository root, P = any scratch directory), one run per counter group, the
program directly after `--`:

  B="python3 $R/bench.py --steps 2 --warmup 1 --no-cpu-baseline --no-layer-calls --no-row-scales --no-rht-sweep --no-context"
  rocprofv3 --kernel-trace --stats -d $P/trace -o bench -- python3 $R/bench.py --steps 5 --warmup 1 \
            --no-cpu-baseline --no-layer-calls --no-row-scales --no-rht-sweep --no-context
  rocprofv3 --pmc FETCH_SIZE -d $P/fetch -o bench -- $B
  rocprofv3 --pmc WRITE_SIZE -d $P/write -o bench -- $B
  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F16 SQ_INSTS_VALU_MFMA_MOPS_F6F4 \
            SQ_VALU_MFMA_COEXEC_CYCLES GRBM_GUI_ACTIVE -d $P/mfma -o bench -- $B
  rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_INSTS_LDS SQ_INSTS_VALU SQ_ACTIVE_INST_VALU SQ_WAVE_CYCLES \
            SQ_WAIT_INST_ANY SQ_WAVES GRBM_GUI_ACTIVE -d $P/sq -o bench -- $B

then, anywhere the databases are (they are large; on the GPU machine itself is simplest):

  python3 bench_profile.py $P [--out DIR] [--commit ID]     # DIR defaults to profiles/

Only this file, bench.py and the library are involved.  Nothing here runs on the GPU.
"""
from __future__ import annotations

import glob
import json
import os
import re
import sqlite3
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
OUT_DIR = os.path.join(ROOT, "profiles")
GEMM_FLOPS = 2.0 * 8192 * 5120 * 20480
CUS, SIMDS_PER_CU, XCDS = 256, 4, 8

BENCH_TAIL = "--no-cpu-baseline --no-layer-calls --no-row-scales --no-rht-sweep --no-context"
COMMANDS = {
    "trace": f"rocprofv3 --kernel-trace --stats -d $P/trace -o bench -- python3 $R/bench.py --steps 5 --warmup 1 {BENCH_TAIL}",
    "fetch": f"rocprofv3 --pmc FETCH_SIZE -d $P/fetch -o bench -- python3 $R/bench.py --steps 2 --warmup 1 {BENCH_TAIL}",
    "write": f"rocprofv3 --pmc WRITE_SIZE -d $P/write -o bench -- python3 $R/bench.py --steps 2 --warmup 1 {BENCH_TAIL}",
    "mfma": "rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F16 SQ_INSTS_VALU_MFMA_MOPS_F6F4 SQ_VALU_MFMA_COEXEC_CYCLES GRBM_GUI_ACTIVE "
            f"-d $P/mfma -o bench -- python3 $R/bench.py --steps 2 --warmup 1 {BENCH_TAIL}",
    "sq": "rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_INSTS_LDS SQ_INSTS_VALU SQ_ACTIVE_INST_VALU SQ_WAVE_CYCLES SQ_WAIT_INST_ANY SQ_WAVES GRBM_GUI_ACTIVE "
          f"-d $P/sq -o bench -- python3 $R/bench.py --steps 2 --warmup 1 {BENCH_TAIL}",
}


def find_db(directory: str):
    hits = sorted(glob.glob(os.path.join(directory, "**", "*_results.db"), recursive=True))
    return hits[-1] if hits else None


def short_name(n: str) -> str:
    """A readable kernel name: template arguments kept, parameter list and namespaces of no interest dropped."""
    m = re.search(r"gemm_f16_kernelILb(\d)ELb(\d)ELb(\d)E", n)
    if m:      # template arguments: bf16 output, per-row tensor scales, split-K partial tiles as output
        return "nvfp4::gemm_f16_kernel<%s>" % ", ".join("true" if g == "1" else "false" for g in m.groups())
    m = re.search(r"splitk_sum_kernelILb(\d)ELb(\d)E", n)
    if m:
        return "nvfp4::splitk_sum_kernel<%s>" % ", ".join("true" if g == "1" else "false" for g in m.groups())
    if "decode_f16_kernel" in n:
        return "nvfp4::decode_f16_kernel"
    n = re.sub(r"\(.*", "", n.replace("void ", "").replace("(anonymous namespace)::", ""))
    return n[:110]


def ours(n: str) -> bool:
    if "amax_finalize_kernel" in n or "mx_tensor_scale_kernel" in n:
        return False                                  # a few microseconds each: left out to keep the summaries short
    return "nvfp4" in n or "stream_copy_kernel" in n or "mfma_rate_kernel" in n


def table_columns(c, table):
    return [r[1] for r in c.execute(f"pragma table_info({table})")]


def kernel_trace(db: str):
    """[(name, calls, total_us, avg_us, min_us, max_us, pct)] over the kernels of the process, ours only."""
    c = sqlite3.connect(db)
    cols = table_columns(c, "kernels")
    name_col = "name" if "name" in cols else [x for x in cols if "name" in x][0]
    tot = c.execute("select sum(end-start) from kernels").fetchone()[0]
    rows = []
    for n, k, s, a, mi, ma in c.execute(f"select {name_col}, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start) "
                                        f"from kernels group by {name_col} order by 3 desc"):
        if ours(n):
            rows.append((short_name(n), k, s / 1e3, a / 1e3, mi / 1e3, ma / 1e3, 100.0 * s / tot))
    return rows


def pmc(db: str):
    """{counter: {kernel: (calls, avg, min, max, avg_us)}}"""
    c = sqlite3.connect(db)
    out = {}
    q = ("select kernel_name, counter_name, count(*), avg(value), min(value), max(value), avg(duration) from counters_collection "
         "group by kernel_name, counter_name")
    for n, cn, k, a, mi, ma, d in c.execute(q):
        if ours(n):
            key = short_name(n)
            prev = out.setdefault(cn, {}).get(key)
            if prev:                                  # two mangled names with one short name: merge
                kk = prev[0] + k
                out[cn][key] = (kk, (prev[1] * prev[0] + a * k) / kk, min(prev[2], mi), max(prev[3], ma), (prev[4] * prev[0] + d * k) / kk)
            else:
                out[cn][key] = (k, a, mi, ma, d)
    return out


def pmc_sum_by_kernel(db: str, counter: str):
    """{kernel: [value per dispatch, in dispatch order]} for one counter."""
    c = sqlite3.connect(db)
    cols = table_columns(c, "counters_collection")
    order = "dispatch_id" if "dispatch_id" in cols else "start"
    out = {}
    for n, v in c.execute(f"select kernel_name, value from counters_collection where counter_name = ? order by {order}", (counter,)):
        if ours(n):
            out.setdefault(short_name(n), []).append(v)
    return out


def fmt_pmc(table, counter):
    lines = [f"{'calls':>5} {'avg':>16} {'min':>16} {'max':>16} {'avg_us':>9}  {counter}  kernel"]
    for kern, (k, a, mi, ma, d) in sorted(table.get(counter, {}).items(), key=lambda kv: -kv[1][1]):
        if ma == 0:
            continue                                  # kernels the counter does not concern
        lines.append(f"{k:5d} {a:16.1f} {mi:16.1f} {ma:16.1f} {d / 1e3:9.1f}  {counter}  {kern}")
    return lines


def git_head() -> str:
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except OSError:
        return "unknown"


def main() -> int:
    global OUT_DIR
    argv = sys.argv[1:]
    commit = git_head()
    if "--commit" in argv:                            # where the tree is not a git checkout (the GPU machine)
        i = argv.index("--commit")
        commit = argv[i + 1]
        del argv[i:i + 2]
    if "--out" in argv:
        i = argv.index("--out")
        OUT_DIR = os.path.abspath(argv[i + 1])
        del argv[i:i + 2]
    if len(argv) != 1:
        print(__doc__)
        return 2
    base = argv[0]
    dbs = {k: find_db(os.path.join(base, k)) for k in COMMANDS}
    os.makedirs(OUT_DIR, exist_ok=True)
    measured = {"source": f"rocprofv3 runs of bench.py summarised by bench_profile.py (tree at commit {commit}); "
                          "see profiles/bench_linear_layer_12B_*.txt for the commands"}
    head = ("bench.py, one NVFP4 linear layer fwd+bwd at the 12B MLP up-projection shape (8192 tokens, 5120 -> 20480), one MI355X;\n"
            "the MXFP4 comparison block of bench.py runs in the same process (gemm_mx_kernel_*, quantize_mx_kernel).\n"
            "Run from /tmp with TMPDIR=/tmp on the GPU box, R = repository root, P = a scratch directory.  Summarised by bench_profile.py.\n")

    if dbs["trace"]:
        rows = kernel_trace(dbs["trace"])
        with open(os.path.join(OUT_DIR, "bench_linear_layer_12B_kernel_trace.txt"), "w") as fh:
            fh.write("rocprofv3 kernel-trace summary: " + head)
            fh.write("Command:\n  " + COMMANDS["trace"] + "\n")
            fh.write("5 timed steps + 1 warm-up step + the side blocks are all in the counts.  One nvfp4_gemm call = decode_f16_kernel +\n"
                     "gemm_f16_kernel<bf16 output, per-row scales, false> (+ for the last partial round of tiles, Dgrad and Wgrad:\n"
                     "gemm_f16_kernel<false, false, true>, which stores split-K partial tiles, and splitk_sum_kernel, which adds them).\n"
                     "Durations in microseconds; pct = share of all GPU kernel time in the process (input generation included).\n\n")
            fh.write(f"{'calls':>6} {'total_us':>12} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'pct':>6}  kernel\n")
            for n, k, s, a, mi, ma, pct in rows:
                fh.write(f"{k:6d} {s:12.1f} {a:10.1f} {mi:10.1f} {ma:10.1f} {pct:6.1f}  {n}\n")
        measured["kernel_avg_us"] = {n: a for n, k, s, a, mi, ma, pct in rows}

    traffic = {}
    if dbs["fetch"] and dbs["write"]:
        f, w = pmc(dbs["fetch"]), pmc(dbs["write"])
        cal_f = f["FETCH_SIZE"].get("stream_copy_kernel")
        cal_w = w["WRITE_SIZE"].get("stream_copy_kernel")
        kib = float(1 << 20)                                    # the calibration copy moves 1 GiB each way
        sf = kib / cal_f[1] if cal_f else 1.0
        sw = kib / cal_w[1] if cal_w else 1.0
        with open(os.path.join(OUT_DIR, "bench_linear_layer_12B_hbm_traffic_pmc.txt"), "w") as fh:
            fh.write("rocprofv3 PMC summary (traffic between L2 and the fabric per dispatch, KiB): " + head)
            fh.write("Two runs, one counter each (FETCH_SIZE takes three of the four TCC counters, WRITE_SIZE two):\n  "
                     + COMMANDS["fetch"] + "\n  " + COMMANDS["write"] + "\n")
            fh.write("Calibration: bench.py issues plain copies of 1 GiB (1048576 KiB read + 1048576 KiB written) with bench_probe.hip's\n"
                     f"stream_copy_kernel before the warm-up.  Scale factor = 1048576 / counter value of that copy: FETCH_SIZE x {sf:.3f}, "
                     f"WRITE_SIZE x {sw:.3f}.\n\n")
            fh.write("\n".join(fmt_pmc(f, "FETCH_SIZE")) + "\n\n" + "\n".join(fmt_pmc(w, "WRITE_SIZE")) + "\n")
            # per nvfp4_gemm call and per step's quantize calls, in bytes
            fv, wv = pmc_sum_by_kernel(dbs["fetch"], "FETCH_SIZE"), pmc_sum_by_kernel(dbs["write"], "WRITE_SIZE")

            def total(kernels, table, scale):
                return sum(sum(table.get(k, [])) for k in kernels) * 1024.0 * scale

            gemm_k = [k for k in fv if "gemm_f16_kernel" in k or "decode_f16_kernel" in k or "splitk_sum_kernel" in k]
            quant_k = [k for k in fv if ("cast_kernel" in k or "amax_kernel" in k or "amax_finalize" in k)]
            steps = 3                                           # --steps 2 --warmup 1
            g_calls = 3 * steps
            traffic["gemm_call_traffic_bytes"] = (total(gemm_k, fv, sf) + total(gemm_k, wv, sw)) / g_calls
            traffic["gemm_call_fetch_bytes"] = total(gemm_k, fv, sf) / g_calls
            traffic["gemm_call_write_bytes"] = total(gemm_k, wv, sw) / g_calls
            traffic["quantize_calls_traffic_bytes"] = (total(quant_k, fv, sf) + total(quant_k, wv, sw)) / steps
            fh.write(f"\nPer nvfp4_gemm call (decode + GEMM kernels, average of the step's three calls): "
                     f"{traffic['gemm_call_fetch_bytes'] / 1e9:.2f} GB fetched + {traffic['gemm_call_write_bytes'] / 1e9:.2f} GB written = "
                     f"{traffic['gemm_call_traffic_bytes'] / 1e9:.2f} GB.\n"
                     f"Per step, the three nvfp4_quantize calls together: {traffic['quantize_calls_traffic_bytes'] / 1e9:.2f} GB.\n")
        measured.update(traffic)

    if dbs["mfma"]:
        m = pmc(dbs["mfma"])
        with open(os.path.join(OUT_DIR, "bench_linear_layer_12B_mfma_pmc.txt"), "w") as fh:
            fh.write("rocprofv3 PMC summary (matrix pipe): " + head)
            fh.write("Command:\n  " + COMMANDS["mfma"] + "\n")
            fh.write("Counters are sums over the chip per dispatch.  SQ_VALU_MFMA_BUSY_CYCLES = cycles the matrix pipe of a SIMD is busy, summed\n"
                     "over the 1024 SIMDs: exactly 16 per v_mfma_f32_16x16x32_f16 and per v_mfma_scale_f32_16x16x128_f8f6f4 with FP4 operands\n"
                     "(BUSY / (MOPS x 512 / flop per instruction) below).  GRBM_GUI_ACTIVE = GPU clock cycles of the dispatch, here summed over\n"
                     f"the {XCDS} XCDs (each counts on its own: divided by {XCDS} and by the duration it gives the clock, 2.1 - 2.5 GHz).\n"
                     f"mfma busy fraction = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / {XCDS} x {CUS} CUs x {SIMDS_PER_CU} SIMDs), rocprofv3's own MfmaUtil formula.\n"
                     "MOPS counters count 512 flop each: MOPS x 512 against 2 M N K proves the timed kernels do the whole contraction.\n\n")
            for cn in sorted(m):
                fh.write("\n".join(fmt_pmc(m, cn)) + "\n\n")
            busy, act = m.get("SQ_VALU_MFMA_BUSY_CYCLES", {}), m.get("GRBM_GUI_ACTIVE", {})
            mops = m.get("SQ_INSTS_VALU_MFMA_MOPS_F16", {})
            fh.write("Derived:\n")
            for kern in busy:
                if kern in act and act[kern][1] > 0:
                    if busy[kern][1] == 0:
                        continue
                    cycles = act[kern][1] / XCDS
                    frac = busy[kern][1] / (cycles * CUS * SIMDS_PER_CU)
                    fh.write(f"  {kern}: mfma busy fraction {frac:.3f} (average over its dispatches), clock {cycles / act[kern][4] :.2f} GHz")
                    if kern in mops and mops[kern][1] > 0:
                        fh.write(f"; MOPS_F16 x 512 = {mops[kern][1] * 512:.4e} flop per dispatch (avg)")
                    fh.write("\n")
                    if "gemm_f16_kernel<true, false, false>" in kern:
                        measured["gemm_f16_kernel_mfma_busy_frac"] = frac
                    if "gemm_mx_kernel_k512" in kern:
                        measured.setdefault("gemm_mx_kernel_mfma_busy_frac", frac)
            tot_mops = sum(v[0] * v[1] for k, v in mops.items() if "gemm_f16_kernel" in k)
            if tot_mops:
                calls = 9                                        # 3 steps x 3 GEMM calls
                fh.write(f"  sum over gemm_f16_kernel dispatches of MOPS_F16 x 512 / {calls} nvfp4_gemm calls = {tot_mops * 512 / calls:.6e} flop; "
                         f"2 M N K = {GEMM_FLOPS:.6e}\n")
                measured["gemm_call_mops_x512_over_2mnk"] = tot_mops * 512 / calls / GEMM_FLOPS

    if dbs["sq"]:
        m = pmc(dbs["sq"])
        with open(os.path.join(OUT_DIR, "bench_linear_layer_12B_sq_pmc.txt"), "w") as fh:
            fh.write("rocprofv3 PMC summary (LDS, VALU, wave counters): " + head)
            fh.write("Command:\n  " + COMMANDS["sq"] + "\n")
            fh.write("Counters are sums over the chip per dispatch.\n\n")
            for cn in sorted(m):
                fh.write("\n".join(fmt_pmc(m, cn)) + "\n\n")
            conf, act = m.get("SQ_LDS_BANK_CONFLICT", {}), m.get("SQ_LDS_IDX_ACTIVE", {})
            fh.write("Derived:\n")
            for kern in conf:
                if kern in act and act[kern][1] > 0:
                    fh.write(f"  {kern}: LDS bank conflict cycles / LDS active cycles = {conf[kern][1] / act[kern][1]:.3f}\n")

    with open(os.path.join(OUT_DIR, "measured_counters.json"), "w") as fh:
        json.dump(measured, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print(json.dumps(measured, indent=1, sort_keys=True))
    return 0


if __name__ == "__main__":
    sys.exit(main())
