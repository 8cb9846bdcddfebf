"""Turns raw rocprofv3 output of bench.py runs into the short text summaries kept under profiles/.

    python3 -m paper_2503_18773_amd.profile_summary        (from the repository root)

Reads <raw>/prof_<workload>[_<variant>]/{trace,fetch,write,sq}/ and <raw>/prof_calib/{fetch,write}/ (raw defaults to
gpurun_out), each written by the rocprofv3 command that the summary quotes, and writes profiles/*.txt.  Per-dispatch
counter values are averaged over the dispatches of the kernel; FETCH_SIZE / WRITE_SIZE are scaled by what the same
counter reads for a plain 1 GiB device copy (bench.py --calib-copy)."""
import collections
import csv
import glob
import os
import sys

RAW = sys.argv[1] if len(sys.argv) > 1 else "gpurun_out"
os.chdir(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

def counters(path, kern):
    acc = collections.defaultdict(list)
    fs = glob.glob(path + "/*counter_collection.csv")
    if not fs: return {}
    for r in csv.DictReader(open(fs[0])):
        if kern in r["Kernel_Name"]:
            acc[r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}

# calibration: 1 GiB copy -> FETCH_SIZE / WRITE_SIZE in KiB per dispatch
calf = counters(RAW + "/prof_calib/fetch", "")  # any kernel
calw = counters(RAW + "/prof_calib/write", "")
def cal(path, name):
    fs = glob.glob(path + "/*counter_collection.csv")
    best = None
    for r in csv.DictReader(open(fs[0])):
        if r["Counter_Name"] == name:
            v = float(r["Counter_Value"])
            if best is None or v > best[0]: best = (v, r["Kernel_Name"])
    return best
cf = cal(RAW + "/prof_calib/fetch", "FETCH_SIZE"); cw = cal(RAW + "/prof_calib/write", "WRITE_SIZE")
KIB = (1 << 30) / 1024
f_fetch = KIB / cf[0]; f_write = KIB / cw[0]
print("calibration: copy 1 GiB: FETCH_SIZE reads", cf, "-> factor", f_fetch, "; WRITE_SIZE reads", cw, "-> factor", f_write)

for cfg, fmt in [("cfg1", "int4"), ("cfg3", "int4"), ("cfg2", "int2"), ("cfg4", "mxfp4")]:
    base = f"{RAW}/prof_{cfg}"
    if not os.path.isdir(base): continue
    kern = "decode_int_kernel" if fmt != "mxfp4" else "decode_mx_kernel"
    lines = []
    lines.append(f"Kernel-trace summary of the benchmark, workload {cfg} ({fmt} KV).")
    lines.append(f"command: rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof_{cfg}/trace -o bench -- python3 bench.py --no-cpu-baseline --no-128k --workload {cfg}")
    lines.append("")
    lines.append(f"{'kernel':70s} {'calls':>6s} {'avg_ns':>10s} {'min_ns':>8s} {'max_ns':>8s} {'pct':>6s}")
    for r in csv.DictReader(open(glob.glob(base + "/trace/*kernel_stats.csv")[0])):
        name = r["Name"].replace("bd::(anonymous namespace)::", "")
        lines.append(f"{name[:70]:70s} {r['Calls']:>6s} {float(r['AverageNs']):10.0f} {r['MinNs']:>8s} {r['MaxNs']:>8s} {float(r['Percentage']):6.2f}")
    lines.append("")
    lines.append("(the decode kernel's calls include the benchmark's 6 x 32 launches of the live roofline timing loop)")
    open(f"profiles/bench_{fmt}_{cfg}_kernel_stats.txt", "w").write("\n".join(lines) + "\n")

    fe = counters(base + "/fetch", kern); wr = counters(base + "/write", kern); sq = counters(base + "/sq", kern)
    lines = []
    lines.append(f"Hardware counters of {kern}, workload {cfg} ({fmt} KV), per dispatch (mean over dispatches).")
    lines.append(f"commands (one counter set per run):")
    lines.append(f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/prof_{cfg}/fetch -o p -- python3 bench.py --no-cpu-baseline --no-128k --workload {cfg} --steps 2 --warmup 1")
    lines.append(f"  rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/prof_{cfg}/write -o p -- python3 bench.py --no-cpu-baseline --no-128k --workload {cfg} --steps 2 --warmup 1")
    lines.append(f"  rocprofv3 --pmc SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY SQ_ACTIVE_INST_VALU SQ_INSTS_VALU SQ_INSTS_MFMA SQ_VALU_MFMA_BUSY_CYCLES --output-format csv -d gpurun_out/prof_{cfg}/sq -o p -- python3 bench.py --no-cpu-baseline --no-128k --workload {cfg} --steps 2 --warmup 1")
    lines.append(f"calibration (plain 1 GiB device copy, torch copy_):")
    lines.append(f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/prof_calib/fetch -o p -- python3 bench.py --calib-copy   -> {cf[0]:.0f} KiB read for 1048576 KiB copied: factor {f_fetch:.4f}")
    lines.append(f"  rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/prof_calib/write -o p -- python3 bench.py --calib-copy   -> {cw[0]:.0f} KiB read for 1048576 KiB copied: factor {f_write:.4f}")
    lines.append("")
    fetch_b = fe["FETCH_SIZE"][0] * 1024 * f_fetch; write_b = wr["WRITE_SIZE"][0] * 1024 * f_write
    lines.append(f"FETCH_SIZE  {fe['FETCH_SIZE'][0]:12.1f} KiB raw  x {f_fetch:.4f} = {fetch_b / 1e6:10.3f} MB   (n={fe['FETCH_SIZE'][1]})")
    lines.append(f"WRITE_SIZE  {wr['WRITE_SIZE'][0]:12.1f} KiB raw  x {f_write:.4f} = {write_b / 1e6:10.3f} MB   (n={wr['WRITE_SIZE'][1]})")
    lines.append(f"traffic_bytes_per_launch: {fetch_b + write_b:.0f}")
    lines.append("")
    for k, (v, n) in sorted(sq.items()):
        lines.append(f"{k:28s} {v:16.1f}")
    if sq:
        w = sq["SQ_WAVES"][0]
        lines.append("")
        lines.append(f"per wave: VALU instructions {sq['SQ_INSTS_VALU'][0] / w:.0f}, MFMA instructions {sq['SQ_INSTS_MFMA'][0] / w:.0f}, "
                     f"MFMA busy cycles per MFMA {sq['SQ_VALU_MFMA_BUSY_CYCLES'][0] / sq['SQ_INSTS_MFMA'][0]:.1f}")
        lines.append(f"share of wave-resident time: VALU issue {sq['SQ_ACTIVE_INST_VALU'][0] / sq['SQ_WAVE_CYCLES'][0]:.3f}, waiting on s_waitcnt {sq['SQ_WAIT_INST_ANY'][0] / sq['SQ_WAVE_CYCLES'][0]:.3f}")
        avg_ns = [float(r["AverageNs"]) for r in csv.DictReader(open(glob.glob(base + "/trace/*kernel_stats.csv")[0])) if kern in r["Name"]][0]
        lines.append(f"MFMA busy: SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x {avg_ns:.0f} ns x 2.4 GHz) = {sq['SQ_VALU_MFMA_BUSY_CYCLES'][0] / (1024 * avg_ns * 2.4):.3f}")
        lines.append("(SQ_WAVE_CYCLES, SQ_ACTIVE_INST_VALU and SQ_WAIT_INST_ANY count in units of 4 clocks, summed over waves)")
    open(f"profiles/decode_{fmt}_{cfg}_pmc.txt", "w").write("\n".join(lines) + "\n")
    print(open(f"profiles/decode_{fmt}_{cfg}_pmc.txt").read())

    # the prefill quantizer of the same runs
    qk = "quant_block_kernel"
    qfe = counters(base + "/fetch", qk); qwr = counters(base + "/write", qk); qsq = counters(base + "/sq", qk)
    if qfe and qwr and qsq:
        ql = []
        ql.append(f"Hardware counters of the prefill quantizer ({'mx_' if fmt == 'mxfp4' else ''}quant_block_kernel), workload {cfg} ({fmt} KV), per dispatch (mean over dispatches).")
        ql.append("Same runs, commands and calibration factors as decode_%s_%s_pmc.txt (the benchmark prefills every layer's cache before its timed steps)." % (fmt, cfg))
        ql.append("")
        qf = qfe["FETCH_SIZE"][0] * 1024 * f_fetch; qw = qwr["WRITE_SIZE"][0] * 1024 * f_write
        ql.append(f"FETCH_SIZE  {qfe['FETCH_SIZE'][0]:12.1f} KiB raw  x {f_fetch:.4f} = {qf / 1e6:10.3f} MB   (n={qfe['FETCH_SIZE'][1]})")
        ql.append(f"WRITE_SIZE  {qwr['WRITE_SIZE'][0]:12.1f} KiB raw  x {f_write:.4f} = {qw / 1e6:10.3f} MB   (n={qwr['WRITE_SIZE'][1]})")
        ql.append(f"traffic_bytes_per_launch: {qf + qw:.0f}")
        ql.append("")
        for k, (v, n) in sorted(qsq.items()):
            ql.append(f"{k:28s} {v:16.1f}")
        qavg = [float(r["AverageNs"]) for r in csv.DictReader(open(glob.glob(base + "/trace/*kernel_stats.csv")[0])) if qk in r["Name"]][0]
        w = qsq["SQ_WAVES"][0]
        ql.append("")
        ql.append(f"average duration (kernel trace of the same workload): {qavg:.0f} ns -> {(qf + qw) / qavg:.0f} GB/s of measured traffic")
        ql.append(f"per wave: VALU instructions {qsq['SQ_INSTS_VALU'][0] / w:.0f}; VALU busy: SQ_ACTIVE_INST_VALU x 4 / (1024 SIMDs x {qavg:.0f} ns x 2.4 GHz) = {qsq['SQ_ACTIVE_INST_VALU'][0] * 4 / (1024 * qavg * 2.4):.3f}")
        ql.append(f"share of wave-resident time: VALU issue {qsq['SQ_ACTIVE_INST_VALU'][0] / qsq['SQ_WAVE_CYCLES'][0]:.3f}, waiting on s_waitcnt {qsq['SQ_WAIT_INST_ANY'][0] / qsq['SQ_WAVE_CYCLES'][0]:.3f}")
        open(f"profiles/quant_{fmt}_{cfg}_pmc.txt", "w").write("\n".join(ql) + "\n")
        print(open(f"profiles/quant_{fmt}_{cfg}_pmc.txt").read())
    print(open(f"profiles/bench_{fmt}_{cfg}_kernel_stats.txt").read())

# ---- workload variants: kernel trace only
for cfg, fmt, var in [("cfg1", "int4", "paged"), ("cfg3", "int4", "paged"), ("cfg4", "mxfp4", "paged"),
                      ("cfg1", "int4_kt", "kt"), ("cfg1", "int4", "gq8"), ("cfg1", "int4", "gq16"),
                      ("cfg1", "int4_g32", "g32"), ("cfg1", "int4_g64", "g64"), ("cfg3", "int4_g32", "g32"),
                      ("cfg1", "int4_kt_g32", "kt_g32"), ("cfg3", "int4_kt_g32", "kt_g32"),
                      ("cfg4", "mxfp4", "gq8"), ("cfg2", "int2", "paged")]:
    base = f"{RAW}/prof_{cfg}_{var}"
    if not os.path.isdir(base): continue
    lines = []
    lines.append(f"Kernel-trace summary of the benchmark, workload {cfg} ({fmt} KV), variant {var}.")
    lines.append(f"command: rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof_{cfg}_{var}/trace -o bench -- python3 bench.py --no-cpu-baseline --no-128k --workload {cfg} --variant {var}")
    lines.append("")
    lines.append(f"{'kernel':70s} {'calls':>6s} {'avg_ns':>10s} {'min_ns':>8s} {'max_ns':>8s} {'pct':>6s}")
    for r in csv.DictReader(open(glob.glob(base + "/trace/*kernel_stats.csv")[0])):
        name = r["Name"].replace("bd::(anonymous namespace)::", "")
        lines.append(f"{name[:70]:70s} {r['Calls']:>6s} {float(r['AverageNs']):10.0f} {r['MinNs']:>8s} {r['MaxNs']:>8s} {float(r['Percentage']):6.2f}")
    lines.append("")
    lines.append("(the decode kernel's calls include the benchmark's 6 x 32 launches of the live roofline timing loop)")
    open(f"profiles/bench_{fmt}_{cfg}_{var}_kernel_stats.txt", "w").write("\n".join(lines) + "\n")
    print(open(f"profiles/bench_{fmt}_{cfg}_{var}_kernel_stats.txt").read())
