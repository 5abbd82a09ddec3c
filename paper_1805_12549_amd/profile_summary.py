"""Turn a rocprofv3 ``*_results.db`` (rocpd SQLite output of ``--kernel-trace --stats``) into
the short per-kernel text table kept under ``profiles/``.

    python -m paper_1805_12549_amd.profile_summary <out-dir>/run_results.db "command line" > profiles/x.txt
"""
import sqlite3
import sys


def summarize(db_path: str, command: str = "") -> str:
    db = sqlite3.connect(db_path)
    cur = db.cursor()
    rows = list(cur.execute(
        "select name, count(*), sum(duration), avg(duration), min(duration), max(duration) "
        "from kernels group by name order by sum(duration) desc"))
    total = sum(r[2] for r in rows) or 1
    out = []
    if command:
        out.append("command: " + command)
    out.append("source: rocprofv3 --kernel-trace --stats (durations in microseconds)")
    out.append("%-9s %-12s %-10s %-10s %-10s %-6s %s" % ("calls", "total_us", "avg_us", "min_us", "max_us", "pct", "kernel"))
    def shorten(name):
        name = name.replace("cg::(anonymous namespace)::", "").replace("void ", "")
        cut = name.find(">(")
        name = name[:cut + 1] if cut > 0 else name
        return name if len(name) < 110 else name[:107] + "..."

    for name, calls, tot, avg, mn, mx in rows[:12]:
        out.append("%-9d %-12.1f %-10.2f %-10.2f %-10.2f %-6.2f %s" % (
            calls, tot / 1e3, avg / 1e3, mn / 1e3, mx / 1e3, 100.0 * tot / total, shorten(name)))
    # all instantiations of the layer kernel together (the figure bench.py's avg_launch_us reports)
    fam = [r for r in rows if "gated_conv_rows_kernel" in r[0]]
    if fam:
        calls = sum(r[1] for r in fam)
        tot = sum(r[2] for r in fam)
        out.append("")
        out.append("gated_conv_rows_kernel, all instantiations: %d calls, average %.2f us" % (calls, tot / calls / 1e3))
    # per-grid breakdown of the dominant kernel (one line per layer shape)
    if rows:
        dom = rows[0][0]
        out.append("")
        out.append("dominant kernel by launch grid (one grid size per layer shape):")
        out.append("%-10s %-8s %-10s %-8s %-8s" % ("grid_x", "calls", "avg_us", "lds", "vgpr"))
        for g, calls, avg, lds, vg, av in cur.execute(
                "select grid_x, count(*), avg(duration), max(lds_size), max(vgpr_count), max(accum_vgpr_count) "
                "from kernels where name = ? group by grid_x order by grid_x desc", (dom,)):
            out.append("%-10d %-8d %-10.2f %-8d %d+%d" % (g, calls, avg / 1e3, lds, vg, av))
    return "\n".join(out) + "\n"


def traffic(fetch_csv: str, write_csv: str, copy_bytes: int = 256 << 20, kernel: str = "gated_conv") -> str:
    """HBM bytes per launch of the layer kernel from two counter runs of traffic_probe, each counter
    scaled by what it reads for the plain copy of known size (the last elementwise copy before the layers)."""
    import csv

    def read(path, counter):
        rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == counter]
        layer = [float(r["Counter_Value"]) for r in rows if kernel in r["Kernel_Name"]]
        copies = [float(r["Counter_Value"]) for r in rows
                  if "copy" in r["Kernel_Name"].lower() and abs(int(r["Grid_Size"]) if r.get("Grid_Size") else 1) > 0]
        big = [v for v in copies if v > 0.5 * max(copies)]
        return layer, big[-1]

    f_layer, f_copy = read(fetch_csv, "FETCH_SIZE")
    w_layer, w_copy = read(write_csv, "WRITE_SIZE")
    f_scale, w_scale = copy_bytes / f_copy, copy_bytes / w_copy
    out = ["source: rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE on paper_1805_12549_amd.traffic_probe",
           "calibration copy of %d bytes: FETCH_SIZE reads %.1f, WRITE_SIZE reads %.1f -> %.2f / %.2f bytes per unit"
           % (copy_bytes, f_copy, w_copy, f_scale, w_scale),
           "%-8s %-14s %-14s %-14s" % ("launch", "fetch_bytes", "write_bytes", "total_bytes")]
    tot = 0.0
    for i, (f, w) in enumerate(zip(f_layer, w_layer)):
        fb, wb = f * f_scale, w * w_scale
        tot += fb + wb
        out.append("%-8d %-14.0f %-14.0f %-14.0f" % (i, fb, wb, fb + wb))
    n = max(1, min(len(f_layer), len(w_layer)))
    out.append("bytes_per_launch: %.0f" % (tot / n))
    out += ["commands (each in its own run, after cd /tmp && export TMPDIR=/tmp, from the repository root):",
            "  rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/prof_fetch -o r -- python3 -m paper_1805_12549_amd.traffic_probe",
            "  rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/prof_write -o r -- python3 -m paper_1805_12549_amd.traffic_probe",
            "  python -m paper_1805_12549_amd.profile_summary --traffic gpurun_out/prof_fetch/r_counter_collection.csv "
            "gpurun_out/prof_write/r_counter_collection.csv",
            "launches 0..6 = the 7 ImageNet-shaped ResNet-18 gated 3x3 layers (64@56, 128@28, 256@14, 512@7, 64>128 s2, "
            "128>256 s2, 256>512 s2), batch 64, bf16, one cold-cache forward each"]
    return "\n".join(out) + "\n"


def mfma_busy(counter_csv: str, trace_us, kernel: str = "gated_conv") -> str:
    """Executed matrix-core work per launch of the layer kernel from SQ_VALU_MFMA_BUSY_CYCLES (summed over
    the SIMDs; a 32x32x16 bf16 MFMA keeps its SIMD busy 32 cycles for 32768 flops, i.e. 1024 flops per busy
    cycle) and the utilisation against the 2.5 PFLOP/s peak for the given per-layer times (microseconds)."""
    import csv
    vals = [float(r["Counter_Value"]) for r in csv.DictReader(open(counter_csv))
            if r["Counter_Name"] == "SQ_VALU_MFMA_BUSY_CYCLES" and kernel in r["Kernel_Name"]]
    out = ["source: rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES on paper_1805_12549_amd.traffic_probe; times: bench.py per_layer us_gated",
           "%-8s %-18s %-16s %-10s %-12s" % ("launch", "mfma_busy_cycles", "executed_gflop", "us_gated", "mfma_util")]
    for i, v in enumerate(vals):
        gflop = v * 1024 / 1e9
        t = trace_us[i] if i < len(trace_us) else float("nan")
        out.append("%-8d %-18.0f %-16.2f %-10.2f %-12.3f" % (i, v, gflop, t, gflop * 1e9 / (t * 1e-6) / 2.5e15))
    if vals and len(trace_us) >= len(vals):
        tot = sum(vals) * 1024
        out.append("all launches: executed %.1f GFLOP in %.1f us -> %.3f of the bf16 MFMA peak" % (
            tot / 1e9, sum(trace_us[:len(vals)]), tot / (sum(trace_us[:len(vals)]) * 1e-6) / 2.5e15))
    out += ["commands (after cd /tmp && export TMPDIR=/tmp, from the repository root):",
            "  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES GRBM_GUI_ACTIVE --output-format csv -d gpurun_out/prof_mfma -o r "
            "-- python3 -m paper_1805_12549_amd.traffic_probe",
            "  python -m paper_1805_12549_amd.profile_summary --mfma gpurun_out/prof_mfma/r_counter_collection.csv <us_gated of the 7 layers>",
            "launches 0..6 = the 7 ImageNet-shaped ResNet-18 gated 3x3 layers, batch 64, bf16, one cold-cache forward each"]
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if sys.argv[1] == "--mfma":
        sys.stdout.write(mfma_busy(sys.argv[2], [float(v) for v in sys.argv[3:]]))
    elif sys.argv[1] == "--traffic":
        sys.stdout.write(traffic(sys.argv[2], sys.argv[3]))
    else:
        sys.stdout.write(summarize(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else ""))
