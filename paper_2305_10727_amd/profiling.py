"""Turns rocprofv3 CSV output of `bench.py --profile-mode` into the short summaries kept under profiles/.

    python -m paper_2305_10727_amd.profiling --stats DIR --fetch DIR --write DIR --out-prefix PREFIX

--stats: output directory of `rocprofv3 --kernel-trace --stats --output-format csv`
--fetch / --write: output directories of `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` (one counter per run).
HBM traffic per launch = counter value of the kernel x (known bytes of the calibration kernel / its counter value);
the calibration kernel is the fp32->fp16 streaming kernel on 2^26 elements (reads 256 MiB, writes 128 MiB).
"""
import argparse
import csv
import glob
import json
import os
from collections import defaultdict

CALIB_KERNEL = "cast_f16_kernel"
CALIB_READ = 4 << 26
CALIB_WRITE = 2 << 26


def _rows(directory, suffix):
    files = glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True)
    for f in files:
        with open(f, newline="") as fh:
            for row in csv.DictReader(fh):
                yield row


def kernel_stats(directory):
    durs = defaultdict(list)
    for r in _rows(directory, "kernel_trace.csv"):
        durs[r["Kernel_Name"]].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    total = sum(sum(v) for v in durs.values()) or 1
    out = []
    for k, v in sorted(durs.items(), key=lambda kv: -sum(kv[1])):
        out.append(dict(kernel=k, calls=len(v), total_ns=sum(v), avg_ns=sum(v) / len(v), min_ns=min(v), max_ns=max(v),
                        percent=100.0 * sum(v) / total))
    return out


def counter_per_kernel(directory, counter):
    vals = defaultdict(list)
    for r in _rows(directory, "counter_collection.csv"):
        if r["Counter_Name"] == counter:
            vals[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in vals.items()}


def pmc_per_kernel(directories, kernel_filter=""):
    """{kernel: {counter: average value per launch}} over several single-pass rocprofv3 --pmc outputs"""
    vals = defaultdict(lambda: defaultdict(list))
    for d in directories:
        for r in _rows(d, "counter_collection.csv"):
            if kernel_filter in r["Kernel_Name"]:
                vals[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: sum(v) / len(v) for c, v in cs.items()} for k, cs in vals.items()}


VALU_CLOCKS = 2.6


def derived(c, simds=1024, xcds=8):
    """Ratios of the raw counters.  rocprofv3 reports a counter summed over the chip.  Time base: SQ_BUSY_CYCLES counts,
    per shader engine (8 dies x 4), the clocks during which the engine holds a wavefront, so busy_cycles / 32 is the
    launch's length in shader clocks (it agrees within 10 % with the traced duration times the shader clock sampled
    during the GEMM; GRBM_GUI_ACTIVE / 8 dies, the fallback, also counts the dispatch's set-up and the collection of the
    counters and reads 30-40 % long).  SQ_WAVE_CYCLES counts the lifetimes of the wavefronts in units of 4 clocks:
    4 x wave_cycles / waves is the mean lifetime, shorter than the launch by what the workgroups that finish early idle.
    The matrix pipe of a SIMD is busy 16 clocks per 16x16 matrix instruction (SQ_VALU_MFMA_BUSY_CYCLES = 16 x
    SQ_INSTS_MFMA), so mfma_util is the share of the launch during which a SIMD's matrix pipe was busy, averaged over all
    `simds` SIMDs."""
    out = {}
    clocks = None
    if c.get("SQ_BUSY_CYCLES"):
        clocks = c["SQ_BUSY_CYCLES"] / (4 * xcds)
        out["launch_clocks (busy_cycles / %d shader engines)" % (4 * xcds)] = clocks
    elif c.get("GRBM_GUI_ACTIVE"):
        clocks = c["GRBM_GUI_ACTIVE"] / xcds
        out["launch_clocks (gui_active / %d XCDs)" % xcds] = clocks
    if c.get("SQ_WAVE_CYCLES") and c.get("SQ_WAVES"):
        out["mean wavefront lifetime in clocks (4 x wave_cycles / waves)"] = 4.0 * c["SQ_WAVE_CYCLES"] / c["SQ_WAVES"]
    if clocks and "SQ_VALU_MFMA_BUSY_CYCLES" in c:
        out["mfma_util = mfma_busy_cycles / (launch_clocks * %d SIMDs)" % simds] = c["SQ_VALU_MFMA_BUSY_CYCLES"] / (clocks * simds)
    if "SQ_VALU_MFMA_BUSY_CYCLES" in c and "SQ_INSTS_MFMA" in c:
        out["mfma_busy_cycles / mfma_insts"] = c["SQ_VALU_MFMA_BUSY_CYCLES"] / max(c["SQ_INSTS_MFMA"], 1.0)
    # SQ_INSTS_VALU includes the matrix instructions.  A SIMD's vector ALU is 32 lanes wide: with two or more wavefronts
    # it takes an fp32 fma every 2.6 clocks (measured, probes: vector_fp32_fma), the instruction mix of the GELU epilogue
    # one instruction every 3.6 clocks; VALU_CLOCKS is the former, so valu_util is a lower bound for epilogue-heavy kernels.
    mfma_insts = c.get("SQ_INSTS_MFMA", 0.0)
    if clocks and "SQ_INSTS_VALU" in c:
        other = c["SQ_INSTS_VALU"] - mfma_insts
        out["vector instructions (matrix ones excluded) per SIMD and clock"] = other / (clocks * simds)
        out["valu_util = %.1f clocks * vector instructions / (launch_clocks * %d SIMDs)" % (VALU_CLOCKS, simds)] = VALU_CLOCKS * other / (clocks * simds)
        if "SQ_VALU_MFMA_BUSY_CYCLES" in c:
            out["mfma_util + valu_util (a busy matrix pipe takes about half of the vector issue away: the two mostly add)"] = \
                (c["SQ_VALU_MFMA_BUSY_CYCLES"] + VALU_CLOCKS * other) / (clocks * simds)
    if clocks and "SQ_LDS_IDX_ACTIVE" in c:
        out["lds_util = lds_idx_active / (launch_clocks * %d CUs)" % (simds // 4)] = c["SQ_LDS_IDX_ACTIVE"] / (clocks * simds / 4)
    if "SQ_INSTS_VALU" in c and "SQ_INSTS_MFMA" in c:
        out["other vector instructions per matrix instruction"] = (c["SQ_INSTS_VALU"] - c["SQ_INSTS_MFMA"]) / max(c["SQ_INSTS_MFMA"], 1.0)
    if "SQ_LDS_BANK_CONFLICT" in c and "SQ_LDS_IDX_ACTIVE" in c:
        out["lds_bank_conflict / lds_idx_active"] = c["SQ_LDS_BANK_CONFLICT"] / max(c["SQ_LDS_IDX_ACTIVE"], 1.0)
    if "SQ_WAVE_CYCLES" in c and "SQ_WAIT_INST_ANY" in c:
        out["wait_inst_any / wave_cycles"] = c["SQ_WAIT_INST_ANY"] / max(c["SQ_WAVE_CYCLES"], 1.0)
    return out


def short(name, n=70):
    return name if len(name) <= n else name[:n - 3] + "..."


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stats")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--out-prefix", required=True)
    ap.add_argument("--command", default="", help="the profiling command line, recorded in the summary")
    ap.add_argument("--pmc", nargs="*", default=[], help="output directories of further `rocprofv3 --pmc` passes: every counter "
                                                         "found there is averaged per kernel")
    ap.add_argument("--kernel", default="", help="with --pmc: only kernels whose name contains this")
    a = ap.parse_args()
    lines = []
    if a.command:
        lines += ["command: " + a.command, ""]
    result = {}
    if a.stats:
        st = kernel_stats(a.stats)
        lines.append("%-72s %6s %12s %10s %10s %10s %6s" % ("kernel", "calls", "total_us", "avg_us", "min_us", "max_us", "%"))
        for r in st:
            lines.append("%-72s %6d %12.1f %10.2f %10.2f %10.2f %6.1f" % (short(r["kernel"]), r["calls"], r["total_ns"] / 1e3,
                                                                      r["avg_ns"] / 1e3, r["min_ns"] / 1e3, r["max_ns"] / 1e3,
                                                                      r["percent"]))
        result["kernel_avg_us"] = {r["kernel"]: r["avg_ns"] / 1e3 for r in st}
    if a.fetch and a.write:
        fetch = counter_per_kernel(a.fetch, "FETCH_SIZE")
        write = counter_per_kernel(a.write, "WRITE_SIZE")
        cf = [v for k, v in fetch.items() if CALIB_KERNEL in k]
        cw = [v for k, v in write.items() if CALIB_KERNEL in k]
        if cf and cw:
            f_scale = CALIB_READ / cf[0]   # bytes per counter unit
            w_scale = CALIB_WRITE / cw[0]
            lines += ["", "FETCH_SIZE / WRITE_SIZE per launch, scaled by the calibration kernel (%s: %d B read -> counter %.1f, "
                      "%d B written -> counter %.1f; bytes per unit %.1f / %.1f)" % (CALIB_KERNEL, CALIB_READ, cf[0], CALIB_WRITE,
                                                                                   cw[0], f_scale, w_scale),
                      "%-72s %14s %14s %14s" % ("kernel", "read_MB", "written_MB", "total_MB")]
            traffic = {}
            for k in sorted(set(fetch) | set(write)):
                rb, wb = fetch.get(k, 0.0) * f_scale, write.get(k, 0.0) * w_scale
                traffic[k] = dict(read_bytes=rb, write_bytes=wb)
                lines.append("%-72s %14.2f %14.2f %14.2f" % (short(k), rb / 1e6, wb / 1e6, (rb + wb) / 1e6))
            result["traffic"] = traffic
            gemm = [v for k, v in traffic.items() if "spgemm_tile_kernel" in k]
            if gemm:
                result["hbm_bytes_per_launch"] = gemm[0]["read_bytes"] + gemm[0]["write_bytes"]
                result["fetch_scale_bytes_per_unit"] = f_scale
                result["write_scale_bytes_per_unit"] = w_scale
    if a.pmc:
        counters = pmc_per_kernel(a.pmc, a.kernel)
        result["counters"] = counters
        for k, cs in counters.items():
            lines += ["", "counters per launch (average over the launches of each pass): " + short(k, 110)]
            for c, v in sorted(cs.items()):
                lines.append("  %-34s %18.1f" % (c, v))
            d = derived(cs)
            for c, v in d.items():
                lines.append("  %-34s %18.4f" % (c, v))
            result.setdefault("derived", {})[k] = d
    with open(a.out_prefix + ".txt", "w") as fh:
        fh.write("\n".join(lines) + "\n")
    with open(a.out_prefix + ".json", "w") as fh:
        json.dump(result, fh, indent=1)
    print("\n".join(lines))


if __name__ == "__main__":
    main()
