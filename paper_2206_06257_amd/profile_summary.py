"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

    python -m paper_2206_06257_amd.profile_summary trace   <dir> <prefix> <workload> [steps_in_trace]
    python -m paper_2206_06257_amd.profile_summary traffic <dir> <workload>
    python -m paper_2206_06257_amd.profile_summary mfma    <dir> <prefix> <workload>

The rocprofv3 commands that produce the inputs are written at the head of every summary.  `traffic` also writes
profiles/traffic_igemm_<workload>.json, which carries a hash of the kernel sources so that bench.py reports the
figure only while the sources are the ones it was measured on."""
import collections
import csv
import hashlib
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")


def source_hash():
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2206_06257_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def _name(n):
    n = n.replace("dat::(anonymous namespace)::", "").replace("void ", "")
    return re.sub(r"\(.*\)$", "", n).replace("unsigned short", "bf16")


def _is_conv(n):
    """conv forward / backward-data launches of the roofline (without those that also form a BN input gradient)."""
    return n.startswith("igemm") and not (n.startswith("igemm_kernel<") and n.rstrip().endswith(", true>"))


TEMPLATES = [
    "# Template arguments: igemm_dma_kernel<TC, TP, WGC, OCC, BK, ANYC> (ANYC = true: k-tiles straddle filter taps), igemm_ring_kernel<TC, TP, WGC, S>,",
    "# igemm_kernel<TC, TP, WGC, PF, FAST, BK, OCC, XF> (XF = true: the operand is a BN input gradient formed while loading),",
    "# bnact_fwd_kernel<T, RES> (RES 0 none, 1 residual, 2 residual normalised on the fly), bnact_bwd_apply_kernel<T, GATE, DXACC, DRES>.",
]


def trace(d, prefix, workload, steps=2):
    rows = list(csv.DictReader(open(os.path.join(d, "%s_kernel_trace.csv" % prefix))))
    agg = collections.OrderedDict()
    for r in rows:
        n = _name(r["Kernel_Name"])
        us = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        e = agg.setdefault(n, [0, 0.0, 1e30, 0.0])
        e[0] += 1; e[1] += us; e[2] = min(e[2], us); e[3] = max(e[3], us)
    tot = sum(e[1] for e in agg.values())
    L = ["# rocprofv3 --kernel-trace --stats --output-format csv -d %s -o %s -- python bench.py --workload %s --steps %d --warmup 1 --no-cpu-baseline --no-launch-events"
         % (d, prefix, workload, steps - 1),
         "# then: python -m paper_2206_06257_amd.profile_summary trace %s %s %s %d" % (d, prefix, workload, steps),
         "# workload %s, bf16 storage / fp32 accumulation; %d steps in the trace (1 warm-up + %d timed), each = the attack iterations"
         % (workload, steps, steps - 1),
         "# (forward + backward-to-input + projected sign step) + outer forward/backward + 8-bit quantize/dequantize.  Durations in microseconds."]
    L += TEMPLATES
    L.append("# The backward-weight launches of the outer step run on a second stream (their durations overlap those of the main stream's kernels).")
    L.append("%-62s %6s %12s %9s %6s %8s %8s" % ("kernel", "calls", "total_us", "avg_us", "pct", "min_us", "max_us"))
    ig = [0, 0.0]
    for n, e in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        L.append("%-62s %6d %12.1f %9.2f %6.2f %8.1f %8.1f" % (n[:62], e[0], e[1], e[1] / e[0], 100 * e[1] / tot, e[2], e[3]))
        if _is_conv(n):
            ig[0] += e[0]; ig[1] += e[1]
    L.append("")
    L.append("total kernel time %.1f ms over %d steps (%.1f ms/step); %d launches per step" % (tot / 1e3, steps, tot / 1e3 / steps, len(rows) // steps))
    L.append("conv forward + backward-data kernels (igemm_dma_kernel + igemm_ring_kernel + igemm_kernel without the XF instantiations): "
             "%d launches, %.1f ms, average %.2f us per launch" % (ig[0], ig[1] / 1e3, ig[1] / max(ig[0], 1)))
    L.append("(bench.py's roofline.avg_launch_ms is the same average, taken with hipEvent pairs around these launches in a second, untimed pass)")
    out = os.path.join(PROFILES, "kernel_trace_%s.txt" % workload)
    open(out, "w").write("\n".join(L) + "\n")
    print("\n".join(L[-4:]))


def _counter(path, counter):
    d = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            d.setdefault(_name(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    return d


def traffic(d, workload):
    cal = {}
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        dd = _counter(os.path.join(d, "copy_%s_counter_collection.csv" % c), c)
        best = max(dd.items(), key=lambda kv: max(kv[1]))          # the 1 GiB copy kernel
        cal[c] = (best[0], max(best[1]))
    ff, wf = 1048576.0 / cal["FETCH_SIZE"][1], 1048576.0 / cal["WRITE_SIZE"][1]
    f = _counter(os.path.join(d, "bench_FETCH_SIZE_counter_collection.csv"), "FETCH_SIZE")
    w = _counter(os.path.join(d, "bench_WRITE_SIZE_counter_collection.csv"), "WRITE_SIZE")
    cmd = "rocprofv3 --pmc %%s --output-format csv -d %s -o %%s -- python bench.py --workload %s --steps 1 --warmup 0 --no-cpu-baseline --no-launch-events" % (d, workload)
    L = ["# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), workload %s" % workload,
         "# commands (each counter in its own run):",
         "#   " + cmd % ("FETCH_SIZE", "bench_FETCH_SIZE"),
         "#   " + cmd % ("WRITE_SIZE", "bench_WRITE_SIZE"),
         "#   rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --output-format csv -d %s -o copy_<counter> -- python bench.py --calibrate-copy" % d,
         "#   python -m paper_2206_06257_amd.profile_summary traffic %s %s" % (d, workload),
         "# calibration: a plain 1 GiB device copy (%s) reads FETCH_SIZE = %.0f KiB and WRITE_SIZE = %.0f KiB per dispatch -> scale factors %.3f (fetch), %.3f (write)"
         % (cal["FETCH_SIZE"][0][:40], cal["FETCH_SIZE"][1], cal["WRITE_SIZE"][1], ff, wf),
         "# one step = the attack iterations + outer step; MiB per launch after scaling",
         "%-48s %6s %18s %18s %12s" % ("kernel", "calls", "fetch MiB/launch", "write MiB/launch", "total GiB")]
    tot, ig, rows = 0.0, [0, 0.0, 0.0], []
    for n in f:
        fv, wv = f[n], w.get(n, [0.0] * len(f[n]))
        fb, wb = sum(fv) * ff / 1024, sum(wv) * wf / 1024
        rows.append((fb + wb, n, len(fv), fb / len(fv), wb / max(len(wv), 1)))
        tot += fb + wb
        if _is_conv(n):
            ig[0] += len(fv); ig[1] += sum(fv) * ff * 1024; ig[2] += sum(wv) * wf * 1024
    for t, n, c, fm, wm in sorted(rows, reverse=True):
        L.append("%-48s %6d %18.1f %18.1f %12.2f" % (n[:48], c, fm, wm, t / 1024))
    L.append("")
    L.append("whole step: %.1f GiB of HBM traffic (%.0f ms at the nominal 8 TB/s)" % (tot / 1024, tot * 1048576 / 8.0e12 * 1e3))
    L.append("conv forward + backward-data kernels (without the <..., true> instantiations that also form a BN input gradient): %d launches, "
             "%.1f MB fetched + %.1f MB written per launch on average" % (ig[0], ig[1] / ig[0] / 1e6, ig[2] / ig[0] / 1e6))
    open(os.path.join(PROFILES, "hbm_traffic_%s.txt" % workload), "w").write("\n".join(L) + "\n")
    json.dump({"kernel": "igemm_dma_kernel + igemm_ring_kernel + igemm_kernel (conv forward + backward-data; without the igemm_kernel<..., true> "
                         "launches that also form a batch-norm input gradient)",
               "workload": workload, "launches": ig[0], "fetch_factor": ff, "write_factor": wf,
               "hbm_fetch_bytes_per_launch": ig[1] / ig[0], "hbm_write_bytes_per_launch": ig[2] / ig[0],
               "hbm_bytes_per_launch": (ig[1] + ig[2]) / ig[0], "whole_step_GiB": tot / 1024, "source_hash": source_hash(),
               "commands": L[2:6]},
              open(os.path.join(PROFILES, "traffic_igemm_%s.json" % workload), "w"), indent=1)
    print("\n".join(L[8:24])); print("\n".join(L[-2:]))


def mfma(d, prefix, workload):
    agg = collections.OrderedDict()
    for r in csv.DictReader(open(os.path.join(d, "%s_counter_collection.csv" % prefix))):
        k = (_name(r["Kernel_Name"]), int(r["Grid_Size"]))
        e = agg.setdefault(k, collections.defaultdict(float))
        e[r["Counter_Name"]] += float(r["Counter_Value"])
        if r["Counter_Name"] == "SQ_WAVE_CYCLES":
            e["_n"] += 1; e["_t"] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    L = ["# MFMA utilisation of the convolution kernels from rocprofv3 SQ counters, workload %s (one step), per kernel and grid size (threads)," % workload,
         "# summed over the launches of the step.",
         "# command: rocprofv3 --pmc SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_INSTS_MFMA SQ_ACTIVE_INST_LDS",
         "#          SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_VMEM --output-format csv -d %s -o %s -- python bench.py --workload %s --steps 1 --warmup 0" % (d, prefix, workload),
         "#          --no-cpu-baseline --no-launch-events ; python -m paper_2206_06257_amd.profile_summary mfma %s %s %s" % (d, prefix, workload),
         "# mfma_busy = SQ_VALU_MFMA_BUSY_CYCLES / (32 x SQ_BUSY_CYCLES): SQ_BUSY_CYCLES is summed over the 32 shader engines, each with 32 SIMDs;",
         "#   every v_mfma_f32_32x32x16_bf16 keeps its SIMD's matrix unit busy for 32 cycles.",
         "# TFLOP/s(mfma) = SQ_INSTS_MFMA x 32768 FLOP / launch time (counts the padded tiles: an upper bound of the algorithmic rate).",
         "# wait = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES: share of a resident wave's cycles spent waiting on an instruction counter.",
         "%-50s %9s %5s %9s %11s %9s %6s %9s" % ("kernel", "grid", "calls", "avg_us", "mfma_insts", "TFLOP/s", "wait", "mfma_busy")]
    rows = []
    for k, e in agg.items():
        if not k[0].startswith(("igemm", "wgrad_kernel")) or not e["_n"]:
            continue
        n = e["_n"]
        rows.append((e["_t"], k, n, e["_t"] / n / 1e3, e["SQ_INSTS_MFMA"] / n, e["SQ_INSTS_MFMA"] * 32768 / (e["_t"] * 1e-9) / 1e12,
                     e["SQ_WAIT_INST_ANY"] / max(e["SQ_WAVE_CYCLES"], 1), e["SQ_VALU_MFMA_BUSY_CYCLES"] / max(32 * e["SQ_BUSY_CYCLES"], 1)))
    for t, k, n, us, mi, tf, wa, mb in sorted(rows, reverse=True):
        L.append("%-50s %9d %5d %9.1f %11.0f %9.0f %6.2f %9.3f" % (k[0][:50], k[1], n, us, mi, tf, wa, mb))
    ig = [r for r in rows if r[1][0].startswith("igemm")]
    num = sum(agg[r[1]]["SQ_VALU_MFMA_BUSY_CYCLES"] for r in ig); den = sum(32 * agg[r[1]]["SQ_BUSY_CYCLES"] for r in ig)
    L.append("")
    L.append("all igemm launches of the step: mfma_busy %.3f (time-weighted)" % (num / max(den, 1)))
    open(os.path.join(PROFILES, "mfma_busy_%s.txt" % workload), "w").write("\n".join(L) + "\n")
    print("\n".join(L[9:]))


if __name__ == "__main__":
    cmd, args = sys.argv[1], sys.argv[2:]
    if cmd == "trace":
        trace(args[0], args[1], args[2], int(args[3]) if len(args) > 3 else 2)
    elif cmd == "traffic":
        traffic(args[0], args[1])
    elif cmd == "mfma":
        mfma(args[0], args[1], args[2])
    else:
        sys.exit(__doc__)
