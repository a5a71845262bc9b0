"""Turn the raw output of rocprofv3 runs of `bench.py --workload <name>` into the short text summary that is kept
under profiles/ (the raw databases and CSV files stay where the profiler wrote them).

    python3 -m paper_2603_24239_amd.profile_summary <workload> <dir> [extra bench.py options ...]

<dir> holds what the four profiler runs of the summary's own command lines wrote:
    <dir>/kt     rocprofv3 --kernel-trace --stats --output-format csv ...
    <dir>/pmcF   rocprofv3 --pmc FETCH_SIZE ...        (with --calibrate-copy)
    <dir>/pmcW   rocprofv3 --pmc WRITE_SIZE ...        (with --calibrate-copy)
    <dir>/pmcSQ  rocprofv3 --pmc SQ_WAVES SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_SMEM SQ_WAIT_INST_ANY SQ_ACTIVE_INST_ANY ...
    <dir>/bench.json   the JSON line of the same bench.py command run without a profiler
(pmcSQ is optional).  Writes profiles/dvm_vm_kernel_<workload>.md and prints it.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SQ = ["SQ_WAVES", "SQ_BUSY_CU_CYCLES", "SQ_WAVE_CYCLES", "SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_SMEM", "SQ_WAIT_INST_ANY",
      "SQ_ACTIVE_INST_ANY"]


def _short(name: str, n: int = 78) -> str:
    return (name[:n] + "...") if len(name) > n else name


def _counter(dirname: str, counter: str):
    """per dispatch values of one counter: {'vm': [...], 'copy': [...], 'dvm_copy': [...]} (a dispatch's value is the sum over
    the rows rocprofv3 wrote for it: one per shader engine / channel where the counter is split)."""
    per = collections.defaultdict(float)
    kind = {}
    for f in glob.glob(os.path.join(dirname, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] != counter:
                continue
            key = (f, r["Dispatch_Id"])
            per[key] += float(r["Counter_Value"])
            k = r["Kernel_Name"]
            kind[key] = "vm" if "dvm_vm_kernel" in k else ("copy" if "copyBuffer" in k else ("dvm_copy" if "dvm_copy_tiles" in k else "x"))
    out = collections.defaultdict(list)
    for key, v in per.items():
        out[kind[key]].append(v)
    return out


def main() -> int:
    if len(sys.argv) < 3:
        print(__doc__)
        return 2
    W, O = sys.argv[1], sys.argv[2]
    extra = (" " + " ".join(sys.argv[3:])) if len(sys.argv) > 3 else ""
    bench = json.loads(open(os.path.join(O, "bench.json")).read().strip().splitlines()[-1])
    pc = bench["per_config"][W]
    roof = bench["roofline"]
    cmd = f"python3 bench.py --workload {W}{extra}"
    out = []
    out.append(f"# rocprofv3 summaries: interpreter kernel, `bench.py --workload {W}{extra}`\n")
    out.append(f"Workload: {pc['workload']}; {pc['instances']} instances, {pc['instances_per_launch']} per launch, "
               f"{pc['launches_per_pass']} launches per pass over the stream.")
    out.append("All commands run from the repository root on the MI355X box; raw output stays outside the repository.\n")

    # ---- kernel trace
    ks = glob.glob(os.path.join(O, "kt", "**", "*kernel_stats.csv"), recursive=True)[0]
    rows = list(csv.DictReader(open(ks)))
    out.append("## Kernel trace\n")
    out.append(f"    rocprofv3 --kernel-trace --stats --output-format csv -d <dir>/kt -o kt -- {cmd} --steps 2 --warmup 1 --no-cpu-baseline --skip-unstacked\n")
    out.append("| kernel | calls | total ms | avg us | min us | max us | % of GPU time |\n|---|---|---|---|---|---|---|")
    vm = [r for r in rows if "dvm_vm_kernel" in r["Name"]]
    for r in vm + [r for r in rows if "dvm_vm_kernel" not in r["Name"]][:3]:
        out.append("| `%s` | %s | %.2f | %.2f | %.2f | %.2f | %s |" % (_short(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e6,
                                                                    float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
                                                                    r["Percentage"]))
    tot_ns = sum(float(r["TotalDurationNs"]) for r in vm)
    calls = sum(int(r["Calls"]) for r in vm)
    avg_us = tot_ns / calls / 1e3
    bpl = roof["bytes_per_launch"]
    out.append("")
    out.append("Interpreter launches (all instantiations together): %d, average %.2f us.  Algorithmic bytes per launch (mean over the launches;"
               % (calls, avg_us))
    out.append("one read of every input element and one write of every output element): %.1f MB -> %.2f TB/s, %.1f %% of the 8 TB/s HBM peak."
               % (bpl / 1e6, bpl / avg_us / 1e6, 100 * bpl / avg_us / 1e6 / 8))
    out.append("The same command without a profiler (HIP events on the launch stream) reported avg_launch_ms %.5f (%.2f TB/s, frac %.4f),"
               % (roof["avg_launch_ms"], roof["achieved"] / 1e3, roof["frac"]))
    out.append("whole-job value %.1f GB/s (encode and launch overhead included), %.1f %% of the library's own copy kernel (%.0f GB/s)."
               % (bench["value"], roof["pct_of_copy_ceiling"], bench["copy_ceiling"]["GBps"]))
    out.append("The other kernels are torch's input generation and the copy-ceiling measurement, outside the timed region.\n")

    # ---- HBM traffic
    f_all, w_all = _counter(os.path.join(O, "pmcF"), "FETCH_SIZE"), _counter(os.path.join(O, "pmcW"), "WRITE_SIZE")
    if f_all["vm"] and w_all["vm"]:
        fcp, wcp = sorted(f_all["copy"])[-3:], sorted(w_all["copy"])[-3:]      # the three 256 MiB calibration copies are the largest copies
        KIB = 256 * 1024
        ff, wf = KIB / (sum(fcp) / len(fcp)), KIB / (sum(wcp) / len(wcp))
        fvm, wvm = f_all["vm"], w_all["vm"]
        fb, wb = sum(fvm) / len(fvm) * ff * 1024, sum(wvm) / len(wvm) * wf * 1024
        out.append("## HBM traffic counters\n")
        out.append(f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir>/pmcF -o p -- {cmd} --steps 1 --warmup 0 --no-cpu-baseline --skip-unstacked --calibrate-copy")
        out.append(f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir>/pmcW -o p -- {cmd} --steps 1 --warmup 0 --no-cpu-baseline --skip-unstacked --calibrate-copy\n")
        out.append("`--calibrate-copy` appends three plain 256 MiB device-to-device copies (`__amd_rocclr_copyBuffer`): a kernel that is known to")
        out.append("read 262144 KiB and write 262144 KiB; its counter readings give the factor from counter units to KiB.\n")
        out.append("| counter | copy kernel reads (mean of %d) | factor to KiB | interpreter kernel (mean of %d launches) | scaled bytes per launch |\n|---|---|---|---|---|"
                   % (len(fcp), len(fvm)))
        out.append("| FETCH_SIZE | %.1f | %.5f | %.1f | %.0f |" % (sum(fcp) / len(fcp), ff, sum(fvm) / len(fvm), fb))
        out.append("| WRITE_SIZE | %.1f | %.5f | %.1f | %.0f |" % (sum(wcp) / len(wcp), wf, sum(wvm) / len(wvm), wb))
        out.append("")
        out.append("Read + written per launch: %.0f bytes against %d algorithmic bytes." % (fb + wb, bpl))
        out.append("")
        out.append("traffic_bytes_per_launch: %d" % round(fb + wb))
        out.append("traffic_ratio: %.4f" % ((fb + wb) / bpl))
        out.append("")

    # ---- SQ counters
    sq_dir = os.path.join(O, "pmcSQ")
    if os.path.isdir(sq_dir):
        vals = {c: _counter(sq_dir, c)["vm"] for c in SQ}
        if vals["SQ_WAVES"]:
            n = len(vals["SQ_WAVES"])
            tot = {c: sum(v) for c, v in vals.items()}
            out.append("## Shader-sequencer counters (issue limits)\n")
            out.append(f"    rocprofv3 --pmc {' '.join(SQ)} --output-format csv -d <dir>/pmcSQ -o p -- {cmd} --steps 1 --warmup 0 --no-cpu-baseline --skip-unstacked\n")
            out.append("Sums over the %d interpreter launches of one pass (SQ_WAVE_CYCLES, SQ_WAIT_INST_ANY and SQ_ACTIVE_INST_ANY count in units of four cycles).\n" % n)
            out.append("| counter | total | per wave |\n|---|---|---|")
            for c in SQ:
                out.append("| %s | %.4g | %.1f |" % (c, tot[c], tot[c] / tot["SQ_WAVES"]))
            out.append("")
            wc = tot["SQ_WAVE_CYCLES"]
            out.append("Per wave: %.0f VALU, %.0f SALU and %.0f SMEM instructions; a wave is resident for %.0f cycles, of which it waits for an"
                       % (tot["SQ_INSTS_VALU"] / tot["SQ_WAVES"], tot["SQ_INSTS_SALU"] / tot["SQ_WAVES"], tot["SQ_INSTS_SMEM"] / tot["SQ_WAVES"],
                          4 * wc / tot["SQ_WAVES"]))
            out.append("instruction to complete (memory, mostly) %.0f %% and issues %.0f %% of the time.  Scalar instructions per vector instruction: %.2f."
                       % (100 * tot["SQ_WAIT_INST_ANY"] / wc, 100 * tot["SQ_ACTIVE_INST_ANY"] / wc, tot["SQ_INSTS_SALU"] / max(1.0, tot["SQ_INSTS_VALU"])))
            out.append("Algorithmic bytes per scalar instruction: %.1f." % (bpl * n / max(1.0, tot["SQ_INSTS_SALU"])))
            out.append("")
    text = "\n".join(out) + "\n"
    path = os.path.join(ROOT, "profiles", f"dvm_vm_kernel_{W}.md")
    with open(path, "w") as f:
        f.write(text)
    print(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
