#!/usr/bin/env python3
"""Turns the raw output of rocprofv3 runs of bench.py into the tracked summaries under profiles/.

Reads a directory of rocprofv3 CSV output (default gpurun_out/prof) laid out as

    copy_fetch/ copy_write/                 --pmc FETCH_SIZE / WRITE_SIZE  -- python3 bench.py --calibrate-copy
    trace_<workload>/t_kernel_stats.csv     --kernel-trace --stats         -- python3 bench.py --workload W --only --steps 200 --cpu-seconds 0
    <workload>_fetch/ <workload>_write/     --pmc FETCH_SIZE / WRITE_SIZE  -- python3 bench.py --workload W --only --steps 5 --warmup 2 --cpu-seconds 0
    <workload>_sq/                          --pmc <matrix-core and LDS counters>, same program

(every counter run also carries --kernel-trace --output-format csv -d <dir> -o p) and writes

    profiles/<kernel>__<workload>.txt       the figures, with the full command of every run
    profiles/traffic.json                   HBM bytes read and written per launch of each workload's
                                            decode kernel, scaled by the copy calibration; bench.py
                                            reports these as roofline.traffic

Usage: python3 profile_summary.py [--raw gpurun_out/prof] [workload ...]
"""
import argparse
import collections
import csv
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

SQ_COUNTERS = ("SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F32 "
               "SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE GRBM_GUI_ACTIVE")
KERNELS = {"split_decode_kernel": "merge_kernel", "mla_decode_kernel": "mla_merge_kernel"}


def short_name(kernel_name):
    for k in ("split_decode_kernel", "mla_decode_kernel", "mla_merge_kernel", "merge_kernel", "copyBuffer"):
        if k in kernel_name:
            return k
    return None


def counters(raw, run):
    """{(kernel, counter): mean value per launch}"""
    agg = collections.defaultdict(list)
    with open(os.path.join(raw, run, "p_counter_collection.csv")) as fh:
        for r in csv.DictReader(fh):
            short = short_name(r["Kernel_Name"])
            if short:
                agg[(short, r["Counter_Name"])].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in agg.items()}


def kernel_stats(raw, run):
    out = {}
    with open(os.path.join(raw, run, "t_kernel_stats.csv")) as fh:
        for r in csv.DictReader(fh):
            short = short_name(r["Name"])
            if short:
                out[short] = r
                out[short + "/full"] = r["Name"]
    return out


def main():
    import workloads
    from bench import kernel_source_hash
    ap = argparse.ArgumentParser()
    ap.add_argument("--raw", default=os.path.join(ROOT, "gpurun_out", "prof"))
    ap.add_argument("workloads", nargs="*")
    args = ap.parse_args()
    raw = args.raw
    names = args.workloads or [w for w in list(workloads.CONFIG_ORDER)[1:] + sorted(workloads.MLA_CONFIGS)
                               if os.path.isdir(os.path.join(raw, "trace_" + w))]
    cf = counters(raw, "copy_fetch")[("copyBuffer", "FETCH_SIZE")]
    cw = counters(raw, "copy_write")[("copyBuffer", "WRITE_SIZE")]
    f_fetch, f_write = (1 << 20) / cf, (1 << 20) / cw          # a 1 GiB copy reads and writes 2^20 KiB
    cal = """Calibration of the two HBM counters against a plain copy of known size (same rocprofv3 options; the program is
python3 bench.py --calibrate-copy: ten 1 GiB device-to-device copies, each reads 1 GiB and writes 1 GiB):
  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT -o p -- python3 bench.py --calibrate-copy
      FETCH_SIZE per copy = %.1f  (nominally KiB; a 1 GiB read = 1048576 KiB)  -> scale factor %.4f
  rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d OUT -o p -- python3 bench.py --calibrate-copy
      WRITE_SIZE per copy = %.1f  -> scale factor %.4f
""" % (cf, f_fetch, cw, f_write)
    traffic_path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(traffic_path) as fh:
            traffic = json.load(fh)
    except (OSError, ValueError):
        traffic = {}
    traffic.setdefault("workloads", {})
    traffic["kernel_source_hash"] = kernel_source_hash()
    traffic["unit"] = "bytes per launch of the decode kernel"
    traffic["how"] = ("rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (KiB per dispatch, one counter per run), each scaled by what "
                      "the same counter reads for a 1 GiB device copy; written by profile_summary.py")
    traffic["calibration"] = {"fetch_factor": f_fetch, "write_factor": f_write}
    for w in names:
        mla = w in workloads.MLA_CONFIGS
        kern = "mla_decode_kernel" if mla else "split_decode_kernel"
        merge = KERNELS[kern]
        cfg = workloads.MLA_CONFIGS[w] if mla else workloads.CONFIGS[w]
        st = kernel_stats(raw, "trace_" + w)
        fe, wr, sq = counters(raw, w + "_fetch"), counters(raw, w + "_write"), counters(raw, w + "_sq")
        alg = cfg.kv_bytes()
        k, m = st[kern], st[merge]
        kf, kw = fe[(kern, "FETCH_SIZE")], wr[(kern, "WRITE_SIZE")]
        mf, mw = fe[(merge, "FETCH_SIZE")], wr[(merge, "WRITE_SIZE")]
        read_b, write_b = kf * f_fetch * 1024, kw * f_write * 1024
        avg_us = float(k["AverageNs"]) / 1e3
        g = lambda c: sq[(kern, c)]                                                   # noqa: E731
        cyc = g("GRBM_GUI_ACTIVE") / 8
        full = st[kern + "/full"]
        shown = full[full.index(kern):].split("(")[0]
        prog = "python3 bench.py --workload %s --only" % w
        roof = "algorithmic K+V bytes per launch: %d -> %.0f GB/s = %.3f of the 8 TB/s HBM peak" % (alg, alg / avg_us / 1e3, alg / avg_us / 1e3 / 8000)
        if mla:
            fl = cfg.flops()
            roof = ("algorithmic flops per launch: %d -> %.0f TFLOP/s = %.3f of the 2.5 PFLOP/s bf16 matrix peak\n   "
                    "algorithmic cache bytes per launch: %d -> %.0f GB/s = %.3f of the 8 TB/s HBM peak"
                    % (fl, fl / avg_us / 1e6, fl / avg_us / 1e6 / 2500, alg, alg / avg_us / 1e3, alg / avg_us / 1e3 / 8000))
        txt = """rocprofv3 summary: %s and %s, workload %s
(one MI355X, ROCm 7.2; all commands run from /tmp with the repository's bench.py; OUT = a scratch directory)

1. Kernel durations
   rocprofv3 --kernel-trace --stats --output-format csv -d OUT -o t -- %s --steps 200 --cpu-seconds 0
   kernel                  calls   avg us    min us    max us
   %-22s  %5d  %8.1f  %8.1f  %8.1f
   %-22s  %5d  %8.1f  %8.1f  %8.1f
   %s
   (bench.py's own HIP-event figure for the decode kernel brackets the launch as well and reads a few us higher.)

2. HBM traffic per launch (one counter per run)
   rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT -o p -- %s --steps 5 --warmup 2 --cpu-seconds 0
   rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d OUT -o p -- %s --steps 5 --warmup 2 --cpu-seconds 0
   kernel                  FETCH_SIZE raw   x factor -> bytes read     WRITE_SIZE raw   x factor -> bytes written
   %-22s  %14.1f   %16.0f     %14.1f   %16.0f
   %-22s  %14.1f   %16.0f     %14.1f   %16.0f
   algorithmic cache bytes per launch: %d   -> bytes read by the decode kernel / algorithmic = %.4f,
   bytes read + written / algorithmic = %.4f

%s
3. Matrix cores and LDS (one run)
   rocprofv3 --pmc %s --kernel-trace --output-format csv -d OUT -o p -- %s --steps 5 --warmup 2 --cpu-seconds 0
   %s, mean per launch, summed over the chip:
     GRBM_GUI_ACTIVE              %14.0f   (8 XCDs: %.0f cycles per launch)
     SQ_VALU_MFMA_BUSY_CYCLES     %14.0f   -> %.1f %% of the 256 CU x 4 SIMD matrix pipes' cycles
     SQ_INSTS_VALU_MFMA_MOPS_BF16 %14.0f
     SQ_INSTS_VALU_MFMA_MOPS_F32  %14.0f
     SQ_LDS_IDX_ACTIVE            %14.0f   -> LDS busy %.1f %% of CU cycles
     SQ_LDS_BANK_CONFLICT         %14.0f   -> %.1f %% of the LDS-active cycles
     SQ_WAVE_CYCLES               %14.0f
     SQ_BUSY_CYCLES               %14.0f
""" % (shown, merge, w, prog,
       kern, int(k["Calls"]), avg_us, int(k["MinNs"]) / 1e3, int(k["MaxNs"]) / 1e3,
       merge, int(m["Calls"]), float(m["AverageNs"]) / 1e3, int(m["MinNs"]) / 1e3, int(m["MaxNs"]) / 1e3, roof,
       prog, prog, kern, kf, read_b, kw, write_b, merge, mf, mf * f_fetch * 1024, mw, mw * f_write * 1024,
       alg, read_b / alg, (read_b + write_b) / alg, cal, SQ_COUNTERS, prog, kern,
       g("GRBM_GUI_ACTIVE"), cyc, g("SQ_VALU_MFMA_BUSY_CYCLES"), 100 * g("SQ_VALU_MFMA_BUSY_CYCLES") / (cyc * 256 * 4),
       g("SQ_INSTS_VALU_MFMA_MOPS_BF16"), g("SQ_INSTS_VALU_MFMA_MOPS_F32"), g("SQ_LDS_IDX_ACTIVE"),
       100 * g("SQ_LDS_IDX_ACTIVE") / (cyc * 256), g("SQ_LDS_BANK_CONFLICT"),
       100 * g("SQ_LDS_BANK_CONFLICT") / max(g("SQ_LDS_IDX_ACTIVE"), 1.0), g("SQ_WAVE_CYCLES"), g("SQ_BUSY_CYCLES"))
        name = "%s__%s.txt" % (kern, w)
        with open(os.path.join(ROOT, "profiles", name), "w") as fh:
            fh.write(txt)
        traffic["workloads"][w] = {"kernel": kern, "bytes_read": int(read_b), "bytes_written": int(write_b),
                                   "algorithmic_bytes": int(alg), "kernel_avg_us": avg_us, "profile": "profiles/" + name}
        print(w, "avg %.1f us" % avg_us, "merge %.1f us" % (float(m["AverageNs"]) / 1e3), "read/alg %.4f" % (read_b / alg),
              "written MB %.1f" % (write_b / 1e6), "mfma busy %.1f%%" % (100 * g("SQ_VALU_MFMA_BUSY_CYCLES") / (cyc * 256 * 4)))
    with open(traffic_path, "w") as fh:
        json.dump(traffic, fh, indent=1, sort_keys=True)
        fh.write("\n")


if __name__ == "__main__":
    main()
