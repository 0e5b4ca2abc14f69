"""Condenses rocprofv3 CSV output of `bench.py` runs into the short text summary that is tracked under profiles/
and that bench.py reads its per-block instruction and traffic counts from.

    python -m paper_2603_11021_amd.profile_summary --trace DIR --sq DIR --fetch DIR --write DIR \
        --blocks-per-step 9103360 --launches-per-step 4 --kernel matmul_kernel --out profiles/NAME.txt

Each DIR holds the CSV files of one rocprofv3 run (`--output-format csv`) of the SAME bench.py command:
  --trace   rocprofv3 --kernel-trace --stats          -> *_kernel_trace.csv   (durations)
  --sq      rocprofv3 --pmc SQ_WAVES SQ_INSTS_VALU SQ_INSTS_LDS SQ_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_LDS_IDX_ACTIVE
                          SQ_LDS_BANK_CONFLICT SQ_THREAD_CYCLES_VALU   -> *_counter_collection.csv
            (matrix-core kernels: SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_MFMA in place of the last two SQ_ACTIVE/THREAD counters)
  --fetch   rocprofv3 --pmc FETCH_SIZE                                  -> *_counter_collection.csv
  --write   rocprofv3 --pmc WRITE_SIZE                                  -> *_counter_collection.csv
Only dispatches whose kernel name contains --kernel are counted; a step is --launches-per-step consecutive ones.
HBM bytes: FETCH_SIZE / WRITE_SIZE are scaled by what the same counters read for the plain 1 GiB device copies that
bench.py runs for its copy-bandwidth figure (the largest copyBuffer dispatches of the same run; the 256 MiB copies of
`bench.py --calib-copy` give the same factors).  Any of the four runs may be omitted.
"""
import argparse
import collections
import csv
import glob
import os


def _rows(directory, suffix):
    out = []
    for f in sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True)):
        with open(f, newline="") as fh:
            out.extend(csv.DictReader(fh))
    return out


def _per_dispatch(rows, match):
    """counter name -> {dispatch id -> value} for kernels whose name contains `match`"""
    acc = collections.defaultdict(dict)
    for r in rows:
        if match in r["Kernel_Name"]:
            acc[r["Counter_Name"]][int(r["Dispatch_Id"])] = acc[r["Counter_Name"]].get(int(r["Dispatch_Id"]), 0.0) + float(r["Counter_Value"])
    return acc


def _copy_factor(rows, counter, copy_bytes):
    """bytes per counter unit from the plain device copies of known size (the copyBuffer dispatches with the largest count)"""
    vals = sorted(float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"] and r["Counter_Name"] == counter)
    if not vals:
        return None, 0
    top = [v for v in vals if v > 0.9 * vals[-1]]
    return copy_bytes / (sum(top) / len(top)), len(top)


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace"); ap.add_argument("--sq"); ap.add_argument("--fetch"); ap.add_argument("--write")
    ap.add_argument("--kernel", default="matmul_kernel")
    ap.add_argument("--blocks-per-step", type=int, required=True)
    ap.add_argument("--launches-per-step", type=int, required=True)
    ap.add_argument("--calib-copy-bytes", type=int, default=1 << 30)
    ap.add_argument("--title", default="")
    ap.add_argument("--command", action="append", default=[], help="the command of a run, quoted in the summary (repeatable)")
    ap.add_argument("--out", required=True)
    a = ap.parse_args(argv)
    L = a.launches_per_step
    lines = []
    put = lines.append
    put("# %s" % (a.title or "counter summary of %s" % a.kernel))
    put("# written by: python -m paper_2603_11021_amd.profile_summary --trace DIR --sq DIR --fetch DIR --write DIR --kernel %s "
        "--blocks-per-step %d --launches-per-step %d (DIR: the CSV output of the runs below)" % (a.kernel, a.blocks_per_step, L))
    for c in a.command:
        put("# run: %s" % c)
    put("# `key = number` lines are read by bench.py; a step = %d consecutive launches of %s = %d blocks of 24 weights" % (L, a.kernel, a.blocks_per_step))
    put("blocks_per_step = %d" % a.blocks_per_step)
    put("launches_per_step = %d" % L)
    if a.trace:
        rows = sorted((r for r in _rows(a.trace, "_kernel_trace.csv") if a.kernel in r["Kernel_Name"]), key=lambda r: int(r["Start_Timestamp"]))
        dur = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in rows]
        nsteps = len(dur) // L
        if nsteps:
            per_step = [sum(dur[i * L:(i + 1) * L]) for i in range(nsteps)]
            mean = sum(per_step) / nsteps
            put("trace_dispatches = %d" % len(dur))
            put("kernel_us_per_step = %.3f   # sum of the kernel durations of a step, mean over %d steps (min %.3f, max %.3f)" % (mean, nsteps, min(per_step), max(per_step)))
            put("kernel_us_per_launch = %.3f" % (mean / L))
            put("packed_GBs_kernel_time = %.1f   # 8 B per block / kernel time" % (8.0 * a.blocks_per_step / mean / 1e3))
            put("hbm_frac_kernel_time = %.4f   # of 8000 GB/s" % (8.0 * a.blocks_per_step / mean / 1e3 / 8000.0))
            by_pos = [sum(dur[i * L + k] for i in range(nsteps)) / nsteps for k in range(L)]
            put("kernel_us_by_launch_of_step = %s" % " ".join("%.2f" % v for v in by_pos))
    if a.sq:
        acc = _per_dispatch(_rows(a.sq, "_counter_collection.csv"), a.kernel)
        n = len(next(iter(acc.values()))) if acc else 0
        nsteps = n // L
        if nsteps:
            tot = {k: sum(v.values()) / nsteps for k, v in acc.items()}      # per step
            put("sq_dispatches = %d" % n)
            for k in sorted(tot):
                put("%s_per_step = %.0f" % (k, tot[k]))
            wb = a.blocks_per_step / 64.0
            if "SQ_INSTS_VALU" in tot:
                put("valu_instructions_per_block = %.1f   # SQ_INSTS_VALU per wave / 64 lanes-blocks, launch prologues included" % (tot["SQ_INSTS_VALU"] / wb))
            if "SQ_INSTS_LDS" in tot:
                put("lds_instructions_per_block = %.1f" % (tot["SQ_INSTS_LDS"] / wb))
            if "SQ_THREAD_CYCLES_VALU" in tot and "SQ_INSTS_VALU" in tot:
                put("mean_active_lanes_per_valu_instruction = %.1f   # of 64" % (tot["SQ_THREAD_CYCLES_VALU"] / tot["SQ_INSTS_VALU"]))
            if "SQ_LDS_BANK_CONFLICT" in tot and tot.get("SQ_LDS_IDX_ACTIVE"):
                put("lds_bank_conflict_share_of_lds_active = %.3f" % (tot["SQ_LDS_BANK_CONFLICT"] / tot["SQ_LDS_IDX_ACTIVE"]))
            if "SQ_BUSY_CYCLES" in tot and "SQ_INSTS_VALU" in tot:
                # SQ_BUSY_CYCLES is summed over the 32 shader engines; one VALU instruction occupies one of 1024 SIMDs for 4 cycles
                cyc = tot["SQ_BUSY_CYCLES"] / 32.0
                put("valu_issue_share_of_busy_cycles = %.3f   # SQ_INSTS_VALU x 4 / 1024 SIMDs against SQ_BUSY_CYCLES / 32" % (tot["SQ_INSTS_VALU"] * 4.0 / 1024.0 / cyc))
                if "SQ_LDS_IDX_ACTIVE" in tot:
                    put("lds_active_share_of_busy_cycles = %.3f   # SQ_LDS_IDX_ACTIVE / 256 CUs" % (tot["SQ_LDS_IDX_ACTIVE"] / 256.0 / cyc))
                if "SQ_VALU_MFMA_BUSY_CYCLES" in tot:
                    put("mfma_busy_share_of_busy_cycles = %.3f   # SQ_VALU_MFMA_BUSY_CYCLES / 1024 SIMDs" % (tot["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024.0 / cyc))
            if "SQ_INSTS_MFMA" in tot and tot.get("SQ_VALU_MFMA_BUSY_CYCLES"):
                put("mfma_busy_cycles_per_mfma_instruction = %.1f" % (tot["SQ_VALU_MFMA_BUSY_CYCLES"] / tot["SQ_INSTS_MFMA"]))
    traffic = 0.0
    have = 0
    for what, d, ctr in (("fetch", a.fetch, "FETCH_SIZE"), ("write", a.write, "WRITE_SIZE")):
        if not d:
            continue
        rows = _rows(d, "_counter_collection.csv")
        factor, ncopies = _copy_factor(rows, ctr, a.calib_copy_bytes)
        acc = _per_dispatch(rows, a.kernel).get(ctr, {})
        nsteps = len(acc) // L
        if factor is None or not nsteps:
            continue
        per_step = sum(acc.values()) / nsteps
        put("%s_counter_per_step = %.1f" % (ctr, per_step))
        put("%s_bytes_per_counter_unit = %.2f   # from %d plain copies of %d bytes" % (ctr, factor, ncopies, a.calib_copy_bytes))
        put("hbm_%s_bytes_per_step = %.0f" % (what, per_step * factor))
        traffic += per_step * factor
        have += 1
    if have == 2:
        put("hbm_traffic_bytes_per_step = %.0f" % traffic)
        put("hbm_traffic_over_algorithmic_bytes = %.3f" % (traffic / (8.0 * a.blocks_per_step)))
    with open(a.out, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
