"""Turn rocprofv3 csv output of `bench.py --case <case>` runs into the short summaries under profiles/.

    python -m paper_2410_07590_amd.profile_summary <dir> [--out profiles]

<dir> holds one folder per run, named <case>.<kind>:

    <case>.trace   rocprofv3 --kernel-trace --stats --output-format csv -d <dir>/<case>.trace -o out -- python3 bench.py --case <case> --iters 12
    <case>.fetch   rocprofv3 --pmc FETCH_SIZE       --output-format csv -d <dir>/<case>.fetch -o out -- python3 bench.py --case <case> --iters 5
    <case>.write   rocprofv3 --pmc WRITE_SIZE       --output-format csv -d <dir>/<case>.write -o out -- python3 bench.py --case <case> --iters 5
    <case>.sq      rocprofv3 --pmc SQ_INSTS_MFMA SQ_INSTS_VALU SQ_VALU_MFMA_BUSY_CYCLES SQ_VALU_MFMA_COEXEC_CYCLES SQ_BUSY_CYCLES
                             SQ_WAIT_INST_LDS SQ_WAVE_CYCLES SQ_ACTIVE_INST_VALU --output-format csv -d <dir>/<case>.sq -o out
                             -- python3 bench.py --case <case> --iters 5

(each from /tmp with TMPDIR=/tmp, one run per counter set).  `copy.fetch` / `copy.write` calibrate the byte counters
on a 256 MiB device copy.  Written: kernel_trace_by_workload.md, hbm_traffic_pmc.md, mfma_utilisation_pmc.md and
traffic.json (HBM bytes per call keyed the way bench.py keys its roofline rows, with the commit and the digest of
the kernel sources they were measured on; bench.py reports them only while that digest still matches).

Only launches of this library's kernels are kept; the first launch of every kernel in a run is dropped as warm-up.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re
import subprocess
import sys

OUR_KERNELS = ("assemble_kernel", "append_kernel", "prefix_attn_kernel", "combine_kernel", "short_attn_kernel",
               "blockdiag_attn_kernel", "gather_attn_kernel", "rope_table_kernel", "rope_rows_kernel", "linear_kernel",
               "linear_combine_kernel", "mfma_loop_probe_kernel", "fill_kernel")
COPY_KIB = 262144.0   # bench.py --case copy moves 256 MiB each way

# case -> [(kernel-name filter or None for "every kernel of the run", bench.py row key)]
BENCH_KEYS = {
    "attn2": [(None, "tr_prefill_attn@qwen2-7b-8x512-q64")],
    "assemble2": [(None, "tr_kv_assemble@qwen2-7b-8x512-q64")],
    "asmapp2": [(None, "tr_kv_assemble_append@qwen2-7b-8x512-q64")],
    "attn4": [(None, "tr_prefill_attn@llama3-8b-32x1024-q256")],
    "assemble4": [(None, "tr_kv_assemble@llama3-8b-32x1024-q256")],
    "asmapp4": [(None, "tr_kv_assemble_append@llama3-8b-32x1024-q256")],
    "raw4": [(None, "tr_kv_assemble_raw@llama3-8b-32x1024-q256")],
    "batched3": [(("assemble_kernel",), "tr_kv_assemble_batched@batched-serving-16req"),
                 (("prefix_attn_kernel", "combine_kernel"), "tr_prefill_attn_batched@batched-serving-16req")],
    "offline5": [(None, "tr_chunk_prefill_attn@offline-64x512")],
    "sequence4": [(None, "tr_sequence_prefill_attn@32x1024-chunks-plus-256-query-llama3-8b")],
    "decode2": [(None, "tr_decode_attn@decode-64x4096-qwen2-7b")],
    "shortq": [(None, "tr_prefill_attn@short-query-16-tokens-over-12288-rows-qwen2-7b")],
    "shortq16": [(None, "tr_prefill_attn_batched@short-query-16req-x-16-tokens-over-12288-rows-qwen2-7b")],
    "linear2": [(None, "tr_linear@qwen2-7b-output-projection-64-tokens")],
    "linearqkv2": [(None, "tr_linear@qwen2-7b-qkv-projection-64-tokens")],
}
SQ_COUNTERS = ["SQ_INSTS_MFMA", "SQ_INSTS_VALU", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_VALU_MFMA_COEXEC_CYCLES", "SQ_BUSY_CYCLES",
               "SQ_WAIT_INST_LDS", "SQ_WAVE_CYCLES", "SQ_ACTIVE_INST_VALU"]
SIMDS = 256 * 4


def short_name(full):
    """`void (anonymous namespace)::prefix_attn_kernel<128, 8, 4, false, 0>(Args)` -> `prefix_attn_kernel<128, 8, 4, false, 0>`"""
    s = re.sub(r"^void\s+", "", full)
    s = s.replace("(anonymous namespace)::", "")
    depth = 0
    for i, ch in enumerate(s):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return s[:i]
    return s


def ours(name):
    return name.startswith(OUR_KERNELS)


def read_csv(folder, pattern):
    rows = []
    for f in sorted(glob.glob(os.path.join(folder, "**", pattern), recursive=True)):
        with open(f, newline="") as fh:
            rows += list(csv.DictReader(fh))
    return rows


def trace_table(folder):
    """kernel -> dict(n, avg_us, min_us, max_us, vgpr, lds, scratch, grid, wg), first launch of each kernel dropped."""
    per = collections.OrderedDict()
    for r in sorted(read_csv(folder, "*kernel_trace.csv"), key=lambda r: int(r["Start_Timestamp"])):
        name = short_name(r["Kernel_Name"])
        if not ours(name):
            continue
        d = per.setdefault(name, {"t": [], "vgpr": r["VGPR_Count"], "agpr": r["Accum_VGPR_Count"], "lds": r["LDS_Block_Size"],
                                  "scratch": r["Scratch_Size"], "grid": set(), "wg": r["Workgroup_Size_X"]})
        d["t"].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
        d["grid"].add(int(r["Grid_Size_X"]) // max(1, int(r["Workgroup_Size_X"])))
    out = collections.OrderedDict()
    for name, d in per.items():
        t = d["t"][1:] if len(d["t"]) > 1 else d["t"]
        out[name] = dict(n=len(t), avg=sum(t) / len(t), min=min(t), max=max(t), vgpr=d["vgpr"], agpr=d["agpr"], lds=d["lds"],
                         scratch=d["scratch"], grid="/".join(str(g) for g in sorted(d["grid"])), wg=d["wg"])
    return out


def counter_table(folder):
    """kernel -> counter -> mean per launch (rows of one dispatch summed first), first launch of each kernel dropped."""
    per = collections.OrderedDict()
    for r in read_csv(folder, "*counter_collection.csv"):
        name = short_name(r["Kernel_Name"])
        if not (ours(name) or name.startswith("__amd_rocclr_copyBuffer") or "copy" in name.lower()):
            continue
        d = per.setdefault(name, collections.OrderedDict())
        key = (int(r["Dispatch_Id"]), r["Counter_Name"])
        d[key] = d.get(key, 0.0) + float(r["Counter_Value"])
    out = collections.OrderedDict()
    for name, d in per.items():
        ids = sorted({k[0] for k in d})
        keep = set(ids[1:] if len(ids) > 1 else ids)
        acc = collections.defaultdict(list)
        for (disp, ctr), v in d.items():
            if disp in keep:
                acc[ctr].append(v)
        out[name] = {c: sum(v) / len(v) for c, v in acc.items()}
        out[name]["_launches"] = len(keep)
    return out


TRACE_ITERS, PMC_ITERS = 12, 5   # the --iters of the runs listed above


def per_call(launches, iters):
    """Launches of a kernel per library call; 0 for a kernel that only the set-up of the case launched."""
    return launches // iters


def git_commit():
    try:
        here = os.path.dirname(os.path.abspath(__file__))
        out = subprocess.run(["git", "-C", here, "rev-parse", "--short", "HEAD"], capture_output=True, text=True)
        dirty = subprocess.run(["git", "-C", here, "status", "--porcelain", "--", "csrc"], capture_output=True, text=True)
        return out.stdout.strip() + ("+local changes to csrc" if dirty.stdout.strip() else "")
    except OSError:
        return "unknown"


def source_digest():
    import hashlib
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
    h = hashlib.sha256()
    for name in sorted(f for f in os.listdir(csrc) if f.endswith((".hip", ".h"))):
        h.update(name.encode())
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("root")
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", "profiles"))
    args = ap.parse_args()
    runs = collections.defaultdict(dict)
    for d in sorted(os.listdir(args.root)):
        if "." in d and os.path.isdir(os.path.join(args.root, d)):
            case, kind = d.rsplit(".", 1)
            runs[case][kind] = os.path.join(args.root, d)
    commit, digest = git_commit(), source_digest()
    stamp = "Kernels as of commit %s (sha256 of the kernel sources %s...).\n" % (commit, digest[:16])
    docline = __doc__.split("<dir> holds")[1].split("(each from")[0]

    # ---------------------------------------------------------------- kernel trace
    lines = ["# Kernel durations, one workload per trace\n", stamp,
             "Each block is one run of `rocprofv3 --kernel-trace --stats --output-format csv -d <dir>/<case>.trace -o out -- "
             "python3 bench.py --case <case> --iters 12` (from /tmp, TMPDIR=/tmp), summarised by "
             "`python -m paper_2410_07590_amd.profile_summary <dir>`; the first launch of each kernel is dropped.  "
             "us = End_Timestamp - Start_Timestamp of the dispatch; `call us` = sum over the kernels of one library call; a kernel "
             "marked set-up was launched by the preparation of the case only (it fills the cache the timed kernel reads).\n"]
    traces = {}
    for case in sorted(runs):
        if "trace" not in runs[case]:
            continue
        t = trace_table(runs[case]["trace"])
        if not t:
            continue
        traces[case] = t
        mult = {name: per_call(d["n"] + 1, TRACE_ITERS) for name, d in t.items()}
        lines.append("\n## %s\n" % case)
        lines.append("| kernel | launches | per call | avg us | min us | max us | workgroups x threads | VGPR+AGPR | static LDS | scratch |")
        lines.append("|---|---|---|---|---|---|---|---|---|---|")
        total = 0.0
        for name, d in t.items():
            total += d["avg"] * mult[name]
            lines.append("| %s | %d | %s | %.2f | %.2f | %.2f | %s x %s | %s+%s | %s | %s |" % (
                name, d["n"], mult[name] or "set-up", d["avg"], d["min"], d["max"], d["grid"], d["wg"], d["vgpr"], d["agpr"], d["lds"], d["scratch"]))
        lines.append("\ncall us (sum of avg x launches per call): %.2f" % total)
    write(args.out, "kernel_trace_by_workload.md", lines)

    # ---------------------------------------------------------------- HBM traffic
    factor = {"FETCH_SIZE": None, "WRITE_SIZE": None}
    for kind, ctr in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        if "copy" in runs and kind in runs["copy"]:
            ct = counter_table(runs["copy"][kind])
            vals = [v[ctr] for v in ct.values() if ctr in v and v[ctr] > 0]
            if vals:
                factor[ctr] = (COPY_KIB / max(vals), max(vals))
    lines = ["# HBM traffic per launch from rocprofv3 counters\n", stamp,
             "Runs (from /tmp, TMPDIR=/tmp; one counter per run):\n",
             "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir>/<case>.fetch -o out -- python3 bench.py --case <case> --iters 5",
             "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir>/<case>.write -o out -- python3 bench.py --case <case> --iters 5\n",
             "summarised by `python -m paper_2410_07590_amd.profile_summary <dir>`.  Calibration: `--case copy` is a 256 MiB "
             "device-to-device copy (262144 KiB read, 262144 KiB written)."]
    for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
        if factor[ctr]:
            lines.append("%s read %.1f per copy launch -> factor %.4f." % (ctr, factor[ctr][1], factor[ctr][0]))
    lines.append("Scaled KiB = counter x factor; mean over the launches after the first of each run.\n")
    lines.append("| case | kernel | per call | FETCH_SIZE | WRITE_SIZE | read MiB | written MiB | total MiB |")
    lines.append("|---|---|---|---|---|---|---|---|")
    traffic = {}
    ff = factor["FETCH_SIZE"][0] if factor["FETCH_SIZE"] else None
    wf = factor["WRITE_SIZE"][0] if factor["WRITE_SIZE"] else None
    for case in sorted(runs):
        if case == "copy" or "fetch" not in runs[case] or "write" not in runs[case] or ff is None or wf is None:
            continue
        fe, wr = counter_table(runs[case]["fetch"]), counter_table(runs[case]["write"])
        sums = collections.defaultdict(float)
        for name in fe:
            if name not in wr or not ours(name):
                continue
            mult = per_call(fe[name]["_launches"] + 1, PMC_ITERS)
            if mult == 0:
                continue   # launched by the set-up of the case only
            f_k, w_k = fe[name].get("FETCH_SIZE", 0.0), wr[name].get("WRITE_SIZE", 0.0)
            rd, wt = f_k * ff / 1024, w_k * wf / 1024
            lines.append("| %s | %s | %d | %.1f | %.1f | %.2f | %.2f | %.2f |" % (case, name, mult, f_k, w_k, rd, wt, rd + wt))
            for filt, key in BENCH_KEYS.get(case, []):
                if filt is None or name.startswith(filt):
                    sums[key] += (rd + wt) * mult * (1 << 20)
        for key, v in sums.items():
            traffic[key] = int(round(v))
    lines.append("\nBytes per library call (kernels of the call summed), as `bench.py` reports them in `traffic`:\n")
    for key, v in sorted(traffic.items()):
        lines.append("    %-90s %14d  (%.2f MiB)" % (key, v, v / (1 << 20)))
    write(args.out, "hbm_traffic_pmc.md", lines)
    if traffic:
        with open(os.path.join(args.out, "traffic.json"), "w") as f:
            json.dump({"commit": commit, "csrc_sha256": digest, "unit": "HBM bytes per library call (FETCH_SIZE + WRITE_SIZE, calibrated)",
                       "bytes_per_launch": traffic}, f, indent=1, sort_keys=True)
            f.write("\n")

    # ---------------------------------------------------------------- MFMA utilisation
    lines = ["# Matrix-unit utilisation of the attention kernels from rocprofv3 counters\n", stamp,
             "Runs (from /tmp, TMPDIR=/tmp):\n",
             "    rocprofv3 --pmc %s --output-format csv -d <dir>/<case>.sq -o out -- python3 bench.py --case <case> --iters 5\n" % " ".join(SQ_COUNTERS),
             "summarised by `python -m paper_2410_07590_amd.profile_summary <dir>`; per launch, mean over the launches after the "
             "first; kernel time from the matching `<case>.trace` run.\n",
             "Reading the counters: SQ_INSTS_VALU counts every vector instruction a wave issues, matrix instructions included, so "
             "`VALU per MFMA` = (SQ_INSTS_VALU - SQ_INSTS_MFMA) / SQ_INSTS_MFMA.  One v_mfma_f32_32x32x16_bf16 occupies its SIMD's "
             "matrix unit for 32 cycles (8 passes of 4; 32768 flops / 32 cycles x 1024 SIMDs x 2.4 GHz is the published 2.5 PFLOP/s), "
             "and SQ_VALU_MFMA_BUSY_CYCLES sums those busy cycles over the chip's 1024 SIMDs; `MFMA busy` = that sum / (kernel time x "
             "clock x 1024).  The clock is not fixed (it follows power), so the share is given for 2.4 GHz, the published peak "
             "clock, and is a lower bound on the share of the cycles the chip really ran.  SQ_BUSY_CYCLES, SQ_WAIT_INST_LDS, "
             "SQ_WAVE_CYCLES and SQ_ACTIVE_INST_VALU are reported by the profiler in units of 4 cycles.\n"]
    lines.append("| case | kernel | us | " + " | ".join(c.replace("SQ_", "") for c in SQ_COUNTERS) + " | VALU per MFMA | MFMA busy @2.4 GHz | MFMA flops / us (TFLOP/s) |")
    lines.append("|---|---|---|" + "---|" * (len(SQ_COUNTERS) + 3))
    for case in sorted(runs):
        if "sq" not in runs[case]:
            continue
        ct = counter_table(runs[case]["sq"])
        for name, v in ct.items():
            if not ours(name) or v.get("SQ_INSTS_MFMA", 0) <= 0:
                continue
            us = traces.get(case, {}).get(name, {}).get("avg")
            mfma, valu = v["SQ_INSTS_MFMA"], v.get("SQ_INSTS_VALU", 0.0)
            busy = v.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0)
            cells = ["%.0f" % v.get(c, float("nan")) for c in SQ_COUNTERS]
            share = "%.3f" % (busy / (us * 1e-6 * 2.4e9 * SIMDS)) if us else "n/a"
            rate = "%.0f" % (mfma * 32768.0 / (us * 1e-6) / 1e12) if us else "n/a"
            lines.append("| %s | %s | %s | %s | %.2f | %s | %s |" % (case, name, "%.2f" % us if us else "n/a", " | ".join(cells),
                                                                  (valu - mfma) / mfma, share, rate))
    write(args.out, "mfma_utilisation_pmc.md", lines)


def write(out_dir, name, lines):
    os.makedirs(out_dir, exist_ok=True)
    with open(os.path.join(out_dir, name), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", os.path.join(out_dir, name))


if __name__ == "__main__":
    main()
