"""Condenses rocprofv3 output of `bench.py` runs into the short tables under profiles/ and into
bench_traffic.json (the `traffic` fields of the bench line).  Reads the CSV files rocprofv3 writes, nothing else;
no GPU is needed.

The runs it expects (from the repository root on the MI355X machine, after `cd /tmp && export TMPDIR=/tmp`; N = 2..5,
`--only` keeps the other configurations' kernels out of the run):

    rocprofv3 --kernel-trace --stats -d OUT/trace_cN -o t --output-format csv -- python3 bench.py --config N --only --no-cpu-baseline
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS \\
              SQ_WAVE_CYCLES SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS -d OUT/sq_cN -o t --output-format csv -- python3 bench.py --config N --only --no-cpu-baseline --steps 2 --warmup 1 --class-reps 2
    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum GRBM_GUI_ACTIVE -d OUT/tcc_cN -o t --output-format csv -- python3 bench.py ... (same flags)
    rocprofv3 --pmc FETCH_SIZE -d OUT/fetch_cN -o t --output-format csv -- python3 bench.py ... (same flags) --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d OUT/write_cN -o t --output-format csv -- python3 bench.py ... (same flags) --calibrate-copy

and then

    python -m paper_2503_06433_amd.profile_summary --config N --dir OUT --profiles profiles --traffic bench_traffic.json

Clock table (how far the package power limit, not the kernels, sets the GEMM rate): two runs that collect the cycle
counter together with the kernel trace, one on the bench's random data and one with `--zero-data` (same instruction
streams, data paths not toggling),

    rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES -d OUT/clk_random_cN -o t --output-format csv -- python3 bench.py --config N --only --no-cpu-baseline --no-reshard --steps 2 --warmup 1
    rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES -d OUT/clk_zero_cN -o t --output-format csv -- python3 bench.py (same flags) --zero-data

are condensed by the same command into profiles/bench_<workload>_gemm_clock.md when those two directories exist.
A yardstick next to it: the vendor library's GEMM on the same projection shapes under the same counters,

    rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES -d OUT/clk_library_cN -o t --output-format csv -- python3 bench.py --config N --library-gemm

goes to profiles/library_gemm_<workload>_clock.md when that directory exists.

The offline engine loop has a kernel trace of its own,

    rocprofv3 --kernel-trace --stats -d OUT/trace_offline -o t --output-format csv -- python3 bench.py --offline-loop > OUT/trace_offline.json

condensed by `python -m paper_2503_06433_amd.profile_summary --offline --dir OUT` into
profiles/offline_loop_c2_shape_2_layers_kernel_trace.md.

`--calibrate-copy` makes bench.py run a plain 1 GiB device-to-device copy first; FETCH_SIZE and WRITE_SIZE (KiB per
dispatch) are scaled by what they read for that copy of known size.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re
import statistics

WORKLOAD = {2: "c2_llama2_7b_layer", 3: "c3_llama2_13b_tp4", 4: "c4_llama3_70b_tp8", 5: "c5_llama3_70b_pp8_slice"}

# kernel class of the bench line <- substring of the kernel name
CLASSES = (
    ("prefill_gemms", ("gemm_mfma_stream_kernel",)),
    ("prefill_attention", ("attn_prefill_lds_kernel", "attn_prefill_mfma_kernel")),
    ("decode_attention", ("attn_decode_mfma_kernel", "attn_decode_merge_kernel")),
    ("decode_gemms", ("gemm_mfma_kernel<", "splitk_reduce_kernel")),
    ("kv_repack", ("kv_repack_kernel",)),
)


def short(name):
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"^ssk(16)?::", "", name)
    name = re.sub(r"\(.*$", "", name)
    return name[:64]


def find(directory, suffix):
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    return hits[0] if hits else None


def read_counters(directory):
    """{kernel: {counter: [value per dispatch]}} of one --pmc run."""
    path = find(directory, "counter_collection.csv")
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    if not path:
        return per
    with open(path) as f:
        for r in csv.DictReader(f):
            per[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return per


def avg(v):
    return sum(v) / len(v) if v else 0.0


def kernel_trace_tables(directory):
    stats, trace = find(directory, "kernel_stats.csv"), find(directory, "kernel_trace.csv")
    lines, durations = [], collections.defaultdict(list)
    if stats:
        lines += ["| kernel | calls | avg us | total ms | % |", "|---|---|---|---|---|"]
        with open(stats) as f:
            for r in list(csv.DictReader(f))[:18]:
                lines.append("| `%s` | %s | %.1f | %.2f | %s |" % (short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3,
                                                                 float(r["TotalDurationNs"]) / 1e6, r["Percentage"]))
    if trace:
        shapes = collections.defaultdict(list)
        with open(trace) as f:
            for r in csv.DictReader(f):
                us = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
                shapes[(short(r["Kernel_Name"]), r["Grid_Size_X"], r["Grid_Size_Y"])].append(us)
                durations[short(r["Kernel_Name"])].append(us)
        lines += ["", "Per launch shape (grid in threads; launches of 15 us and more, at least 3 of them):", "",
                  "| kernel | grid | launches | min us | median us |", "|---|---|---|---|---|"]
        for (k, gx, gy), v in sorted(shapes.items(), key=lambda kv: -sum(kv[1])):
            if len(v) >= 3 and statistics.median(v) >= 15:
                lines.append("| `%s` | %s x %s | %d | %.1f | %.1f |" % (k, gx, gy, len(v), min(v), statistics.median(v)))
    return lines, durations


def counter_table(sq, tcc, durations):
    lines = ["| kernel | launches | GPU cycles | MFMA busy | MFMA ops (bf16) | LDS conflict cycles / active LDS cycle | "
             "waiting / wave cycles | L2 hit rate |", "|---|---|---|---|---|---|---|---|"]
    rows = []
    for k in sorted(set(sq) | set(tcc)):
        gui = avg(tcc[k]["GRBM_GUI_ACTIVE"]) / 8 if k in tcc else 0.0            # summed over the 8 XCDs
        if gui < 20000:
            continue
        mf = avg(sq[k]["SQ_VALU_MFMA_BUSY_CYCLES"]) / 1024                        # summed over 256 CUs x 4 SIMDs
        req, hit = avg(tcc[k]["TCC_REQ_sum"]), avg(tcc[k]["TCC_HIT_sum"])
        act = avg(sq[k]["SQ_ACTIVE_INST_LDS"])
        wc = avg(sq[k]["SQ_WAVE_CYCLES"])
        rows.append((gui, "| `%s` | %d | %.0f | %.1f %% | %.3g | %.2f | %.2f | %s |" % (
            k, len(tcc[k]["GRBM_GUI_ACTIVE"]), gui, 100 * mf / gui if gui else 0,
            avg(sq[k]["SQ_INSTS_VALU_MFMA_MOPS_BF16"]), avg(sq[k]["SQ_LDS_BANK_CONFLICT"]) / act if act else 0,
            avg(sq[k]["SQ_WAIT_INST_ANY"]) / wc if wc else 0, ("%.1f %%" % (100 * hit / req)) if req else "-")))
    return lines + [r[1] for r in sorted(rows, key=lambda r: -r[0])]


def clock_rows(directory):
    """Per kernel of a run that has both a kernel trace and GRBM_GUI_ACTIVE / SQ_VALU_MFMA_BUSY_CYCLES per dispatch:
    [(kernel, launches, median us, median GHz, median MFMA busy %)] for launches of a millisecond and more."""
    tr_path, cc_path = find(directory, "kernel_trace.csv"), find(directory, "counter_collection.csv")
    if not tr_path or not cc_path:
        return []
    us = {}
    with open(tr_path) as f:
        for r in csv.DictReader(f):
            us[r["Dispatch_Id"]] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
    per = collections.defaultdict(dict)
    with open(cc_path) as f:
        for r in csv.DictReader(f):
            per[r["Dispatch_Id"]][r["Counter_Name"]] = float(r["Counter_Value"])
            per[r["Dispatch_Id"]]["kernel"] = short(r["Kernel_Name"])
    by_kernel = collections.defaultdict(list)
    for did, c in per.items():
        t = us.get(did, 0.0)
        if t < 1000 or "GRBM_GUI_ACTIVE" not in c:
            continue
        cycles = c["GRBM_GUI_ACTIVE"] / 8
        by_kernel[c["kernel"]].append((t, cycles / t / 1e3, 100 * c.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / 1024 / cycles))
    rows = []
    for k, v in sorted(by_kernel.items(), key=lambda kv: -sum(x[0] for x in kv[1])):
        rows.append((k, len(v), statistics.median(x[0] for x in v), statistics.median(x[1] for x in v),
                     statistics.median(x[2] for x in v)))
    return rows


def library_rows(directory):
    """The run of `bench.py --library-gemm` under the clock counters: its long launches in dispatch order come in
    groups of 7 (2 warm-up + 5 timed) per data kind (random, zeros) and shape (qkv, o, gate_up, down).
    [(data, shape, median us, median GHz, median MFMA busy %)] over the timed launches of each group."""
    tr_path, cc_path = find(directory, "kernel_trace.csv"), find(directory, "counter_collection.csv")
    if not tr_path or not cc_path:
        return []
    us = {}
    with open(tr_path) as f:
        for r in csv.DictReader(f):
            us[r["Dispatch_Id"]] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
    per = collections.defaultdict(dict)
    with open(cc_path) as f:
        for r in csv.DictReader(f):
            per[r["Dispatch_Id"]][r["Counter_Name"]] = float(r["Counter_Value"])
    long = []
    for did in sorted(per, key=int):
        c, t = per[did], us.get(did, 0.0)
        if t >= 1000 and "GRBM_GUI_ACTIVE" in c:
            cycles = c["GRBM_GUI_ACTIVE"] / 8
            long.append((t, cycles / t / 1e3, 100 * c.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / 1024 / cycles))
    if len(long) != 56:
        return []
    rows = []
    for i, (data, shape) in enumerate((dk, sh) for dk in ("random", "zeros") for sh in ("qkv", "o", "gate_up", "down")):
        g = long[7 * i + 2:7 * i + 7]
        rows.append((data, shape, statistics.median(x[0] for x in g), statistics.median(x[1] for x in g),
                     statistics.median(x[2] for x in g)))
    return rows


def traffic(fetch, write):
    """HBM-side GB per class and the per-kernel table; counters scaled by the 1 GiB calibration copy."""
    def calib(per, ctr):
        vals = [v for k, c in per.items() if "copy" in k.lower() or "elementwise" in k.lower() for v in c[ctr]]
        return max(vals) if vals else None
    cf, cw = calib(fetch, "FETCH_SIZE"), calib(write, "WRITE_SIZE")
    kib = float(1 << 20)                                      # the copy reads and writes 1 048 576 KiB
    sf = kib / cf if cf else 2.0
    sw = kib / cw if cw else 1.0
    lines = ["| kernel | launches | FETCH_SIZE avg (KiB, raw) | WRITE_SIZE avg (KiB, raw) | scaled read GB | scaled write GB |",
             "|---|---|---|---|---|---|"]
    total = {}
    for k in sorted(fetch, key=lambda k: -sum(fetch[k]["FETCH_SIZE"])):
        f, w = fetch[k]["FETCH_SIZE"], (write[k]["WRITE_SIZE"] if k in write else [])
        if not f:
            continue
        total[k] = (len(f), sum(f) * sf * 1024, sum(w) * sw * 1024 if w else 0.0)
        lines.append("| `%s` | %d | %.0f | %.0f | %.3f | %.3f |" % (k, len(f), avg(f), avg(w), avg(f) * sf * 1024 / 1e9,
                                                                   avg(w) * sw * 1024 / 1e9))
    return lines, total, (cf, cw, sf, sw)


def class_bytes(total, config):
    """Bytes per layer call (per launch for the repack) of every kernel class present."""
    def count(sub):
        return sum(v[0] for k, v in total.items() if sub in k)

    def size(subs):
        return sum(v[1] + v[2] for k, v in total.items() if any(s in k for s in subs))
    n_prefill = count("attn_prefill_lds_kernel") + count("attn_prefill_mfma_kernel")
    n_decode = count("attn_decode_mfma_kernel")
    out = {}
    for cls, subs in CLASSES:
        b = size(subs)
        if not b:
            continue
        if cls == "kv_repack" and config not in (2, 5):
            continue                    # only these two configurations time the repack (the others scatter their synthetic caches once)
        if cls == "kv_repack":          # the export of a whole batch is what bench.py times: the largest gather launches
            per = [(v[1] + v[2]) / v[0] for k, v in total.items() if "kv_repack_kernel<unsigned short, true>" in k]
            out[cls] = max(per) if per else b
        else:
            calls = n_prefill if cls.startswith("prefill") else n_decode
            if calls:
                out[cls] = b / calls
    return out, n_prefill, n_decode


def offline_summary(directory, profiles):
    lines, _ = kernel_trace_tables(os.path.join(directory, "trace_offline"))
    if not lines:
        raise SystemExit("no kernel trace under %s/trace_offline" % directory)
    runs = {}
    try:
        with open(os.path.join(directory, "trace_offline.json")) as f:
            runs = json.loads(f.read().strip().splitlines()[-1]).get("runs", {})
    except (OSError, ValueError, IndexError):
        pass
    with open(os.path.join(profiles, "offline_loop_c2_shape_2_layers_kernel_trace.md"), "w") as f:
        f.write("# Kernel trace of the offline engine loop (`bench.py --offline-loop`)\n\nCommand (from the repository root on the MI355X "
                "box, after `cd /tmp && export TMPDIR=/tmp`):\n\n    rocprofv3 --kernel-trace --stats -d OUT/trace_offline -o t --output-format csv "
                "-- python3 bench.py --offline-loop > OUT/trace_offline.json\n\nWorkload: 64 requests of 3000 prompt + 64 output tokens, two layers "
                "of the configuration-2 shape, vocabulary 2048, bf16, greedy decoding, weights reloaded at every switch; four runs (CPU store for all "
                "64 requests, the same with swap-ins in groups of 4, for 16 requests, for 4 requests), each executed twice (the first execution "
                "allocates).  All runs together; summarised by `python -m paper_2503_06433_amd.profile_summary --offline`.\n\n")
        f.write("\n".join(lines) + "\n")
        if runs:
            f.write("\nThe same command printed (under the profiler; prompt+output tokens/s, stage changes, seconds in prefill / decode / "
                    "switch issue):\n\n")
            for name, r in runs.items():
                f.write("* `%s`: %.0f tokens/s, %s switches, %.3f / %.3f / %.3f s\n" % (
                    name, r.get("tokens_per_s", 0.0), r.get("switches", "?"), r.get("prefill_s", 0.0), r.get("decode_s", 0.0), r.get("switch_s", 0.0)))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--offline", action="store_true", help="summarise OUT/trace_offline (the offline engine loop) instead of a configuration")
    ap.add_argument("--config", type=int, choices=[2, 3, 4, 5])
    ap.add_argument("--dir", required=True, help="directory that holds trace_cN, sq_cN, tcc_cN, fetch_cN, write_cN")
    ap.add_argument("--profiles", default="profiles")
    ap.add_argument("--traffic", default="bench_traffic.json")
    a = ap.parse_args()
    os.makedirs(a.profiles, exist_ok=True)
    if a.offline:
        offline_summary(a.dir, a.profiles)
        return
    if a.config is None:
        ap.error("--config N or --offline")
    n, wl = a.config, WORKLOAD[a.config]
    d = lambda kind: os.path.join(a.dir, "%s_c%d" % (kind, n))
    flags = "--config %d --only --no-cpu-baseline" % n
    short_flags = flags + " --steps 2 --warmup 1 --class-reps 2"
    os.makedirs(a.profiles, exist_ok=True)

    trace_lines, durations = kernel_trace_tables(d("trace"))
    if trace_lines:
        with open(os.path.join(a.profiles, "bench_%s_kernel_trace.md" % wl), "w") as f:
            f.write("# Kernel trace of `bench.py %s` (%s)\n\nCommand (from the repository root on the MI355X box, after "
                    "`cd /tmp && export TMPDIR=/tmp`):\n\n    rocprofv3 --kernel-trace --stats -d OUT/trace_c%d -o t --output-format csv "
                    "-- python3 bench.py %s\n\nAll passes of the run together (the timed steps, then the per-class timing passes); "
                    "summarised by `python -m paper_2503_06433_amd.profile_summary`.\n\n" % (flags, wl, n, flags))
            f.write("\n".join(trace_lines) + "\n")
    sq, tcc = read_counters(d("sq")), read_counters(d("tcc"))
    if sq or tcc:
        with open(os.path.join(a.profiles, "bench_%s_counters.md" % wl), "w") as f:
            f.write("# Hardware counters of the kernels of `bench.py %s` (%s)\n\nTwo runs (rocprofv3 does not split counters over "
                    "passes):\n\n    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_LDS_BANK_CONFLICT "
                    "SQ_ACTIVE_INST_LDS SQ_WAVE_CYCLES SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS -d OUT/sq_c%d -o t --output-format csv -- python3 "
                    "bench.py %s\n    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum GRBM_GUI_ACTIVE -d OUT/tcc_c%d -o t --output-format "
                    "csv -- python3 bench.py %s\n\nAverages per launch (while KV mover jobs are pending the runtime cuts the prefill GEMMs into launches "
                    "of 8 tiles per block, so their rows average whole and partial launches).  GPU cycles = GRBM_GUI_ACTIVE / 8 (the counter sums "
                    "the 8 XCDs); MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / 1024 (256 CUs x 4 SIMDs) / GPU cycles.\n\n" % (flags, wl, n, short_flags, n, short_flags))
            f.write("\n".join(counter_table(sq, tcc, durations)) + "\n")
    clk_random, clk_zero = clock_rows(d("clk_random")), clock_rows(d("clk_zero"))
    if clk_random and clk_zero:
        zero = {r[0]: r for r in clk_zero}
        cflags = flags + " --no-reshard --steps 2 --warmup 1"
        with open(os.path.join(a.profiles, "bench_%s_gemm_clock.md" % wl), "w") as f:
            f.write("# Clock and matrix-pipe occupancy of the long kernels of `bench.py %s`, on the bench's data and on zeros (%s)\n\n"
                    "Two runs; each collects the cycle counter and the kernel trace together, so cycles / duration is the clock the "
                    "chip held during that launch:\n\n    rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES -d OUT/clk_random_c%d "
                    "-o t --output-format csv -- python3 bench.py %s\n    rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES "
                    "-d OUT/clk_zero_c%d -o t --output-format csv -- python3 bench.py %s --zero-data\n\n`--zero-data` runs the same instruction "
                    "streams on all-zero weights and inputs.  Medians over launches of 1 ms and more; clock = GRBM_GUI_ACTIVE / 8 / "
                    "duration; MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / 1024 / (GRBM_GUI_ACTIVE / 8).  The nominal matrix peak (2.5 PFLOP/s) "
                    "assumes 2.4 GHz; at the clock the chip holds on random data the pipes could deliver clock / 2.4 of it.\n\n"
                    "| kernel | launches | median us (random) | clock GHz (random) | MFMA busy (random) | median us (zeros) | clock GHz (zeros) | "
                    "MFMA busy (zeros) | zeros / random speed |\n|---|---|---|---|---|---|---|---|---|\n" % (cflags, wl, n, cflags, n, cflags))
            for k, cnt, t, ghz, busy in clk_random:
                if k in zero:
                    z = zero[k]
                    f.write("| `%s` | %d | %.0f | %.2f | %.1f %% | %.0f | %.2f | %.1f %% | %.2f |\n" % (k, cnt, t, ghz, busy, z[2], z[3], z[4], t / z[2]))
    lib = library_rows(d("clk_library"))
    if lib:
        with open(os.path.join(a.profiles, "library_gemm_%s_clock.md" % wl), "w") as f:
            f.write("# Yardstick: the vendor library's GEMM (`torch.matmul`) on the prefill projection shapes of %s\n\n"
                    "Not a kernel of this library: the same four contractions without the fused epilogues, timed by "
                    "`bench.py --config %d --library-gemm` (2 warm-up + 5 timed launches per shape, on random data and on zeros) "
                    "under the clock counters:\n\n    rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES -d OUT/clk_library_c%d "
                    "-o t --output-format csv -- python3 bench.py --config %d --library-gemm\n\nMedians over the timed launches; clock = "
                    "GRBM_GUI_ACTIVE / 8 / duration; MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / 1024 / (GRBM_GUI_ACTIVE / 8).  Compare with "
                    "`bench_%s_gemm_clock.md` (this library's kernels on the same box class).\n\n"
                    "| data | shape | median us | clock GHz | MFMA busy |\n|---|---|---|---|---|\n" % (wl, n, n, n, wl))
            for data, shape, t, ghz, busy in lib:
                f.write("| %s | %s | %.0f | %.2f | %.1f %% |\n" % (data, shape, t, ghz, busy))
    fetch, write = read_counters(d("fetch")), read_counters(d("write"))
    if fetch:
        lines, total, (cf, cw, sf, sw) = traffic(fetch, write)
        per_class, n_pf, n_dec = class_bytes(total, n)
        with open(os.path.join(a.profiles, "bench_%s_hbm_traffic.md" % wl), "w") as f:
            f.write("# Traffic between L2 and the memory fabric of the kernels of `bench.py %s` (%s)\n\nFETCH_SIZE / WRITE_SIZE count what "
                    "leaves the eight L2s towards memory: reads that the memory-side cache (256 MB, in front of HBM) serves are included, "
                    "so this is an upper bound of the HBM traffic.  Two runs, one counter each:\n\n    rocprofv3 --pmc FETCH_SIZE -d "
                    "OUT/fetch_c%d -o t --output-format csv -- python3 bench.py %s --calibrate-copy\n    rocprofv3 --pmc WRITE_SIZE -d OUT/write_c%d "
                    "-o t --output-format csv -- python3 bench.py %s --calibrate-copy\n\nCalibration: `--calibrate-copy` runs a plain 1 GiB "
                    "device-to-device copy (1 048 576 KiB read, 1 048 576 KiB written); the counters read %s (FETCH_SIZE) and %s (WRITE_SIZE) for "
                    "it, so FETCH_SIZE is scaled by %.3f and WRITE_SIZE by %.3f.\n\n" % (
                        flags, wl, n, short_flags, n, short_flags, "%.0f" % cf if cf else "nothing", "%.0f" % cw if cw else "nothing", sf, sw))
            f.write("\n".join(lines) + "\n\nPer layer call (sums over the launches of a class divided by the %d prefill / %d decode calls "
                    "of the run; per launch for the repack), as written to `bench_traffic.json`:\n\n| class | GB beyond L2 |\n|---|---|\n"
                    % (n_pf, n_dec))
            for cls, b in per_class.items():
                f.write("| %s | %.3f |\n" % (cls, b / 1e9))
        tj = {}
        if os.path.exists(a.traffic):
            with open(a.traffic) as f:
                tj = json.load(f)
        tj = {k: v for k, v in tj.items() if "." in k or k == "_note"}       # drop entries of the older, unprefixed form
        for cls, b in per_class.items():
            tj["c%d.%s" % (n, cls)] = b
        tj["_note"] = ("bytes between L2 and the memory fabric (memory-side cache hits included: an upper bound of the HBM bytes) per layer "
                       "call (per launch for the repack) from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, scaled by the factors a 1 GiB "
                       "device copy gives; written by python -m paper_2503_06433_amd.profile_summary, see profiles/")
        with open(a.traffic, "w") as f:
            json.dump(tj, f, indent=1)
        print(json.dumps({k: v for k, v in tj.items() if k.startswith("c%d." % n)}, indent=1))


if __name__ == "__main__":
    main()
