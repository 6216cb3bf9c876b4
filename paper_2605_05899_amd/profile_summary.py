"""Turns rocprofv3 CSV output of a bench.py run into the short text summaries kept under profiles/.

    python -m paper_2605_05899_amd.profile_summary stats  <..._kernel_stats.csv>
    python -m paper_2605_05899_amd.profile_summary pmc    <..._counter_collection.csv> [more csv ...]
    python -m paper_2605_05899_amd.profile_summary traffic <workload> <fetch csv> <write csv>
    python -m paper_2605_05899_amd.profile_summary regen   <raw dir>

`regen` rebuilds every file under profiles/ from the raw output of paper_2605_05899_amd/collect_profiles.sh (run on a
GPU machine) and stamps profiles/hbm_traffic.json with the commit of the tree it is run on.

`stats` prints calls / average / min / max duration per kernel of this library (give the kernel trace CSV as a second
file to add the median). `traffic` prints the JSON fragment kept in profiles/hbm_traffic.json. `pmc` prints the mean of every
counter per kernel and per dispatch; FETCH_SIZE and WRITE_SIZE (KiB) are also scaled by the reading of the 1 GiB
device-to-device copy that `bench.py --calib-copy` issues (a copy kernel of known size: 1 GiB read, 1 GiB written).
"""
import collections
import csv
import sys

GIB_KIB = float(1 << 20)


def short(name: str) -> str:
    name = name.split("(")[0]
    for pre in ("void ", "vismoe::"):
        name = name.replace(pre, "")
    return name.strip()


def stats(path, trace_path=None):
    rows = list(csv.DictReader(open(path)))
    med = {}
    if trace_path:
        durs = collections.defaultdict(list)
        for r in csv.DictReader(open(trace_path)):
            durs[short(r["Kernel_Name"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
        med = {k: sorted(v)[len(v) // 2] / 1e3 for k, v in durs.items()}
    print(f"{'kernel':40s} {'calls':>6s} {'avg us':>10s} {'median us':>10s} {'min us':>10s} {'max us':>10s}")
    for r in rows:
        n = short(r["Name"])
        if "at::native" in r["Name"] or "rocclr" in r["Name"]:
            continue
        m = f"{med[n]:10.1f}" if n in med else f"{'-':>10s}"
        print(f"{n[:40]:40s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:10.1f} {m} {float(r['MinNs']) / 1e3:10.1f} "
              f"{float(r['MaxNs']) / 1e3:10.1f}")


def traffic(workload, fetch_csv, write_csv, quiet=False):
    import json
    out = {}
    for cname, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        agg = collections.defaultdict(list)
        calib = None
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != cname:
                continue
            k, v = short(r["Kernel_Name"]), float(r["Counter_Value"])
            agg[k].append(v)
            if ("copy" in k.lower() or "elementwise" in k) and v > 0.5 * GIB_KIB * 0.9:
                calib = GIB_KIB / v
        if calib is None:
            raise SystemExit(f"no 1 GiB calibration copy found in {path} (run bench.py with --calib-copy)")
        for k, v in agg.items():
            if "at::native" in k or "rocclr" in k:
                continue
            out.setdefault(k, {})["fetch_bytes" if cname == "FETCH_SIZE" else "write_bytes"] = round(
                sum(v) / len(v) * calib * 1024)
            out[k]["fetch_scale" if cname == "FETCH_SIZE" else "write_scale"] = round(calib, 4)
    if not quiet:
        print(json.dumps({workload: out}, indent=1))
    return {workload: out}


def pmc(paths):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in paths:
        for r in csv.DictReader(open(path)):
            agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    calib = {}
    for kname, d in agg.items():
        # the calibration copy is the elementwise copy kernel that moves 1 GiB: by far the largest reading
        if "elementwise" in kname or "copyBuffer" in kname or "copy" in kname.lower():
            for c in ("FETCH_SIZE", "WRITE_SIZE"):
                if c in d and max(d[c]) > 0.5 * GIB_KIB:
                    calib[c] = GIB_KIB / max(d[c])
    for c, f in calib.items():
        print(f"calibration: a 1 GiB copy reads {c} = {GIB_KIB / f:.4g} KiB -> scale factor {f:.4f}")
    for kname, d in sorted(agg.items()):
        if "at::native" in kname or "rocclr" in kname:
            continue
        print(kname)
        for c, v in sorted(d.items()):
            mean = sum(v) / len(v)
            extra = ""
            if c in calib:
                extra = f"   -> {mean * calib[c] * 1024 / 1e6:10.1f} MB per launch (scaled)"
            print(f"   {c:34s} n={len(v):4d} mean={mean:12.5g}{extra}")


SQ_COUNTERS = ("SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_LDS_BANK_CONFLICT "
               "SQ_ACTIVE_INST_LDS SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS")
TCC_COUNTERS = "TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum GRBM_GUI_ACTIVE"


def regen(raw, out_dir="profiles"):
    """profiles/*.txt and profiles/hbm_traffic.json from the raw rocprofv3 output of collect_profiles.sh."""
    import contextlib
    import io
    import json
    import os
    import subprocess

    def captured(fn, *a):
        buf = io.StringIO()
        with contextlib.redirect_stdout(buf):
            fn(*a)
        return buf.getvalue()

    os.makedirs(out_dir, exist_ok=True)
    traffic_all = {}
    workloads = [w for w in ("C1", "C2", "C3", "C4", "C5") if os.path.isdir(os.path.join(raw, f"{w}_trace"))]
    for W in workloads:
        B = f"python3 bench.py --config {W} --no-cpu-baseline --no-also"
        p = lambda kind, name: os.path.join(raw, f"{W}_{kind}", name)
        txt = [f"# rocprofv3 summaries, workload {W} (bench.py --config {W}), one MI355X, kernels of libvismoe",
               "# commands are run from the repository root (paper_2605_05899_amd/collect_profiles.sh runs them all); "
               "-d/-o only name the output", "",
               "## kernel durations",
               f"command: rocprofv3 --kernel-trace --stats -d OUT -o t --output-format csv -- {B} --steps 50 --warmup 10",
               "(calls per kernel: the untimed spin-up of 0.1 s, then 10 warm-up + 50 timed + 50 stage-timing + 1 "
               "routing-statistics step)",
               captured(stats, p("trace", "t_kernel_stats.csv"), p("trace", "t_kernel_trace.csv")),
               "## HBM traffic per launch",
               f"command: rocprofv3 --pmc FETCH_SIZE -d OUT -o p --output-format csv -- {B} --steps 5 --warmup 2 --calib-copy",
               f"command: rocprofv3 --pmc WRITE_SIZE -d OUT -o p --output-format csv -- {B} --steps 5 --warmup 2 --calib-copy",
               captured(pmc, [p("fetch", "p_counter_collection.csv"), p("write", "p_counter_collection.csv")]),
               "## SQ counters (MFMA busy, LDS, waits), summed over the chip per launch",
               f"command: rocprofv3 --pmc {SQ_COUNTERS} -d OUT -o p --output-format csv -- {B} --steps 5 --warmup 2",
               captured(pmc, [p("sq", "p_counter_collection.csv")]),
               "## L2 (TCC) counters per launch; GRBM_GUI_ACTIVE is summed over the 8 XCDs",
               f"command: rocprofv3 --pmc {TCC_COUNTERS} -d OUT -o p --output-format csv -- {B} --steps 5 --warmup 2",
               captured(pmc, [p("tcc", "p_counter_collection.csv")])]
        with open(os.path.join(out_dir, f"moe_layer_{W}.txt"), "w") as f:
            f.write("\n".join(txt))
        traffic_all.update(traffic(W, p("fetch", "p_counter_collection.csv"), p("write", "p_counter_collection.csv"),
                                   quiet=True))
    try:
        root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
        commit = subprocess.run(["git", "rev-parse", "HEAD"], capture_output=True, text=True, cwd=root).stdout.strip()
        dirty = bool(subprocess.run(["git", "status", "--porcelain", "--", "paper_2605_05899_amd/csrc", "include"],
                                    capture_output=True, text=True, cwd=root).stdout.strip())
    except OSError:
        commit, dirty = "", False
    traffic_all["_meta"] = {"commit": commit + ("+uncommitted kernel changes" if dirty else ""),
                            "note": "HBM bytes per launch: rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB copy's readings"}
    with open(os.path.join(out_dir, "hbm_traffic.json"), "w") as f:
        json.dump(traffic_all, f, indent=1, sort_keys=True)
    for W, cfg, what, calls in (
            ("P2", "P2 --no-cpu-baseline", "token compressor workload P2",
             "50 spin-up + 200 timed calls of moe_token_compress"),
            ("P3", "P3 --no-cpu-baseline", "token compressor workload P3 (32 768 tokens: the many-workgroup path)",
             "50 spin-up + 200 timed calls of moe_token_compress"),
            ("PF", "PF", "predictor feature construction",
             "50 spin-up + 200 timed calls each of moe_mean_pool, moe_routing_histogram, moe_lookahead_target, "
             "moe_predictor_forward")):
        d = os.path.join(raw, f"{W}_trace")
        if not os.path.isdir(d):
            continue
        name = {"P2": "token_compress_P2.txt", "P3": "token_compress_P3.txt"}.get(W, "predictor_features_PF.txt")
        with open(os.path.join(out_dir, name), "w") as f:
            f.write(f"# rocprofv3 summary, {what} (bench.py --config {W}), one MI355X, kernels of libvismoe\n\n"
                    "## kernel durations\n"
                    f"command: rocprofv3 --kernel-trace --stats -d OUT -o t --output-format csv -- python3 bench.py "
                    f"--config {cfg} --steps 200 --warmup 10\n(calls per kernel: {calls})\n"
                    + captured(stats, os.path.join(d, "t_kernel_stats.csv"), os.path.join(d, "t_kernel_trace.csv")))
    print("wrote", sorted(os.listdir(out_dir)))


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "regen":
        regen(sys.argv[2])
        sys.exit(0)
    if len(sys.argv) < 3 or sys.argv[1] not in ("stats", "pmc", "traffic"):
        sys.exit(__doc__)
    if sys.argv[1] == "stats":
        stats(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else None)
    elif sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        pmc(sys.argv[2:])
