"""Turns the raw output of three rocprofv3 runs of bench.py into the short text summary kept under profiles/.

    python3 profile_summary.py <workload> <raw dir>          (the folder the three runs below wrote into)

expects, for workload W in c2 / c3 / c4a / c4b / c5 / f1 (the commands are repeated in every summary):

    cd /tmp && export TMPDIR=/tmp
    B="python3 <repo>/bench.py --workload W --modes fused --skip-extra --skip-cpu --steps 10 --warmup 2"
    rocprofv3 --kernel-trace --stats --output-format csv -d <raw>/trace -o run -- $B > <raw>/trace.json
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <raw>/fetch -o run -- $B > <raw>/fetch.json
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <raw>/write -o run -- $B > <raw>/write.json

and writes profiles/W.txt: per kernel the calls and average duration, FETCH_SIZE / WRITE_SIZE per dispatch, the
counter scale read off the plain copy kernel of known size that every bench run starts with, and the workload's
roofline fraction recomputed from these figures alone (algorithmic bytes per step from the run's own JSON line).
"""
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
COPY_KIB = 65536.0          # bench.py's clock spin-up copies 64 MiB per dispatch: 65536 KiB read, 65536 KiB written
PEAK = 8000.0               # GB/s


def find(raw, sub, pattern):
    hits = glob.glob(os.path.join(raw, sub, "**", pattern), recursive=True)
    return hits[0] if hits else None


def kernel_stats(path):
    out = {}
    for r in csv.DictReader(open(path)):
        name = r.get("Name") or r.get("Kernel_Name")
        out[name] = {"calls": int(r["Calls"]), "avg_ns": float(r["AverageNs"]), "total_ns": float(r["TotalDurationNs"])}
    return out


def counters(path, which):
    acc = {}
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != which:
            continue
        e = acc.setdefault(r["Kernel_Name"], [0, 0.0])
        e[0] += 1
        e[1] += float(r["Counter_Value"])
    return {k: (n, v / n) for k, (n, v) in acc.items()}


def short(name, width=110):
    name = name.replace("void redist::", "").replace("redist::", "")
    return name[:width]


def main():
    w = sys.argv[1]
    if len(sys.argv) < 3:
        sys.exit(__doc__)
    raw = sys.argv[2]
    line = json.loads(open(os.path.join(raw, "trace.json")).read().strip().splitlines()[-1])
    stats = kernel_stats(find(raw, "trace", "*kernel_stats.csv"))
    fetch = counters(find(raw, "fetch", "*counter_collection.csv"), "FETCH_SIZE")
    write = counters(find(raw, "write", "*counter_collection.csv"), "WRITE_SIZE")
    copy_f = [v for k, v in fetch.items() if "redist_copy_kernel" in k][0][1]
    copy_w = [v for k, v in write.items() if "redist_copy_kernel" in k][0][1]
    fs, ws = COPY_KIB / copy_f, COPY_KIB / copy_w
    steps, warm = line["steps"], line["warmup"]
    calls_per_case = warm + 2 * steps       # warm-up, the timed region, the same calls again with an event after each
    mine = {k: v for k, v in stats.items() if "redist_" in k and "redist_copy_kernel" not in k and "ptr_" not in k
            and "upload" not in k}
    total_ns = sum(v["total_ns"] for v in mine.values())
    bytes_step = line["config"]["bytes_per_step"]
    ns_step = total_ns / calls_per_case
    gbs = bytes_step / ns_step
    fetched = sum(fetch[k][0] * fetch[k][1] for k in mine if k in fetch) * fs * 1024
    written = sum(write[k][0] * write[k][1] for k in mine if k in write) * ws * 1024
    n_steps_pmc = calls_per_case
    head = mine and max(mine, key=lambda k: mine[k]["total_ns"])
    out = []
    out.append("rocprofv3 summary -- workload %s, fused mode" % w)
    out.append(line["config"]["workload"])
    out.append("")
    out.append("Commands (from /tmp with TMPDIR=/tmp on a 1-GPU MI355X box; three separate runs of committed files):")
    b = "python3 <repo>/bench.py --workload %s --modes fused --skip-extra --skip-cpu --steps %d --warmup %d" % (w, steps, warm)
    out.append("  rocprofv3 --kernel-trace --stats --output-format csv -d <raw>/trace -o run -- %s > <raw>/trace.json" % b)
    out.append("  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <raw>/fetch -o run -- %s > <raw>/fetch.json" % b)
    out.append("  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <raw>/write -o run -- %s > <raw>/write.json" % b)
    out.append("  python3 <repo>/profile_summary.py %s <raw>" % w)
    out.append("")
    out.append("Every case of the workload is called %d times per run (%d warm-up + %d timed + the same %d again with an event"
               % (calls_per_case, warm, steps, steps))
    out.append("after each call).  Algorithmic bytes per step (every distinct source byte read once + every destination byte")
    out.append("written once, summed over the workload's cases): %d." % bytes_step)
    out.append("Counter scale from the plain copy kernel of known size in the same runs (redist_copy_kernel, 65536 KiB read and")
    out.append("65536 KiB written per dispatch): FETCH_SIZE reads %.1f -> x%.3f; WRITE_SIZE reads %.1f -> x%.3f." % (copy_f, fs, copy_w, ws))
    out.append("")
    out.append("Recomputed from the figures below:")
    out.append("  kernel time per step = sum(calls x average) / %d = %.2f us  ->  %d B / %.2f us = %.0f GB/s = %.1f %% of 8 TB/s"
               % (calls_per_case, ns_step / 1e3, bytes_step, ns_step / 1e3, gbs, gbs / PEAK * 100))
    out.append("  bench.py's own line in the trace run (events around the timed region): %.0f GB/s = %.1f %%"
               % (line["value"], line["value"] / PEAK * 100))
    out.append("  HBM traffic per step: fetched %.0f B + written %.0f B = %.0f B = %.3f x the algorithmic bytes"
               % (fetched / n_steps_pmc, written / n_steps_pmc, (fetched + written) / n_steps_pmc,
                  (fetched + written) / n_steps_pmc / bytes_step))
    out.append("traffic_bytes_per_step: %d" % int((fetched + written) / n_steps_pmc))
    if head:
        k = head
        per_launch = bytes_step if len(mine) == 1 and mine[k]["calls"] == calls_per_case else None
        out.append("  dominant kernel: %s" % short(k, 160))
        out.append("    calls %d, average %.2f us%s" % (mine[k]["calls"], mine[k]["avg_ns"] / 1e3,
                   ("  ->  %d B per launch / %.2f us = %.0f GB/s = %.1f %%" % (per_launch, mine[k]["avg_ns"] / 1e3,
                    per_launch / mine[k]["avg_ns"], per_launch / mine[k]["avg_ns"] / PEAK * 100)) if per_launch else ""))
        if k in fetch and k in write:
            out.append("    HBM traffic per launch: fetch %.1f x %.3f = %.0f KiB, write %.1f x %.3f = %.0f KiB"
                       % (fetch[k][1], fs, fetch[k][1] * fs, write[k][1], ws, write[k][1] * ws))
            out.append("traffic_bytes_per_launch: %d" % int((fetch[k][1] * fs + write[k][1] * ws) * 1024))
    out.append("")
    out.append("== kernels of the library (rocprofv3 --kernel-trace --stats) ==")
    for k, v in sorted(mine.items(), key=lambda kv: -kv[1]["total_ns"]):
        f = fetch.get(k, (0, float("nan")))[1] * fs
        wv = write.get(k, (0, float("nan")))[1] * ws
        out.append("  calls %6d  avg %10.2f us  total %10.3f ms  fetch %10.0f KiB  write %10.0f KiB per dispatch  %s"
                   % (v["calls"], v["avg_ns"] / 1e3, v["total_ns"] / 1e6, f, wv, short(k)))
    out.append("== other kernels in the run ==")
    for k, v in sorted(stats.items(), key=lambda kv: -kv[1]["total_ns"]):
        if k not in mine:
            out.append("  calls %6d  avg %10.2f us  %s" % (v["calls"], v["avg_ns"] / 1e3, short(k, 90)))
    path = os.path.join(ROOT, "profiles", w + ".txt")
    open(path, "w").write("\n".join(out) + "\n")
    print("\n".join(out[:40]))


if __name__ == "__main__":
    main()
