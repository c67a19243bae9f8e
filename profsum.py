"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

  python profsum.py kernels <dir-with-*_kernel_stats.csv> "<command that produced it>"
  python profsum.py traffic <fetch-dir> <write-dir> <kernel-name-substring> <copy-bytes>
  python profsum.py counters <dir-with-*_counter_collection.csv> "<command that produced it>"

`counters` prints, per kernel, the mean over its dispatches of every counter of one --pmc run (ten largest kernels
by dispatch count x first counter).  `traffic` reads the per-dispatch FETCH_SIZE / WRITE_SIZE counters (KiB) of two --pmc runs, scales
them by what the same counters report for the known-size copy kernel that `bench.py --copy-probe`
launches (torch.neg over <copy-bytes> bytes: that many read and as many written) and prints the HBM bytes per launch of the
chosen kernel.
"""
import csv
import glob
import os
import sys


def find(d, suffix):
    hits = glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True)
    if not hits:
        raise SystemExit(f"no *{suffix} under {d}")
    return hits[0]


def short(name):
    name = name.replace("void ", "").replace("sd::", "")
    return name.split("(")[0].replace(" ", "")


def kernels(d, command):
    rows = list(csv.DictReader(open(find(d, "kernel_stats.csv"))))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print(f"# rocprofv3 kernel statistics\n# command: {command}\n# total kernel time {total / 1e6:.3f} ms\n")
    print(f"{'kernel':64s} {'calls':>7s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'share':>7s}")
    for r in rows[:24]:
        print(f"{short(r['Name'])[:64]:64s} {r['Calls']:>7s} {float(r['AverageNs']) / 1e3:9.2f} {float(r['MinNs']) / 1e3:9.2f} "
              f"{float(r['MaxNs']) / 1e3:9.2f} {float(r['Percentage']):6.2f}%")


def counter_rows(d):
    rows = list(csv.DictReader(open(find(d, "counter_collection.csv"))))
    return rows


def per_kernel(rows, counter, substr):
    vals = [float(r["Counter_Value"]) for r in rows if r["Counter_Name"] == counter and substr in r["Kernel_Name"].replace(" ", "")]
    return (sum(vals) / len(vals), len(vals)) if vals else (None, 0)


def traffic(fetch_dir, write_dir, substr, copy_bytes):
    copy_bytes = float(copy_bytes)
    f, w = counter_rows(fetch_dir), counter_rows(write_dir)
    cf, ncf = per_kernel(f, "FETCH_SIZE", "neg_kernel")
    cw, ncw = per_kernel(w, "WRITE_SIZE", "neg_kernel")
    kf, nkf = per_kernel(f, "FETCH_SIZE", substr.replace(" ", ""))
    kw, nkw = per_kernel(w, "WRITE_SIZE", substr.replace(" ", ""))
    print(f"# HBM traffic of kernels matching '{substr}' from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch)")
    print(f"copy kernel ({copy_bytes / 2**20:.0f} MiB read + written): FETCH_SIZE {cf:.1f} KiB over {ncf} dispatches, WRITE_SIZE {cw:.1f} KiB over {ncw}")
    sf, sw = copy_bytes / (cf * 1024.0), copy_bytes / (cw * 1024.0)
    print(f"scale factors (true bytes / counter bytes): fetch {sf:.4f}, write {sw:.4f}")
    print(f"kernel: FETCH_SIZE {kf:.1f} KiB over {nkf} dispatches, WRITE_SIZE {kw:.1f} KiB over {nkw}")
    total = kf * 1024.0 * sf + kw * 1024.0 * sw
    print(f"HBM bytes per launch: read {kf * 1024 * sf:.0f} + written {kw * 1024 * sw:.0f} = {total:.0f}")


def counters(d, command):
    rows = counter_rows(d)
    names = sorted({r["Counter_Name"] for r in rows})
    per = {}
    for r in rows:
        k = short(r["Kernel_Name"])
        per.setdefault(k, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    print(f"# rocprofv3 --pmc counters, mean per dispatch\n# command: {command}\n")
    print(f"{'kernel':56s} {'dispatches':>10s} " + " ".join(f"{n:>16s}" for n in names))
    order = sorted(per, key=lambda k: -sum(per[k].get(names[0], [0.0])))
    for k in order[:12]:
        n_disp = max(len(v) for v in per[k].values())
        cells = []
        for n in names:
            v = per[k].get(n, [])
            cells.append(f"{sum(v) / len(v):16.4g}" if v else f"{'-':>16s}")
        print(f"{k[:56]:56s} {n_disp:10d} " + " ".join(cells))


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "kernels":
        kernels(sys.argv[2], sys.argv[3])
    elif len(sys.argv) >= 4 and sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3])
    elif len(sys.argv) == 6 and sys.argv[1] == "traffic":
        traffic(*sys.argv[2:6])
    else:
        raise SystemExit(__doc__)
