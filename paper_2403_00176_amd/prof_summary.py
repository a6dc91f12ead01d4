"""Condenses rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2403_00176_amd.prof_summary stats  <..._kernel_stats.csv>
  python -m paper_2403_00176_amd.prof_summary pmc    <..._counter_collection.csv> COUNTER [copy_bytes]

`stats`: per kernel calls / total / average duration (kernel-trace --stats run).
`pmc`:   per kernel the average of COUNTER per dispatch.  With copy_bytes, the dispatches of the plain
         copy kernel of that size found in the same run give the scale of the counter (bytes per unit),
         and the per-dispatch averages are also printed in bytes.
"""
import csv
import collections
import sys


def short(name: str) -> str:
    name = name.replace("void sod2::", "sod2::")
    cut = name.find("(")
    return name if cut < 0 else name[:cut]


def stats(path):
    rows = list(csv.DictReader(open(path)))
    print("# kernel | calls | total ms | average us | % | min us | max us")
    for r in rows:
        print(f"{short(r['Name'])} | {r['Calls']} | {float(r['TotalDurationNs']) / 1e6:.3f} | {float(r['AverageNs']) / 1e3:.2f} | "
              f"{r['Percentage']} | {float(r['MinNs']) / 1e3:.2f} | {float(r['MaxNs']) / 1e3:.2f}")


def pmc(path, counter, copy_bytes=None):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            per[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    scale = None
    if copy_bytes:
        # the calibration copy: the dispatches with the largest counter value among copy / elementwise kernels
        cands = {k: v for k, v in per.items() if "copy" in k.lower() or "elementwise" in k.lower()}
        if cands:
            k, v = max(cands.items(), key=lambda kv: max(kv[1]))
            big = [x for x in v if x > 0.5 * max(v)]
            scale = float(copy_bytes) / (sum(big) / len(big))
            print(f"# calibration: {len(big)} dispatches of {k} moving {copy_bytes} bytes read {sum(big) / len(big):.1f} {counter} units"
                  f" -> {scale:.2f} bytes per unit")
    print(f"# kernel | dispatches | average {counter} per dispatch" + (" | average bytes per dispatch" if scale else ""))
    total = collections.defaultdict(float)
    count = collections.defaultdict(int)
    for k, v in sorted(per.items(), key=lambda kv: -sum(kv[1])):
        line = f"{k} | {len(v)} | {sum(v) / len(v):.1f}"
        if scale:
            line += f" | {scale * sum(v) / len(v):.0f}"
        print(line)
        fam = "gemm" if ("gemm" in k or "gemv" in k or "splitk" in k) else ("attention" if "attention" in k else None)
        if fam:
            total[fam] += sum(v)
            if "splitk" not in k:            # the partial-sum pass belongs to the contraction launched before it
                count[fam] += len(v)
    for fam in total:
        line = f"ALL {fam} kernels | {count[fam]} | {total[fam] / count[fam]:.1f}"
        if scale:
            line += f" | {scale * total[fam] / count[fam]:.0f}"
        print(line)


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 4 and sys.argv[1] == "pmc":
        pmc(sys.argv[2], sys.argv[3], sys.argv[4] if len(sys.argv) > 4 else None)
    else:
        print(__doc__)
        sys.exit(2)
