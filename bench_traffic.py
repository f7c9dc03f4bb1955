"""Writes profiles/hbm_traffic.json: HBM bytes per launch of a workload's forward kernel.

Counters cannot be read from inside a timed run, so the bench line's "roofline.traffic" comes
from two rocprofv3 counter runs of bench.py itself (run on the GPU machine, from the repository
root, after `cd /tmp && export TMPDIR=/tmp`):

  rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT/fetch -o t -- python3 bench.py --only --config 2 --copy-probe-mib 256 > OUT/fetch.log
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT/write -o t -- python3 bench.py --only --config 2 --copy-probe-mib 256 > OUT/write.log
  python3 bench_traffic.py OUT/fetch OUT/write OUT/fetch.log

Both counters are in KiB per dispatch; each is scaled by what the same counter reads for the
plain device-to-device copy of --copy-probe-mib (whose traffic is known: its size read, its
size written).  The entry records the kernel's name from the bench line of the same run;
bench.py ignores an entry whose kernel is not the one it has just run.
"""
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))


def counter_rows(folder, counter):
    for f in glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True):
        with open(f) as fh:
            for r in csv.DictReader(fh):
                if r["Counter_Name"] == counter:
                    yield r["Kernel_Name"], float(r["Counter_Value"])


def mean_per_kernel(folder, counter):
    acc = {}
    for name, v in counter_rows(folder, counter):
        acc.setdefault(name, []).append(v)
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def largest_copy(folder, counter):
    """The copy probe is the largest device-to-device copy of the run (a workload with beta != 0 also copies its y)."""
    return max(v for name, v in counter_rows(folder, counter) if "copy" in name.lower())


def main():
    if len(sys.argv) != 4:
        print(__doc__)
        sys.exit(2)
    fetch_dir, write_dir, bench_log = sys.argv[1:]
    line = [l for l in open(bench_log) if l.startswith("{")][-1]
    bench = json.loads(line)
    workload, kernel = bench["config"]["workload"], bench["config"]["kernel"]
    out = {}
    for key, folder, counter in (("read", fetch_dir, "FETCH_SIZE"), ("written", write_dir, "WRITE_SIZE")):
        per = mean_per_kernel(folder, counter)
        conv = {k: v for k, v in per.items() if "igconv_fwd" in k}
        assert conv, "need the forward kernel in %s" % folder
        kname, (kib, calls) = max(conv.items(), key=lambda kv: kv[1][1])     # the kernel launched most often
        ckib = largest_copy(folder, counter)
        scale = (bench["config"]["copy_probe_mib"] * 1024) / ckib    # the copy probe reads and writes its size once
        out[key] = {"kib_per_dispatch": kib, "dispatches": calls, "scale": scale, "bytes": kib * 1024 * scale,
                    "rocprof_kernel": kname}
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    table = json.load(open(path)) if os.path.exists(path) else {}
    table[workload] = {
        "kernel": kernel,
        "bytes_per_launch": int(out["read"]["bytes"] + out["written"]["bytes"]),
        "read_bytes": int(out["read"]["bytes"]), "written_bytes": int(out["written"]["bytes"]),
        "scale_fetch": out["read"]["scale"], "scale_write": out["written"]["scale"],
        "algorithmic_bytes": bench["roofline"].get("algorithmic_bytes"),
    }
    with open(path, "w") as fh:
        json.dump(table, fh, indent=1)
    print(json.dumps(table[workload]))


if __name__ == "__main__":
    main()
