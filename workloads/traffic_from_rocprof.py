"""Turns two rocprofv3 counter runs of bench.py into workloads/measured_traffic_gfx950.json,
which bench.py reads for the `traffic` field of its roofline object.

    cd /tmp && export TMPDIR=/tmp
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d /tmp/pmcF -- python3 <repo>/bench.py --only step --steps 10 --calib-copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d /tmp/pmcW -- python3 <repo>/bench.py --only step --steps 10 --calib-copy
    python3 <repo>/workloads/traffic_from_rocprof.py /tmp/pmcF /tmp/pmcW [out.json]

Kernels already in the output file that the two runs did not launch keep their
stored figures; kernels the runs did launch are replaced.

Both counters are in KiB per dispatch up to a constant factor; the factor is
taken from the plain copy kernel that --calib-copy runs, which reads and writes
256 MiB per launch.  Kernels are keyed by template instantiation and grid size
(threads), averages over all dispatches of the run."""
import collections
import csv
import glob
import json
import os
import re
import sys

COPY_KIB = 262144.0


def norm(name):
    name = re.sub(r"^void\s+", "", name)
    name = name.replace("alt::", "").replace("(anonymous namespace)::", "")
    return re.sub(r"\(.*$", "", name).strip()


def collect(d):
    agg = collections.defaultdict(list)
    for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
        with open(f) as fh:
            for r in csv.DictReader(fh):
                agg[(norm(r["Kernel_Name"]), int(r["Grid_Size"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in agg.items()}


def main():
    fdir, wdir = sys.argv[1], sys.argv[2]
    out = sys.argv[3] if len(sys.argv) > 3 else os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                            "measured_traffic_gfx950.json")
    vals = collect(fdir)
    vals.update(collect(wdir))
    copy_f = [v for (n, g, c), v in vals.items() if n.startswith("stream_copy_kernel") and c == "FETCH_SIZE"]
    copy_w = [v for (n, g, c), v in vals.items() if n.startswith("stream_copy_kernel") and c == "WRITE_SIZE"]
    if not copy_f or not copy_w:
        raise SystemExit("no stream_copy_kernel dispatches found: run bench.py with --calib-copy")
    sf, sw = COPY_KIB / copy_f[0], COPY_KIB / copy_w[0]
    kernels = {}
    for (n, g, c), v in sorted(vals.items()):
        if not (n.startswith("dconv_kernel") or n.startswith("dstream_kernel") or n.startswith("igemm")
                or n.startswith("permute") or n.startswith("splitk")):
            continue
        e = kernels.setdefault("%s|%d" % (n, g), {})
        e["fetch_bytes" if c == "FETCH_SIZE" else "write_bytes"] = round(v * (sf if c == "FETCH_SIZE" else sw) * 1024.0)
    if os.path.exists(out):
        with open(out) as fh:
            old = json.load(fh).get("kernels", {})
        kernels = dict(old, **kernels)
    doc = dict(source="rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE over bench.py --only <target> --calib-copy",
               scale=dict(fetch=round(sf, 4), write=round(sw, 4),
                          note="factor from counter units to KiB, from the 256 MiB copy kernel"),
               kernels=kernels)
    with open(out, "w") as fh:
        json.dump(doc, fh, indent=1, sort_keys=True)
    print("wrote %s: %d kernels, scale fetch %.3f write %.3f" % (out, len(kernels), sf, sw))


if __name__ == "__main__":
    main()
