"""Reads rocprofv3 counter-collection and kernel-trace CSV files and prints per-kernel means.

    python -m paper_2604_26666_amd.counters summarise FILE.csv [FILE.csv ...]
    python -m paper_2604_26666_amd.counters runs KERNEL_TRACE.csv [MIN_LAUNCHES]
    python -m paper_2604_26666_amd.counters traffic-json FETCH.csv WRITE.csv PROBE_STDOUT OUT.json

`summarise` groups the dispatches of each file by (kernel, grid, work-group size) and prints the
mean of every counter, or of the duration for a kernel trace.  FETCH_SIZE and WRITE_SIZE (KiB per
dispatch) are also given in bytes, scaled by what the same counter read for the plain 1 GiB
device-to-device copies that `bench.py --probe` and `bench.py --traffic-probe` append to their
launches (the last three dispatches of the copy kernel): scale = 2^30 / (1024 x the copy's reading).

`runs` lists, in time order, every run of at least MIN_LAUNCHES (default 20) consecutive launches of
one (kernel, grid): the timing loops of `bench.py --all`, one per shape, with the average duration
of the run's second half (its timed part).

`traffic-json` turns the two counter files of `bench.py --traffic-probe` and the line that
the probe printed into the small file that bench.py quotes as `roofline.traffic`.
No arithmetic of the GEMM itself lives here.
"""
import csv
import json
import re
import sys
from collections import OrderedDict

COPY_BYTES = 1 << 30
COPY_KERNEL = "copyBuffer"


def short_name(name):
    name = name.replace("void ", "").replace("fact::", "")
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    cut = name.find("(")
    if cut > 0 and not name.startswith("("):
        name = name[:cut]
    return name[:72]


def read(path):
    with open(path, newline="") as f:
        return list(csv.DictReader(f))


def groups(rows):
    """OrderedDict: (kernel, grid, work-group) -> {"n": dispatches, counter or "duration_us": [values]}"""
    out = OrderedDict()
    seen = set()
    for r in sorted(rows, key=lambda r: int(r.get("Start_Timestamp", 0) or 0)):
        grid = r.get("Grid_Size") or "x".join(r.get(k, "1") for k in ("Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"))
        wg = r.get("Workgroup_Size") or r.get("Workgroup_Size_X", "")
        key = (short_name(r["Kernel_Name"]), grid, wg)
        g = out.setdefault(key, {"n": 0})
        disp = (r.get("Dispatch_Id"), r.get("Start_Timestamp"))
        if disp not in seen:
            seen.add(disp)
            g["n"] += 1
        if "Counter_Name" in r:
            g.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
        else:
            g.setdefault("duration_us", []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return out


def copy_scale(gr, counter):
    """bytes per KiB reported, from the last three dispatches of the copy kernel (the 1 GiB copies)"""
    vals = []
    for (name, _, _), g in gr.items():
        if COPY_KERNEL in name and counter in g:
            vals += g[counter]
    vals = [v for v in vals[-3:] if v > 1e5]
    if not vals:
        return None
    return COPY_BYTES / (sum(vals) / len(vals))


def mean(v):
    return sum(v) / len(v)


def summarise(paths, out=sys.stdout):
    for path in paths:
        gr = groups(read(path))
        print(f"== {path}", file=out)
        scales = {c: copy_scale(gr, c) for c in ("FETCH_SIZE", "WRITE_SIZE")}
        for c, s in scales.items():
            if s:
                print(f"   {c}: 1 GiB copy reads {COPY_BYTES / s:.0f} KiB -> {s:.1f} bytes per unit (x{s / 1024:.3f} of KiB)", file=out)
        for (name, grid, wg), g in gr.items():
            if g["n"] < 3 and COPY_KERNEL not in name:
                continue
            parts = []
            for c, v in g.items():
                if c == "n":
                    continue
                if COPY_KERNEL in name:
                    v = v[-3:]                                  # the 1 GiB copies come last; clones of operands before them
                if c == "duration_us":
                    half = v[len(v) // 2:]
                    parts.append(f"avg_us {mean(v):.2f} second_half_avg_us {mean(half):.2f} min_us {min(v):.2f}")
                elif c in scales and scales[c]:
                    parts.append(f"{c} {mean(v):.0f} KiB = {mean(v) * scales[c] / 1e6:.2f} MB")
                else:
                    parts.append(f"{c} {mean(v):.4g}")
            print(f"   {name}  grid {grid} wg {wg}  dispatches {g['n']}:  " + "; ".join(parts), file=out)


def runs(path, min_launches=20, out=sys.stdout):
    rows = sorted(read(path), key=lambda r: int(r["Start_Timestamp"]))
    found = []
    for r in rows:
        grid = "x".join(r.get(k, "1") for k in ("Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"))
        key = (short_name(r["Kernel_Name"]), grid, r.get("Workgroup_Size_X", ""))
        d = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        if found and found[-1][0] == key:
            found[-1][1].append(d)
        else:
            found.append((key, [d]))
    for (name, grid, wg), d in found:
        if len(d) >= min_launches:
            half = d[len(d) // 2:]
            print(f"{name}  grid {grid} wg {wg}  launches {len(d)}  second_half_avg_us {mean(half):.2f}  min_us {min(d):.2f}", file=out)


def traffic_json(fetch_csv, write_csv, probe_stdout, out_path):
    probe = None
    with open(probe_stdout) as f:
        for line in f:
            if line.startswith("{") and "traffic_probe" in line:
                probe = json.loads(line)
    if probe is None:
        raise SystemExit(f"{probe_stdout}: no traffic-probe line")
    doc = {"n": probe["n"], "kernel_tag": probe["kernel_tag"], "unit": "bytes per launch"}
    total = 0.0
    for counter, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        gr = groups(read(path))
        scale = copy_scale(gr, counter)
        if scale is None:
            raise SystemExit(f"{path}: no 1 GiB copy to scale {counter} by")
        vals = [v for (name, _, _), g in gr.items() if "gemm_kernel" in name for v in g.get(counter, [])]
        if not vals:
            raise SystemExit(f"{path}: no gemm_kernel dispatch")
        doc[counter] = {"kib_per_dispatch": mean(vals), "bytes_per_kib_from_copy": scale, "bytes": mean(vals) * scale,
                        "dispatches": len(vals)}
        total += mean(vals) * scale
    doc["bytes_per_launch"] = total
    with open(out_path, "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")
    print(json.dumps(doc))


def main(argv):
    if len(argv) >= 2 and argv[0] == "summarise":
        summarise(argv[1:])
    elif len(argv) in (2, 3) and argv[0] == "runs":
        runs(argv[1], int(argv[2]) if len(argv) == 3 else 20)
    elif len(argv) == 5 and argv[0] == "traffic-json":
        traffic_json(*argv[1:])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv[1:])
