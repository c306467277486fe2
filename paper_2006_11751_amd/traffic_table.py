"""Builds the table of measured HBM bytes per launch that bench.py reads.

Input: the outputs of two counter runs of the benchmark under rocprofv3, one per counter
(FETCH_SIZE, then WRITE_SIZE; KiB per dispatch), each made with

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o p -- \\
        python3 bench.py --config <i> --profile-run --calibrate-copy --steps 3 --warmup 1 > <dir>/bench.json

A profile run ends with whole steps, so the last len(ops) dispatches of the trace are one step's
launches in order.  Each counter is scaled by what it reads for the plain copy kernel of known
size in the same run (copy16_kernel, 256 MiB in and out).  The entry is keyed by workload, batch,
launch sequence and the hash of the library sources, so that bench.py reports traffic only for
the kernels it was measured on.

    python -m paper_2006_11751_amd.traffic_table --fetch <dir1> --write <dir2> --profile <name of the summary>
"""
import argparse
import csv
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")
COPY_KIB = 256 * 1024
HEADER = ("# HBM traffic per launch of sf_policy_step, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs\n"
          "# (KiB per dispatch, scaled by the same counter's reading for a 256 MiB plain copy).\n"
          "# Written by `python -m paper_2006_11751_amd.traffic_table`; read by bench.py.\n")


def _dispatches(directory, counter):
    path = os.path.join(directory, "p_counter_collection.csv")
    rows = {}
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                d = int(r["Dispatch_Id"])
                rows[d] = (r["Kernel_Name"], rows.get(d, ("", 0.0))[1] + float(r["Counter_Value"]))
    return [rows[d] for d in sorted(rows)]


def _bench_line(directory):
    for line in open(os.path.join(directory, "bench.json")):
        line = line.strip()
        if line.startswith("{"):
            return json.loads(line)
    raise SystemExit("no JSON line in %s/bench.json" % directory)


def _per_op(directory, counter, n_ops):
    disp = _dispatches(directory, counter)
    copies = [v for name, v in disp if "copy16_kernel" in name]
    if not copies:
        raise SystemExit("%s: no copy16_kernel dispatch (run bench.py with --calibrate-copy)" % directory)
    scale = COPY_KIB / copies[-1]
    last = disp[-n_ops:]
    return [name for name, _ in last], [v * scale for _, v in last], scale


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--profile", default="", help="name of the summary under profiles/ that documents the runs")
    args = ap.parse_args()
    a, b = _bench_line(args.fetch), _bench_line(args.write)
    for k in ("name", "B", "source_hash", "launch_pipes"):
        if a["config"][k] != b["config"][k]:
            raise SystemExit("the two runs differ in %s" % k)
    ops = list(a["config"]["launch_pipes"].items())
    kf, fetch, sf = _per_op(args.fetch, "FETCH_SIZE", len(ops))
    kw, write, sw = _per_op(args.write, "WRITE_SIZE", len(ops))
    if kf != kw:
        raise SystemExit("the two runs end in different kernels:\n%s\n%s" % (kf, kw))
    entry = {"workload": a["config"]["name"], "B": a["config"]["B"], "source_hash": a["config"]["source_hash"],
             "profile": args.profile, "fetch_scale": round(sf, 4), "write_scale": round(sw, 4),
             "ops": [{"op": op, "pipe": pipe, "kernel": k.replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0][:120], "fetch_kib": round(f, 1),
                      "write_kib": round(wv, 1), "hbm_kib": round(f + wv, 1)}
                     for (op, pipe), k, f, wv in zip(ops, kf, fetch, write)]}
    table = []
    if os.path.exists(TABLE):
        table = json.loads("".join(l for l in open(TABLE) if not l.startswith("#")))
    table = [e for e in table if not (e["workload"] == entry["workload"] and e["B"] == entry["B"])]
    table.append(entry)
    with open(TABLE, "w") as f:
        f.write(HEADER)
        f.write(json.dumps(table, indent=1))
        f.write("\n")
    print(json.dumps(entry, indent=1))


if __name__ == "__main__":
    main()
