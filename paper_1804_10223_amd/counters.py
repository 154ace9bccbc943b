"""Turn rocprofv3 --pmc output of a bench.py run into the short counter summary that bench.py reads back.

    python -m paper_1804_10223_amd.counters --fetch DIR --write DIR --kernel persistent_kernel --workload cfg3 \
        --out profiles/persistent_kernel_cfg3_traffic.txt

DIR is the -d directory of one `rocprofv3 --pmc FETCH_SIZE -- python3 bench.py ...` (resp. WRITE_SIZE) pass.  Both
counters are in KiB per dispatch; each is scaled by what the same counter reads for the run's reference dispatch of known
size: bench.py issues one plain device-to-device copy of 256 MiB (kernel `__amd_rocclr_copyBuffer`, 256 MiB read and
256 MiB written) for exactly that purpose.  The summary is `key = value` text: averages per dispatch of every kernel whose
name contains --kernel (the first match with the most dispatches is the one reported as the workload's kernel).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os

REFERENCE_KERNEL = "copyBuffer"
REFERENCE_BYTES = 256 << 20


def read_counter(directory: str, counter: str):
    """{kernel name: [values per dispatch]} of one counter from every *counter_collection.csv below directory."""
    per_kernel = collections.defaultdict(list)
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if row.get("Counter_Name") == counter:
                    per_kernel[row["Kernel_Name"]].append(float(row["Counter_Value"]))
    return per_kernel


def scaled_bytes(directory: str, counter: str, kernel_substring: str):
    """(kernel name, dispatches, bytes per dispatch, scale factor, raw KiB per dispatch) for the matching kernel."""
    data = read_counter(directory, counter)
    ref = [v for k, vals in data.items() if REFERENCE_KERNEL in k for v in vals if v > 0]
    if not ref:
        raise SystemExit("no reference copy dispatch (%s) with %s in %s" % (REFERENCE_KERNEL, counter, directory))
    # the largest reference dispatch is the 256 MiB copy (smaller copies of the run use the same kernel)
    scale = (REFERENCE_BYTES / 1024.0) / max(ref)
    hits = [(k, vals) for k, vals in data.items() if kernel_substring in k]
    if not hits:
        raise SystemExit("no kernel matching %r in %s" % (kernel_substring, directory))
    name, vals = max(hits, key=lambda kv: len(kv[1]))
    raw = sum(vals) / len(vals)
    return name, len(vals), raw * scale * 1024.0, scale, raw


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--fetch", required=True, help="output directory of the FETCH_SIZE pass")
    ap.add_argument("--write", required=True, help="output directory of the WRITE_SIZE pass")
    ap.add_argument("--kernel", default="persistent_kernel", help="substring of the kernel's name")
    ap.add_argument("--workload", required=True, help="workload name bench.py was run with (cfg3, ...)")
    ap.add_argument("--command", default="", help="the profiled command, recorded in the summary")
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    kf, nf, fetch, sf, rawf = scaled_bytes(args.fetch, "FETCH_SIZE", args.kernel)
    kw, nw, write, sw, raww = scaled_bytes(args.write, "WRITE_SIZE", args.kernel)
    lines = [
        "# HBM traffic of one launch, from rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE passes (KiB per dispatch),",
        "# each scaled by the same counter's reading for the run's 256 MiB reference copy.  Written by",
        "# python -m paper_1804_10223_amd.counters; read by bench.py (--traffic-file).",
        "workload = %s" % args.workload,
        "kernel = %s" % kf,
        "command = %s" % args.command,
        "dispatches = %d" % nf,
        "fetch_raw_kib_per_launch = %.1f" % rawf,
        "fetch_scale = %.4f" % sf,
        "fetch_bytes_per_launch = %.0f" % fetch,
        "write_raw_kib_per_launch = %.1f" % raww,
        "write_scale = %.4f" % sw,
        "write_bytes_per_launch = %.0f" % write,
    ]
    if kw != kf or nw != nf:
        lines.append("# note: the WRITE_SIZE pass matched kernel %s with %d dispatches" % (kw, nw))
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
