"""HBM traffic readings of the library's kernels, kept as data next to the profile summaries.

``profiles/traffic.json`` holds, per (kernel, workload, layout), the bytes one launch moved
through HBM as read from two ``rocprofv3 --pmc`` runs (``FETCH_SIZE``, then ``WRITE_SIZE``; KiB
per dispatch), each scaled by what the same counter reads for a plain device copy of 2^30 bytes
issued by ``bench.py --copy-probe`` in the same run.  Every entry carries the revision of the
kernel source it was measured on (a hash of the ``.hip`` file that defines the kernel and of
the shared headers); ``lookup`` returns nothing for an entry of another revision, so a changed
kernel never inherits an old reading, and a change to another kernel's file does not discard
this one's.

Regenerate (from the repo root, on a GPU machine; ``cd /tmp && export TMPDIR=/tmp`` first)::

    rocprofv3 --pmc FETCH_SIZE -d <dirF> -o bench --output-format csv -- \
        python3 bench.py --workload 2 --workloads 2 --no-extras --steps 3 --warmup 1 \
        --no-cpu-baseline --copy-probe
    rocprofv3 --pmc WRITE_SIZE -d <dirW> -o bench --output-format csv -- \
        python3 bench.py --workload 2 --workloads 2 --no-extras --steps 3 --warmup 1 \
        --no-cpu-baseline --copy-probe
    python3 -m paper_2510_25979_amd.traffic --fetch <dirF> --write <dirW> \
        --workload llama-3.2-1b-shaped --layout packed --kernel apply_bf16_kernel
    python3 -m paper_2510_25979_amd.traffic --fetch <dirF> --write <dirW> \
        --workload llama-3.2-1b-shaped --kernel exact_bf16_kernel --largest

(the same with ``--workload 3 --workloads 3`` / ``4`` and the kernels that serve them:
``apply_bf16_kernel`` and ``apply_bf16_long_kernel``).
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import statistics
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
DATA = os.path.join(ROOT, "profiles", "traffic.json")
COPY_KERNEL = "copyBuffer"          # the runtime's device-to-device copy kernel
COPY_KIB = 1 << 20                  # the probe copies 2^30 bytes: 2^20 KiB read, 2^20 KiB written


def source_file(kernel: str) -> str:
    """The file under csrc/ that defines a kernel: kernels are named <file stem>_..."""
    stem = kernel.split("_")[0]
    name = stem + ".hip"
    if not os.path.exists(os.path.join(HERE, "csrc", name)):
        raise ValueError(f"no source file csrc/{name} for kernel {kernel!r}")
    return name


def source_revision(kernel: str) -> str:
    """Hash of the kernel's source file and of the shared headers: the revision a reading of
    that kernel belongs to."""
    h = hashlib.sha256()
    csrc = os.path.join(HERE, "csrc")
    names = [source_file(kernel)] + sorted(n for n in os.listdir(csrc) if n.endswith(".hpp"))
    for name in names:
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def _key(kernel: str, workload: str, layout: str) -> str:
    return f"{kernel}|{workload}|{layout}"


def lookup(kernel: str, workload: str, layout: str) -> Optional[dict]:
    """The stored reading for this kernel and workload, or None when there is none for the
    current revision of the kernel sources."""
    if not os.path.exists(DATA):
        return None
    entry = json.load(open(DATA)).get(_key(kernel, workload, layout))
    if entry is None or entry.get("revision") != source_revision(kernel):
        return None
    return entry


def _readings(directory: str, counter: str):
    """(dispatch id, counter value) per dispatch, grouped by kernel name, from rocprofv3's CSV."""
    out = {}
    for f in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] == counter:
                out.setdefault(r["Kernel_Name"], []).append(
                    (int(r.get("Dispatch_Id") or 0), float(r["Counter_Value"])))
    return out


def _pick(readings: dict, needle: str):
    vals = [v for k, vs in readings.items() if needle in k for _, v in vs]
    if not vals:
        raise SystemExit(f"no dispatch of a kernel named *{needle}* in the counter output")
    return vals


def _probe(readings: dict) -> float:
    """Reading of the copy probe: the LAST device copy of the run (bench.py issues it after all
    timed work; torch's own copies of other sizes come earlier)."""
    rows = [dv for k, vs in readings.items() if COPY_KERNEL in k for dv in vs]
    if not rows:
        raise SystemExit("no device copy in the counter output: run bench.py with --copy-probe")
    return max(rows)[1]


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--fetch", required=True, help="output directory of the FETCH_SIZE run")
    ap.add_argument("--write", required=True, help="output directory of the WRITE_SIZE run")
    ap.add_argument("--kernel", required=True, help="kernel name (substring), e.g. apply_bf16_kernel")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--layout", default="packed")
    ap.add_argument("--largest", action="store_true",
                    help="take the largest dispatch instead of the median (kernels that are also "
                         "launched on a part of the batch)")
    args = ap.parse_args()
    fetch, write = _readings(args.fetch, "FETCH_SIZE"), _readings(args.write, "WRITE_SIZE")
    f_scale = COPY_KIB / _probe(fetch)
    w_scale = COPY_KIB / _probe(write)
    agg = max if args.largest else statistics.median
    f_raw, w_raw = agg(_pick(fetch, args.kernel)), agg(_pick(write, args.kernel))
    entry = {"revision": source_revision(args.kernel), "source": source_file(args.kernel),
             "fetch_raw": f_raw, "fetch_scale": round(f_scale, 4),
             "write_raw": w_raw, "write_scale": round(w_scale, 4),
             "read_bytes": int(f_raw * f_scale * 1024), "written_bytes": int(w_raw * w_scale * 1024),
             "dispatches": len(_pick(fetch, args.kernel))}
    entry["bytes"] = entry["read_bytes"] + entry["written_bytes"]
    data = json.load(open(DATA)) if os.path.exists(DATA) else {}
    data[_key(args.kernel, args.workload, args.layout)] = entry
    os.makedirs(os.path.dirname(DATA), exist_ok=True)
    json.dump(data, open(DATA, "w"), indent=1, sort_keys=True)
    print(json.dumps(entry))


if __name__ == "__main__":
    main()
