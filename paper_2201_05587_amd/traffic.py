"""HBM traffic per kernel launch from rocprofv3 counters, calibrated with a plain copy.

Usage (on a GPU machine, from the repository root; each counter needs a run of its own)::

    rocprofv3 --pmc FETCH_SIZE -d OUT/fetch -o run --output-format csv -- python3 bench.py --no-cpu-baseline --steps 3 --warmup 1
    rocprofv3 --pmc WRITE_SIZE -d OUT/write -o run --output-format csv -- python3 bench.py --no-cpu-baseline --steps 3 --warmup 1
    rocprofv3 --pmc FETCH_SIZE -d OUT/copy_fetch -o run --output-format csv -- python3 -m paper_2201_05587_amd.traffic copy
    rocprofv3 --pmc WRITE_SIZE -d OUT/copy_write -o run --output-format csv -- python3 -m paper_2201_05587_amd.traffic copy
    python3 -m paper_2201_05587_amd.traffic summarise OUT cfg5

Any other counters (matrix-core utilisation, LDS conflicts, latencies) of the same command are tabulated
per kernel symbol with ``python3 -m paper_2201_05587_amd.traffic counters OUT/<run> [OUT/<run> ...]``.

``copy`` launches a device-to-device copy of a known size, so the counters' unit
can be checked against bytes that certainly crossed HBM: the calibration
factor is known bytes / counter reading.  ``summarise`` averages each counter
over the dispatches of every contraction kernel symbol, scales by the factor
and writes ``tuned/traffic_<workload>.json`` together with a digest of the
kernel sources; ``bench.py`` reports the figure only while the digest still
matches the sources the library was built from.
"""
from __future__ import annotations

import csv
import glob
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
COPY_BYTES = 256 << 20
COPY_LAUNCHES = 6
COPY_KERNEL_HINT = ("elementwise", "copy")  # the kernels a tensor copy turns into


def source_digest() -> str:
    """SHA-256 over the sources the kernels are built from."""
    h = hashlib.sha256()
    csrc = os.path.join(HERE, "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h", ".cpp", ".py")) or name == "Makefile":
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()


def run_copy() -> None:
    import torch
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(COPY_LAUNCHES):
        dst.copy_(src)
    torch.cuda.synchronize()
    assert int(dst[-1]) == 3


def _rows(directory: str):
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise FileNotFoundError(f"no counter_collection.csv under {directory}")
    for path in files:
        with open(path) as f:
            yield from csv.DictReader(f)


def _symbol(name: str) -> str:
    name = name.strip()
    if name.startswith("void "):
        name = name[5:]
    name = name.replace("(anonymous namespace)::", "")
    for args in ("(tt::ContractArgs", "(tt::DwArgs"):
        cut = name.find(args)
        if cut >= 0:
            return name[:cut]
    return name


def per_symbol_kib(directory: str, counter: str) -> dict:
    """symbol -> (mean counter value per dispatch, dispatches)."""
    acc = {}
    for r in _rows(directory):
        if r["Counter_Name"] != counter:
            continue
        s = _symbol(r["Kernel_Name"])
        tot, n = acc.get(s, (0.0, 0))
        acc[s] = (tot + float(r["Counter_Value"]), n + 1)
    return {s: (tot / n, n) for s, (tot, n) in acc.items()}


def copy_factor(directory: str, counter: str) -> float:
    """Known bytes of the copy / what the counter read for it (bytes per counter unit).

    The copy's dispatches are the COPY_LAUNCHES largest readings among the copy-like kernels (the
    process also makes a small fill and a tiny read-back); their median is the reading of one copy.
    """
    values = sorted((float(r["Counter_Value"]) for r in _rows(directory)
                     if r["Counter_Name"] == counter and any(h in r["Kernel_Name"].lower() for h in COPY_KERNEL_HINT)),
                    reverse=True)[:COPY_LAUNCHES]
    if len(values) < COPY_LAUNCHES or values[-1] <= 0:
        raise RuntimeError(f"copy kernel not found in {directory}")
    return COPY_BYTES / values[len(values) // 2]


def summarise(out_dir: str, workload: str) -> str:
    f_fetch = copy_factor(os.path.join(out_dir, "copy_fetch"), "FETCH_SIZE")
    f_write = copy_factor(os.path.join(out_dir, "copy_write"), "WRITE_SIZE")
    fetch = per_symbol_kib(os.path.join(out_dir, "fetch"), "FETCH_SIZE")
    write = per_symbol_kib(os.path.join(out_dir, "write"), "WRITE_SIZE")
    kernels = {}
    for s in sorted(set(fetch) & set(write)):
        if "tt::" not in s:
            continue
        kernels[s] = dict(fetch_bytes_per_launch=fetch[s][0] * f_fetch, write_bytes_per_launch=write[s][0] * f_write,
                          dispatches=fetch[s][1])
    doc = dict(workload=workload, source_digest=source_digest(), copy_bytes=COPY_BYTES,
               bytes_per_unit=dict(FETCH_SIZE=f_fetch, WRITE_SIZE=f_write), kernels=kernels)
    path = os.path.join(HERE, "tuned", f"traffic_{workload}.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")
    mirror = os.path.join(os.path.dirname(HERE), "gpurun_out", "tuned")
    if os.path.isdir(os.path.dirname(mirror)):
        os.makedirs(mirror, exist_ok=True)
        with open(os.path.join(mirror, os.path.basename(path)), "w") as f:
            json.dump(doc, f, indent=1)
            f.write("\n")
    return path


def lookup(workload: str, symbol: str):
    """Measured HBM bytes per launch of `symbol`, or None if never measured or measured on other sources."""
    path = os.path.join(HERE, "tuned", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        doc = json.load(f)
    if doc.get("source_digest") != source_digest() or symbol not in doc.get("kernels", {}):
        return None
    k = doc["kernels"][symbol]
    return k["fetch_bytes_per_launch"] + k["write_bytes_per_launch"]


def counters_table(directories) -> str:
    """Per kernel symbol of this library: the mean of every counter found under the given output
    directories (one rocprofv3 --pmc run each), and the number of dispatches it was averaged over."""
    acc = {}
    names = []
    for d in directories:
        for r in _rows(d):
            s = _symbol(r["Kernel_Name"])
            if "tt::" not in s or "probe_" in s:
                continue
            c = r["Counter_Name"]
            if c not in names:
                names.append(c)
            tot, n = acc.setdefault(s, {}).get(c, (0.0, 0))
            acc[s][c] = (tot + float(r["Counter_Value"]), n + 1)
    lines = ["# symbol | dispatches | " + " | ".join(names)]
    for s in sorted(acc, key=lambda s: -max(n for _, n in acc[s].values())):
        n = max(n for _, n in acc[s].values())
        cells = [f"{acc[s][c][0] / acc[s][c][1]:.4g}" if c in acc[s] else "-" for c in names]
        lines.append(f"{s.replace('tt::', '')} | {n} | " + " | ".join(cells))
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    if len(sys.argv) >= 2 and sys.argv[1] == "copy":
        run_copy()
    elif len(sys.argv) >= 3 and sys.argv[1] == "counters":
        sys.stdout.write(counters_table(sys.argv[2:]))
    elif len(sys.argv) >= 4 and sys.argv[1] == "summarise":
        print(summarise(sys.argv[2], sys.argv[3]))
    else:
        print(__doc__)
        sys.exit(2)
