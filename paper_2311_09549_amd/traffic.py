"""HBM traffic of a kernel from hardware counters, calibrated against a copy of known size.

Two `rocprofv3 --pmc` runs of `bench.py --calibrate-copy` (one collecting FETCH_SIZE, one
WRITE_SIZE, both in KiB per dispatch) hold, next to the kernel of interest, dispatches of the
library's plain copy kernel, which reads and writes a known number of bytes.  The ratio of
what a counter reads for the copy to the copy's true size turns the kernel's counter value
into bytes.  The result is stored with a digest of the kernel sources; `lookup` returns it
only while the sources are unchanged.

Usage (from the repository root, after the two counter runs):

    python3 -m paper_2311_09549_amd.traffic <dir of the FETCH_SIZE run> <dir of the WRITE_SIZE run> \\
        --kernel mttkrp3_fused_kernel --key 2:mttkrp3_fused --out paper_2311_09549_amd/traffic.json
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT_PATH = os.path.join(HERE, "traffic.json")
COPY_KERNEL = "stream_copy_kernel"
COPY_BYTES = 1 << 30  # size of the calibration copy bench.py queues (well beyond the 256 MB last-level cache)


def source_digest() -> str:
    """sha256 over the kernel and host sources the library is built from."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(HERE, "csrc", "*")))
    files.append(os.path.join(HERE, "..", "include", "sparsecontract.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _per_dispatch_mean(run_dir: str, counter: str, kernel_substr: str) -> float:
    """Mean over dispatches of `counter` (summed over the chip's instances) for kernels whose
    name contains `kernel_substr`."""
    per = {}
    for f in glob.glob(os.path.join(run_dir, "**", "*counter_collection.csv"), recursive=True):
        with open(f, newline="") as fh:
            for row in csv.DictReader(fh):
                if row["Counter_Name"] != counter or kernel_substr not in row["Kernel_Name"]:
                    continue
                key = (f, row["Dispatch_Id"])
                per[key] = per.get(key, 0.0) + float(row["Counter_Value"])
    if not per:
        raise SystemExit(f"no {counter} rows for a kernel named *{kernel_substr}* under {run_dir}")
    return sum(per.values()) / len(per)


def lookup(key: str, path: str = DEFAULT_PATH):
    """Stored traffic record for `key` ("<config id>:<launch name>"), or None when there is
    none or the sources changed after the counters were taken."""
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        rec = json.load(fh)
    ent = rec.get("entries", {}).get(key)
    if ent is None or ent.get("source_sha256") != source_digest():
        return None
    return ent


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("fetch_dir")
    ap.add_argument("write_dir")
    ap.add_argument("--kernel", required=True, help="substring of the profiled kernel's name")
    ap.add_argument("--key", required=True, help='"<config id>:<launch name>" as bench.py reports it')
    ap.add_argument("--out", default=DEFAULT_PATH)
    ap.add_argument("--mfma-dir", default=None,
                    help="directory of a third counter run (SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_MFMA): "
                         "stores the matrix cores' busy fraction of the kernel")
    a = ap.parse_args()
    kib = 1024.0
    k_fetch = _per_dispatch_mean(a.fetch_dir, "FETCH_SIZE", a.kernel) * kib
    k_write = _per_dispatch_mean(a.write_dir, "WRITE_SIZE", a.kernel) * kib
    c_fetch = _per_dispatch_mean(a.fetch_dir, "FETCH_SIZE", COPY_KERNEL) * kib
    c_write = _per_dispatch_mean(a.write_dir, "WRITE_SIZE", COPY_KERNEL) * kib
    f_fetch, f_write = c_fetch / COPY_BYTES, c_write / COPY_BYTES
    ent = {
        "kernel": a.kernel, "fetch_counter_bytes": k_fetch, "write_counter_bytes": k_write,
        "copy_bytes": COPY_BYTES, "copy_fetch_counter_bytes": c_fetch, "copy_write_counter_bytes": c_write,
        "fetch_factor": f_fetch, "write_factor": f_write,
        "hbm_read_bytes": k_fetch / f_fetch, "hbm_write_bytes": k_write / f_write,
        "hbm_bytes": k_fetch / f_fetch + k_write / f_write,
        "source_sha256": source_digest(),
    }
    if a.mfma_dir:
        # busy cycles of the matrix pipes summed over the four SIMDs of every CU, over the CUs' busy cycles
        busy = _per_dispatch_mean(a.mfma_dir, "SQ_VALU_MFMA_BUSY_CYCLES", a.kernel)
        cu = _per_dispatch_mean(a.mfma_dir, "SQ_BUSY_CU_CYCLES", a.kernel)
        ent["mfma_busy"] = busy / (4.0 * cu) if cu else None
        ent["mfma_instructions"] = _per_dispatch_mean(a.mfma_dir, "SQ_INSTS_MFMA", a.kernel)
    rec = {"entries": {}}
    if os.path.exists(a.out):
        with open(a.out) as fh:
            rec = json.load(fh)
    rec.setdefault("entries", {})[a.key] = ent
    with open(a.out, "w") as fh:
        json.dump(rec, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print(json.dumps(ent, indent=1))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
