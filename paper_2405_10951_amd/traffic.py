"""Turn two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE; both with
--calibrate-copy) into the HBM bytes per GEMM launch that bench.py reports as roofline.traffic.

    python -m paper_2405_10951_amd.traffic <fetch_counter_collection.csv> <write_counter_collection.csv> [steps] [workload/batchN]

Only the GEMM launches of the last `steps` steps count (default 7 = 1 warm-up + 3 timed + 3 bracketed steps
of `bench.py --steps 3 --warmup 1`): the tile-tuning passes before them launch other tile shapes.

Each counter is scaled by what it reads for the plain 256 MiB copy kernel of the same run (the
counters are in KiB per dispatch; the copy reads 256 MiB and writes 256 MiB).  Writes
profiles/gemm_traffic.json together with a hash of the GEMM source, so that the figure is dropped
once the kernel changes."""
from __future__ import annotations

import csv
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 256 << 20


def per_kernel(path: str, counter: str, last_steps: int):
    """Counter values of the GEMM dispatches of the last `last_steps` steps (a step starts at its
    patchify dispatch: what runs before them is set-up, e.g. the tile tuning passes) and of the copies."""
    rows = []
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                rows.append((int(r["Dispatch_Id"]), r["Kernel_Name"], float(r["Counter_Value"])))
    rows.sort()
    starts = [i for i, r in enumerate(rows) if "patchify" in r[1]]
    first = starts[-last_steps] if 0 < last_steps <= len(starts) else 0
    gemm = [v for _, n, v in rows[first:] if "gemm_nt_kernel" in n or "gemm_ntd_kernel" in n or "gemm_tn_kernel" in n]
    copy = [v for _, n, v in rows if "copybuffer" in n.lower()]    # the runtime's plain device-to-device copy kernel
    return gemm, copy


def main(fetch_csv: str, write_csv: str, last_steps: int = 7, key: str = "c3_vit_b/batch32") -> None:
    gf, cf = per_kernel(fetch_csv, "FETCH_SIZE", last_steps)
    gw, cw = per_kernel(write_csv, "WRITE_SIZE", last_steps)
    if not (gf and gw and cf and cw):
        sys.exit("counter files lack GEMM or copy-kernel rows")
    # the calibration copy is the largest copy dispatch of the run
    scale_f = COPY_BYTES / max(cf)
    scale_w = COPY_BYTES / max(cw)
    fetch = sum(gf) / len(gf) * scale_f
    write = sum(gw) / len(gw) * scale_w
    with open(os.path.join(ROOT, "paper_2405_10951_amd", "csrc", "k_gemm_mfma.hip"), "rb") as f:
        sha = hashlib.sha256(f.read()).hexdigest()
    rec = {"hbm_bytes_per_launch": fetch + write, "fetch_bytes_per_launch": fetch,
           "write_bytes_per_launch": write, "gemm_launches_counted": len(gf),
           "copy_fetch_counter_KiB": max(cf), "copy_write_counter_KiB": max(cw),
           "bytes_per_counter_unit_fetch": scale_f, "bytes_per_counter_unit_write": scale_w,
           "kernel_source_sha256": sha}
    out = os.path.join(ROOT, "profiles", "gemm_traffic.json")
    try:
        with open(out) as f:
            allrec = json.load(f)
        if "records" not in allrec:
            allrec = {"records": {}}
    except (OSError, ValueError):
        allrec = {"records": {}}
    allrec["records"][key] = rec          # one record per workload and batch: bench.py looks its own up
    with open(out, "w") as f:
        json.dump(allrec, f, indent=1)
    print(json.dumps(rec))


if __name__ == "__main__":
    main(sys.argv[1], sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 7,
         sys.argv[4] if len(sys.argv) > 4 else "c3_vit_b/batch32")
