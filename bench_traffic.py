"""Turn two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE) of `bench.py --calibrate-copy`
into the HBM-traffic figure that bench.py reports for the dominant attention kernel.

    python bench_traffic.py <fetch_dir> <write_dir> <out.md> [kernel-substring]

Each directory holds rocprofv3's *_counter_collection.csv.  The counters (KiB per dispatch) are
scaled by what the same counter reads for the plain copy kernel of known size that bench.py runs
first (`--calibrate-copy`: a 1 GiB device-to-device copy, i.e. 1 GiB fetched and 1 GiB written).
The result is written as a small markdown file with one machine-readable line

    TRAFFIC_JSON {"kernel": ..., "bytes_per_launch": ..., "source_sha256": ...}

which bench.py picks up as `roofline.traffic` as long as the kernel source still has that hash.
"""
from __future__ import annotations

import csv
import glob
import hashlib
import json
import os
import sys

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2505_01068_amd")
COPY_BYTES = 1 << 30
KERNEL_SOURCES = {"mfma_": ["csrc/mfma_attn.hip", "csrc/mfma_common.hpp", "csrc/common.hpp"],
                  "rowlane_": ["csrc/attn_rowlane.hip", "csrc/common.hpp"]}


def source_hash(kernel_name: str) -> str:
    """sha256 over the sources the named kernel is compiled from ("" if unknown)."""
    for key, rels in KERNEL_SOURCES.items():
        if key in kernel_name:
            h = hashlib.sha256()
            for rel in rels:
                h.update(open(os.path.join(HERE, rel), "rb").read())
            return h.hexdigest()
    return ""


def read_counter(directory: str, counter: str):
    """{kernel name: [values per dispatch]} for one counter."""
    out = {}
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] == counter:
                out.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return out


def pick(d, substr):
    hits = {k: v for k, v in d.items() if substr in k}
    if not hits:
        raise SystemExit(f"no kernel matching {substr!r}")
    k = max(hits, key=lambda n: len(hits[n]))
    return k, hits[k]


def main(argv):
    fetch_dir, write_dir, out_md = argv[1:4]
    substr = argv[4] if len(argv) > 4 else "mfma_dkv_kernel"
    fetch, write = read_counter(fetch_dir, "FETCH_SIZE"), read_counter(write_dir, "WRITE_SIZE")
    # the calibration copy is the elementwise copy kernel with the largest reading
    def copy_reading(d):
        cands = {k: max(v) for k, v in d.items() if "copy" in k.lower() or "elementwise" in k.lower()}
        k = max(cands, key=cands.get)
        return k, cands[k]
    ck_f, cf = copy_reading(fetch)
    ck_w, cw = copy_reading(write)
    kf, vf = pick(fetch, substr)
    kw, vw = pick(write, substr)
    f_scale, w_scale = COPY_BYTES / cf, COPY_BYTES / cw      # bytes per counter unit
    f_bytes = sum(vf) / len(vf) * f_scale
    w_bytes = sum(vw) / len(vw) * w_scale
    rec = {"kernel": kf.split("(")[0], "fetch_bytes_per_launch": round(f_bytes), "write_bytes_per_launch": round(w_bytes),
           "bytes_per_launch": round(f_bytes + w_bytes), "launches_averaged": len(vf),
           "copy_kernel": ck_f.split("(")[0][:60], "fetch_scale_bytes_per_unit": round(f_scale, 2),
           "write_scale_bytes_per_unit": round(w_scale, 2), "source_sha256": source_hash(kf)}
    lines = [
        f"# HBM traffic of `{rec['kernel']}` from rocprofv3 counters",
        "",
        "FETCH_SIZE and WRITE_SIZE (one --pmc run each), scaled by the reading of the same counter for a 1 GiB",
        "device-to-device copy in the same run.",
        "",
        f"- copy kernel: `{rec['copy_kernel']}`: FETCH_SIZE {cf:.0f}, WRITE_SIZE {cw:.0f} per 1 GiB -> "
        f"{f_scale:.1f} / {w_scale:.1f} bytes per unit",
        f"- kernel: fetch {f_bytes / 1e6:.1f} MB, write {w_bytes / 1e6:.1f} MB per launch "
        f"(mean of {len(vf)} launches)",
        "",
        "Commands (TMPDIR=/tmp, from the repository root), then this module on the two directories:",
        "",
        "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch_dir> -o p -- python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --calibrate-copy",
        "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write_dir> -o p -- python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --calibrate-copy",
        "    python bench_traffic.py <fetch_dir> <write_dir> profiles/c5_attn_dkv_traffic.md mfma_dkv_kernel",
        "",
        "TRAFFIC_JSON " + json.dumps(rec),
        "",
    ]
    open(out_md, "w").write("\n".join(lines))
    print("\n".join(lines))


if __name__ == "__main__":
    main(sys.argv)
