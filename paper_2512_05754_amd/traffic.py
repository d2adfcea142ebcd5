"""Book-keeping for the measured HBM-side traffic figures that bench.py reports as `roofline.traffic`.

The figures come from rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same
counter reads for a plain copy of known size) and are stored in profiles/traffic.json, one entry per
workload, together with a digest of the kernel sources they were measured with.  A figure whose digest
no longer matches the sources in the tree is STALE: bench.py then reports `traffic: null` and says why in
`traffic_source`, and `python -m paper_2512_05754_amd.traffic check` exits non-zero, so a kernel change
cannot silently keep an old measurement.

    python -m paper_2512_05754_amd.traffic check
    python -m paper_2512_05754_amd.traffic record <entry> <bytes_key> <fetch_raw_KiB> <write_raw_KiB>
                                                  <copy_fetch_raw_KiB> <copy_write_raw_KiB> <copy_KiB> <profile.md>
"""
from __future__ import annotations

import hashlib
import json
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
PATH = os.path.join(ROOT, "profiles", "traffic.json")

# kernel sources behind each kind of entry (the entry name's prefix before ':' picks the kind)
SOURCES = {
    "attention": ("usv_attn_bf16.hip", "usv_internal.h"),
    "raster": ("usv_attn_bf16.hip", "usv_internal.h"),
    "cubes": ("usv_attn_bf16.hip", "usv_internal.h"),
    "reorder": ("usv_reorder.hip", "usv_internal.h"),
    "merge": ("usv_merge.hip", "usv_internal.h"),
}


def kind_of(entry: str) -> str:
    return entry.split(":", 1)[0] if ":" in entry else "attention"


def source_digest(kind: str) -> str:
    h = hashlib.sha256()
    for name in SOURCES[kind]:
        with open(os.path.join(PKG_DIR, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _load() -> dict:
    try:
        with open(PATH) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def lookup(entry: str, key: str = "attn_hbm_bytes_per_launch"):
    """(bytes per launch or None, one-line provenance) for bench.py."""
    e = _load().get(entry)
    if not e or key not in e:
        return None, "no rocprofv3 measurement recorded for this workload"
    where = f"{e.get('source', 'profiles/traffic.json')} (kernel sources {e.get('kernel_digest', '?')}, tree at {e.get('commit', '?')})"
    if e.get("kernel_digest") != source_digest(kind_of(entry)):
        return None, "STALE, not reported: the kernel sources changed after " + where
    return e[key], where


def record(entry, key, fetch_raw, write_raw, copy_fetch_raw, copy_write_raw, copy_kib, profile):
    fs, ws = copy_kib / copy_fetch_raw, copy_kib / copy_write_raw
    fetch, write = fetch_raw * 1024 * fs, write_raw * 1024 * ws
    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except OSError:
        commit = ""
    data = _load()
    data[entry] = {
        key: int(fetch + write), "fetch_bytes": int(fetch), "write_bytes": int(write),
        "fetch_scale": round(fs, 4), "write_scale": round(ws, 4), "source": profile,
        "kernel_digest": source_digest(kind_of(entry)), "commit": commit or "unknown",
    }
    with open(PATH, "w") as f:
        json.dump(data, f, indent=1)
        f.write("\n")
    return data[entry]


def check() -> int:
    bad = 0
    for entry, e in sorted(_load().items()):
        ok = e.get("kernel_digest") == source_digest(kind_of(entry))
        print(f"{'ok   ' if ok else 'STALE'} {entry}: {e.get('source')} (digest {e.get('kernel_digest')}, now {source_digest(kind_of(entry))})")
        bad += not ok
    return 1 if bad else 0


if __name__ == "__main__":
    if len(sys.argv) >= 2 and sys.argv[1] == "check":
        sys.exit(check())
    if len(sys.argv) == 10 and sys.argv[1] == "record":
        a = sys.argv
        print(record(a[2], a[3], float(a[4]), float(a[5]), float(a[6]), float(a[7]), float(a[8]), a[9]))
        sys.exit(0)
    print(__doc__)
    sys.exit(2)
