"""Per-kernel HBM bytes from two hardware-counter runs of ``traffic_probe``.

    rocprofv3 --pmc FETCH_SIZE -d OUT/fetch -o run -- paper_2507_17307_amd/traffic_probe m7 2 6
    rocprofv3 --pmc WRITE_SIZE -d OUT/write -o run -- paper_2507_17307_amd/traffic_probe m7 2 6
    python -m paper_2507_17307_amd.pmc_summary OUT/fetch/run_results.db OUT/write/run_results.db

Each counter (KiB per dispatch) is scaled by what the same counter reads for the
probe's copy kernel, which moves exactly 2^28 bytes each way per launch.
"""
from __future__ import annotations

import collections
import sqlite3
import statistics
import sys

COPY_BYTES = 1 << 28


def per_kernel(db_path: str) -> dict:
    cur = sqlite3.connect(db_path).cursor()
    out = collections.defaultdict(list)
    for name, value in cur.execute("select kernel_name, value from counters_collection"):
        out[name].append(value)
    return out


def main(argv) -> int:
    if len(argv) != 3:
        print(__doc__, file=sys.stderr)
        return 2
    fetch, write = per_kernel(argv[1]), per_kernel(argv[2])
    copy = [n for n in fetch if "k_probe_copy" in n]
    if not copy or copy[0] not in write:
        print("the copy kernel is missing from a run", file=sys.stderr)
        return 1
    f_scale = COPY_BYTES / statistics.mean(fetch[copy[0]])      # bytes per counter unit
    w_scale = COPY_BYTES / statistics.mean(write[copy[0]])
    print(f"copy kernel: FETCH_SIZE {statistics.mean(fetch[copy[0]]):.1f}, WRITE_SIZE {statistics.mean(write[copy[0]]):.1f} "
          f"per launch of {COPY_BYTES} bytes each way -> {f_scale:.1f} and {w_scale:.1f} bytes per unit "
          f"(a unit is nominally 1024 bytes)")
    print(f"{'kernel':64s} {'launches':>8s} {'fetched MB':>12s} {'written MB':>12s}")
    for name in sorted(fetch, key=lambda n: -statistics.mean(fetch[n])):
        if "rs::" not in name:
            continue
        fb = statistics.mean(fetch[name]) * f_scale / 1e6
        wb = statistics.mean(write.get(name, [0.0])) * w_scale / 1e6
        print(f"{name[:64]:64s} {len(fetch[name]):8d} {fb:12.3f} {wb:12.3f}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
