"""HBM traffic per launch from profiler counters -> profiles/hbm_traffic_pmc.{json,md}.

Input: per workload, two directories written by rocprofv3 counter runs of `bench.py`
(one with FETCH_SIZE, one with WRITE_SIZE; rocprofv3 does not split counters over passes):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT_F -- python3 bench.py --workload W \
        --steps 5 --warmup 2 --no-cpu-baseline --no-lean-extra --no-configs --copy-probe-mib 1024
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT_W -- python3 bench.py (the same flags)

`--copy-probe-mib 1024` makes the same process run the library's stream probe as a plain copy of
known size (1 GiB read, 1 GiB written), which scales the counters (both are reported in KiB per
dispatch, FETCH_SIZE at half the bytes on this part).

    python -m paper_1810_08297_amd.pmc_traffic cfg3:OUT_F:OUT_W [cfg4:OUT_F:OUT_W ...]

The JSON holds, per workload and kernel role, the kernel's name and its HBM bytes per launch, and a
hash of the kernel sources it was measured on; `bench.py` reports these figures as `traffic` and
says whether the hash still matches the sources it runs.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import json
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
OUT_JSON = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.json")
OUT_MD = os.path.join(ROOT, "profiles", "hbm_traffic_pmc.md")


def source_hash() -> str:
    """sha256 over the library's sources (csrc/ and the public header), file names included."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(HERE, "csrc", "*")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def counter_means(directory, counter):
    """kernel name -> (mean counter value per dispatch, dispatches) from the newest CSV under `directory`
    (a directory that several runs wrote into holds one file per run)."""
    agg = collections.defaultdict(list)
    files = sorted(glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True), key=os.path.getmtime)
    for f in files[-1:]:
        with open(f, newline="") as fh:
            for r in csv.DictReader(fh):
                if r["Counter_Name"] == counter:
                    agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in agg.items()}


def role_of(kernel):
    if "stream_probe_kernel" in kernel:
        return "copy"
    if "fwd_tiled_kernel" in kernel or "fwd_generic_kernel" in kernel:
        return "forward"
    if "bwd_pass2_kernel" in kernel:
        return "second_pass"
    if "bwd_sig_kernel" in kernel or "bwd_tiled_kernel" in kernel or "bwdr_tiled_kernel" in kernel:
        return "backward"
    return None


def summarise(workload, dir_fetch, dir_write, copy_mib):
    fetch, write = counter_means(dir_fetch, "FETCH_SIZE"), counter_means(dir_write, "WRITE_SIZE")
    by_role = {}
    for k in set(fetch) | set(write):
        role = role_of(k)
        if role is None:
            continue
        if role in by_role:
            raise SystemExit(f"{workload}: two kernels in the role {role}: {by_role[role]['kernel'][:60]} and {k[:60]}")
        by_role[role] = {"kernel": k, "fetch_kib": fetch.get(k, (0.0, 0))[0], "write_kib": write.get(k, (0.0, 0))[0],
                         "dispatches": max(fetch.get(k, (0, 0))[1], write.get(k, (0, 0))[1])}
    if "copy" not in by_role:
        raise SystemExit(f"{workload}: no stream_probe_kernel dispatch found (run bench.py with --copy-probe-mib)")
    known_kib = copy_mib * 1024.0
    sf, sw = known_kib / by_role["copy"]["fetch_kib"], known_kib / by_role["copy"]["write_kib"]
    out = {"scale": {"fetch": sf, "write": sw, "copy_mib": copy_mib,
                     "copy_fetch_kib": by_role["copy"]["fetch_kib"], "copy_write_kib": by_role["copy"]["write_kib"]}}
    for role in ("forward", "backward", "second_pass"):
        if role not in by_role:
            continue
        r = by_role[role]
        r["read_bytes"] = r["fetch_kib"] * sf * 1024.0
        r["written_bytes"] = r["write_kib"] * sw * 1024.0
        r["traffic_bytes"] = r["read_bytes"] + r["written_bytes"]
        out[role] = r
    if "second_pass" in out and "backward" in out:  # the reverse step's traffic is both of its launches
        for key in ("read_bytes", "written_bytes", "traffic_bytes"):
            out["backward"][key] += out["second_pass"][key]
        out["backward"]["includes_second_pass"] = True
    return out


def main(argv):
    copy_mib = 1024
    table = {"source_hash": source_hash(), "workloads": {}}
    try:
        table["commit"] = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True,
                                         text=True).stdout.strip() or None
    except OSError:
        table["commit"] = None
    for spec in argv:
        workload, dir_fetch, dir_write = spec.split(":")
        table["workloads"][workload] = summarise(workload, dir_fetch, dir_write, copy_mib)
    with open(OUT_JSON, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    lines = ["# HBM traffic per launch from counters (rocprofv3 --pmc)", "",
             "Written by `python -m paper_1810_08297_amd.pmc_traffic` from two counter runs per workload W (on the MI355X box,",
             "from /tmp with TMPDIR=/tmp), one counter each:", "",
             "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -- python3 bench.py --workload W --steps 5 --warmup 2 --no-cpu-baseline --no-lean-extra --no-configs --copy-probe-mib 1024",
             "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -- python3 bench.py (the same flags)", "",
             f"`--copy-probe-mib {copy_mib}` runs `bd::stream_probe_kernel` as a plain copy of {copy_mib} MiB in the same process: the known",
             "size that scales the counters.  Mean counter value per dispatch in KiB; bytes after scaling.",
             f"Kernel sources at measurement: hash {table['source_hash']} (commit {table['commit']}).", ""]
    for wl, t in table["workloads"].items():
        lines += [f"## {wl}", "",
                  f"Scale from the copy: FETCH_SIZE x {t['scale']['fetch']:.5f}, WRITE_SIZE x {t['scale']['write']:.5f}.", "",
                  "| Kernel | dispatches | FETCH_SIZE KiB | WRITE_SIZE KiB | read MB | written MB | HBM traffic MB |", "|---|---|---|---|---|---|---|"]
        for role in ("forward", "backward", "second_pass"):
            if role in t:
                r = t[role]
                note = " (+ second pass)" if r.get("includes_second_pass") else ""
                lines.append(f"| {role}{note}: `{r['kernel'][:90]}` | {r['dispatches']} | {r['fetch_kib']:.0f} | {r['write_kib']:.0f} | "
                             f"{r['read_bytes'] / 1e6:.1f} | {r['written_bytes'] / 1e6:.1f} | {r['traffic_bytes'] / 1e6:.1f} |")
        lines.append("")
    with open(OUT_MD, "w") as f:
        f.write("\n".join(lines))
    print(f"wrote {OUT_JSON} and {OUT_MD}")


if __name__ == "__main__":
    main(sys.argv[1:])
