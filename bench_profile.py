#!/usr/bin/env python3
"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

  kernel trace : python bench_profile.py trace  <dir with *_kernel_stats.csv>
  HBM traffic  : python bench_profile.py traffic <FETCH_SIZE run dir> <WRITE_SIZE run dir> [--json profiles/traffic.json]
                 [--workload NAME]   (the key in the JSON file; default llama128k; a workload of 167 772 160 packed bytes)
  counters     : python bench_profile.py counters <--pmc run dir> [<--pmc run dir> ...]
                 (per-dispatch means of every counter collected for the decode kernels, and what follows from them)

The traffic mode expects both runs to come from `bench.py --calibrate-copy`: the plain device copy of
known size in that run gives the factor between the counter's reading and real bytes.
"""
from __future__ import annotations

import csv
import glob
import json
import statistics
import sys

PARTIAL = "decode_partial_mfma_kernel"
COPY_KERNEL = "__amd_rocclr_copyBuffer"      # what torch's same-dtype device copy_ launches


def _rows(d, suffix):
    out = []
    for f in sorted(glob.glob(f"{d}/**/*{suffix}", recursive=True)):
        out += list(csv.DictReader(open(f)))
    return out


def trace(d):
    rows = _rows(d, "kernel_stats.csv")
    print(f"{'kernel':70s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>7s}")
    for r in rows:
        name = r["Name"]
        if "tq::" not in name and COPY_KERNEL not in name:
            continue
        name = name.replace("void tq::(anonymous namespace)::", "").replace("tq::(anonymous namespace)::", "")
        name = name.split("(")[0][:70]
        print(f"{name:70s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:10.2f} {float(r['MinNs']) / 1e3:10.2f} "
              f"{float(r['MaxNs']) / 1e3:10.2f} {float(r['Percentage']):7.2f}")


def _counter(d, counter):
    vals = {}
    for r in _rows(d, "counter_collection.csv"):
        if r["Counter_Name"] == counter:
            vals.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return vals


def traffic(fetch_dir, write_dir, json_path=None, workload="llama128k", known_bytes=167772160):
    out = {}
    for label, d, counter in (("read", fetch_dir, "FETCH_SIZE"), ("write", write_dir, "WRITE_SIZE")):
        vals = _counter(d, counter)
        copy = [v for k, vs in vals.items() if COPY_KERNEL in k for v in vs if v * 1024 > 0.25 * known_bytes]
        part = [v for k, vs in vals.items() if PARTIAL in k for v in vs]
        part = part[len(part) // 4:]
        copy_kib, part_kib = statistics.median(copy), statistics.fmean(part)
        factor = known_bytes / (copy_kib * 1024)
        out[label] = {"counter": counter, "copy_reading_KiB": copy_kib, "copy_true_bytes": known_bytes,
                      "factor": factor, "partial_reading_KiB": part_kib, "partial_bytes": part_kib * 1024 * factor}
        print(f"{counter}: plain copy of {known_bytes} B reads {copy_kib:.0f} KiB -> factor {factor:.3f}; "
              f"partial kernel reads {part_kib:.0f} KiB per dispatch -> {part_kib * 1024 * factor / 1e6:.2f} MB")
    total = out["read"]["partial_bytes"] + out["write"]["partial_bytes"]
    print(f"HBM traffic of the partial kernel: {total / 1e6:.2f} MB per launch "
          f"(algorithmic {known_bytes / 1e6:.2f} MB packed int4 + scales + zero-points)")
    if json_path:
        try:
            cur = json.load(open(json_path))
        except Exception:
            cur = {}
        cur[workload] = {"read_bytes": round(out["read"]["partial_bytes"]), "write_bytes": round(out["write"]["partial_bytes"]),
                         "total_bytes": round(total), "read_factor": round(out["read"]["factor"], 4),
                         "write_factor": round(out["write"]["factor"], 4), "unit": "bytes per launch of the partial kernel"}
        json.dump(cur, open(json_path, "w"), indent=1)
        print(f"wrote {json_path}")


def counters(dirs):
    """Per-dispatch means of the counters of the decode kernels (first quarter of the dispatches dropped: warm-up)."""
    acc = {}
    for d in dirs:
        for r in _rows(d, "counter_collection.csv"):
            k = r["Kernel_Name"]
            if "decode_partial" not in k:
                continue
            name = "decode_partial" + k.split("decode_partial")[1].split("(")[0]
            acc.setdefault(name, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    for name, cs in acc.items():
        m = {c: statistics.fmean(v[len(v) // 4:]) for c, v in cs.items()}
        print(f"kernel {name}  ({len(next(iter(cs.values())))} dispatches)")
        for c in sorted(m):
            print(f"  {c:30s} {m[c]:16.1f}")
        w = m.get("SQ_WAVES")
        if w:
            simds = 1024.0                                 # 256 compute units x 4
            print(f"  -- per wave: VALU instructions {m.get('SQ_INSTS_VALU', 0) / w:.0f} (of which matrix {m.get('SQ_INSTS_MFMA', 0) / w:.0f}), "
                  f"scalar {m.get('SQ_INSTS_SALU', 0) / w:.0f}, LDS {m.get('SQ_INSTS_LDS', 0) / w:.0f}, vector memory {m.get('SQ_INSTS_VMEM_RD', 0) / w:.0f}")
            if "SQ_WAVE_CYCLES" in m and "SQ_ACTIVE_INST_VALU" in m:
                # SQ_WAVE_CYCLES and SQ_ACTIVE_INST_* count in units of 4 cycles, summed over waves / SIMDs
                wave_q = m["SQ_WAVE_CYCLES"] / w
                print(f"  -- a wave lives {4 * wave_q:.0f} cycles; its SIMD's vector ALU is busy {100 * (m['SQ_ACTIVE_INST_VALU'] / simds) / wave_q:.0f} % "
                      f"of that; matrix cores busy {100 * (m.get('SQ_VALU_MFMA_BUSY_CYCLES', 0) / simds) / (4 * wave_q):.0f} %; "
                      f"waves waiting on any counter {100 * m.get('SQ_WAIT_INST_ANY', 0) / m['SQ_WAVE_CYCLES']:.0f} % of their time")
            if "SQ_LDS_BANK_CONFLICT" in m and m.get("SQ_LDS_IDX_ACTIVE"):
                print(f"  -- LDS bank-conflict cycles / LDS active cycles: {100 * m['SQ_LDS_BANK_CONFLICT'] / m['SQ_LDS_IDX_ACTIVE']:.0f} %")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "trace":
        trace(sys.argv[2])
    elif len(sys.argv) >= 3 and sys.argv[1] == "counters":
        counters(sys.argv[2:])
    elif len(sys.argv) >= 4 and sys.argv[1] == "traffic":
        jp = sys.argv[sys.argv.index("--json") + 1] if "--json" in sys.argv else None
        wl = sys.argv[sys.argv.index("--workload") + 1] if "--workload" in sys.argv else "llama128k"
        traffic(sys.argv[2], sys.argv[3], jp, workload=wl)
    else:
        sys.exit(__doc__)
