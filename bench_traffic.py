#!/usr/bin/env python3
"""Turns rocprofv3 byte-counter runs of bench.py into profiles/hbm_traffic.json and profiles/hbm_traffic_pmc.md.

The runs (on the GPU machine, from /tmp with TMPDIR=/tmp; one call and one counter per run, so that every
dispatch after the copy probe belongs to the call that is named):

    for CALL in select_reuse attend_reuse ...; do for C in FETCH_SIZE WRITE_SIZE; do
      rocprofv3 --pmc $C --output-format csv -d OUT/$C/$CALL -o p -- \\
          python3 bench.py --calls $CALL --steps 3 --warmup 1 --no-warm --copy-probe
    done; done

then, anywhere:   python3 bench_traffic.py OUT

`--copy-probe` makes bench.py run one plain elementwise launch of known size (dst = src + 1 on 2^28 int32:
reads 1 GiB, writes 1 GiB) right before the call's launches.  The counters are in KiB per dispatch; each is
scaled by what it reads for that launch.  A kernel's figure is the mean over the three timed launches.
bench.py loads the JSON file for its `roofline.traffic` fields; tests/test_bench_contract.py checks that
the JSON file and the summary agree.
"""
from __future__ import annotations

import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
STEPS = 3
PROBE_BYTES = float(1 << 30)
COUNTERS = ("FETCH_SIZE", "WRITE_SIZE")


def short(name: str) -> str:
    return name.split("(")[0].replace("void ", "").replace("dllm::", "").strip()


def read_run(path: str, counter: str):
    """-> (probe KiB, {kernel: (grid, mean KiB of the last STEPS launches after the probe)})"""
    files = glob.glob(os.path.join(path, "**", "*counter_collection.csv"), recursive=True)
    if len(files) != 1:
        raise SystemExit(f"{path}: expected one counter_collection.csv, found {len(files)}")
    rows = [r for r in csv.DictReader(open(files[0])) if r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    # the probe is torch's elementwise add over 2^28 int32 (the only add functor bench.py launches)
    big = [i for i, r in enumerate(rows)
           if "elementwise" in r["Kernel_Name"] and "Functor" in r["Kernel_Name"] and "_add" in r["Kernel_Name"]
           and int(r["Grid_Size"]) >= 1 << 24]
    if not big:
        raise SystemExit(f"{path}: no copy-probe launch found (run bench.py with --copy-probe)")
    probe = float(rows[big[-1]]["Counter_Value"])
    per = {}
    for r in rows[big[-1] + 1:]:
        if "dllm::" not in r["Kernel_Name"]:
            continue
        k = short(r["Kernel_Name"])
        grid = f'{int(r["Grid_Size"]) // int(r["Workgroup_Size"])} x {r["Workgroup_Size"]}'
        per.setdefault(k, (grid, []))[1].append(float(r["Counter_Value"]))
    return probe, {k: (g, sum(v[-STEPS:]) / len(v[-STEPS:])) for k, (g, v) in per.items()}


def algorithmic_bytes():
    """per call: (description, bytes) from the workload generators (no GPU needed)"""
    sys.path.insert(0, ROOT)
    from paper_2512_17077_amd import synth
    w3, w4, w5 = synth.config(3), synth.config(4), synth.config(5)
    e, d = 2, 128
    dense4 = 4 * w4.total_kv * w4.n_q_heads * d * e            # Q, K, V once each + O
    nd = int((w5.seq_mode == 1).sum()) * int(w5.kv_lens[w5.seq_mode == 1][0])
    dense5 = nd * (2 * w5.n_q_heads + 2 * w5.n_kv_heads) * d * e   # Q and O of 32 heads, K and V of 8
    return {
        "select_reuse": ("whole call", w3.select_bytes()),
        "attend_reuse": ("", w3.attend_sparse_bytes()),
        "attend_shared_list_reuse": ("", w3.attend_sparse_bytes()),
        "pack_reuse": ("", w3.pack_bytes()),
        "attend_packed_reuse": ("", w3.attend_packed_bytes()),
        "dense_refresh": ("Q, K, V once each + O", dense4),
        "select_mixed": ("whole call", w5.select_bytes()),
        "attend_mixed": ("sparse part per head + dense part with K, V of 8 heads", w5.attend_sparse_bytes() + dense5),
        "attend_mixed_reuse_part_alone": ("per-head rows", w5.attend_sparse_bytes()),
        "attend_mixed_refresh_part_alone": ("Q and O of 32 heads, K and V of 8", dense5),
    }


def main():
    if len(sys.argv) != 2:
        raise SystemExit(__doc__)
    out_dir = sys.argv[1]
    calls = sorted(os.path.basename(p) for p in glob.glob(os.path.join(out_dir, COUNTERS[0], "*")) if os.path.isdir(p))
    if not calls:
        raise SystemExit(f"no runs under {out_dir}/{COUNTERS[0]}/")
    data = {"steps": STEPS, "probe_bytes_read": PROBE_BYTES, "probe_bytes_written": PROBE_BYTES, "probe_kib": {}, "calls": {}}
    probes = {c: [] for c in COUNTERS}
    raw = {}
    for call in calls:
        raw[call] = {}
        for c in COUNTERS:
            probe, per = read_run(os.path.join(out_dir, c, call), c)
            probes[c].append(probe)
            raw[call][c] = per
    factor = {}
    for c in COUNTERS:
        mean = sum(probes[c]) / len(probes[c])
        data["probe_kib"][c] = mean
        factor[c] = PROBE_BYTES / 1024.0 / mean
    data["factor"] = factor
    for call in calls:
        data["calls"][call] = {}
        for k, (grid, fetch) in raw[call]["FETCH_SIZE"].items():
            write = raw[call]["WRITE_SIZE"].get(k, (grid, 0.0))[1]
            data["calls"][call][k] = {"grid": grid, "fetch_kib": round(fetch, 1), "write_kib": round(write, 1),
                                      "read_bytes": round(fetch * 1024.0 * factor["FETCH_SIZE"]),
                                      "write_bytes": round(write * 1024.0 * factor["WRITE_SIZE"])}
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    with open(os.path.join(ROOT, "profiles", "hbm_traffic.json"), "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")
    alg = algorithmic_bytes()
    md = ["# HBM traffic per launch from rocprofv3 byte counters (MI355X)\n",
          "Commands (one call and one counter per run; from /tmp with TMPDIR=/tmp; OUT is any scratch folder):\n",
          "    for CALL in " + " ".join(calls) + "; do for C in FETCH_SIZE WRITE_SIZE; do",
          "      rocprofv3 --pmc $C --output-format csv -d OUT/$C/$CALL -o p -- python3 bench.py --calls $CALL --steps 3 --warmup 1 --no-warm --copy-probe",
          "    done; done",
          "    python3 bench_traffic.py OUT        # writes this file and profiles/hbm_traffic.json, which bench.py loads\n",
          "`--copy-probe` adds one plain elementwise launch of known size (`dst = src + 1` on 2^28 int32: reads 1 GiB, writes 1 GiB) "
          "right before the call's launches. The counters are in KiB per dispatch; each is scaled by what it reads for that launch. "
          "Means over the 3 timed launches of each call.\n",
          f"Copy probe: FETCH_SIZE reads {data['probe_kib']['FETCH_SIZE']:.0f} KiB for 1048576 KiB read -> factor {factor['FETCH_SIZE']:.3f}; "
          f"WRITE_SIZE reads {data['probe_kib']['WRITE_SIZE']:.0f} KiB for 1048576 KiB written -> factor {factor['WRITE_SIZE']:.3f}.\n",
          "| call | kernel (workgroups x threads) | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled read MB | scaled write MB | algorithmic MB of the call |",
          "|---|---|---|---|---|---|---|"]
    for call in calls:
        first = True
        for k, t in data["calls"][call].items():
            a = alg.get(call)
            note = f"{a[1] / 1e6:.1f}" + (f" ({a[0]})" if a[0] else "") if (a and first) else ""
            md.append(f"| {call} | {k} ({t['grid']}) | {t['fetch_kib']:.0f} | {t['write_kib']:.0f} | {t['read_bytes'] / 1e6:.1f} | "
                      f"{t['write_bytes'] / 1e6:.1f} | {note} |")
            first = False
    notes_path = os.path.join(ROOT, "profiles", "hbm_traffic_notes.md")
    md.append("")
    with open(os.path.join(ROOT, "profiles", "hbm_traffic_pmc.md"), "w") as f:
        f.write("\n".join(md))
        if os.path.exists(notes_path):
            f.write("\n" + open(notes_path).read())
    print(f"wrote profiles/hbm_traffic.json and profiles/hbm_traffic_pmc.md ({len(calls)} calls)")


if __name__ == "__main__":
    main()
