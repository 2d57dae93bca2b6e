#!/usr/bin/env python3
"""Turn raw rocprofv3 output of bench.py runs into the short text summaries kept
under profiles/ and into profiles/hbm_traffic.json (HBM bytes per launch of each
layer's kernel, which bench.py reports as roofline.traffic).

    python -m paper_1608_01409_amd.profile_summary RAW_DIR OUT_DIR

RAW_DIR holds one sub-directory per profiler run, named as in the header of the
kernel summary under profiles/: kt (kernel trace + stats), fetch (FETCH_SIZE),
write (WRITE_SIZE), sq1, sq2 (SQ counters), l2 (TCC request counters).  The byte
counters and the L2 request counters are scaled by what the same counter reads
for the plain device copy bench.py launches with --copy-probe-mb (a kernel that
moves a known number of bytes each way).
"""
from __future__ import annotations

import csv
import glob
import json
import os
import sys
from collections import defaultdict

LAYERS = ["conv2", "conv3", "conv4", "conv5"]
COPY_MB = 256


def find(raw, run, suffix):
    hits = glob.glob(os.path.join(raw, run, "**", f"*{suffix}"), recursive=True)
    return hits[0] if hits else None


def counters(raw, run):
    """{counter: {"layers": {layer: mean per launch}, "copy": value}} for one --pmc run."""
    path = find(raw, run, "counter_collection.csv")
    if not path:
        return {}
    rows = list(csv.DictReader(open(path)))
    per = defaultdict(lambda: defaultdict(list))   # counter -> dispatch -> values
    name = {}
    for r in rows:
        d = int(r["Dispatch_Id"])
        per[r["Counter_Name"]][d].append(float(r["Counter_Value"]))
        name[d] = r["Kernel_Name"]
    sconv = sorted(d for d, n in name.items() if "sconv_lds" in n or "sconv_direct" in n)
    copies = sorted(d for d, n in name.items() if "copy" in n.lower() or "elementwise" in n.lower())
    out = {}
    for c, by_d in per.items():
        lay = defaultdict(list)
        for i, d in enumerate(sconv):
            lay[LAYERS[i % len(LAYERS)]].append(sum(by_d.get(d, [0.0])))
        # the probe copy is the largest copy-like dispatch
        cp = max((sum(by_d.get(d, [0.0])) for d in copies), default=None)
        out[c] = {"layers": {k: sum(v) / len(v) for k, v in lay.items()}, "copy": cp, "launches": len(sconv)}
    return out


def main() -> int:
    raw, out_dir = sys.argv[1], sys.argv[2]
    os.makedirs(out_dir, exist_ok=True)
    lines = []
    kt = find(raw, "kt", "kernel_stats.csv")
    if kt:
        lines.append("kernel trace (rocprofv3 --kernel-trace --stats), all launches of bench.py's run")
        lines.append(f"{'kernel':70s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}")
        for r in csv.DictReader(open(kt)):
            lines.append(f"{r['Name'][:70]:70s} {r['Calls']:>6s} {float(r['AverageNs'])/1e3:9.2f} "
                         f"{float(r['MinNs'])/1e3:9.2f} {float(r['MaxNs'])/1e3:9.2f} {float(r['Percentage']):6.2f}")
        lines.append("")
    traffic = {}
    fetch, write = counters(raw, "fetch").get("FETCH_SIZE"), counters(raw, "write").get("WRITE_SIZE")
    if fetch and write and fetch["copy"] and write["copy"]:
        expect_kib = COPY_MB * 1024.0
        fs, ws = expect_kib / fetch["copy"], expect_kib / write["copy"]
        lines.append(f"HBM traffic per launch (FETCH_SIZE / WRITE_SIZE, KiB; scale factors from a {COPY_MB} MiB copy: "
                     f"read x{fs:.3f}, write x{ws:.3f})")
        for l in LAYERS:
            rd = fetch["layers"].get(l, 0.0) * fs * 1024.0
            wr = write["layers"].get(l, 0.0) * ws * 1024.0
            traffic[l] = {"read_bytes": round(rd), "write_bytes": round(wr), "bytes": round(rd + wr)}
            lines.append(f"  {l}: read {rd/1e6:8.1f} MB  write {wr/1e6:8.1f} MB")
        lines.append("")
        json.dump(traffic, open(os.path.join(out_dir, "hbm_traffic.json"), "w"), indent=1)
    for run in ("sq1", "sq2"):
        cs = counters(raw, run)
        if cs:
            lines.append(f"SQ counters per launch ({run})")
            for c in sorted(cs):
                lines.append(f"  {c:28s} " + "  ".join(f"{l} {cs[c]['layers'].get(l, 0):.4g}" for l in LAYERS))
            lines.append("")
    l2 = counters(raw, "l2")
    l2_read_bytes = {}
    if l2 and "TCC_READ_sum" in l2 and l2["TCC_READ_sum"]["copy"]:
        per_req = COPY_MB * 2.0 ** 20 / l2["TCC_READ_sum"]["copy"]
        lines.append(f"L2 (TCC) counters per launch; one read request = {per_req:.1f} B (from the {COPY_MB} MiB copy)")
        for c in sorted(l2):
            lines.append(f"  {c:28s} " + "  ".join(f"{l} {l2[c]['layers'].get(l, 0):.4g}" for l in LAYERS))
        for l in LAYERS:
            l2_read_bytes[l] = l2["TCC_READ_sum"]["layers"].get(l, 0.0) * per_req
        if "TCC_HIT_sum" in l2 and "TCC_MISS_sum" in l2:
            hr = {l: l2["TCC_HIT_sum"]["layers"].get(l, 0.0) /
                  max(1.0, l2["TCC_HIT_sum"]["layers"].get(l, 0.0) + l2["TCC_MISS_sum"]["layers"].get(l, 0.0)) for l in LAYERS}
            lines.append("  hit rate                     " + "  ".join(f"{l} {hr[l]:.1%}" for l in LAYERS))
        lines.append("")
    # rates derived from the counters, beside the ceilings measured by the microbenchmark
    # (`paper_1608_01409_amd/sconv_ceilings`: v_fma_f32 60 lanes-FMA/clk/CU, ds_read_b128 242 B/clk/CU, copy 4.9 TB/s)
    sq1, sq2 = counters(raw, "sq1"), counters(raw, "sq2")
    if sq1 and sq2 and "GRBM_GUI_ACTIVE" in sq1:
        lines.append("derived per layer (kernel cycles = GRBM_GUI_ACTIVE / 8 XCDs; SQ instruction counters are per wave, "
                     "x64 lanes; one LDS instruction of this kernel moves 1 KiB)")
        lines.append(f"  {'layer':6s} {'us@2.4GHz':>10s} {'FMA lanes/clk/CU':>17s} {'of 64':>6s} {'LDS B/clk/CU':>13s} {'VALU busy':>10s} "
                     f"{'HBM TB/s':>9s} {'L2 read TB/s':>13s} {'bank conflict cyc':>18s}")
        for l in LAYERS:
            cyc = sq1["GRBM_GUI_ACTIVE"]["layers"].get(l, 0.0) / 8.0
            if cyc <= 0:
                continue
            fma = sq2.get("SQ_INSTS_VALU_FMA_F32", {"layers": {}})["layers"].get(l, 0.0) * 64.0 / (cyc * 256.0)
            lds = sq2.get("SQ_INSTS_LDS", {"layers": {}})["layers"].get(l, 0.0) * 1024.0 / (cyc * 256.0)
            busy = sq1.get("SQ_ACTIVE_INST_VALU", {"layers": {}})["layers"].get(l, 0.0) * 4.0 / (cyc * 1024.0)
            hbm = traffic.get(l, {}).get("bytes", 0) / (cyc / 2.4e9) / 1e12 if traffic else 0.0
            bc = sq2.get("SQ_LDS_BANK_CONFLICT", {"layers": {}})["layers"].get(l, 0.0)
            l2bw = l2_read_bytes.get(l, 0.0) / (cyc / 2.4e9) / 1e12
            lines.append(f"  {l:6s} {cyc/2.4e3:10.1f} {fma:17.2f} {fma/64:6.1%} {lds:13.1f} {busy:10.1%} {hbm:9.2f} {l2bw:13.2f} {bc:18.0f}")
        lines.append("")
    text = "\n".join(lines)
    print(text)
    open(os.path.join(out_dir, "_summary_body.txt"), "w").write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
