#!/usr/bin/env python3
"""Turn raw rocprofv3 output of profile_run.py (or bench.py) runs into the short text summaries kept under
profiles/, and, for the alexnet configuration, into profiles/hbm_traffic.json (HBM bytes per launch of each
layer's kernel, which bench.py reports as roofline.traffic).

    python -m paper_1608_01409_amd.profile_summary RAW_DIR OUT_FILE [--traffic-json PATH]

RAW_DIR holds one sub-directory per profiler run: kt (kernel trace), fetch (FETCH_SIZE), write (WRITE_SIZE),
sq1, sq2 (SQ counters), l2 (TCC request counters), each with the profiler's CSV files and the log.json that
profile_run.py wrote for that run (which forward call launched which dispatches).  Dispatches are attributed to
layers from the end of the run backwards, so launches that precede the log (library set-up) do not matter.  The
byte counters and the L2 request counters are scaled by what the same counter reads for the plain device copy
of --copy-probe-mb (a kernel that moves a known number of bytes each way).  Rates are set beside the ceilings
of profiles/ceilings_gfx950.txt.
"""
from __future__ import annotations

import csv
import glob
import json
import os
import sys
from collections import defaultdict

MAIN = ("sconv_lds2_kernel", "sconv_lds_kernel", "sconv_direct_kernel")
CEIL = dict(fma_lanes=59.0, lds_b_clk=253.7, copy_tbs=4.83, l2_read_tbs=34.5)   # per CU per clock; whole chip


def find(raw, run, suffix):
    hits = glob.glob(os.path.join(raw, run, "**", f"*{suffix}"), recursive=True)
    return hits[0] if hits else None


def load_log(raw, run):
    p = os.path.join(raw, run, "log.json")
    return json.load(open(p)) if os.path.exists(p) else None


def attribute(dispatches, log):
    """dispatches: [(id, kernel name)] in launch order.  Returns {id: (layer, phase, role)} for the library's
    kernels, matched to the log's calls from the end backwards; role = main / aux (phase images, reduction)."""
    ours = [(d, n) for d, n in dispatches if "sconv" in n]
    out = {}
    i = len(ours)
    for call in reversed(log["calls"]):
        k = call["kernels"]
        if i - k < 0:
            break
        for d, n in ours[i - k:i]:
            out[d] = (call["layer"], call["phase"], "main" if any(m in n for m in MAIN) else "aux")
        i -= k
    return out


def counters(raw, run):
    """({counter: {layer: mean per timed forward call, main kernel + aux}}, {counter: copy value}, log)"""
    path, log = find(raw, run, "counter_collection.csv"), load_log(raw, run)
    if not path or not log:
        return {}, {}, log
    per = defaultdict(lambda: defaultdict(float))   # counter -> dispatch -> value (summed over instances)
    name = {}
    for r in csv.DictReader(open(path)):
        d = int(r["Dispatch_Id"])
        per[r["Counter_Name"]][d] += float(r["Counter_Value"])
        name[d] = r["Kernel_Name"]
    order = sorted(name)
    who = attribute([(d, name[d]) for d in order], log)
    copies = [d for d in order if "sconv" not in name[d] and ("copy" in name[d].lower() or "elementwise" in name[d].lower())]
    n_timed = defaultdict(int)
    for c in log["calls"]:
        if c["phase"] == "timed":
            n_timed[c["layer"]] += 1
    out, cp = {}, {}
    for c, by_d in per.items():
        lay = defaultdict(float)
        for d, (layer, phase, role) in who.items():
            if phase == "timed":
                lay[layer] += by_d.get(d, 0.0)
        out[c] = {l: v / max(1, n_timed[l]) for l, v in lay.items()}
        cp[c] = max((by_d.get(d, 0.0) for d in copies), default=None)
    return out, cp, log


def kernel_times(raw):
    path, log = find(raw, "kt", "kernel_trace.csv"), load_log(raw, "kt")
    if not path or not log:
        return None, log
    rows = sorted(((int(r["Dispatch_Id"]), r["Kernel_Name"], int(r["Start_Timestamp"]), int(r["End_Timestamp"]))
                   for r in csv.DictReader(open(path))), key=lambda r: r[0])
    who = attribute([(d, n) for d, n, _, _ in rows], log)
    by = defaultdict(lambda: defaultdict(list))      # layer -> kernel name -> durations (timed phase)
    for d, n, t0, t1 in rows:
        if d in who and who[d][1] == "timed":
            by[who[d][0]][n].append((t1 - t0) / 1e3)
    return by, log


def main() -> int:
    args = [a for a in sys.argv[1:] if not a.startswith("--")]
    raw, out_file = args[0], args[1]
    traffic_json = None
    if "--traffic-json" in sys.argv:
        traffic_json = sys.argv[sys.argv.index("--traffic-json") + 1]
    lines = []
    by, log = kernel_times(raw)
    if not log:
        print("no kt/log.json under", raw, file=sys.stderr)
        return 2
    layers = [L["name"] for L in log["layers"]]
    meta = {L["name"]: L for L in log["layers"]}
    copy_mb = None
    lines.append(f"configuration: {log['config']}; tilings in use:")
    for l in layers:
        p = meta[l]["plan"]
        lines.append(f"  {l:16s} N {meta[l]['N']:4d}  kernel {p['kernel']} cb {p['cb']} waves {p['waves']} cg {p['cg']} rows_w {p['rows_w']} t {p['t']} "
                     f"band {p['band']} strip {p['strip']} splits {p['splits']};  {meta[l]['flops'] / 1e9:.2f} GFLOP (nonzeros only), "
                     f"{meta[l]['bytes'] / 1e6:.1f} MB algorithmic HBM bytes per launch")
    lines.append("")
    kt_main = {}
    if by:
        lines.append("kernel trace (rocprofv3 --kernel-trace), timed launches only, per layer in launch order")
        lines.append(f"  {'layer':16s} {'kernel':62s} {'calls':>5s} {'avg_us':>8s} {'min_us':>8s} {'max_us':>8s} {'TFLOP/s':>8s} {'of 78.6':>7s}")
        for l in layers:
            for n, ds in by.get(l, {}).items():
                is_main = any(m in n for m in MAIN)
                avg = sum(ds) / len(ds)
                if is_main:
                    kt_main[l] = avg
                tf = meta[l]["flops"] / avg / 1e6 if is_main else 0.0
                lines.append(f"  {l:16s} {n.replace('void sconv::', '')[:62]:62s} {len(ds):5d} {avg:8.2f} {min(ds):8.2f} {max(ds):8.2f} "
                             + (f"{tf:8.2f} {tf / 78.6:7.1%}" if is_main else f"{'':8s} {'':7s}"))
        lines.append("")
    traffic = {}
    fetch, fcopy, flog = counters(raw, "fetch")
    write, wcopy, _ = counters(raw, "write")
    if fetch.get("FETCH_SIZE") and write.get("WRITE_SIZE") and fcopy.get("FETCH_SIZE") and wcopy.get("WRITE_SIZE"):
        copy_mb = flog["copy_probe_mb"]
        expect_kib = copy_mb * 1024.0
        fs, ws = expect_kib / fcopy["FETCH_SIZE"], expect_kib / wcopy["WRITE_SIZE"]
        lines.append(f"HBM traffic per launch (FETCH_SIZE / WRITE_SIZE, KiB; scale factors from a {copy_mb} MiB copy: "
                     f"read x{fs:.3f}, write x{ws:.3f}); 'x alg' = measured / algorithmic bytes")
        for l in layers:
            rd = fetch["FETCH_SIZE"].get(l, 0.0) * fs * 1024.0
            wr = write["WRITE_SIZE"].get(l, 0.0) * ws * 1024.0
            traffic[l] = {"read_bytes": round(rd), "write_bytes": round(wr), "bytes": round(rd + wr)}
            lines.append(f"  {l:16s} read {rd / 1e6:8.1f} MB  write {wr / 1e6:8.1f} MB  x alg {(rd + wr) / meta[l]['bytes']:.2f}")
        lines.append("")
        if traffic_json:
            json.dump(traffic, open(traffic_json, "w"), indent=1)
    sq1, _, _ = counters(raw, "sq1")
    sq2, _, _ = counters(raw, "sq2")
    for tag, cs in (("sq1", sq1), ("sq2", sq2)):
        if cs:
            lines.append(f"SQ counters per launch ({tag})")
            for c in sorted(cs):
                lines.append(f"  {c:26s} " + "  ".join(f"{l} {cs[c].get(l, 0):.4g}" for l in layers))
            lines.append("")
    l2, l2copy, l2log = counters(raw, "l2")
    l2_read = {}
    if l2.get("TCC_READ_sum") and l2copy.get("TCC_READ_sum"):
        per_req = l2log["copy_probe_mb"] * 2.0 ** 20 / l2copy["TCC_READ_sum"]
        lines.append(f"L2 (TCC) counters per launch; one read request = {per_req:.1f} B (from the {l2log['copy_probe_mb']} MiB copy)")
        for c in sorted(l2):
            lines.append(f"  {c:26s} " + "  ".join(f"{l} {l2[c].get(l, 0):.4g}" for l in layers))
        for l in layers:
            l2_read[l] = l2["TCC_READ_sum"].get(l, 0.0) * per_req
        if "TCC_HIT_sum" in l2 and "TCC_MISS_sum" in l2:
            lines.append("  hit rate                   " + "  ".join(
                f"{l} {l2['TCC_HIT_sum'].get(l, 0.0) / max(1.0, l2['TCC_HIT_sum'].get(l, 0.0) + l2['TCC_MISS_sum'].get(l, 0.0)):.1%}" for l in layers))
        lines.append("")
    if sq1 and sq2 and "GRBM_GUI_ACTIVE" in sq1:
        lines.append("derived per layer, each beside its ceiling (kernel cycles = GRBM_GUI_ACTIVE / 8 XCDs; SQ instruction counters "
                     "are per wave, x 64 lanes; one LDS instruction of these kernels moves 1 KiB)")
        lines.append(f"  ceilings (profiles/ceilings_gfx950.txt): v_fma_f32 {CEIL['fma_lanes']} lanes-FMA/clk/CU of 64, ds_read_b128 "
                     f"{CEIL['lds_b_clk']} B/clk/CU, device copy {CEIL['copy_tbs']} TB/s, L2 read {CEIL['l2_read_tbs']} TB/s")
        lines.append(f"  {'layer':16s} {'us@2.4GHz':>10s} {'FMA lanes/clk/CU':>17s} {'of 64':>6s} {'LDS B/clk/CU':>13s} {'of peak':>8s} {'VALU busy':>10s} "
                     f"{'HBM TB/s':>9s} {'of copy':>8s} {'L2 read TB/s':>13s} {'of peak':>8s} {'bank confl':>10s}")
        for l in layers:
            cyc = sq1["GRBM_GUI_ACTIVE"].get(l, 0.0) / 8.0
            if cyc <= 0:
                continue
            fma = sq2.get("SQ_INSTS_VALU_FMA_F32", {}).get(l, 0.0) * 64.0 / (cyc * 256.0)
            lds = sq2.get("SQ_INSTS_LDS", {}).get(l, 0.0) * 1024.0 / (cyc * 256.0)
            busy = sq1.get("SQ_ACTIVE_INST_VALU", {}).get(l, 0.0) * 4.0 / (cyc * 1024.0)
            hbm = traffic.get(l, {}).get("bytes", 0) / (cyc / 2.4e9) / 1e12 if traffic else 0.0
            bc = sq2.get("SQ_LDS_BANK_CONFLICT", {}).get(l, 0.0)
            l2bw = l2_read.get(l, 0.0) / (cyc / 2.4e9) / 1e12
            lines.append(f"  {l:16s} {cyc / 2.4e3:10.1f} {fma:17.2f} {fma / 64:6.1%} {lds:13.1f} {lds / CEIL['lds_b_clk']:8.1%} {busy:10.1%} "
                         f"{hbm:9.2f} {hbm / CEIL['copy_tbs']:8.1%} {l2bw:13.2f} {l2bw / CEIL['l2_read_tbs']:8.1%} {bc:10.0f}")
        lines.append("")
    text = "\n".join(lines)
    print(text)
    open(out_file, "w").write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
