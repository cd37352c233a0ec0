"""Short text summaries of rocprofv3 runs of bench.py: the files kept under profiles/ are the output of this module.

    python -m paper_2603_07685_amd.profile_summary trace   DIR [BENCH_JSON]      kernel-trace run (per kernel, per call site)
    python -m paper_2603_07685_amd.profile_summary traffic FETCH_DIR WRITE_DIR BENCH_JSON   FETCH_SIZE / WRITE_SIZE passes
    python -m paper_2603_07685_amd.profile_summary mfma    DIR BENCH_JSON        SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES GRBM_GUI_ACTIVE pass
    python -m paper_2603_07685_amd.profile_summary moves   TRACE_DIR FETCH_DIR WRITE_DIR BENCH_JSON   data-movement kernels

DIR is the -d directory of a `rocprofv3 ... --output-format csv -- python3 bench.py ...` run; BENCH_JSON the JSON line
bench.py printed in that run (its "kernels" keys, in call order, label the call sites).  Only parsing and arithmetic on
the profiler's numbers happen here; nothing is measured and nothing of the layer is computed.
"""
from __future__ import annotations

import csv
import glob
import json
import os
import re
import sys
from collections import OrderedDict

GIB = 1 << 30
LEGEND = ("gg_kernel<MODE,EPI,F32,F8,NW>: MODE 0 fwd / 1 dgrad / 2 wgrad; EPI 0 store / 1 SwiGLU / 2 SwiGLU-bwd; "
          "F8 0 bf16 / 1 blockwise fp8 / 2 MXFP8; NW waves per workgroup")


def _short(name: str) -> str:
    return re.sub(r"\(.*", "", name).replace("void ", "")[:70]


def _csv(d: str, suffix: str):
    hits = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit(f"no *{suffix} under {d}")
    with open(hits[-1]) as fh:
        return list(csv.DictReader(fh))


def _bench(path: str) -> dict:
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if line.startswith("{") and '"metric"' in line:
                return json.loads(line)
    raise SystemExit(f"no bench.py JSON line in {path}")


def _gemm_labels(bench: dict):
    return [k for k in bench["kernels"] if re.search(r"_(fwd|dgrad|wgrad)(_|$)", k)]


def _is_site(name: str) -> bool:
    return any(t in name for t in ("gg_kernel", "combine", "permute_rows", "quant"))


def _last_step(rows, name_of):
    """Rows of the last fwd+bwd step: from the last router launch up to the vendor GEMM bench.py times afterwards."""
    idx = [i for i, r in enumerate(rows) if "route_topk" in name_of(r)]
    out = []
    for r in rows[idx[-1]:]:
        if "Cijk" in name_of(r):
            break
        out.append(r)
    return out


def trace(d: str, bench_path: str | None = None):
    rows = sorted(_csv(d, "kernel_trace.csv"), key=lambda r: int(r["Start_Timestamp"]))
    agg = OrderedDict()
    for r in rows:
        a = agg.setdefault(_short(r["Kernel_Name"]), [0, 0.0])
        a[0] += 1
        a[1] += (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
    # (bench.py's context measurements -- the vendor GEMM and the register-resident MFMA loop -- are listed but left
    # out of the percentages)
    context = lambda n: "ceiling_kernel" in n or "Cijk" in n
    tot = sum(v[1] for n, v in agg.items() if not context(n))
    if bench_path:
        b = _bench(bench_path)
        print(f"# bench.py reported in the same run: {b['ms_per_step']} ms per fwd+bwd step, {b['value']} {b['unit']}; "
              f"roofline kernel {b['roofline']['kernel']}: {b['roofline']['achieved']} TFLOP/s by its own HIP-event timing")
    print("# " + LEGEND)
    print("# durations in microseconds")
    print(f"{'kernel':72s} {'calls':>6s} {'total_us':>12s} {'avg_us':>10s} {'pct':>6s}")
    for n, (cnt, t) in sorted(agg.items(), key=lambda kv: -kv[1][1])[:22]:
        pct = "   ctx" if context(n) else f"{100 * t / tot:6.2f}"
        print(f"{n:72s} {cnt:6d} {t:12.1f} {t / cnt:10.1f} {pct}")
    steps, cur = [], None
    for r in rows:
        sn = _short(r["Kernel_Name"])
        if sn.startswith("route_topk"):
            cur = []
            steps.append(cur)
        if cur is not None and _is_site(sn) and "Cijk" not in sn:
            cur.append((sn, (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3))
    steps = [s for s in steps if len(s) == len(steps[-1])]
    labels = _gemm_labels(_bench(bench_path)) if bench_path else []
    print(f"\nper call site, averaged over {len(steps)} steps (dispatch order inside one fwd+bwd step):")
    gi = 0
    for i in range(len(steps[-1])):
        name = steps[-1][i][0]
        avg = sum(s[i][1] for s in steps) / len(steps)
        lab = ""
        if name.startswith("gg_kernel") and gi < len(labels):
            lab = labels[gi]
            gi += 1
        print(f"  {i:2d} {name:44s} {lab:36s} {avg:10.1f} us")


def _pmc(d: str):
    rows = _csv(d, "counter_collection.csv")
    out = OrderedDict()
    for r in rows:
        e = out.setdefault(int(r["Dispatch_Id"]), {"name": r["Kernel_Name"], "s": int(r.get("Start_Timestamp", 0) or 0),
                                                    "e": int(r.get("End_Timestamp", 0) or 0)})
        e[r["Counter_Name"]] = float(r["Counter_Value"])
    return [v for _, v in sorted(out.items())]


def _calibration(F, W):
    for f, w in zip(F, W):
        if f["FETCH_SIZE"] * 1024 > 0.3 * GIB and ("copy" in f["name"].lower() or "elementwise" in f["name"]):
            return f["name"], f["FETCH_SIZE"] * 1024, w["WRITE_SIZE"] * 1024
    raise SystemExit("calibration copy not found")


def _traffic_rows(fd: str, wd: str):
    F, W = _pmc(fd), _pmc(wd)
    cal = _calibration(F, W)
    kf, kw = GIB / cal[1], GIB / cal[2]
    Fs, Ws = _last_step(F, lambda r: r["name"]), _last_step(W, lambda r: r["name"])
    # (the two passes are two runs: what bench.py launches after its timed steps may differ in count, a step may not)
    assert [r["name"] for r in Fs] == [r["name"] for r in Ws], (len(Fs), len(Ws))
    rows = [(_short(f["name"]), f["FETCH_SIZE"] * 1024 * kf / 1e9, w["WRITE_SIZE"] * 1024 * kw / 1e9)
            for f, w in zip(Fs, Ws) if _is_site(f["name"])]
    return cal, rows


def traffic(fd: str, wd: str, bench_path: str):
    cal, rows = _traffic_rows(fd, wd)
    labels = _gemm_labels(_bench(bench_path))
    print("# " + LEGEND)
    print("# counters are KiB per dispatch; each is divided by what it read for the 1 GiB device copy bench.py runs first")
    print("# (FETCH_SIZE counts what the L2 caches fetch from the fabric: reads served by the memory-side cache are included)")
    print(f"calibration copy: {_short(cal[0])} FETCH_SIZE reads {cal[1] / GIB:.4f} x, WRITE_SIZE {cal[2] / GIB:.4f} x of 1 GiB")
    print("scaled HBM-side bytes per launch in the last step, in call order (GB read, GB written); bench.py reads the labelled rows:")
    gi = 0
    for name, rd, wr in rows:
        lab = "-"
        if name.startswith("gg_kernel") and gi < len(labels):
            lab = labels[gi]
            gi += 1
        print(f"  {lab:36s} {name:44s} read {rd:8.3f}  write {wr:8.3f}")


def mfma(d: str, bench_path: str):
    rows = _last_step(_pmc(d), lambda r: r["name"])
    labels = _gemm_labels(_bench(bench_path))
    print("# " + LEGEND)
    print("# SQ_VALU_MFMA_BUSY_CYCLES is summed over the 1024 SIMDs, SQ_BUSY_CU_CYCLES over the 256 CUs, GRBM_GUI_ACTIVE over the 8 XCDs")
    print("#   clock               = GRBM_GUI_ACTIVE / 8 / kernel duration (the sustained clock during the launch)")
    print("#   MFMA busy / CU busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES)")
    print("#   vs 2.4 GHz peak     = SQ_VALU_MFMA_BUSY_CYCLES / 1024 / (duration * 2.4 GHz)")
    print(f"  {'call site':36s} {'kernel':30s} {'dur_us':>8s} {'clock_GHz':>9s} {'MFMA busy / CU busy':>20s} {'vs 2.4 GHz peak':>16s}")
    gi = 0
    for v in rows:
        if "gg_kernel" not in v["name"]:
            continue
        dur = (v["e"] - v["s"]) / 1e3
        clk = v["GRBM_GUI_ACTIVE"] / 8 / (dur * 1e3)
        busy = v["SQ_VALU_MFMA_BUSY_CYCLES"] / (4 * v["SQ_BUSY_CU_CYCLES"])
        vs = v["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024 / (dur * 1e3 * 2.4)
        lab = labels[gi] if gi < len(labels) else "-"
        gi += 1
        print(f"  {lab:36s} {_short(v['name']):30s} {dur:8.1f} {clk:9.2f} {100 * busy:19.1f}% {100 * vs:15.1f}%")


def moves(td: str, fd: str, wd: str, bench_path: str):
    b = _bench(bench_path)
    trows = sorted(_csv(td, "kernel_trace.csv"), key=lambda r: int(r["Start_Timestamp"]))
    steps, cur = [], None
    for r in trows:
        sn = _short(r["Kernel_Name"])
        if sn.startswith("route_topk"):
            cur = []
            steps.append(cur)
        if cur is not None and any(t in sn for t in ("combine", "permute_rows")):
            cur.append((sn, (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3))
    steps = [s for s in steps if len(s) == len(steps[-1])]
    _, rows = _traffic_rows(fd, wd)
    meas = [(n, rd + wr) for n, rd, wr in rows if any(t in n for t in ("combine", "permute_rows"))]
    alg = {k: v for k, v in b["kernels"].items() if k in ("permute", "combine", "combine_bwd", "unpermute_sum_dx")}

    def label_of(i):   # call site of the i-th move kernel of a step, by kernel and order (a step without a bf16 permuted
        name = steps[-1][i][0]   # copy launches no permute_rows kernel, one whose dO is quantised on the fly no full combine backward)
        if "permute_rows" in name:
            return "permute"
        if "combine_bwd" in name:
            return "combine_bwd"
        return "combine" if not any("combine_kernel" in steps[-1][j][0] for j in range(i)) else "unpermute_sum_dx"
    print("# durations: rocprofv3 --kernel-trace averages per call site; bytes: FETCH_SIZE / WRITE_SIZE passes scaled by the calibration copy;")
    print("# algorithmic bytes: bench.py's figures for the same calls (its GB/s x its ms).  Peak 8000 GB/s.")
    print(f"{'call site':20s} {'kernel':30s} {'avg_us':>8s} {'alg_GB':>8s} {'meas_GB':>8s} {'alg_GB/s':>9s} {'% of peak':>9s} {'meas_GB/s':>10s}")
    for i, (name, _) in enumerate(steps[-1]):
        avg = sum(s[i][1] for s in steps) / len(steps)
        lab = label_of(i)
        a = alg.get(lab)
        alg_gb = a["gbs"] * a["ms"] / 1e3 if a else float("nan")
        m = meas[i][1] if i < len(meas) else float("nan")
        print(f"{lab:20s} {name:30s} {avg:8.1f} {alg_gb:8.3f} {m:8.3f} {alg_gb / avg * 1e6:9.0f} {alg_gb / avg * 1e6 / 80:8.1f}% {m / avg * 1e6:10.0f}")


if __name__ == "__main__":
    cmd, args = sys.argv[1], sys.argv[2:]
    {"trace": trace, "traffic": traffic, "mfma": mfma, "moves": moves}[cmd](*args)
