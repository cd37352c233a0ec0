#!/usr/bin/env python3
"""Benchmark of the one-GPU MoE expert-layer hot path (router -> permute -> grouped-GEMM SwiGLU MLP
-> combine, forward + backward) at the DeepSeek-V3-style local shape.

One "step" = one forward + backward pass of the whole path over one synthetic batch whose inputs are
already resident in HBM.  Prints ONE JSON line: the layer's model TFLOP/s, the roofline figure of the
dominant kernel (measured with events inside the timed region) and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
FP8_PEAK_TFLOPS = 5000.0    # MI355X dense fp8 MFMA
HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
CAL_COPY_BYTES = 1 << 30    # size of the calibration copy (read 1 GiB, write 1 GiB)

def measured_traffic(workload: str, label: str):
    """(GB read, GB written) per launch of one grouped-GEMM call site, from the tracked summary of the two rocprofv3
    counter passes over this script (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch, each scaled by what the same
    counter read for the 1 GiB calibration copy below): profiles/gg_kernel_<workload>_hbm_traffic.txt, written by
    paper_2603_07685_amd.profile_summary.  Offline measurements: they describe the committed kernels at the default
    load pattern, not this run.  None when the workload has no summary."""
    import re
    path = os.path.join(ROOT, "profiles", f"gg_kernel_{workload.lower()}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        for line in fh:
            m = re.match(r"\s+(\S+)\s+gg_kernel<[^>]*>\s+read\s+([0-9.]+)\s+write\s+([0-9.]+)", line)
            if m and m.group(1) == label:
                return float(m.group(2)), float(m.group(3))
    return None


def mfma_ceiling():
    """Context only: what the matrix pipes of this box sustain with every operand in registers (no LDS, no memory),
    measured by paper_2603_07685_amd/csrc/mfma_ceiling.hip for the two MFMA shapes the grouped GEMMs use, on zeros
    (nominal rate) and on random operands (the power-limited rate a kernel on real data can approach).  None if the
    probe library is not built."""
    import ctypes
    path = os.path.join(ROOT, "paper_2603_07685_amd", "libmfma_ceiling.so")
    if not os.path.exists(path):
        return None
    lib = ctypes.CDLL(path)
    lib.mfma_ceiling.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float)]
    res = {"what": "register-resident MFMA loop, TFLOP/s: v_mfma_f32_16x16x32_bf16 / v_mfma_scale_f32_32x32x64_f8f6f4 (E4M3)"}
    for name, fp8, rnd in (("bf16_zeros", 0, 0), ("bf16_random", 0, 1), ("fp8_zeros", 1, 0), ("fp8_random", 1, 1)):
        v = ctypes.c_float(0.0)
        rc = lib.mfma_ceiling(fp8, rnd, 300, ctypes.byref(v))
        res[name] = round(v.value, 1) if rc == 0 else None
    return res


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4",
                    help="C1 | MID | C2 | C3 | C4 | C4G (C4 behind the group-limited, bias-corrected router) | C5 (blockwise fp8) | C6 (MXFP8) (default: the metric's config, C4)")
    ap.add_argument("--variant", default=None,
                    help="load pattern override: uniform | zeros | hot | cv | zipf | router (the router's own top-k over "
                         "the global experts; only hits on the local experts become rows)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--wgrad-f32", action="store_true", help="fp32 weight gradients (default bf16)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture the step in a HIP graph and report the time of its replays (field 'graph')")
    ap.add_argument("--bf16-wgrad", action="store_true",
                    help="blockwise fp8 workloads: weight gradients from the bf16 tensors instead of the 128x1 E4M3 copies")
    ap.add_argument("--no-epilogue-quant", action="store_true",
                    help="one-byte recipes: quantise A and dZ with stand-alone quantiser launches instead of in the GEMM epilogues")
    ap.add_argument("--gather", action="store_true",
                    help="bf16 workloads: no permuted copy of the tokens (with --eq2: nor of dY); the GEMMs that would read it "
                         "fetch the rows of X / dY through the row map")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed step and the box reference (profiler runs: no second pass with gathered operands)")
    ap.add_argument("--eq2", action="store_true",
                    help="memory-efficient permutation: routing weights applied in the fc1 epilogue, plain-sum combine")
    return ap.parse_args()


def describe_call(name, args, st):
    """(label, flops or None, bytes or None) of one library call, from its own arguments."""
    cfg = st.cfg
    T, k = cfg.T, cfg.k
    # routed rows (unpadded): the algorithmic row count of the grouped calls.  With the router's own top-k over more
    # experts than live on this GPU (--variant router) only the local hits are rows: counted after the warm-up
    R = getattr(st, "R_live", None) or T * k
    if name == "moe_gather_row_prob":
        return "gather_row_prob", None, args[3] * 12
    if name == "moe_scatter_row_dprob":
        return "scatter_row_dprob", None, T * k * (8 + 4 * args[2])
    q_out = 0   # quantised copies a quantising epilogue writes besides its bf16 output (bytes per output element)
    gath = ""
    if name.startswith("moe_grouped_gemm_") and name.endswith("_gather"):
        # one operand fetched through the row map: the same algorithmic work as the plain call (a row per permuted row,
        # plus the map); arguments brought into the plain call's order
        gath = "_gather"
        if "fwd" in name:      # (ctx, X, T, src_of, k, B, offsets, E, N, K, Rcap, epi, ...)
            args = [args[0], args[1], args[5], args[6], args[7], args[8], args[9], args[10], 0, args[11]]
        elif "dgrad" in name:  # (ctx, G, T, src_of, k, B, offsets, E, N, K, Rcap, Z_saved, ...)
            args = [args[0], args[1], args[5], args[6], args[7], args[8], args[9], args[10], 0, args[11]]
        else:                  # (ctx, A, dC, which, T, src_of, k, offsets, E, N, K, Rcap, accumulate, out_dt, dB)
            args = [args[0], args[1], args[2], args[7], args[8], args[9], args[10], args[11], 0, None, None, args[12], args[13]]
        name = name[:-len("_gather")]
    if name.endswith("_quant_mx"):   # (ctx, P, W, offsets, E, N, K, Rcap, [Z_saved,] scales ...): MXFP8 implied
        fwd = "fwd" in name
        q_out = 1 + (args[-2] is not None)
        args = list(args[:8]) + [3, 1 if fwd else args[8]]
        name = "moe_grouped_gemm_" + ("fwd" if fwd else "dgrad")
    for sfx in ("_weighted", "_quant"):
        if name.endswith(sfx):
            name = name[:-len(sfx)]
    if name in ("moe_grouped_gemm_fwd", "moe_grouped_gemm_dgrad", "moe_grouped_gemm_wgrad"):
        E, N, K, dt = args[4], args[5], args[6], args[8]
        rows = R if E > 1 else T
        kind = name.rsplit("_", 1)[1]
        tag = {1: "fp8", 3: "mxfp8"}.get(dt, "bf16")
        if kind == "fwd":
            extra = "_swiglu" if args[9] == 1 else ""
        elif kind == "dgrad":
            extra = "_swiglu_bwd" if args[9] is not None else ""
        else:
            extra = ""
        which = ("fc1" if (kind == "fwd" and K == cfg.h) or (kind != "fwd" and K == cfg.h) else "fc2")
        label = f"{'shared_' if E == 1 else ''}{which}_{kind}{extra}_{tag}{gath}"
        es = 1 if dt in (1, 3) else 2
        if kind == "fwd":      # read A and the weights once, write C (SwiGLU: pre-activations + activation)
            by = rows * K * es + E * N * K * es + rows * N * 2 + (rows * (N // 2) * (2 + q_out) if extra else 0)
        elif kind == "dgrad":  # read dC and the weights once, write dA (SwiGLU-bwd: read Z, write dZ, both [rows, 2K])
            by = rows * N * es + E * N * K * es + (rows * 2 * K * (2 * 2 + q_out) if extra else rows * K * 2)
        else:                  # read A and dC once, write the weight gradients
            by = rows * (N + K) * es + E * N * K * (4 if args[12] == 2 else 2)
        if gath:
            by += rows * 4
        return label, 2.0 * rows * N * K, by
    if name == "moe_route_topk_grouped":
        Tn, E = args[3], args[4]
        return "route_topk_grouped", None, Tn * E * 4 + Tn * args[5] * 8 + E * 8
    if name == "moe_route_topk":
        Tn, E = args[2], args[3]
        return "route_topk", None, Tn * E * 4 + Tn * args[4] * 8 + E * 4
    if name == "moe_permute":
        h = args[6]
        if args[1] is None:   # the maps alone: read the expert ids, write row_of and src_of
            return "permute_maps", None, T * k * 8 + R * 4
        return "permute", None, (T + R) * h * 2 + T * k * 12
    if name == "moe_unpermute_combine":
        h = args[8]
        res = args[5] is not None
        return ("combine" if args[4] is not None else "unpermute_sum_dx"), None, (R + T) * h * 2 + T * k * 8 + (T * h * 2 if res else 0)
    if name == "moe_unpermute_combine_bwd":
        h = args[9]
        # read dY, read O (when dprob is wanted), write dO (unless only dprob is wanted)
        return "combine_bwd", None, (T + ((args[2] is not None) + (args[11] is not None)) * R) * h * 2
    if name == "moe_mx_quantize":
        block, groups, rows, cols, live = args[2], args[3], args[4], args[5], args[6]
        rows_alg = R if live is not None else rows
        n = groups * rows_alg * cols
        return f"mx_quantize_{['1x32', '32x1'][block]}[{groups * rows}x{cols}]", None, n * 3 + n // 32
    if name == "moe_mx_quantize_rowcol":  # read bf16 once, write two one-byte copies and their scales
        rows, cols, live = args[2], args[3], args[4]
        n = (R if live is not None else rows) * cols
        return f"mx_quantize_rowcol[{rows}x{cols}]", None, n * 4 + n // 16
    if name == "moe_mx_quantize_rowcol_gather":  # read the source rows, write two one-byte copies and their scales
        cols = args[7]
        n = R * cols
        src = "tokens" if args[1] is st.X else "dY"
        return f"mx_quantize_gather_{src}[{args[6]}x{cols}]", None, T * cols * 2 + n * 2 + n // 16 + R * 4
    if name == "moe_fp8_quantize_rowcol":  # read bf16 once, write one or two one-byte copies and their scales
        rows, cols, live = args[2], args[3], args[4]
        n = (R if live is not None else rows) * cols
        copies = (args[5] is not None) + (args[7] is not None)
        return f"fp8_quantize_rowcol[{rows}x{cols},{copies}]", None, n * (2 + copies) + copies * (n // 128) * 4
    if name == "moe_fp8_quantize_rowcol_gather":
        cols = args[7]
        n = R * cols
        src = "tokens" if args[1] is st.X else "dY"
        return f"fp8_quantize_gather_{src}[{args[6]}x{cols}]", None, T * cols * 2 + n * 2 + (n // 128) * 8 + R * 4
    if name == "moe_fp8_quantize":
        block, groups, rows, cols, live = args[2], args[3], args[4], args[5], args[6]
        rows_alg = R if live is not None else rows          # grouped row tensors: only the routed rows count
        n = groups * rows_alg * cols
        return f"quantize_{['1x128', '128x1', '128x128'][block]}[{rows}x{cols}]", None, n * 3 + n // 128 * 4
    return name, None, None


HOOKED = ["moe_fp8_quantize_rowcol", "moe_fp8_quantize_rowcol_gather", "moe_mx_quantize", "moe_mx_quantize_rowcol", "moe_mx_quantize_rowcol_gather", "moe_route_topk", "moe_route_topk_grouped", "moe_permute", "moe_grouped_gemm_fwd", "moe_grouped_gemm_dgrad", "moe_grouped_gemm_wgrad",
          "moe_unpermute_combine", "moe_unpermute_combine_bwd", "moe_fp8_quantize",
          "moe_grouped_gemm_fwd_weighted", "moe_grouped_gemm_dgrad_weighted",
          "moe_grouped_gemm_fwd_quant", "moe_grouped_gemm_dgrad_quant", "moe_grouped_gemm_fwd_quant_mx",
          "moe_grouped_gemm_dgrad_quant_mx", "moe_gather_row_prob",
          "moe_scatter_row_dprob", "moe_grouped_gemm_fwd_gather", "moe_grouped_gemm_dgrad_gather",
          "moe_grouped_gemm_wgrad_gather"]


def timed_step_with_events(st, torch, sync=True):
    """One step with an event after every library call.  Returns (records, events): records[i] =
    (label, flops, bytes) of call i in issue order, bracketed by events[i] and events[i + 1]."""
    from paper_2603_07685_amd import binding as B
    recs, evs, orig = [], [torch.cuda.Event(enable_timing=True)], {}

    def wrap(name, fn):
        def inner(*a, **kw):
            r = fn(*a, **kw)
            ev = torch.cuda.Event(enable_timing=True)
            ev.record()
            evs.append(ev)
            recs.append(describe_call(name, a, st))
            return r
        return inner

    evs[0].record()
    for n in HOOKED:
        orig[n] = getattr(B, n)
        setattr(B, n, wrap(n, orig[n]))
    try:
        st.step()
    finally:
        for n in HOOKED:
            setattr(B, n, orig[n])
    if sync:
        torch.cuda.synchronize()
    return recs, evs


def _rows_of(st, torch, which, rows):
    """Rows of the permuted tokens / of the combine's backward for the CPU baseline's inputs: as stored, or, when the
    layer quantises them straight from X / dY and keeps no bf16 copy, gathered here through the row map."""
    t = getattr(st, which)
    if t is not None:
        return t[rows]
    s = st.src_of[rows].long()
    tok = torch.div(s.clamp(min=0), st.cfg.k, rounding_mode="floor")
    x = (st.X if which == "Xp" else st.dY)[tok].float()
    if which == "dO" and not st.eq2:
        x = x * st.topk_prob.reshape(-1)[s.clamp(min=0)][:, None]
    x[s < 0] = 0
    return x.to(torch.bfloat16)


def cpu_baseline(st, torch):
    """The fp32 CPU oracle on a bounded sample of the same workload: 16 experts x 512 rows through
    fc1+SwiGLU+fc2 forward and both data gradients, and 512x512 weight-gradient windows contracted over
    all rows of those experts.  Returns (TFLOP/s, threads, description)."""
    import numpy as np
    import oracle as orc
    orc.build()
    cfg = st.cfg
    E, h, f = cfg.E, cfg.h, cfg.f
    offs = st.offsets.cpu().numpy()
    experts = [e for e in np.linspace(0, E - 1, num=min(16, E)).astype(int).tolist() if offs[e + 1] > offs[e]]
    nrow, win = 512, 512
    flops, secs = 0.0, 0.0
    for e in experts:
        lo, hi = int(offs[e]), int(offs[e + 1])
        rows = np.unique(np.linspace(lo, hi - 1, num=min(nrow, hi - lo)).astype(np.int64))
        n = len(rows)
        ridx = torch.from_numpy(rows).cuda()
        xp = _rows_of(st, torch, "Xp", ridx).float().cpu().numpy()
        do = _rows_of(st, torch, "dO", ridx).float().cpu().numpy()
        w1 = st.W1[e].float().cpu().numpy()[None]
        w2 = st.W2[e].float().cpu().numpy()[None]
        o1 = np.array([0, n], np.int32)
        # wgrad windows over all rows of the expert
        wn, wk = min(win, h), min(win, f)
        allr = torch.arange(lo, hi, device="cuda")
        dO_all = _rows_of(st, torch, "dO", allr)[:, :wn].float().cpu().numpy()
        A_all = st.A[lo:hi, :wk].float().cpu().numpy()
        dZ_all = st.dZ[lo:hi, :min(win, 2 * f)].float().cpu().numpy()
        Xp_all = _rows_of(st, torch, "Xp", allr)[:, :min(win, h)].float().cpu().numpy()
        oall = np.array([0, hi - lo], np.int32)
        t0 = time.perf_counter()
        z = orc.grouped_gemm_nt(xp, w1, o1, prec="f32")
        a = orc.swiglu(z, prec="f32")
        orc.grouped_gemm_nt(a, w2, o1, prec="f32")
        da = orc.grouped_gemm_nn(do, w2, o1, prec="f32")
        dz = orc.swiglu_bwd(da, z, prec="f32")
        orc.grouped_gemm_nn(dz, w1, o1, prec="f32")
        orc.grouped_gemm_tn(dO_all, A_all, oall, prec="f32")
        orc.grouped_gemm_tn(dZ_all, Xp_all, oall, prec="f32")
        secs += time.perf_counter() - t0
        flops += 12.0 * n * h * f  # fwd + dgrad of fc1 and fc2
        flops += 2.0 * (hi - lo) * (dO_all.shape[1] * A_all.shape[1] + dZ_all.shape[1] * Xp_all.shape[1])
    desc = (f"{len(experts)} experts x {nrow} rows through fc1+SwiGLU+fc2 forward and both dgrads, plus "
            f"{win}x{win} wgrad windows over all rows of those experts; fp32 oracle, {secs:.1f} s")
    return flops / secs / 1e12, orc.num_threads(), desc


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is the one-GPU expert-layer path; it has no multi-GPU mode "
              "(no collectives, no sharding). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_07685_amd import binding as B
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl

    B.lib()  # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.workload]
    small = cfg.T * cfg.h <= 4 * 1024 * 1024
    hin = L.host_inputs(cfg) if small else None
    st = L.LayerState(cfg, hin, variant=args.variant, wgrad_f32=args.wgrad_f32, eq2=args.eq2,
                      fp8_wgrad=False if args.bf16_wgrad else None,
                      epilogue_quant=False if args.no_epilogue_quant else None, gather=args.gather)

    # one plain device copy of known size, outside the timed region: the reference dispatch the HBM byte
    # counters (FETCH_SIZE / WRITE_SIZE) of a profiler run are scaled by
    cal_src = torch.empty(CAL_COPY_BYTES, dtype=torch.uint8, device="cuda").fill_(1)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    del cal_src, cal_dst

    for _ in range(args.warmup):
        st.step()
    torch.cuda.synchronize()
    if st.forced_idx is None and cfg.E_router > cfg.E:
        st.R_live = int(st.counts.sum().item())   # rows whose expert lives here (outside the timed region)
    # timed region: K steps; every library call is followed by an event on the launch stream, so the
    # per-kernel durations come from the timed region itself (an event record costs about a microsecond)
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    per_step = [timed_step_with_events(st, torch, sync=False) for _ in range(args.steps)]
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms = e0.elapsed_time(e1) / args.steps
    ms = max(ms, 1e-6)
    assert st.ctx.poll_error() == 0
    calls = None
    for recs, evs in per_step:
        cur = [(lab, fl, by, evs[i].elapsed_time(evs[i + 1])) for i, (lab, fl, by) in enumerate(recs)]
        calls = cur if calls is None else [(a[0], a[1], a[2], a[3] + b[3]) for a, b in zip(calls, cur)]
    calls = [(lab, fl, by, t / args.steps) for lab, fl, by, t in calls]
    breakdown = {}
    for lab, fl, by, t in calls:
        d = {"ms": round(t, 4)}
        if fl:
            d["tflops"] = round(fl / t / 1e9, 1)
        if by:
            d["gbs"] = round(by / t / 1e6, 1)
        key, n = lab, 2
        while key in breakdown:
            key = f"{lab}#{n}"
            n += 1
        breakdown[key] = d
    gemm = [(t, lab, fl) for lab, fl, by, t in calls if fl]
    t_dom, n_dom, fl_dom = max(gemm)
    by_dom = next(by for lab, fl, by, t in calls if lab == n_dom)
    rw = measured_traffic(args.workload, n_dom) if args.variant is None else None
    traffic = round(sum(rw), 3) if rw else None
    achieved = fl_dom / t_dom / 1e9
    gemm_ms = sum(t for t, _, _ in gemm)
    gemm_fl = sum(fl for _, _, fl in gemm)
    peak = FP8_PEAK_TFLOPS if n_dom.endswith("fp8") else BF16_PEAK_TFLOPS  # ("..._fp8" and "..._mxfp8")

    flops = cfg.model_flops()
    if getattr(st, "R_live", None):
        flops = 18.0 * st.R_live * cfg.h * cfg.f + 18.0 * cfg.T * cfg.h * st.sf
    out = {
        "metric": "MoE-layer fwd+bwd TFLOPS/GPU at DeepSeek-V3 local shape" if args.workload == "C4"
                  else f"MoE-layer fwd+bwd TFLOPS/GPU ({cfg.name})",
        "value": round(flops / ms / 1e9, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "wall_ms_per_step": round(wall_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("mxfp8_e4m3 (fwd/dgrad/wgrad GEMMs) + bf16 moves" if cfg.mx else
                  "fp8_e4m3 (fwd/dgrad/wgrad GEMMs) + bf16 moves" if cfg.fp8 and st.fp8_wgrad else
                  "fp8_e4m3 (fwd/dgrad GEMMs) + bf16 (wgrad, moves)" if cfg.fp8 else "bf16"), "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} h={cfg.h} f={cfg.f} E_local={cfg.E} top{cfg.k} "
                               f"shared_f={cfg.shared_f} load={args.variant or cfg.load} "
                               f"wgrad_out={'f32' if args.wgrad_f32 else 'bf16'}"
                               f"{' weights-in-fc1 (eq. 2)' if args.eq2 else ''}"
                               f"{' gathered-operands' if args.gather else ''}",
                   "model_tflop_per_step": round(flops / 1e12, 3)},
        "pct_bf16_mfma_peak": round(100.0 * flops / ms / 1e9 / BF16_PEAK_TFLOPS, 2),
        "gemm_only": {"tflops": round(gemm_fl / gemm_ms / 1e9, 1),
                      "pct_peak": round(100.0 * gemm_fl / gemm_ms / 1e9 / BF16_PEAK_TFLOPS, 2)},
        "roofline": {"bound": "mfma", "kernel": f"gg_kernel ({n_dom})", "achieved": round(achieved, 1),
                     "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "traffic": traffic, "traffic_unit": "GB per launch (HBM-side read + write, offline counters: profiles/gg_kernel_<workload>_hbm_traffic.txt)",
                     "traffic_read_write_gb": list(rw) if rw else None,
                     "algorithmic_gb": round(by_dom / 1e9, 2) if by_dom else None},
        "kernels": breakdown,
    }
    if args.graph:
        # the same step captured once in a HIP graph (no allocation, copy or host sync inside it: every extent is read
        # on the device) and replayed K times; launch overhead is what differs from the eager figure above
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            st.step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(args.steps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        gms = g0.elapsed_time(g1) / args.steps
        assert st.ctx.poll_error() == 0
        out["graph"] = {"ms_per_step": round(gms, 4), "tflops": round(flops / gms / 1e9, 2)}
    if not (cfg.fp8 or cfg.mx) and not args.gather and not args.variant and not args.no_extras:
        # the same step with the permute's row move fused into the GEMMs that read the permuted tokens (no bf16 Xp; with
        # --eq2 no dO either): bit-identical results (tests/test_gpu_layer.py), reported beside the figure above, which
        # keeps the stand-alone permute kernel in the timed step
        sg = L.LayerState(cfg, hin, wgrad_f32=args.wgrad_f32, eq2=args.eq2, gather=True)
        for _ in range(max(args.warmup, 1)):
            sg.step()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(args.steps):
            sg.step()
        g1.record()
        torch.cuda.synchronize()
        gms = g0.elapsed_time(g1) / args.steps
        assert sg.ctx.poll_error() == 0
        out["gathered_operands"] = {"ms_per_step": round(gms, 4), "tflops": round(flops / gms / 1e9, 2)}
        sg.ctx.close()
        del sg
    # context only: the vendor dense bf16 GEMM through torch on this very box, at the size of one fc1 call of this
    # workload (rows = routed tokens, capped), same operand distribution, output preallocated
    m_ref = min(cfg.T * cfg.k, 131072)
    a_ref = torch.randn((m_ref, cfg.h), dtype=torch.bfloat16, device="cuda") * 0.02
    b_ref = torch.randn((4096, cfg.h), dtype=torch.bfloat16, device="cuda") * 0.02
    o_ref = torch.empty((m_ref, 4096), dtype=torch.bfloat16, device="cuda")
    for _ in range(3):
        torch.matmul(a_ref, b_ref.T, out=o_ref)
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record()
    for _ in range(10):
        torch.matmul(a_ref, b_ref.T, out=o_ref)
    r1.record()
    torch.cuda.synchronize()
    out["box_reference"] = {"what": f"torch.matmul bf16 {m_ref}x4096x{cfg.h} (dense, hipBLASLt) on this box",
                            "tflops": round(2.0 * m_ref * 4096 * cfg.h * 10 / r0.elapsed_time(r1) / 1e9, 1)}
    del o_ref
    del a_ref, b_ref
    out["box_reference"]["mfma_ceiling"] = mfma_ceiling()
    if not args.no_cpu_baseline:
        v, cores, desc = cpu_baseline(st, torch)
        out["cpu_baseline"] = {"value": round(v, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle", "sample": desc}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
