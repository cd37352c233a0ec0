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
HBM_PEAK_GBS = 8000.0       # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", help="C1 | MID | C2 | C3 | C4 (default: the metric's config)")
    ap.add_argument("--variant", default=None, help="load pattern override: uniform | zeros | hot | cv | zipf")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--wgrad-f32", action="store_true", help="fp32 weight gradients (default bf16)")
    return ap.parse_args()


def call_table(st):
    """(name, flops or None, bytes or None) for every library call of one step, in issue order."""
    cfg = st.cfg
    T, k, h, f, sf = cfg.T, cfg.k, cfg.h, cfg.f, st.sf
    R = T * k  # routed rows (unpadded)
    b = 2
    calls = [
        ("route_topk", None, T * cfg.E_router * 4 + T * k * 8 + cfg.E_router * 4),
        ("permute", None, (T + R) * h * b + T * k * 12),
        ("fc1_fwd_swiglu", 2.0 * R * 2 * f * h, None),
        ("fc2_fwd", 2.0 * R * f * h, None),
    ]
    if sf:
        calls += [("shared_fc1_fwd_swiglu", 2.0 * T * 2 * sf * h, None), ("shared_fc2_fwd", 2.0 * T * sf * h, None)]
    calls += [
        ("combine", None, (R + T) * h * b + T * k * 8 + (T * h * b if sf else 0)),
        ("combine_bwd", None, (T + 2 * R) * h * b),
        ("fc2_wgrad", 2.0 * R * f * h, None),
        ("fc2_dgrad_swiglu_bwd", 2.0 * R * f * h, None),
        ("fc1_wgrad", 2.0 * R * 2 * f * h, None),
        ("fc1_dgrad", 2.0 * R * 2 * f * h, None),
    ]
    if sf:
        calls += [("shared_fc2_wgrad", 2.0 * T * sf * h, None), ("shared_fc2_dgrad_swiglu_bwd", 2.0 * T * sf * h, None),
                  ("shared_fc1_wgrad", 2.0 * T * 2 * sf * h, None), ("shared_fc1_dgrad", 2.0 * T * 2 * sf * h, None)]
    calls += [("unpermute_sum_dx", None, (R + T) * h * b + (T * h * b if sf else 0))]
    return calls


def timed_step_with_events(st, torch):
    """One step with an event after every library call; returns per-call milliseconds."""
    from paper_2603_07685_amd import binding as B
    names = [c[0] for c in call_table(st)]
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)]
    it = iter(evs)
    orig = {}

    def wrap(fn):
        def inner(*a, **kw):
            r = fn(*a, **kw)
            next(it).record()
            return r
        return inner

    hooked = ["moe_route_topk", "moe_permute", "moe_grouped_gemm_fwd", "moe_grouped_gemm_dgrad",
              "moe_grouped_gemm_wgrad", "moe_unpermute_combine", "moe_unpermute_combine_bwd"]
    next(it).record()
    for n in hooked:
        orig[n] = getattr(B, n)
        setattr(B, n, wrap(orig[n]))
    try:
        st.step()
    finally:
        for n in hooked:
            setattr(B, n, orig[n])
    torch.cuda.synchronize()
    return [evs[i].elapsed_time(evs[i + 1]) for i in range(len(names))]


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
        xp = st.Xp[ridx].float().cpu().numpy()
        do = st.dO[ridx].float().cpu().numpy()
        w1 = st.W1[e].float().cpu().numpy()[None]
        w2 = st.W2[e].float().cpu().numpy()[None]
        o1 = np.array([0, n], np.int32)
        # wgrad windows over all rows of the expert
        wn, wk = min(win, h), min(win, f)
        dO_all = st.dO[lo:hi, :wn].float().cpu().numpy()
        A_all = st.A[lo:hi, :wk].float().cpu().numpy()
        dZ_all = st.dZ[lo:hi, :min(win, 2 * f)].float().cpu().numpy()
        Xp_all = st.Xp[lo:hi, :min(win, h)].float().cpu().numpy()
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
    st = L.LayerState(cfg, hin, variant=args.variant, wgrad_f32=args.wgrad_f32)

    for _ in range(args.warmup):
        st.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        st.step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms = e0.elapsed_time(e1) / args.steps
    ms = max(ms, 1e-6)
    assert st.ctx.poll_error() == 0

    # per-call durations (events on the same stream, extra instrumented steps after the timed region)
    reps = max(3, min(10, args.steps))
    per = None
    for _ in range(reps):
        cur = timed_step_with_events(st, torch)
        per = cur if per is None else [a + b for a, b in zip(per, cur)]
    per = [p / reps for p in per]
    calls = call_table(st)
    breakdown = {}
    for (name, fl, by), t in zip(calls, per):
        d = {"ms": round(t, 4)}
        if fl:
            d["tflops"] = round(fl / t / 1e9, 1)
        if by:
            d["gbs"] = round(by / t / 1e6, 1)
        breakdown[name] = d
    gemm = [(t, name, fl) for (name, fl, by), t in zip(calls, per) if fl]
    t_dom, n_dom, fl_dom = max(gemm)
    achieved = fl_dom / t_dom / 1e9
    gemm_ms = sum(t for t, _, _ in gemm)
    gemm_fl = sum(fl for _, _, fl in gemm)

    flops = cfg.model_flops()
    out = {
        "metric": "MoE-layer fwd+bwd TFLOPS/GPU at DeepSeek-V3 local shape" if args.workload == "C4"
                  else f"MoE-layer fwd+bwd TFLOPS/GPU ({cfg.name})",
        "value": round(flops / ms / 1e9, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "wall_ms_per_step": round(wall_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} h={cfg.h} f={cfg.f} E_local={cfg.E} top{cfg.k} "
                               f"shared_f={cfg.shared_f} load={args.variant or cfg.load} "
                               f"wgrad_out={'f32' if args.wgrad_f32 else 'bf16'}",
                   "model_tflop_per_step": round(flops / 1e12, 3)},
        "pct_bf16_mfma_peak": round(100.0 * flops / ms / 1e9 / BF16_PEAK_TFLOPS, 2),
        "gemm_only": {"tflops": round(gemm_fl / gemm_ms / 1e9, 1),
                      "pct_peak": round(100.0 * gemm_fl / gemm_ms / 1e9 / BF16_PEAK_TFLOPS, 2)},
        "roofline": {"bound": "mfma", "kernel": f"gg_kernel ({n_dom})", "achieved": round(achieved, 1),
                     "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / BF16_PEAK_TFLOPS, 4),
                     "traffic": None},
        "kernels": breakdown,
    }
    # context only: the vendor dense bf16 GEMM through torch on this very box (boxes differ by +-20 %)
    a_ref = torch.randn((16384, cfg.h), dtype=torch.bfloat16, device="cuda") * 0.02
    b_ref = torch.randn((4096, cfg.h), dtype=torch.bfloat16, device="cuda") * 0.02
    for _ in range(3):
        a_ref @ b_ref.T
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record()
    for _ in range(10):
        a_ref @ b_ref.T
    r1.record()
    torch.cuda.synchronize()
    out["box_reference"] = {"what": f"torch.matmul bf16 16384x4096x{cfg.h} (dense, hipBLASLt) on this box",
                            "tflops": round(2.0 * 16384 * 4096 * cfg.h * 10 / r0.elapsed_time(r1) / 1e9, 1)}
    del a_ref, b_ref
    if not args.no_cpu_baseline:
        v, cores, desc = cpu_baseline(st, torch)
        out["cpu_baseline"] = {"value": round(v, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle", "sample": desc}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
