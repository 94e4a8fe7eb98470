#!/usr/bin/env python3
"""Benchmark of the FLuRKA attention hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: sequence projection, key-side state, query stream,
and (for a workload with a backward pass) the full backward.  Prints ONE JSON
line.  `value` is tokens*heads per second of the whole step.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--algo auto]

The `roofline` object describes the stage that takes the most time, measured
with HIP events recorded on the stream the kernels run on (the library's
built-in stage timer), in a second loop of the same K steps so that the
events do not sit inside the region that `value` is computed from.
`cpu_baseline` times the fp64 oracle on a bounded sample of the same
workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0          # GB/s
PEAK_MFMA_BF16_TFLOPS = 2500.0  # dense bf16, TFLOP/s
PEAK_FP32_TFLOPS = 157.3        # vector fp32


def stage_model(w, stage: str):
    """Algorithmic (flops, bytes) of one stage for workload w: every caller tensor the
    stage needs read once, every result written once, no n x k or n x m matrix in HBM."""
    es = 2 if w.dtype == "bf16" else 4
    BH, n, d, k = w.B * w.H, w.n, w.d, w.k
    mf = w.d if w.phi == "elu1" else w.m
    perf = w.phi != "elu1"
    om = (w.H if w.omega_per_head else 1) * w.m * d * es if perf else 0
    small = 4 * BH * (2 * k * d + mf * d + mf)          # K', V', S, z in fp32
    if stage == "project":
        return 4.0 * k * n * d * BH, es * (2 * BH * n * d + 2 * k * n) + 4 * BH * 2 * k * d
    if stage == "key_state":
        fl = (2 * k * d * mf + 2 * k * mf * d + k * mf) * BH if perf else (2 * k * d * d + k * d) * BH
        return float(fl), small + om
    if stage == "query_stream":
        fl = (2 * n * d * mf + 2 * n * mf * d + 2 * n * mf) * BH if perf else (2 * n * d * d + 2 * n * d) * BH
        return float(fl), es * 2 * BH * n * d + om + 4 * BH * (mf * d + mf)
    if stage == "bwd_query":
        # with the forward's log-denominators and out at hand: u, G S^T, dQ, dS (performer)
        gemms = 4 if perf else 3
        return 2.0 * gemms * n * mf * d * BH, es * 4 * BH * n * d + om + 4 * BH * 2 * (mf * d + mf)
    if stage == "bwd_key":
        return float((4 * k * mf * d + (2 * k * mf * d if perf else 0)) * BH), 2 * small
    if stage == "bwd_dk_dv":
        return 4.0 * n * k * d * BH, es * (2 * k * n + 2 * BH * n * d) + 4 * BH * 2 * k * d
    if stage == "bwd_de_df":
        return 4.0 * k * n * d * BH, es * (2 * BH * n * d + 2 * k * n) + 4 * BH * 2 * k * d
    raise KeyError(stage)


# timer name of an MFMA-path kernel -> (name in rocprofv3 traces, stage it belongs to)
KERNEL_TRACE_NAME = {
    "gemm_mfma_proj": "gemm_mfma_kernel<ProjPolicy<{d}>, false>",        # one item per workgroup
    "proj_finish": "proj_finish_kernel",
    "key_state": "key_state_kernel<{d}, false>",
    "merge_pack": "merge_pack_kernel",
    "query_stream": "query_stream_kernel<{d}, {elu}, {qs_waves}, 1, {elu}>",     # staged tiles: elu1 only
    "bwd_query_x": "bwd_query_x_kernel<{d}, {ring}>",              # ring: d = 128 with more than 192 features
    "bwd_query_y": "bwd_query_y_kernel<{d}, 8, false>",
    "bwd_merge": "bwd_merge_kernel",
    "bwd_key": "bwd_key_kernel<{d}>",
    "gemm_mfma_gradx": "gemm_mfma_kernel<GradXPolicy<{d}>, true>",      # several items per workgroup
    "gemm_mfma_grade": "gemm_mfma_kernel<GradEPolicy<{d}, false>, false>",
    "sum_splits": "sum_splits_bf16_kernel",
}


def kernel_model(w, kernel: str):
    """Algorithmic (flops, bytes) of one kernel of the MFMA path (recomputation is not counted: the
    backward's four n*m*d contractions are split 3 : 1 between bwd_query_x, which forms u, G S^T and
    dQ, and bwd_query_y, whose second evaluation of u is not counted)."""
    es = 2 if w.dtype == "bf16" else 4
    BH, n, d, k = w.B * w.H, w.n, w.d, w.k
    mf = w.d if w.phi == "elu1" else w.m
    if kernel == "gemm_mfma_proj":
        return stage_model(w, "project")
    if kernel == "query_stream":
        return stage_model(w, "query_stream")
    if kernel == "key_state":
        return stage_model(w, "key_state")
    if kernel == "bwd_query_x":
        return 6.0 * n * mf * d * BH, es * 4 * BH * n * d + 8 * BH * n
    if kernel == "bwd_query_y":
        return 2.0 * n * mf * d * BH, es * 2 * BH * n * d + 8 * BH * n + 4 * BH * mf * d
    if kernel == "bwd_key":
        return stage_model(w, "bwd_key")
    if kernel == "gemm_mfma_gradx":
        return stage_model(w, "bwd_dk_dv")
    if kernel == "gemm_mfma_grade":
        return stage_model(w, "bwd_de_df")
    # small helper kernels: data movement only
    small = 4 * BH * (2 * k * d + mf * d + mf)
    return 0.0, float(small)


def whole_model(w):
    stages = ["project", "key_state", "query_stream"]
    if w.backward:
        stages += ["bwd_query", "bwd_key", "bwd_dk_dv", "bwd_de_df"]
    fl = sum(stage_model(w, s)[0] for s in stages)
    es = 2 if w.dtype == "bf16" else 4
    BH, n, d, k = w.B * w.H, w.n, w.d, w.k
    om = (w.H if w.omega_per_head else 1) * w.m * d * es if w.phi != "elu1" else 0
    by = es * (4 * BH * n * d + 2 * k * n) + om                       # forward: Q,K,V,E,F,omega in, out out
    if w.backward:
        # backward: Q, K, V, out, dOut, E, F, omega in; dQ, dK, dV, dE, dF out
        by += es * (5 * BH * n * d + 2 * k * n) + om + es * (3 * BH * n * d + 2 * k * n)
    return fl, by


def roofline_entry(w, stage, avg_ms, launches_note, model=None):
    fl, by = (model or stage_model)(w, stage)
    sec = avg_ms * 1e-3
    peak_fl = PEAK_MFMA_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS
    t_fl = fl / (peak_fl * 1e12)
    t_by = by / (PEAK_HBM_GBS * 1e9)
    if t_fl >= t_by:
        bound = "mfma" if w.dtype == "bf16" else "alu"
        achieved, peak, unit = fl / sec / 1e12, peak_fl, "TFLOP/s"
    else:
        bound, achieved, peak, unit = "hbm", by / sec / 1e9, PEAK_HBM_GBS, "GB/s"
    return {"kernel": stage, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
            "frac": round(achieved / peak, 4), "traffic": None, "avg_ms": round(avg_ms, 5),
            "alg_flops": fl, "alg_bytes": by,
            "tflops": round(fl / sec / 1e12, 3), "gbs": round(by / sec / 1e9, 2), "note": launches_note}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C5", help="C1..C5 (C5 = forward+backward, the headline metric); C4T = C4's shape with a backward pass")
    ap.add_argument("--algo", default="auto", choices=["auto", "generic", "fast"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the device copy and library GEMM that give the box's achievable HBM and MFMA rates")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target wall time of the oracle sample")
    args = ap.parse_args()

    if args.gpus != 1:
        print(f"bench.py: this build runs on exactly one GPU; --gpus {args.gpus} is not supported "
              "(no collectives, no sharding in this library)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2306_15799_amd import binding as fb
    from paper_2306_15799_amd import inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    fb.load_library()          # raises if the HIP library has not been built: there is no fallback

    w = {**inputs.WORKLOADS, **inputs.DERIVED_WORKLOADS}[args.workload]
    t = inputs.make_inputs(w, seed=0)
    td = torch.float32 if w.dtype == "f32" else torch.bfloat16
    dev = torch.device("cuda:0")
    g = {k: (None if v is None else torch.from_numpy(v).to(dev).to(td).contiguous()) for k, v in t.items()}
    if w.backward and "dOut" not in g:
        raise RuntimeError("workload has a backward pass but no dOut")

    code = fb.BF16 if w.dtype == "bf16" else fb.F32
    m_eff = w.d if w.phi == "elu1" else w.m
    dims = (w.B, w.H, w.n, w.d, w.k, m_eff)
    ctx = fb.alloc_buffer(fb.ctx_bytes(*dims, code, w.phi), dev)
    ws_f = fb.alloc_buffer(fb.workspace_bytes(*dims, code, w.phi, fb.PASS_FWD, args.algo), dev)
    out = torch.empty_like(g["Q"])
    grads = ws_b = None
    if w.backward:
        ws_b = fb.alloc_buffer(fb.workspace_bytes(*dims, code, w.phi, fb.PASS_BWD, args.algo), dev)
        grads = (torch.empty_like(g["Q"]), torch.empty_like(g["Q"]), torch.empty_like(g["Q"]),
                 torch.empty_like(g["E"]), torch.empty_like(g["E"]))

    def step():
        fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], phi=w.phi, algo=args.algo,
                           out=out, ctx=ctx, workspace=ws_f)
        if w.backward:
            fb.flurka_attn_bwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx,
                               phi=w.phi, algo=args.algo, workspace=ws_b, grads=grads)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = ev0.elapsed_time(ev1) / args.steps

    # per-stage times from HIP events on the kernels' own stream, same K steps again
    fb.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    rec = fb.profile_read()
    fb.profile_enable(False)
    # timer entries are "stage" (generic kernels) or "stage:kernel" (MFMA path, one kernel each)
    steps_seen = max(1, args.steps)
    stage_tot, kernel_tot, kernel_cnt = {}, {}, {}
    for name, ms in rec:
        stage, _, kern = name.partition(":")
        stage_tot[stage] = stage_tot.get(stage, 0.0) + ms
        if kern:
            kernel_tot[kern] = kernel_tot.get(kern, 0.0) + ms
            kernel_cnt[kern] = kernel_cnt.get(kern, 0) + 1
    stage_avg = {k: v / steps_seen for k, v in stage_tot.items()}
    stages_out = {}
    for name, ms in stage_avg.items():
        fl, by = stage_model(w, name)
        stages_out[name] = {"ms": round(ms, 5), "tflops": round(fl / ms / 1e9, 2), "gbs": round(by / ms / 1e6, 1)}
    kernels_out = {k: {"avg_ms": round(kernel_tot[k] / kernel_cnt[k], 5), "launches_per_step": kernel_cnt[k] / steps_seen}
                   for k in kernel_tot}
    if kernel_tot:
        # dominant kernel = largest time per step; its average launch duration from the HIP events
        dominant = max(kernel_tot, key=kernel_tot.get)
        avg_launch = kernel_tot[dominant] / kernel_cnt[dominant]
        roof = roofline_entry(w, dominant, avg_launch,
                              "HIP events around each launch of this kernel, on the stream it runs on",
                              model=kernel_model)
        trace = KERNEL_TRACE_NAME[dominant].format(d=w.d, elu="true" if w.phi == "elu1" else "false",
                                                   qs_waves=12 if w.d == 64 else 8,
                                                   ring="true" if (w.d == 128 and m_eff > 192) else "false")
        roof["kernel_in_trace"] = trace
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            tr = json.load(open(tpath)).get(w.name, {}).get("kernels", {}).get(trace)
            if tr:
                roof["traffic"] = tr["read_bytes"] + tr["write_bytes"]
                roof["traffic_note"] = "HBM bytes per launch from rocprofv3 FETCH_SIZE/WRITE_SIZE runs (profiles/hbm_traffic_%s.txt)" % w.name
    else:
        dominant = max(stage_avg, key=stage_avg.get)
        roof = roofline_entry(w, dominant, stage_avg[dominant],
                              "stage time = HIP events around the stage's launches on their stream")

    fl_all, by_all = whole_model(w)
    sec = ms_per_step * 1e-3
    value = w.tokens_heads / sec

    result = {
        "metric": "FLuRKA attn fwd+bwd tokens*heads/s" if w.backward else "FLuRKA attn fwd tokens*heads/s",
        "value": round(value, 1), "unit": "tokens*heads/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "wall_ms_per_step": round(wall_ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} n={w.n} d={w.d} k={w.k} m={m_eff} {w.dtype} "
                               f"{w.phi} {'fwd+bwd' if w.backward else 'fwd'}", "algo": args.algo,
                   "fast_path": bool(fb.fast_path_supported(*dims, code, w.phi, fb.PASS_FWD))},
        "whole_step": {"tflops": round(fl_all / sec / 1e12, 3), "gbs": round(by_all / sec / 1e9, 2),
                       "alg_flops": fl_all, "alg_bytes": by_all,
                       "frac_of_binding_roof": round(max(fl_all / (PEAK_MFMA_BF16_TFLOPS * 1e12 if w.dtype == "bf16" else PEAK_FP32_TFLOPS * 1e12),
                                                         by_all / (PEAK_HBM_GBS * 1e9)) / sec, 4)},
        "stages": stages_out,
        "kernels": kernels_out,
        "roofline": roof,
    }

    if not args.no_measured_peaks:
        # What this machine sustains, beside the published peaks: a plain device copy (read + write) and the
        # vendor library's bf16 GEMM, both through torch.  Context for the fractions above, not a target.
        def timed(fn, reps):
            fn(); torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / reps
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev)       # 1 GiB
        dst = torch.empty_like(src)
        t_copy = timed(lambda: dst.copy_(src), 10)
        del dst
        a_ = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
        b_ = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
        t_mm = timed(lambda: torch.matmul(a_, b_), 10)
        copy_gbs = 2.0 * src.numel() * 4 / t_copy / 1e9
        mm_tflops = 2.0 * 8192 ** 3 / t_mm / 1e12
        del src, a_, b_
        result["measured_peaks"] = {"hbm_copy_gbs": round(copy_gbs, 1), "bf16_gemm_tflops": round(mm_tflops, 1),
                                    "how": "torch copy_ of 1 GiB fp32 (bytes read + written); torch.matmul 8192^3 bf16"}
        meas = copy_gbs if roof["bound"] == "hbm" else (mm_tflops if roof["bound"] == "mfma" else None)
        if meas:
            roof["frac_of_measured_peak"] = round(roof["achieved"] / meas, 4)

    if not args.no_cpu_baseline:
        from oracle import flurka_oracle as fo
        import threadpoolctl
        threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
        # bounded sample: whole heads of the same workload, one after another, until the time target
        heads = [(b, h) for b in range(w.B) for h in range(w.H)]
        done, t_start = 0, time.perf_counter()
        errs = []
        passes = 0
        while time.perf_counter() - t_start < args.cpu_seconds and passes < 64:
          passes += 1
          for (b, h) in heads:
            om = None if t["omega"] is None else np.asarray(t["omega"][h if t["omega"].shape[0] > 1 else 0], np.float64)
            ref = fo.flurka_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["E"], t["F"], om, w.phi)
            if w.backward:
                fo.flurka_head_bwd(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["E"], t["F"], om,
                                   t["dOut"][b, h], w.phi)
            done += 1
            if passes == 1:
                errs.append(fo.rel_l2(out[b, h].float().cpu().numpy(), ref))
            if time.perf_counter() - t_start >= args.cpu_seconds:
                break
        cpu_s = time.perf_counter() - t_start
        result["cpu_baseline"] = {"value": round(done * w.n / cpu_s, 1), "unit": "tokens*heads/s",
                                  "cores": int(threads), "kind": "oracle",
                                  "sample": f"{done} (batch, head) slices ({len(heads)} distinct) of {w.name}, "
                                            f"{'fwd+bwd' if w.backward else 'fwd'}, fp64 numpy, {cpu_s:.1f} s"}
        result["parity_sample_rel_l2_out"] = float(max(errs))

    print(json.dumps(result))


if __name__ == "__main__":
    main()
