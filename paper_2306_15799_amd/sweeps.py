"""Attention-level counterparts of the paper's three speed experiments, on one MI355X.

    python -m paper_2306_15799_amd.sweeps [--steps 30] [--out profiles/sweeps_attention_level.txt]

The paper times whole models (Sec. 4.1 "Model speed": sequence length N from 7k to 55k; Sec. 4.3: the
downsampling factor d_k against the low-rank method, the model width d_m against the kernel method).
Here the same three sweeps run on the attention path alone, forward, bf16, synthetic inputs of the
benchmark recipe, through the library's own entry points:

  flurka        flurka_attn_fwd                         (projection + kernel attention over k keys)
  kernel        flurka_baseline_fwd(KERNEL_ATTN)        (kernel attention over all n keys)
  linformer     flurka_baseline_fwd(LINFORMER)          (softmax over the k projected keys)
  paper order   flurka_attn_fwd_fused_w                 (projection of the model-wide input, then W)
  kernel + W    torch.matmul for X W over n positions + kernel baseline   (what a kernel method pays)

Shapes follow the paper's where the kernels allow (head size 64 as in its Table 6; its k = 1500 .. 20000
exceed what the Linformer baseline keeps in LDS, so k stays <= 512 there).  Times are medians over
`steps` calls after a warm-up; every figure is a single-GPU forward time in milliseconds.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _time(torch, fn, steps):
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.15:        # leave the idle power state, warm the code caches
        fn()
        torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evs[0].record()
    for i in range(steps):
        fn()
        evs[i + 1].record()
    torch.cuda.synchronize()
    return statistics.median(evs[i].elapsed_time(evs[i + 1]) for i in range(steps))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--out", default=None, help="also write the tables to this file")
    args = ap.parse_args()

    import torch
    from paper_2306_15799_amd import binding as fb
    from paper_2306_15799_amd import inputs
    from paper_2306_15799_amd.inputs import Workload, PHI_PERFORMER

    if not torch.cuda.is_available():
        sys.exit("sweeps: no GPU visible")
    fb.load_library()
    dev = torch.device("cuda:0")
    lines, records = [], []

    def emit(s=""):
        print(s, flush=True)
        lines.append(s)

    def upload(t):
        return {k: (None if v is None else torch.from_numpy(v).to(dev).to(torch.bfloat16).contiguous()) for k, v in t.items()}

    def three_ways(B, H, n, d, k, m):
        """ms of flurka, kernel attention and Linformer on one input set (None where unsupported)."""
        w = Workload("sweep", B, H, n, d, k, m, "bf16", PHI_PERFORMER, False)
        g = upload(inputs.make_inputs(w, 0))
        dims = (B, H, n, d, k, m)
        out = torch.empty_like(g["Q"])
        ctx = fb.alloc_buffer(fb.ctx_bytes(*dims, fb.BF16, w.phi), dev)
        ws = fb.alloc_buffer(fb.workspace_bytes(*dims, fb.BF16, w.phi, fb.PASS_FWD, "auto"), dev)
        res = {"flurka": _time(torch, lambda: fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"],
                                                                  phi=w.phi, out=out, ctx=ctx, workspace=ws), args.steps)}
        lib = fb.load_library()
        for name, which, kk, mm in (("kernel", fb.BASELINE_KERNEL_ATTN, n, m), ("linformer", fb.BASELINE_LINFORMER, k, 32)):
            if not fb.baseline_supported(which, B, H, n, d, kk, mm, fb.BF16, w.phi):
                res[name] = None
                continue
            bctx = fb.alloc_buffer(lib.flurka_baseline_ctx_bytes(which, B, H, n, d, kk, mm, fb.BF16, 0), dev)
            bws = fb.alloc_buffer(lib.flurka_baseline_workspace_bytes(which, B, H, n, d, kk, mm, fb.BF16, 0), dev)
            res[name] = _time(torch, lambda: fb.flurka_baseline_fwd(which, g["Q"], g["K"], g["V"], E=g["E"], F=g["F"],
                                                                    omega=g["omega"], phi=w.phi, out=out, ctx=bctx,
                                                                    workspace=bws), args.steps)
        del g, out, ctx, ws
        torch.cuda.empty_cache()
        return res

    def fmt(x):
        return "     -  " if x is None else f"{x:8.3f}"

    def ratio(a, b):
        return "    - " if (a is None or b is None) else f"{a / b:6.2f}"

    emit("Attention-level sweeps, forward, bf16, one MI355X (milliseconds, median of %d calls)" % args.steps)
    emit("command (from the repository root on the GPU box): python -m paper_2306_15799_amd.sweeps --steps %d" % args.steps)
    emit()
    emit("1. Sequence length (Sec. 4.1 \"Model speed\"): B=1 H=16 d=64 k=512 m=256")
    emit(f"{'N':>8s} {'flurka':>8s} {'kernel':>8s} {'linformer':>9s}   kernel/flurka  linformer/flurka")
    for n in range(7040, 55489, 6016):
        r = three_ways(1, 16, n, 64, 512, 256)
        records.append({"sweep": "N", "n": n, **r})
        emit(f"{n:8d} {fmt(r['flurka'])} {fmt(r['kernel'])} {fmt(r['linformer']):>9s}   {ratio(r['kernel'], r['flurka']):>13s}  {ratio(r['linformer'], r['flurka']):>16s}")
    emit()
    emit("2. Downsampling factor (Sec. 4.3, against the low-rank method): B=1 H=16 N=20032 d=64 m=256")
    emit(f"{'k':>8s} {'flurka':>8s} {'linformer':>9s}   linformer/flurka")
    for k in (128, 256, 384, 512):
        r = three_ways(1, 16, 20032, 64, k, 256)
        records.append({"sweep": "k", "k": k, **r})
        emit(f"{k:8d} {fmt(r['flurka'])} {fmt(r['linformer']):>9s}   {ratio(r['linformer'], r['flurka']):>16s}")
    emit()
    emit("3. Model width (Sec. 4.3, against the kernel method): B=1 N=20032 d=64 H=dm/64 k=512 m=256; the layer")
    emit("   inputs are (B, N, dm); the kernel method transforms all N positions (vendor GEMM), the paper's order")
    emit("   transforms the k projected rows")
    emit(f"{'dm':>8s} {'paper order':>12s} {'kernel + W':>11s}   (kernel + W)/paper order")
    for dm in (512, 1024, 2048, 4096):
        H, n, d, k, m = dm // 64, 20032, 64, 512, 256
        w = Workload("sweep_dm", 1, H, n, d, k, m, "bf16", PHI_PERFORMER, False)
        g = upload(inputs.make_paper_order_inputs(w, dm, 0))
        dims = (1, H, n, d, k, m)
        lib = fb.load_library()
        out = torch.empty_like(g["Q"])
        ctx = fb.alloc_buffer(fb.ctx_bytes(*dims, fb.BF16, w.phi), dev)
        ws = fb.alloc_buffer(lib.flurka_fused_w_workspace_bytes(*dims, dm, fb.BF16, 0), dev)
        t_po = _time(torch, lambda: fb.flurka_attn_fwd_fused_w(g["Q"], g["XK"], g["XV"], g["E"], g["F"], g["WK"], g["WV"],
                                                              g["omega"], phi=w.phi, out=out, ctx=ctx, workspace=ws), args.steps)
        wk2 = g["WK"].reshape(H * d, dm).t().contiguous()
        wv2 = g["WV"].reshape(H * d, dm).t().contiguous()
        bctx = fb.alloc_buffer(lib.flurka_baseline_ctx_bytes(fb.BASELINE_KERNEL_ATTN, 1, H, n, d, n, m, fb.BF16, 0), dev)
        bws = fb.alloc_buffer(lib.flurka_baseline_workspace_bytes(fb.BASELINE_KERNEL_ATTN, 1, H, n, d, n, m, fb.BF16, 0), dev)

        def kernel_method():
            K = torch.matmul(g["XK"], wk2).view(1, n, H, d).permute(0, 2, 1, 3).contiguous()
            V = torch.matmul(g["XV"], wv2).view(1, n, H, d).permute(0, 2, 1, 3).contiguous()
            fb.flurka_baseline_fwd(fb.BASELINE_KERNEL_ATTN, g["Q"], K, V, omega=g["omega"], phi=w.phi, out=out, ctx=bctx,
                                   workspace=bws)
        t_kw = _time(torch, kernel_method, args.steps)
        records.append({"sweep": "dm", "dm": dm, "paper_order": t_po, "kernel_plus_w": t_kw})
        emit(f"{dm:8d} {t_po:12.3f} {t_kw:11.3f}   {t_kw / t_po:24.2f}")
        del g, out, ctx, ws, bctx, bws
        torch.cuda.empty_cache()
    emit()
    print(json.dumps(records))
    if args.out:
        with open(os.path.join(ROOT, args.out) if not os.path.isabs(args.out) else args.out, "w") as f:
            f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
