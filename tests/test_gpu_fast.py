"""GPU parity of the bf16 MFMA kernels (algo = fast) against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import flurka_oracle as fo
from paper_2306_15799_amd import binding as fb
from paper_2306_15799_amd import inputs
from paper_2306_15799_amd.inputs import Workload, PHI_ELU1, PHI_PERFORMER

import gpu_util as gu

pytestmark = pytest.mark.gpu

# (B, H, n, d, k, m): several 256-wide column tiles, ragged head count per tile, ragged k,
# a sequence split over several workgroups, both head sizes
# the last two: more (head, tile) pairs than resident workgroups, so one workgroup's share crosses
# from one head into the next and refills its LDS image; many heads with few tiles each
FWD_SHAPES = [
    (1, 3, 192, 64, 100, 96),
    (2, 5, 1024, 64, 256, 256),
    (1, 3, 640, 128, 300, 160),
    (3, 2, 2048, 128, 512, 32),
    (1, 1, 64, 64, 1, 32),
    (3, 5, 1088, 64, 96, 128),
    (8, 16, 128, 128, 40, 64),
    # sequence lengths that are multiples of 8 only: a ragged last reduction step of the projection (whose
    # missing positions would otherwise read the next head's rows), a ragged last query tile
    (1, 3, 200, 64, 100, 96),
    (2, 5, 1000, 64, 256, 256),
    (2, 2, 72, 128, 8, 32),
    (1, 3, 1048, 128, 300, 160),
    (2, 3, 8, 64, 4, 32),
    # more projection tiles than one resident round of workgroups: every workgroup streams several tiles,
    # the requests for a tile's first steps being issued during the previous tile's last ones (with a
    # ragged last step in each)
    (8, 40, 200, 128, 40, 32),
    # feature counts that are not multiples of 32: the last feature tile is padded with features of weight 0
    (1, 3, 192, 64, 100, 72),
    (2, 2, 1000, 128, 300, 200),
    (1, 2, 256, 64, 64, 8),
    (2, 3, 640, 128, 96, 250),
    (1, 2, 512, 64, 200, 500),
]


@pytest.mark.parametrize("shape", FWD_SHAPES)
def test_forward_performer(shape):
    B, H, n, d, k, m = shape
    w = Workload("fast", B, H, n, d, k, m, "bf16", PHI_PERFORMER, False)
    assert fb.fast_path_supported(B, H, n, d, k, m, fb.BF16, w.phi)
    err = gu.check_forward(w, seed=7, algo="fast")
    print(shape, f"rel-L2 {err:.3e}")


@pytest.mark.parametrize("shape", [(1, 3, 192, 64, 100), (2, 4, 1024, 64, 256), (1, 2, 320, 128, 64),
                                   (1, 3, 200, 64, 100), (2, 2, 328, 128, 64)])
def test_forward_elu(shape):
    B, H, n, d, k = shape
    w = Workload("fast", B, H, n, d, k, d, "bf16", PHI_ELU1, False)
    err = gu.check_forward(w, seed=8, algo="fast")
    print(shape, f"rel-L2 {err:.3e}")


@pytest.mark.parametrize("n", [4096, 4120])
def test_fast_projection_matches_oracle_projection(n):
    w = Workload("proj", 1, 6, n, 64, 256, 64, "bf16", PHI_PERFORMER, False)
    t = inputs.make_inputs(w, 9)
    _, _, ctx = gu.run_forward(w, t, "fast")
    v = fb.ctx_views(ctx, w.B, w.H, w.n, w.d, w.k, w.m, fb.BF16, w.phi)
    Kp = np.matmul(t["E"].astype(np.float64), t["K"].astype(np.float64))
    Vp = np.matmul(t["F"].astype(np.float64), t["V"].astype(np.float64))
    # bf16 x bf16 products are exact in fp32; only the fp32 summation order differs
    assert fo.rel_l2(gu.to_host(v["Kp"]), Kp) < 2e-6
    assert fo.rel_l2(gu.to_host(v["Vp"]), Vp) < 2e-6
    # the forward also leaves the log of every row's denominator for the backward pass
    for h in range(w.H):
        om = t["omega"][h].astype(np.float64)
        e = Kp[0, h] @ om.T - 0.5 * np.sum(Kp[0, h] ** 2, axis=1, keepdims=True)
        lse = gu.log_denominator(t["Q"][0, h], om, e)
        assert np.max(np.abs(gu.to_host(v["lse"][0, h]) - lse)) < 2e-3 * max(1.0, np.abs(lse).max())


def test_shared_omega_and_determinism():
    w = Workload("shared", 2, 3, 512, 64, 128, 64, "bf16", PHI_PERFORMER, False, omega_per_head=False)
    t = inputs.make_inputs(w, 10)
    _, out1, _ = gu.run_forward(w, t, "fast")
    _, out2, _ = gu.run_forward(w, t, "fast")
    assert torch.equal(out1, out2)
    assert fo.rel_l2(gu.to_host(out1), gu.oracle_forward(w, t)) < 2e-2


def test_unsupported_shapes_are_refused_not_miscomputed():
    # n not a multiple of 8, head size other than 64/128, fp32 storage
    assert not fb.fast_path_supported(1, 1, 100, 64, 8, 32, fb.BF16, "performer")
    assert not fb.fast_path_supported(1, 1, 128, 48, 8, 32, fb.BF16, "performer")
    assert not fb.fast_path_supported(1, 1, 128, 64, 8, 32, fb.F32, "performer")
    w = Workload("odd", 1, 1, 100, 64, 8, 32, "bf16", PHI_PERFORMER, False)
    t = inputs.make_inputs(w, 11)
    g = gu.to_device(t, "bf16")
    with pytest.raises(fb.FlurkaError) as e:
        fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], algo="fast")
    assert e.value.status == fb.ERR_UNSUPPORTED
    # auto falls back to the generic kernels and still matches
    assert gu.check_forward(w, seed=11, algo="auto") < 2e-2


# ---- backward ------------------------------------------------------------------------------
# (3, 5, 1088, ...): 34 query tiles per head -- shares of the resident grid cross head boundaries, and
# the last 128-query block of each range of the dS kernel is only half filled
BWD_SHAPES = [
    (1, 3, 192, 64, 100, 96),
    (2, 5, 1024, 64, 256, 256),
    (2, 2, 2048, 64, 64, 32),
    (3, 5, 1088, 64, 96, 128),
    (8, 16, 128, 64, 40, 64),
    # head size 128: rows move between memory and registers directly (up to 192 features fit LDS)
    (1, 3, 640, 128, 300, 160),
    (2, 2, 1024, 128, 256, 192),
    (3, 2, 2048, 128, 512, 32),
    (4, 8, 192, 128, 40, 96),
    # head size 128 with 256 features: the lo terms of S/z pass through a two-slot LDS ring, the
    # wavefronts of a workgroup walk the feature tiles in step (rounds with idle wavefronts; shares that
    # cross from one head into the next)
    (2, 2, 1024, 128, 256, 256),
    (1, 3, 2112, 128, 300, 256),
    (8, 16, 128, 128, 40, 256),
    # many tiles: the dE/dF contraction fills the chip without splitting its reduction and stores its
    # result directly (ragged k and a ragged last column tile; both head sizes)
    (1, 1, 8256, 64, 1000, 32),
    (1, 2, 4160, 128, 1000, 32),
    # attention concentrated on few (key, feature) pairs (long sequence, few features, |k'|^2 ~ 500): the
    # sums of the chain rule cancel almost completely; a g_i taken from the rounded output alone, or S
    # rounded to a single bf16 term, puts tens of percent of error on dK here
    (1, 1, 32832, 64, 500, 32),
    # sequence lengths that are odd multiples of 32: a last reduction step of the projection and last
    # position tiles of the gradient GEMMs that are only partly there (both head sizes, the ring variant)
    (1, 3, 96, 64, 40, 64),
    (2, 2, 1056, 64, 100, 96),
    (1, 2, 2080, 128, 300, 160),
    (2, 2, 1056, 128, 256, 256),
    # feature counts that are not multiples of 32 (the last feature tile padded with features of weight 0);
    # 250 features at head size 128 run the ring variant
    (1, 3, 192, 64, 100, 72),
    (2, 2, 1056, 128, 300, 200),
    (1, 2, 256, 64, 64, 8),
    (2, 2, 640, 128, 96, 250),
    (1, 2, 512, 64, 200, 280),
]


@pytest.mark.parametrize("shape", BWD_SHAPES)
def test_forward_backward_performer(shape):
    B, H, n, d, k, m = shape
    w = Workload("fastbwd", B, H, n, d, k, m, "bf16", PHI_PERFORMER, True)
    assert fb.fast_path_supported(B, H, n, d, k, m, fb.BF16, w.phi, fb.PASS_BWD)
    errs = gu.check_forward_backward(w, seed=12, algo="fast")
    print(shape, {k_: f"{v:.2e}" for k_, v in errs.items()})


# elu1: dQ, dS, dz on MFMA kernels of their own, the key side on the generic kernels, the four
# sequence-length GEMMs shared with the random-feature map
@pytest.mark.parametrize("shape", [(1, 3, 192, 64, 100), (2, 4, 1024, 64, 256), (1, 2, 320, 128, 64),
                                   (3, 5, 1088, 64, 96), (1, 2, 16384, 64, 256), (2, 2, 2048, 128, 300),
                                   (2, 3, 160, 64, 100), (1, 2, 1056, 128, 300)])
def test_forward_backward_elu(shape):
    B, H, n, d, k = shape
    w = Workload("fastbwd_elu", B, H, n, d, k, d, "bf16", PHI_ELU1, True)
    assert fb.fast_path_supported(B, H, n, d, k, d, fb.BF16, w.phi, fb.PASS_BWD)
    errs = gu.check_forward_backward(w, seed=16, algo="fast")
    print(shape, {k_: f"{v:.2e}" for k_, v in errs.items()})


@pytest.mark.parametrize("phi", [PHI_PERFORMER, PHI_ELU1])
@pytest.mark.parametrize("B,H,n,d,k,m", [(1, 1, 64, 64, 1, 32), (2, 1, 64, 128, 3, 32), (1, 2, 128, 64, 200, 32)])
def test_degenerate_shapes_through_the_mfma_kernels(phi, B, H, n, d, k, m):
    """Smallest sequence the path takes (one 64-row step), k = 1 (the output ignores Q and K: dQ, dK, dE are
    exactly zero and are measured against unit scale), fewer keys than one tile, more keys than positions."""
    mm = d if phi == PHI_ELU1 else m
    w = Workload("tiny", B, H, n, d, k, mm, "bf16", phi, True)
    assert fb.fast_path_supported(B, H, n, d, k, mm, fb.BF16, phi, fb.PASS_BWD)
    errs = gu.check_forward_backward(w, seed=18, algo="fast", floor=1.0 if k == 1 else 0.0)
    print((phi, B, H, n, d, k, mm), {k_: f"{v:.2e}" for k_, v in errs.items()})


@pytest.mark.parametrize("qs,ks", [(3.0, 1.0), (1.0, 2.5), (0.05, 0.05)])
def test_large_and_small_input_norms(qs, ks):
    """Exponents far from the synthetic workloads' range: queries three times longer (u up to ~ +-60 with a
    spread of e^40 between the features of one row), keys 2.5 times longer (|k'|^2/2 in the hundreds, key
    weights spanning hundreds of e-folds), and nearly uniform attention (everything scaled down)."""
    w = Workload("norms", 1, 2, 1024, 64, 128, 128, "bf16", PHI_PERFORMER, True)
    t = inputs.make_inputs(w, 19)
    t["Q"] = inputs.round_to_bf16(t["Q"] * qs)
    t["K"] = inputs.round_to_bf16(t["K"] * ks)
    g, out, ctx = gu.run_forward(w, t, "fast")
    errs = {"out": fo.rel_l2(gu.to_host(out), gu.oracle_forward(w, t))}
    grads = gu.run_backward(w, g, out, ctx, "fast")
    for name, a, b in zip(["dQ", "dK", "dV", "dE", "dF"], grads, gu.oracle_backward(w, t)):
        errs[name] = gu.rel_err(gu.to_host(a), b)
    print((qs, ks), {k_: f"{v:.2e}" for k_, v in errs.items()})
    assert all(v <= 2e-2 for v in errs.values()), errs
    assert all(torch.isfinite(x.float()).all() for x in (out, *grads))


@pytest.mark.parametrize("phi,d,m", [(PHI_PERFORMER, 64, 96), (PHI_PERFORMER, 128, 256), (PHI_ELU1, 64, 64)])
def test_backward_is_linear_in_the_upstream_gradient(phi, d, m):
    """Every gradient is linear in dOut, and scaling by a power of two commutes with every rounding on
    the way: grads(4 dOut) = 4 grads(dOut) bit for bit, and grads(0) = 0 exactly."""
    w = Workload("lin", 2, 2, 512, d, 96, m, "bf16", phi, True)
    t = inputs.make_inputs(w, 20)
    g, out, ctx = gu.run_forward(w, t, "fast")
    base = gu.run_backward(w, g, out, ctx, "fast")
    g4 = dict(g); g4["dOut"] = g["dOut"] * 4
    quad = gu.run_backward(w, g4, out, ctx, "fast")
    g0 = dict(g); g0["dOut"] = torch.zeros_like(g["dOut"])
    zero = gu.run_backward(w, g0, out, ctx, "fast")
    for name, a, b, z in zip(["dQ", "dK", "dV", "dE", "dF"], base, quad, zero):
        assert torch.equal(a * 4, b), name
        assert not z.float().abs().max().item(), name


def test_backward_matches_generic_kernels_closely():
    """Same inputs through both kernel families: they differ only by bf16 rounding of operands."""
    w = Workload("cmp", 1, 2, 512, 64, 128, 64, "bf16", PHI_PERFORMER, True)
    t = inputs.make_inputs(w, 13)
    g, out, ctx = gu.run_forward(w, t, "fast")
    fast = gu.run_backward(w, g, out, ctx, "fast")
    g2, out2, ctx2 = gu.run_forward(w, t, "generic")
    gen = gu.run_backward(w, g2, out2, ctx2, "generic")
    for name, a, b in zip(["dQ", "dK", "dV", "dE", "dF"], fast, gen):
        assert fo.rel_l2(gu.to_host(a), gu.to_host(b)) < 2e-2, name


def test_sequence_length_that_only_the_forward_kernels_take():
    """n = 200 is a multiple of 8 but not of 32: algo = auto runs the MFMA forward and the generic backward."""
    w = Workload("ragged_n", 2, 3, 200, 64, 100, 96, "bf16", PHI_PERFORMER, True)
    dims = (w.B, w.H, w.n, w.d, w.k, w.m)
    assert fb.fast_path_supported(*dims, fb.BF16, w.phi, fb.PASS_FWD)
    assert not fb.fast_path_supported(*dims, fb.BF16, w.phi, fb.PASS_BWD)
    errs = gu.check_forward_backward(w, seed=24, algo="auto")
    print({k_: f"{v:.2e}" for k_, v in errs.items()})


def test_one_context_serves_both_kernel_families():
    """What the forward leaves in ctx (K', V', S, z, c, lse) means the same to the MFMA kernels and to
    the generic ones.  With 320 features at head size 64, algo = auto runs the MFMA forward and the
    generic backward on one ctx; the second case forces the opposite pairing."""
    w = Workload("cross", 1, 2, 512, 64, 96, 320, "bf16", PHI_PERFORMER, True)
    dims = (w.B, w.H, w.n, w.d, w.k, w.m)
    assert fb.fast_path_supported(*dims, fb.BF16, w.phi, fb.PASS_FWD)
    assert not fb.fast_path_supported(*dims, fb.BF16, w.phi, fb.PASS_BWD)
    errs = gu.check_forward_backward(w, seed=22, algo="auto")
    print("mfma fwd + generic bwd", {k_: f"{v:.2e}" for k_, v in errs.items()})

    w = Workload("cross2", 1, 2, 512, 64, 96, 64, "bf16", PHI_PERFORMER, True)
    t = inputs.make_inputs(w, 23)
    g, out, ctx = gu.run_forward(w, t, "generic")
    grads = gu.run_backward(w, g, out, ctx, "fast")
    errs = {}
    for name, a, b in zip(["dQ", "dK", "dV", "dE", "dF"], grads, gu.oracle_backward(w, t)):
        errs[name] = gu.rel_err(gu.to_host(a), b)
    print("generic fwd + mfma bwd", {k_: f"{v:.2e}" for k_, v in errs.items()})
    assert all(v <= 2e-2 for v in errs.values()), errs


@pytest.mark.parametrize("shape,phi", [((2, 2, 512, 64, 96, 64), PHI_PERFORMER), ((2, 3, 512, 128, 96, 256), PHI_PERFORMER),
                                       ((2, 3, 512, 64, 96, 64), PHI_ELU1)])
def test_backward_is_deterministic(shape, phi):
    """Both head sizes (128 with 256 features: the ring variant of the dQ kernel, whose wavefronts meet
    at a barrier per feature tile) and both feature maps."""
    w = Workload("det", *shape, "bf16", phi, True)
    t = inputs.make_inputs(w, 14)
    g, out, ctx = gu.run_forward(w, t, "fast")
    a = gu.run_backward(w, g, out, ctx, "fast")
    b = gu.run_backward(w, g, out, ctx, "fast")
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("d,m", [(64, 128), (128, 256)])
def test_backward_with_one_omega_for_all_heads(d, m):
    w = Workload("shared", 2, 3, 512, d, 128, m, "bf16", PHI_PERFORMER, True, omega_per_head=False)
    errs = gu.check_forward_backward(w, seed=15, algo="fast")
    print((d, m), {k_: f"{v:.2e}" for k_, v in errs.items()})


# ---- scratch independence ------------------------------------------------------------------
@pytest.mark.parametrize("algo,d,m,phi", [("fast", 64, 96, PHI_PERFORMER), ("generic", 64, 96, PHI_PERFORMER),
                                          ("fast", 128, 256, PHI_PERFORMER), ("fast", 64, 64, PHI_ELU1)])
def test_results_do_not_depend_on_what_the_scratch_buffers_held(algo, d, m, phi):
    """ctx, workspace and the result tensors are filled with NaN bit patterns (0xFF bytes) before the
    calls: every byte a kernel reads must have been written by an earlier kernel of the same call.
    Shape with ragged k (tile rows past k), ragged heads per projection tile and an odd step count."""
    w = Workload("poison", 1, 3, 192, d, 100, m, "bf16", phi, True)
    t = inputs.make_inputs(w, 21)
    g = gu.to_device(t, w.dtype)
    dims = (w.B, w.H, w.n, w.d, w.k, w.m)
    dev = g["Q"].device

    def run(fill):
        ctx = fb.alloc_buffer(fb.ctx_bytes(*dims, fb.BF16, w.phi), dev).fill_(fill)
        wf = fb.alloc_buffer(fb.workspace_bytes(*dims, fb.BF16, w.phi, fb.PASS_FWD, algo), dev).fill_(fill)
        wb = fb.alloc_buffer(fb.workspace_bytes(*dims, fb.BF16, w.phi, fb.PASS_BWD, algo), dev).fill_(fill)
        out = torch.empty_like(g["Q"]).view(torch.uint8).fill_(fill).view(torch.bfloat16).view(g["Q"].shape)
        fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], phi=w.phi, algo=algo,
                           out=out, ctx=ctx, workspace=wf)
        grads = tuple(torch.empty_like(x).view(torch.uint8).fill_(fill).view(torch.bfloat16).view(x.shape)
                      for x in (g["Q"], g["K"], g["V"], g["E"], g["F"]))
        fb.flurka_attn_bwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx,
                           phi=w.phi, algo=algo, workspace=wb, grads=grads)
        torch.cuda.synchronize()
        return (out,) + grads

    clean, dirty = run(0), run(0xFF)
    for name, a, b in zip(["out", "dQ", "dK", "dV", "dE", "dF"], clean, dirty):
        assert torch.isfinite(b.float()).all(), name
        assert torch.equal(a, b), name


# ---- stream capture --------------------------------------------------------------------------
def test_forward_and_backward_replay_from_a_captured_graph():
    """The library allocates nothing, never synchronises and clears no memory with runtime calls, so a
    forward+backward pair can be captured into a graph.  The graph is replayed several times with eager
    calls (and synchronisations) in between; every replay must reproduce the eager result bit for bit."""
    w = Workload("graph", 2, 3, 512, 64, 96, 64, "bf16", PHI_PERFORMER, True)
    t = inputs.make_inputs(w, 17)
    g = gu.to_device(t, w.dtype)
    dims = (w.B, w.H, w.n, w.d, w.k, w.m)
    dev = g["Q"].device
    ctx = fb.alloc_buffer(fb.ctx_bytes(*dims, fb.BF16, w.phi), dev)
    wf = fb.alloc_buffer(fb.workspace_bytes(*dims, fb.BF16, w.phi, fb.PASS_FWD, "auto"), dev)
    wb = fb.alloc_buffer(fb.workspace_bytes(*dims, fb.BF16, w.phi, fb.PASS_BWD, "auto"), dev)
    out = torch.empty_like(g["Q"])
    grads = tuple(torch.empty_like(x) for x in (g["Q"], g["K"], g["V"], g["E"], g["F"]))

    def step():
        fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], phi=w.phi, out=out, ctx=ctx,
                           workspace=wf)
        fb.flurka_attn_bwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi,
                           workspace=wb, grads=grads)

    step()                                   # eager: reference values (and one-time kernel attribute calls)
    torch.cuda.synchronize()
    ref = [out.clone()] + [x.clone() for x in grads]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                               # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep in range(3):
        for x in [out, *grads]:
            x.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(["out", "dQ", "dK", "dV", "dE", "dF"], [out, *grads], ref):
            assert torch.equal(a, b), (rep, name)
        # eager work between replays, on another shape, through the same library
        gu.check_forward(Workload("between", 1, 2, 256, 64, 40, 32, "bf16", PHI_PERFORMER, False), seed=rep, algo="fast")
