"""GPU parity of the generic (fp32-arithmetic) kernels against the fp64 oracle,
element by element on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import flurka_oracle as fo
from paper_2306_15799_amd import binding as fb
from paper_2306_15799_amd import inputs
from paper_2306_15799_amd.inputs import Workload, PHI_ELU1, PHI_PERFORMER

import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_c1_fp32_forward():
    err = gu.check_forward(inputs.WORKLOADS["C1"], seed=0, algo="generic")
    print(f"C1 fwd rel-L2 {err:.3e}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("phi", [PHI_PERFORMER, PHI_ELU1])
def test_ragged_shapes_forward_backward(dtype, phi):
    # several 64-wide tiles plus a ragged tail in every dimension
    m = 150 if phi == PHI_PERFORMER else 72
    w = Workload("ragged", 2, 3, 333, 72, 77, m, dtype, phi, True)
    errs = gu.check_forward_backward(w, seed=1, algo="generic")
    print(dtype, phi, {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("shape", [(1, 1, 1, 1, 1, 1), (1, 2, 5, 3, 1, 4), (2, 1, 64, 8, 64, 1),
                                   (1, 1, 7, 130, 3, 9)])
def test_degenerate_sizes(shape):
    B, H, n, d, k, m = shape
    w = Workload("edge", B, H, n, d, k, m, "f32", PHI_PERFORMER, True)
    # with k = 1 the output ignores Q and K (dQ, dK, dE are exactly zero), with m = 1 it ignores Q;
    # what the GPU returns there is fp32 cancellation noise: measure it against unit scale, not zero
    floor = 1.0 if (k == 1 or m == 1) else 0.0
    errs = gu.check_forward_backward(w, seed=2, algo="generic", floor=floor)
    print(shape, "performer", {k_: f"{v:.2e}" for k_, v in errs.items()})
    w = Workload("edge", B, H, n, d, k, d, "f32", PHI_ELU1, True)
    errs = gu.check_forward_backward(w, seed=2, algo="generic", floor=floor)
    print(shape, "elu1", {k_: f"{v:.2e}" for k_, v in errs.items()})


def test_shared_omega_equals_per_head_copy():
    w = Workload("shared", 2, 3, 96, 16, 24, 40, "f32", PHI_PERFORMER, False, omega_per_head=False)
    t = inputs.make_inputs(w, 3)
    assert t["omega"].shape[0] == 1
    _, out_shared, _ = gu.run_forward(w, t, "generic")
    t2 = dict(t)
    t2["omega"] = np.repeat(t["omega"], w.H, axis=0)
    _, out_rep, _ = gu.run_forward(w, t2, "generic")
    assert torch.equal(out_shared, out_rep)
    assert fo.rel_l2(gu.to_host(out_shared), gu.oracle_forward(w, t)) < 1e-5


def test_context_holds_the_key_side_state():
    w = Workload("ctx", 1, 2, 200, 32, 40, 48, "f32", PHI_PERFORMER, False)
    t = inputs.make_inputs(w, 4)
    _, _, ctx = gu.run_forward(w, t, "generic")
    v = fb.ctx_views(ctx, w.B, w.H, w.n, w.d, w.k, w.m, fb.F32, w.phi)
    Kp = np.matmul(t["E"].astype(np.float64), t["K"].astype(np.float64))
    Vp = np.matmul(t["F"].astype(np.float64), t["V"].astype(np.float64))
    assert fo.rel_l2(gu.to_host(v["Kp"]), Kp) < 1e-6
    assert fo.rel_l2(gu.to_host(v["Vp"]), Vp) < 1e-6
    for h in range(w.H):
        om = t["omega"][h].astype(np.float64)
        # the library shifts every feature by its own column maximum; the oracle by one constant:
        # compare after undoing each side's shift (S_j / z_j and z_j * exp(c_j) are shift-free)
        e = Kp[0, h] @ om.T - 0.5 * np.sum(Kp[0, h] ** 2, axis=1, keepdims=True)
        gc = gu.to_host(v["c"][0, h])
        assert np.max(np.abs(gc - e.max(axis=0))) < 1e-4 * max(1.0, np.abs(e).max())
        Phi, S, z, c = fo.key_state(Kp[0, h], Vp[0, h], om, w.phi)
        gS, gz = gu.to_host(v["S"][0, h]), gu.to_host(v["z"][0, h])
        assert fo.rel_l2(gS / gz[:, None], S / z[:, None]) < 1e-5
        assert fo.rel_l2(np.log(gz) + gc, np.log(z) + c) < 1e-5
        # lse_i = ln sum_j exp(omega_j . q_i) sum_r exp(e_rj): the denominator without any shift
        lse = gu.log_denominator(t["Q"][0, h], om, e)
        assert np.max(np.abs(gu.to_host(v["lse"][0, h]) - lse)) < 1e-4 * max(1.0, np.abs(lse).max())


def test_large_exponent_scale_stays_finite():
    """Key norms as in the long-sequence workload (|k'|^2/2 of several hundred)."""
    w = Workload("range", 1, 1, 4096, 128, 32, 64, "bf16", PHI_PERFORMER, False)
    t = inputs.make_inputs(w, 5)
    _, out, _ = gu.run_forward(w, t, "generic")
    o = gu.to_host(out)
    assert np.all(np.isfinite(o))
    assert fo.rel_l2(o, gu.oracle_forward(w, t)) < 2e-2


def test_results_are_deterministic():
    w = Workload("det", 2, 2, 300, 32, 50, 70, "bf16", PHI_PERFORMER, True)
    t = inputs.make_inputs(w, 6)
    g, out1, ctx = gu.run_forward(w, t, "generic")
    grads1 = gu.run_backward(w, g, out1, ctx, "generic")
    _, out2, ctx2 = gu.run_forward(w, t, "generic")
    grads2 = gu.run_backward(w, g, out2, ctx2, "generic")
    assert torch.equal(out1, out2)
    for a, b in zip(grads1, grads2):
        assert torch.equal(a, b)
