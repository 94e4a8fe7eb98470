"""GPU parity of the variants behind the extended entry points (flurka_attn_fwd_ex / _bwd_ex): one
projection pair per head, float32 dE / dF, the gradient for omega -- against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import flurka_oracle as fo
from paper_2306_15799_amd import binding as fb
from paper_2306_15799_amd import inputs
from paper_2306_15799_amd.inputs import Workload, PHI_ELU1, PHI_PERFORMER

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _per_head_inputs(w, seed):
    t = inputs.make_inputs(w, seed)
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    scale = np.float32(float(w.k) ** -0.5)
    for name in ("E", "F"):
        x = rng.standard_normal(size=(w.H, w.k, w.n), dtype=np.float32) * scale
        t[name] = inputs.round_to_bf16(x) if w.dtype == "bf16" else x
    return t


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("phi", [PHI_PERFORMER, PHI_ELU1])
def test_one_projection_pair_per_head(dtype, phi):
    m = 70 if phi == PHI_PERFORMER else 40
    w = Workload("per_head", 2, 3, 200, 40, 33, m, dtype, phi, True)
    t = _per_head_inputs(w, 80)
    g = gu.to_device(t, dtype)
    out, ctx = fb.flurka_attn_fwd_ex(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], phi=phi, ef_per_head=True)
    grads = fb.flurka_attn_bwd_ex(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=phi,
                                  ef_per_head=True)
    torch.cuda.synchronize()
    bar = gu.TOL[dtype]
    ref_out = fo.flurka_attention_per_head(t["Q"], t["K"], t["V"], t["E"], t["F"], t["omega"], phi)
    errs = {"out": fo.rel_l2(gu.to_host(out), ref_out)}
    ref = fo.flurka_attention_per_head_bwd(t["Q"], t["K"], t["V"], t["E"], t["F"], t["omega"], t["dOut"], phi)
    for name, a, b in zip(["dQ", "dK", "dV", "dE", "dF"], grads, ref):
        errs[name] = fo.rel_l2(gu.to_host(a), b)
    print(dtype, phi, {k_: f"{v:.2e}" for k_, v in errs.items()})
    assert all(v <= bar for v in errs.values()), errs
    # H copies of one pair through the per-head path = the shared pair through the plain path, bit for bit
    # in fp32 arithmetic order (same kernels, same strides but for the head offset)
    gc = dict(g)
    gc["E"] = g["E"][:1].repeat(w.H, 1, 1).contiguous()
    gc["F"] = g["F"][:1].repeat(w.H, 1, 1).contiguous()
    out_c, _ = fb.flurka_attn_fwd_ex(g["Q"], g["K"], g["V"], gc["E"], gc["F"], g["omega"], phi=phi, ef_per_head=True)
    out_s, _ = fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"][0].contiguous(), g["F"][0].contiguous(), g["omega"],
                                  phi=phi, algo="generic")
    assert torch.equal(out_c, out_s)


def test_float32_projection_gradients_from_bf16_storage():
    """dE, dF as float32: the same sums as the bf16 outputs before their final rounding, so closer to the
    oracle than bf16 can be, and equal to the bf16 outputs after rounding."""
    w = Workload("ef32", 2, 3, 256, 64, 48, 64, "bf16", PHI_PERFORMER, True)
    t = inputs.make_inputs(w, 81)
    g = gu.to_device(t, "bf16")
    out, ctx = fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], phi=w.phi, algo="generic")
    g32 = fb.flurka_attn_bwd_ex(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi,
                                grad_ef_f32=True)
    g16 = fb.flurka_attn_bwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi,
                             algo="generic")
    torch.cuda.synchronize()
    assert g32[3].dtype == torch.float32 and g32[4].dtype == torch.float32
    ref = gu.oracle_backward(w, t)
    for i, name in ((3, "dE"), (4, "dF")):
        e32, e16 = fo.rel_l2(gu.to_host(g32[i]), ref[i]), fo.rel_l2(gu.to_host(g16[i]), ref[i])
        print(name, f"f32 {e32:.2e} bf16 {e16:.2e}")
        assert e32 <= gu.TOL["bf16"] and e32 <= e16
        assert torch.equal(g32[i].to(torch.bfloat16), g16[i])


@pytest.mark.parametrize("dtype,shared", [("f32", False), ("bf16", False), ("bf16", True)])
def test_gradient_for_omega(dtype, shared):
    w = Workload("domega", 2, 3, 300, 32, 40, 48, dtype, PHI_PERFORMER, True, omega_per_head=not shared)
    t = inputs.make_inputs(w, 82)
    g = gu.to_device(t, dtype)
    out, ctx = fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], phi=w.phi, algo="generic")
    res = fb.flurka_attn_bwd_ex(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi,
                                want_d_omega=True)
    torch.cuda.synchronize()
    ref = fo.flurka_attention_bwd_omega(t["Q"], t["K"], t["V"], t["E"], t["F"], t["omega"], t["dOut"])
    err = fo.rel_l2(gu.to_host(res[5]), ref)
    print(dtype, "shared" if shared else "per head", f"d_omega rel-L2 {err:.2e}")
    assert res[5].shape == g["omega"].shape and err <= gu.TOL[dtype]
    # the other gradients are unaffected by asking for d_omega
    plain = fb.flurka_attn_bwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi,
                               algo="generic")
    for a, b in zip(res[:5], plain):
        assert torch.equal(a, b)


def test_options_are_refused_by_the_mfma_kernels_and_for_elu():
    w = Workload("opts", 1, 2, 128, 64, 32, 64, "bf16", PHI_PERFORMER, True)
    t = inputs.make_inputs(w, 83)
    g = gu.to_device(t, "bf16")
    out, ctx = fb.flurka_attn_fwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], phi=w.phi)
    with pytest.raises(fb.FlurkaError) as e:
        fb.flurka_attn_bwd_ex(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi,
                              algo="fast", grad_ef_f32=True)
    assert e.value.status == fb.ERR_UNSUPPORTED
    # no options: the extended entry point is the plain one, MFMA kernels included
    a = fb.flurka_attn_bwd_ex(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi, algo="fast")
    b = fb.flurka_attn_bwd(g["Q"], g["K"], g["V"], g["E"], g["F"], g["omega"], out, g["dOut"], ctx, phi=w.phi, algo="fast")
    for x, y in zip(a, b):
        assert torch.equal(x, y)
