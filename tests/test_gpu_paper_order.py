"""GPU parity of the forward in the paper's order, K' = (E X_K) W^K (flurka_attn_fwd_fused_w), against
the fp64 oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import flurka_oracle as fo
from paper_2306_15799_amd import binding as fb
from paper_2306_15799_amd import inputs
from paper_2306_15799_amd.inputs import Workload, PHI_ELU1, PHI_PERFORMER

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _run(w, dm, seed):
    t = inputs.make_paper_order_inputs(w, dm, seed)
    g = gu.to_device(t, "bf16")
    out, ctx = fb.flurka_attn_fwd_fused_w(g["Q"], g["XK"], g["XV"], g["E"], g["F"], g["WK"], g["WV"], g["omega"],
                                          phi=w.phi)
    torch.cuda.synchronize()
    return t, g, out, ctx


# (B, H, n, d, k, m, dm): several column tiles per batch in both products, ragged k, a model width that is
# not a multiple of the 256-column tile, more than one batch, both head sizes
SHAPES = [
    (1, 4, 512, 64, 100, 96, 256),
    (2, 8, 1024, 64, 256, 128, 320),
    (2, 2, 640, 128, 300, 160, 192),
    (1, 4, 2048, 128, 512, 64, 512),
    # a sequence length that is a multiple of 8 only (ragged last reduction step of the first product)
    (2, 4, 712, 64, 100, 96, 256),
    # a feature count that is not a multiple of 32
    (1, 4, 512, 64, 100, 100, 256),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_forward_performer(shape):
    B, H, n, d, k, m, dm = shape
    w = Workload("paper_order", B, H, n, d, k, m, "bf16", PHI_PERFORMER, False)
    assert fb.fused_w_supported(B, H, n, d, k, m, dm, fb.BF16, w.phi)
    t, g, out, ctx = _run(w, dm, 41)
    ref = fo.flurka_attention_paper_order(t["Q"], t["XK"], t["XV"], t["E"], t["F"], t["WK"], t["WV"], t["omega"], w.phi)
    got = gu.to_host(out)
    err = fo.rel_l2(got, ref)
    wb = gu.worst_block(got, ref, 32, -2)
    print(shape, f"rel-L2 {err:.3e} worst block {wb:.3e}")
    assert err <= gu.TOL["bf16"] and wb <= gu.BLOCK_FACTOR * gu.TOL["bf16"]
    # the projected keys and values the transform leaves in ctx: fp32-accurate (three-term operands)
    v = fb.ctx_views(ctx, B, H, n, d, k, m, fb.BF16, w.phi)
    Kp = np.einsum("bkc,hdc->bhkd", np.matmul(t["E"].astype(np.float64), t["XK"].astype(np.float64)), t["WK"].astype(np.float64))
    Vp = np.einsum("bkc,hdc->bhkd", np.matmul(t["F"].astype(np.float64), t["XV"].astype(np.float64)), t["WV"].astype(np.float64))
    assert fo.rel_l2(gu.to_host(v["Kp"]), Kp) < 3e-6
    assert fo.rel_l2(gu.to_host(v["Vp"]), Vp) < 3e-6


def test_forward_elu():
    B, H, n, d, k, dm = 2, 4, 1024, 64, 128, 256
    w = Workload("paper_order_elu", B, H, n, d, k, d, "bf16", PHI_ELU1, False)
    t, g, out, _ = _run(w, dm, 42)
    ref = fo.flurka_attention_paper_order(t["Q"], t["XK"], t["XV"], t["E"], t["F"], t["WK"], t["WV"], None, w.phi)
    assert fo.rel_l2(gu.to_host(out), ref) <= gu.TOL["bf16"]


def test_matches_the_transform_first_entry_point():
    """Same data through both entry points: X W formed outside (rounded to bf16 as the caller of
    flurka_attn_fwd must) and inside (never rounded).  They agree to the rounding of K, V."""
    B, H, n, d, k, m, dm = 1, 4, 1024, 64, 128, 128, 256
    w = Workload("both", B, H, n, d, k, m, "bf16", PHI_PERFORMER, False)
    t, g, out, _ = _run(w, dm, 43)
    K = torch.einsum("bnc,hdc->bhnd", g["XK"].float(), g["WK"].float()).to(torch.bfloat16).contiguous()
    V = torch.einsum("bnc,hdc->bhnd", g["XV"].float(), g["WV"].float()).to(torch.bfloat16).contiguous()
    out2, _ = fb.flurka_attn_fwd(g["Q"], K, V, g["E"], g["F"], g["omega"], phi=w.phi, algo="fast")
    torch.cuda.synchronize()
    rel = ((out.float() - out2.float()).norm() / out2.float().norm()).item()
    print(f"paper order vs transform first rel-L2 {rel:.2e}")
    assert rel < 2e-2


def test_unsupported_shapes_are_refused():
    # model width not a multiple of 64; H*d not a multiple of 256; fp32 storage
    assert not fb.fused_w_supported(1, 4, 512, 64, 64, 64, 100, fb.BF16, "performer")
    assert not fb.fused_w_supported(1, 3, 512, 64, 64, 64, 256, fb.BF16, "performer")
    assert not fb.fused_w_supported(1, 4, 512, 64, 64, 64, 256, fb.F32, "performer")
    w = Workload("odd", 1, 3, 512, 64, 64, 64, "bf16", PHI_PERFORMER, False)
    t = inputs.make_paper_order_inputs(w, 256, 44)
    g = gu.to_device(t, "bf16")
    with pytest.raises(fb.FlurkaError) as e:
        fb.flurka_attn_fwd_fused_w(g["Q"], g["XK"], g["XV"], g["E"], g["F"], g["WK"], g["WV"], g["omega"],
                                   workspace=fb.alloc_buffer(1 << 20, g["Q"].device))
    assert e.value.status == fb.ERR_UNSUPPORTED


def test_results_do_not_depend_on_what_the_buffers_held():
    """ctx, workspace and out filled with NaN bit patterns before the call (ragged k, a model width that
    leaves the last 256-column tile of the first product half empty, an odd number of reduction steps)."""
    B, H, n, d, k, m, dm = 2, 4, 704, 64, 100, 96, 320
    w = Workload("poison", B, H, n, d, k, m, "bf16", PHI_PERFORMER, False)
    t = inputs.make_paper_order_inputs(w, dm, 45)
    g = gu.to_device(t, "bf16")
    lib = fb.load_library()

    def run(fill):
        ctx = fb.alloc_buffer(fb.ctx_bytes(B, H, n, d, k, m, fb.BF16, w.phi), g["Q"].device).fill_(fill)
        ws = fb.alloc_buffer(lib.flurka_fused_w_workspace_bytes(B, H, n, d, k, m, dm, fb.BF16, 0), g["Q"].device).fill_(fill)
        out = torch.empty_like(g["Q"]).view(torch.uint8).fill_(fill).view(torch.bfloat16).view(g["Q"].shape)
        fb.flurka_attn_fwd_fused_w(g["Q"], g["XK"], g["XV"], g["E"], g["F"], g["WK"], g["WV"], g["omega"], phi=w.phi,
                                   out=out, ctx=ctx, workspace=ws)
        torch.cuda.synchronize()
        return out

    clean, dirty = run(0), run(0xFF)
    assert torch.isfinite(dirty.float()).all()
    assert torch.equal(clean, dirty)
