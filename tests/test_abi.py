"""Host-side checks of the C ABI: the library loads, exports what the header
declares, sizes its buffers sensibly and rejects bad arguments before any
launch.  No compute call is made, so this runs without a GPU."""
import ctypes
import os
import re

import pytest

from paper_2306_15799_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000          # 256-byte aligned, never dereferenced: validation fails first


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fb.LIB_PATH):
        from paper_2306_15799_amd import build
        build.build()
    return fb.load_library()


def test_every_declared_entry_point_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "flurka.h")).read()
    declared = set(re.findall(r"FLURKA_API\s+[\w\s\*]+?\b(flurka_\w+)\s*\(", header))
    assert declared == set(fb.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.flurka_version() == 150


def test_status_strings(lib):
    seen = {fb.status_str(i) for i in range(8)}
    assert len(seen) == 8 and fb.status_str(0) == "ok"
    assert fb.status_str(99) == "unknown status"


def test_buffer_sizes(lib):
    # C1: K',V' 2*4096 + S 4096 + z 64 + c 64 + lse 512 floats
    assert fb.ctx_bytes(1, 1, 512, 64, 64, 64, fb.F32, "performer") == 4 * (3 * 4096 + 64 + 64 + 512)
    assert fb.ctx_bytes(1, 1, 512, 64, 64, 63, fb.F32, "elu1") == 0          # m != d
    assert fb.ctx_bytes(0, 1, 512, 64, 64, 64, fb.F32, "performer") == 0
    fwd = fb.workspace_bytes(4, 12, 8192, 64, 256, 256, fb.BF16, "performer", fb.PASS_FWD, "generic")
    bwd = fb.workspace_bytes(4, 12, 8192, 64, 256, 256, fb.BF16, "performer", fb.PASS_BWD, "generic")
    assert 0 < fwd < bwd
    auto = fb.workspace_bytes(4, 12, 8192, 64, 256, 256, fb.BF16, "performer", fb.PASS_FWD, "auto")
    assert auto >= fwd
    offs = (ctypes.c_size_t * 6)()
    assert lib.flurka_ctx_layout(1, 1, 512, 64, 64, 64, fb.F32, 0, offs) == fb.OK
    assert list(offs) == [0, 4096, 8192, 12288, 12352, 12416]
    assert lib.flurka_ctx_layout(1, 1, 512, 64, 64, 64, fb.F32, 0, None) == fb.ERR_NULL


def _fwd(lib, **over):
    a = dict(Q=FAKE, K=FAKE, V=FAKE, E=FAKE, F=FAKE, omega=FAKE, out=FAKE, ctx=FAKE, ctx_bytes=1 << 40,
             ws=FAKE, ws_bytes=1 << 40, B=1, H=1, n=512, d=64, k=64, m=64, per_head=1,
             dtype=fb.F32, phi=fb.PHI_PERFORMER, algo=fb.ALGO_GENERIC)
    a.update(over)
    return lib.flurka_attn_fwd(a["Q"], a["K"], a["V"], a["E"], a["F"], a["omega"], a["out"], a["ctx"],
                               a["ctx_bytes"], a["ws"], a["ws_bytes"], a["B"], a["H"], a["n"], a["d"],
                               a["k"], a["m"], a["per_head"], a["dtype"], a["phi"], a["algo"], None)


def _bwd(lib, **over):
    a = dict(Q=FAKE, K=FAKE, V=FAKE, E=FAKE, F=FAKE, omega=FAKE, out=FAKE, dOut=FAKE, ctx=FAKE,
             ctx_bytes=1 << 40, dQ=FAKE, dK=FAKE, dV=FAKE, dE=FAKE, dF=FAKE, ws=FAKE, ws_bytes=1 << 40,
             B=1, H=1, n=512, d=64, k=64, m=64, per_head=1, dtype=fb.F32, phi=fb.PHI_PERFORMER,
             algo=fb.ALGO_GENERIC)
    a.update(over)
    return lib.flurka_attn_bwd(a["Q"], a["K"], a["V"], a["E"], a["F"], a["omega"], a["out"], a["dOut"],
                               a["ctx"], a["ctx_bytes"], a["dQ"], a["dK"], a["dV"], a["dE"], a["dF"], a["ws"],
                               a["ws_bytes"], a["B"], a["H"], a["n"], a["d"], a["k"], a["m"],
                               a["per_head"], a["dtype"], a["phi"], a["algo"], None)


def test_forward_rejects_bad_arguments_before_launching(lib):
    for name in ["Q", "K", "V", "E", "F", "omega", "out", "ctx", "ws"]:
        assert _fwd(lib, **{name: None}) == fb.ERR_NULL, name
    for dim in ["B", "H", "n", "d", "k", "m"]:
        assert _fwd(lib, **{dim: 0}) == fb.ERR_SHAPE, dim
        assert _fwd(lib, **{dim: -3}) == fb.ERR_SHAPE, dim
    assert _fwd(lib, B=256, H=256) == fb.ERR_SHAPE                 # B*H above the grid limit
    assert _fwd(lib, d=4097) == fb.ERR_SHAPE
    assert _fwd(lib, n=(1 << 24) + 1) == fb.ERR_SHAPE
    assert _fwd(lib, phi=fb.PHI_ELU1, m=32) == fb.ERR_SHAPE        # elu1 needs m == d
    assert _fwd(lib, dtype=7) == fb.ERR_DTYPE
    assert _fwd(lib, phi=5) == fb.ERR_DTYPE
    assert _fwd(lib, algo=9) == fb.ERR_DTYPE
    assert _fwd(lib, Q=FAKE + 2) == fb.ERR_ALIGN
    assert _fwd(lib, ctx=FAKE + 64) == fb.ERR_ALIGN
    assert _fwd(lib, ctx_bytes=1000) == fb.ERR_WORKSPACE
    assert _fwd(lib, ws_bytes=1000) == fb.ERR_WORKSPACE
    assert _fwd(lib, algo=fb.ALGO_FAST) == fb.ERR_UNSUPPORTED      # fp32 storage has no MFMA path
    # the elu1 map takes no omega: NULL is fine there, and validation moves on to the next check
    assert _fwd(lib, phi=fb.PHI_ELU1, omega=None, ws_bytes=8) == fb.ERR_WORKSPACE


def test_backward_rejects_bad_arguments_before_launching(lib):
    for name in ["Q", "K", "V", "E", "F", "omega", "out", "dOut", "ctx", "dQ", "dK", "dV", "dE", "dF", "ws"]:
        assert _bwd(lib, **{name: None}) == fb.ERR_NULL, name
    assert _bwd(lib, k=0) == fb.ERR_SHAPE
    assert _bwd(lib, dtype=2) == fb.ERR_DTYPE
    assert _bwd(lib, dE=FAKE + 1) == fb.ERR_ALIGN
    assert _bwd(lib, ctx_bytes=16) == fb.ERR_WORKSPACE
    assert _bwd(lib, ws_bytes=16) == fb.ERR_WORKSPACE


def test_shapes_whose_byte_offsets_leave_32_bits_are_not_taken_by_the_mfma_kernels(lib):
    # the bf16 images of dK', dV' are addressed with 32-bit byte offsets: many projected keys (k > n is
    # allowed) times many (head, coordinate) rows must fall back to the generic kernels
    assert fb.fast_path_supported(64, 1, 64, 128, 1 << 10, 32, fb.BF16, "performer", fb.PASS_BWD)
    assert not fb.fast_path_supported(64, 1, 64, 128, 1 << 18, 32, fb.BF16, "performer", fb.PASS_BWD)
    assert _bwd(lib, B=64, n=64, d=128, k=1 << 18, m=32, dtype=fb.BF16, algo=fb.ALGO_FAST) == fb.ERR_UNSUPPORTED
    # forward: one projection tile's rows of E must stay below 2 GiB
    assert not fb.fast_path_supported(1, 1, 1 << 22, 64, 512, 32, fb.BF16, "performer", fb.PASS_FWD)


def test_static_scratch_entry_point_validates_like_the_forward(lib):
    def call(**over):
        a = dict(Q=FAKE, K=FAKE, V=FAKE, E=FAKE, F=FAKE, omega=FAKE, out=FAKE, ctx=FAKE, ctx_bytes=1 << 40,
                 B=1, H=1, n=512, d=64, k=64, m=64, per_head=1, dtype=fb.F32, phi=fb.PHI_PERFORMER,
                 algo=fb.ALGO_GENERIC)
        a.update(over)
        return lib.flurka_attn_fwd_static(a["Q"], a["K"], a["V"], a["E"], a["F"], a["omega"], a["out"], a["ctx"],
                                          a["ctx_bytes"], a["B"], a["H"], a["n"], a["d"], a["k"], a["m"],
                                          a["per_head"], a["dtype"], a["phi"], a["algo"], None)
    assert call(Q=None) == fb.ERR_NULL
    assert call(n=0) == fb.ERR_SHAPE
    assert call(ctx=FAKE + 64) == fb.ERR_ALIGN
    assert call(ctx_bytes=16) == fb.ERR_WORKSPACE
    # a workspace beyond the library's own array is refused before anything is launched
    assert fb.workspace_bytes(4, 12, 8192, 64, 256, 256, fb.BF16, "performer", fb.PASS_FWD, "generic") > fb.STATIC_WORKSPACE_BYTES
    assert call(B=4, H=12, n=8192, d=64, k=256, m=256, dtype=fb.BF16) == fb.ERR_WORKSPACE


def test_paper_order_entry_point_validates_before_launching(lib):
    def call(**over):
        a = dict(Q=FAKE, XK=FAKE, XV=FAKE, E=FAKE, F=FAKE, WK=FAKE, WV=FAKE, omega=FAKE, out=FAKE, ctx=FAKE,
                 ctx_bytes=1 << 40, ws=FAKE, ws_bytes=1 << 40, B=1, H=4, n=512, d=64, k=64, m=64, dm=256,
                 per_head=1, dtype=fb.BF16, phi=fb.PHI_PERFORMER)
        a.update(over)
        return lib.flurka_attn_fwd_fused_w(a["Q"], a["XK"], a["XV"], a["E"], a["F"], a["WK"], a["WV"], a["omega"],
                                           a["out"], a["ctx"], a["ctx_bytes"], a["ws"], a["ws_bytes"], a["B"],
                                           a["H"], a["n"], a["d"], a["k"], a["m"], a["dm"], a["per_head"],
                                           a["dtype"], a["phi"], None)
    for name in ["Q", "XK", "XV", "E", "F", "WK", "WV", "omega", "out", "ctx", "ws"]:
        assert call(**{name: None}) == fb.ERR_NULL, name
    assert call(dm=0) == fb.ERR_SHAPE
    assert call(n=0) == fb.ERR_SHAPE
    assert call(dm=100) == fb.ERR_UNSUPPORTED              # not whole 64-deep reduction steps
    assert call(H=3) == fb.ERR_UNSUPPORTED                 # H*d not a multiple of the 256-column tile
    assert call(dtype=fb.F32) == fb.ERR_UNSUPPORTED
    assert call(WK=FAKE + 2) == fb.ERR_UNSUPPORTED         # vector loads need 16-byte alignment
    assert call(ws_bytes=1000) == fb.ERR_WORKSPACE
    assert call(ctx_bytes=1000) == fb.ERR_WORKSPACE
    assert lib.flurka_fused_w_supported(1, 4, 512, 64, 64, 64, 256, fb.BF16, 0) == 1
    assert lib.flurka_fused_w_workspace_bytes(1, 4, 512, 64, 64, 64, 256, fb.BF16, 0) > 0
    assert lib.flurka_fused_w_workspace_bytes(1, 3, 512, 64, 64, 64, 256, fb.BF16, 0) == 0


def test_extended_entry_points_validate_their_options(lib):
    def bwd(opt, **over):
        a = dict(algo=fb.ALGO_GENERIC, dtype=fb.F32, phi=fb.PHI_PERFORMER, ws_bytes=1 << 40, dE=FAKE)
        a.update(over)
        return lib.flurka_attn_bwd_ex(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, FAKE, FAKE, FAKE,
                                      a["dE"], FAKE, FAKE, a["ws_bytes"], 1, 1, 512, 64, 64, 64, 1, a["dtype"],
                                      a["phi"], a["algo"], opt, None)
    import ctypes as ct
    none = fb.FlurkaOptions(0, 0, None)
    assert bwd(None, ws_bytes=16) == fb.ERR_WORKSPACE                 # NULL options = the plain call
    assert bwd(ct.byref(none), ws_bytes=16) == fb.ERR_WORKSPACE
    f32ef = fb.FlurkaOptions(0, 1, None)
    assert bwd(ct.byref(f32ef), dtype=fb.BF16, algo=fb.ALGO_FAST, n=512) == fb.ERR_UNSUPPORTED
    assert bwd(ct.byref(f32ef), dtype=fb.BF16, dE=FAKE + 2) == fb.ERR_ALIGN     # float32 dE needs 4-byte alignment
    dom = fb.FlurkaOptions(0, 0, FAKE)
    assert bwd(ct.byref(dom), phi=fb.PHI_ELU1) == fb.ERR_SHAPE       # the elu1 map has no omega
    assert bwd(ct.byref(fb.FlurkaOptions(0, 0, FAKE + 2))) == fb.ERR_ALIGN
    assert bwd(ct.byref(dom), ws_bytes=16) == fb.ERR_WORKSPACE


def test_binding_refuses_cpu_tensors(lib):
    import torch
    q = torch.zeros(1, 1, 8, 4)
    e = torch.zeros(2, 8)
    om = torch.zeros(1, 3, 4)
    with pytest.raises(ValueError):
        fb.flurka_attn_fwd(q, q, q, e, e, om)
