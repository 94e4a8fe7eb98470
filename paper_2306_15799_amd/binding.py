"""ctypes binding of libflurka (see include/flurka.h for the ABI).

Argument marshalling only: tensors in, raw device pointers and sizes out.
PyTorch is used for device memory and streams; every step of the attention
runs inside the library's HIP kernels.  There is no CPU fallback: if the
shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libflurka.so")

# enums of include/flurka.h
OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH, ERR_ALIGN = range(8)
F32, BF16 = 0, 1
PHI_PERFORMER, PHI_ELU1 = 0, 1
ALGO_AUTO, ALGO_GENERIC, ALGO_FAST = 0, 1, 2
PASS_FWD, PASS_BWD = 0, 1

_PHI = {"performer": PHI_PERFORMER, "elu1": PHI_ELU1, PHI_PERFORMER: PHI_PERFORMER, PHI_ELU1: PHI_ELU1}
_ALGO = {"auto": ALGO_AUTO, "generic": ALGO_GENERIC, "fast": ALGO_FAST,
         ALGO_AUTO: ALGO_AUTO, ALGO_GENERIC: ALGO_GENERIC, ALGO_FAST: ALGO_FAST}

EXPORTED_SYMBOLS = (
    "flurka_version", "flurka_status_str", "flurka_ctx_bytes", "flurka_ctx_layout", "flurka_workspace_bytes",
    "flurka_fast_path_supported", "flurka_attn_fwd", "flurka_attn_fwd_static", "flurka_attn_bwd",
    "flurka_fused_w_supported", "flurka_fused_w_workspace_bytes", "flurka_attn_fwd_fused_w",
    "flurka_attn_fwd_ex", "flurka_attn_bwd_ex",
    "flurka_baseline_supported", "flurka_baseline_ctx_bytes", "flurka_baseline_workspace_bytes", "flurka_baseline_fwd",
    "flurka_profile_enable", "flurka_profile_read", "flurka_profile_stage_name",
)

class FlurkaOptions(ctypes.Structure):
    """flurka_options of include/flurka.h."""
    _fields_ = [("ef_per_head", ctypes.c_int), ("grad_ef_f32", ctypes.c_int), ("d_omega", ctypes.c_void_p)]


_lib: Optional[ctypes.CDLL] = None


class FlurkaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} (status {status})")


def load_library() -> ctypes.CDLL:
    """Load libflurka.so built in-tree; raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build it first (python -m paper_2306_15799_amd.build); "
            "there is no fallback implementation")
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_size, c_void = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
    lib.flurka_version.restype = c_int
    lib.flurka_version.argtypes = []
    lib.flurka_status_str.restype = ctypes.c_char_p
    lib.flurka_status_str.argtypes = [c_int]
    lib.flurka_ctx_bytes.restype = c_size
    lib.flurka_ctx_bytes.argtypes = [c_int] * 8
    lib.flurka_ctx_layout.restype = c_int
    lib.flurka_ctx_layout.argtypes = [c_int] * 8 + [ctypes.POINTER(c_size)]
    lib.flurka_workspace_bytes.restype = c_size
    lib.flurka_workspace_bytes.argtypes = [c_int] * 10
    lib.flurka_fast_path_supported.restype = c_int
    lib.flurka_fast_path_supported.argtypes = [c_int] * 9
    lib.flurka_attn_fwd.restype = c_int
    lib.flurka_attn_fwd.argtypes = ([c_void] * 7 + [c_void, c_size, c_void, c_size]
                                    + [c_int] * 6 + [c_int] + [c_int] * 3 + [c_void])
    lib.flurka_attn_fwd_static.restype = c_int
    lib.flurka_attn_fwd_static.argtypes = ([c_void] * 7 + [c_void, c_size]
                                           + [c_int] * 6 + [c_int] + [c_int] * 3 + [c_void])
    lib.flurka_fused_w_supported.restype = c_int
    lib.flurka_fused_w_supported.argtypes = [c_int] * 9
    lib.flurka_fused_w_workspace_bytes.restype = c_size
    lib.flurka_fused_w_workspace_bytes.argtypes = [c_int] * 9
    lib.flurka_attn_fwd_fused_w.restype = c_int
    lib.flurka_attn_fwd_fused_w.argtypes = ([c_void] * 9 + [c_void, c_size, c_void, c_size]
                                            + [c_int] * 7 + [c_int] + [c_int] * 2 + [c_void])
    lib.flurka_baseline_supported.restype = c_int
    lib.flurka_baseline_supported.argtypes = [c_int] * 9
    lib.flurka_baseline_ctx_bytes.restype = c_size
    lib.flurka_baseline_ctx_bytes.argtypes = [c_int] * 9
    lib.flurka_baseline_workspace_bytes.restype = c_size
    lib.flurka_baseline_workspace_bytes.argtypes = [c_int] * 9
    lib.flurka_baseline_fwd.restype = c_int
    lib.flurka_baseline_fwd.argtypes = ([c_int] + [c_void] * 7 + [c_void, c_size, c_void, c_size]
                                        + [c_int] * 6 + [c_int] + [c_int] * 2 + [c_void])
    lib.flurka_attn_fwd_ex.restype = c_int
    lib.flurka_attn_fwd_ex.argtypes = ([c_void] * 7 + [c_void, c_size, c_void, c_size]
                                       + [c_int] * 6 + [c_int] + [c_int] * 3 + [ctypes.POINTER(FlurkaOptions), c_void])
    lib.flurka_attn_bwd_ex.restype = c_int
    lib.flurka_attn_bwd_ex.argtypes = ([c_void] * 8 + [c_void, c_size] + [c_void] * 5 + [c_void, c_size]
                                       + [c_int] * 6 + [c_int] + [c_int] * 3 + [ctypes.POINTER(FlurkaOptions), c_void])
    lib.flurka_attn_bwd.restype = c_int
    lib.flurka_attn_bwd.argtypes = ([c_void] * 8 + [c_void, c_size] + [c_void] * 5 + [c_void, c_size]
                                    + [c_int] * 6 + [c_int] + [c_int] * 3 + [c_void])
    lib.flurka_profile_enable.restype = c_int
    lib.flurka_profile_enable.argtypes = [c_int]
    lib.flurka_profile_read.restype = c_int
    lib.flurka_profile_read.argtypes = [ctypes.POINTER(c_int), ctypes.POINTER(ctypes.c_float), c_int]
    lib.flurka_profile_stage_name.restype = ctypes.c_char_p
    lib.flurka_profile_stage_name.argtypes = [c_int]
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load_library().flurka_status_str(int(status)).decode()


def profile_enable(on: bool) -> None:
    st = load_library().flurka_profile_enable(1 if on else 0)
    if st != OK:
        raise FlurkaError(st, "flurka_profile_enable")


def profile_read() -> list:
    """[(stage name, milliseconds), ...] recorded since the last read, in launch order."""
    lib = load_library()
    cap = 4096
    ids = (ctypes.c_int * cap)()
    ms = (ctypes.c_float * cap)()
    cnt = lib.flurka_profile_read(ids, ms, cap)
    return [(lib.flurka_profile_stage_name(ids[i]).decode(), float(ms[i])) for i in range(cnt)]


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}; use float32 or bfloat16")


def ctx_bytes(B, H, n, d, k, m, dtype, phi) -> int:
    return load_library().flurka_ctx_bytes(B, H, n, d, k, m, dtype, _PHI[phi])


def ctx_views(ctx: torch.Tensor, B, H, n, d, k, m, dtype, phi) -> dict:
    """float32 views of the context buffer's segments (K', V', S, z, c, lse)."""
    lib = load_library()
    offs = (ctypes.c_size_t * 6)()
    st = lib.flurka_ctx_layout(B, H, n, d, k, m, dtype, _PHI[phi], offs)
    if st != OK:
        raise FlurkaError(st, "flurka_ctx_layout")
    mf = d if _PHI[phi] == PHI_ELU1 else m
    f = ctx.view(torch.float32)
    shapes = {"Kp": (B, H, k, d), "Vp": (B, H, k, d), "S": (B, H, mf, d), "z": (B, H, mf), "c": (B, H, mf),
              "lse": (B, H, n)}
    views = {}
    for (name, shape), off in zip(shapes.items(), offs):
        cnt = 1
        for v in shape:
            cnt *= v
        views[name] = f[off:off + cnt].view(shape)
    return views


def workspace_bytes(B, H, n, d, k, m, dtype, phi, pass_, algo=ALGO_AUTO) -> int:
    return load_library().flurka_workspace_bytes(B, H, n, d, k, m, dtype, _PHI[phi], pass_, _ALGO[algo])


def fast_path_supported(B, H, n, d, k, m, dtype, phi, pass_=PASS_FWD) -> bool:
    return bool(load_library().flurka_fast_path_supported(B, H, n, d, k, m, dtype, _PHI[phi], pass_))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _check(t: torch.Tensor, name: str, shape, dtype, device):
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if t.device != device or not t.is_cuda:
        raise ValueError(f"{name}: must live on {device}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")


def _shapes(Q, E, omega, phi):
    if Q.dim() != 4 or E.dim() != 2:
        raise ValueError("Q must be (B,H,n,d) and E (k,n)")
    B, H, n, d = Q.shape
    k = E.shape[0]
    if _PHI[phi] == PHI_PERFORMER:
        if omega is None or omega.dim() != 3 or omega.shape[0] not in (1, H):
            raise ValueError("omega must be (H,m,d) or (1,m,d) for the performer map")
        m = omega.shape[1]
        per_head = 1 if (omega.shape[0] == H and H > 1) else 0
        omega_shape = (omega.shape[0], m, d)
    else:
        m, per_head, omega_shape = d, 0, None
    return B, H, n, d, k, m, per_head, omega_shape


def alloc_buffer(nbytes: int, device) -> torch.Tensor:
    """Device scratch of at least `nbytes` (torch's allocator returns >= 256-byte aligned blocks)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def flurka_attn_fwd(Q, K, V, E, F, omega, phi="performer", algo="auto", out=None, ctx=None,
                    workspace=None, stream=None):
    """out, ctx = forward of FLuRKA attention (Eq. 2 with the App. D normaliser).

    Q, K, V: (B,H,n,d); E, F: (k,n); omega: (H|1,m,d) or None for "elu1".
    Returns the output tensor and the context buffer the backward needs.
    """
    lib = load_library()
    B, H, n, d, k, m, per_head, omega_shape = _shapes(Q, E, omega, phi)
    dt, dev = Q.dtype, Q.device
    code = _dtype_code(Q)
    for t, name in ((Q, "Q"), (K, "K"), (V, "V")):
        _check(t, name, (B, H, n, d), dt, dev)
    for t, name in ((E, "E"), (F, "F")):
        _check(t, name, (k, n), dt, dev)
    if omega_shape is not None:
        _check(omega, "omega", omega_shape, dt, dev)
    if out is None:
        out = torch.empty_like(Q)
    _check(out, "out", (B, H, n, d), dt, dev)
    cb = lib.flurka_ctx_bytes(B, H, n, d, k, m, code, _PHI[phi])
    wb = lib.flurka_workspace_bytes(B, H, n, d, k, m, code, _PHI[phi], PASS_FWD, _ALGO[algo])
    if ctx is None:
        ctx = alloc_buffer(cb, dev)
    if workspace is None:
        workspace = alloc_buffer(wb, dev)
    s = stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    st = lib.flurka_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(E), _ptr(F),
                             _ptr(omega) if omega_shape is not None else None, _ptr(out),
                             _ptr(ctx), ctx.numel() * ctx.element_size(),
                             _ptr(workspace), workspace.numel() * workspace.element_size(),
                             B, H, n, d, k, m, per_head, code, _PHI[phi], _ALGO[algo], s)
    if st != OK:
        raise FlurkaError(st, "flurka_attn_fwd")
    return out, ctx


def fused_w_supported(B, H, n, d, k, m, dm, dtype, phi) -> bool:
    return bool(load_library().flurka_fused_w_supported(B, H, n, d, k, m, dm, dtype, _PHI[phi]))


def flurka_attn_fwd_fused_w(Q, XK, XV, E, F, WK, WV, omega, phi="performer", out=None, ctx=None, workspace=None,
                            stream=None):
    """out, ctx = forward in the paper's order: K' = (E X_K) W^K, V' = (F X_V) W^V (Eq. 2).

    Q: (B,H,n,d); XK, XV: (B,n,dm); WK, WV: (H,d,dm) (each head's transform, transposed); E, F: (k,n)."""
    lib = load_library()
    B, H, n, d, k, m, per_head, omega_shape = _shapes(Q, E, omega, phi)
    dt, dev = Q.dtype, Q.device
    code = _dtype_code(Q)
    dm = XK.shape[-1]
    _check(Q, "Q", (B, H, n, d), dt, dev)
    for t, name in ((XK, "XK"), (XV, "XV")):
        _check(t, name, (B, n, dm), dt, dev)
    for t, name in ((WK, "WK"), (WV, "WV")):
        _check(t, name, (H, d, dm), dt, dev)
    for t, name in ((E, "E"), (F, "F")):
        _check(t, name, (k, n), dt, dev)
    if omega_shape is not None:
        _check(omega, "omega", omega_shape, dt, dev)
    if out is None:
        out = torch.empty_like(Q)
    _check(out, "out", (B, H, n, d), dt, dev)
    if ctx is None:
        ctx = alloc_buffer(lib.flurka_ctx_bytes(B, H, n, d, k, m, code, _PHI[phi]), dev)
    if workspace is None:
        workspace = alloc_buffer(lib.flurka_fused_w_workspace_bytes(B, H, n, d, k, m, dm, code, _PHI[phi]), dev)
    s = stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    st = lib.flurka_attn_fwd_fused_w(_ptr(Q), _ptr(XK), _ptr(XV), _ptr(E), _ptr(F), _ptr(WK), _ptr(WV),
                                     _ptr(omega) if omega_shape is not None else None, _ptr(out),
                                     _ptr(ctx), ctx.numel() * ctx.element_size(),
                                     _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     B, H, n, d, k, m, dm, per_head, code, _PHI[phi], s)
    if st != OK:
        raise FlurkaError(st, "flurka_attn_fwd_fused_w")
    return out, ctx


def flurka_attn_fwd_ex(Q, K, V, E, F, omega, phi="performer", algo="auto", ef_per_head=False, stream=None):
    """flurka_attn_fwd with options (include/flurka.h: flurka_options).  With ef_per_head E, F are (H,k,n).
    Returns out, ctx."""
    lib = load_library()
    Eh = E[0] if ef_per_head else E
    B, H, n, d, k, m, per_head, omega_shape = _shapes(Q, Eh, omega, phi)
    dt, dev = Q.dtype, Q.device
    code = _dtype_code(Q)
    for t, name in ((Q, "Q"), (K, "K"), (V, "V")):
        _check(t, name, (B, H, n, d), dt, dev)
    for t, name in ((E, "E"), (F, "F")):
        _check(t, name, (H, k, n) if ef_per_head else (k, n), dt, dev)
    if omega_shape is not None:
        _check(omega, "omega", omega_shape, dt, dev)
    out = torch.empty_like(Q)
    ctx = alloc_buffer(lib.flurka_ctx_bytes(B, H, n, d, k, m, code, _PHI[phi]), dev)
    a = ALGO_GENERIC if ef_per_head else _ALGO[algo]
    ws = alloc_buffer(lib.flurka_workspace_bytes(B, H, n, d, k, m, code, _PHI[phi], PASS_FWD, a), dev)
    opt = FlurkaOptions(1 if ef_per_head else 0, 0, None)
    s = stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    st = lib.flurka_attn_fwd_ex(_ptr(Q), _ptr(K), _ptr(V), _ptr(E), _ptr(F),
                                _ptr(omega) if omega_shape is not None else None, _ptr(out),
                                _ptr(ctx), ctx.numel(), _ptr(ws), ws.numel(),
                                B, H, n, d, k, m, per_head, code, _PHI[phi], _ALGO[algo], ctypes.byref(opt), s)
    if st != OK:
        raise FlurkaError(st, "flurka_attn_fwd_ex")
    return out, ctx


def flurka_attn_bwd_ex(Q, K, V, E, F, omega, out, dOut, ctx, phi="performer", algo="auto", ef_per_head=False,
                       grad_ef_f32=False, want_d_omega=False, stream=None):
    """flurka_attn_bwd with options.  Returns dQ, dK, dV, dE, dF and, with want_d_omega, d_omega (float32)."""
    lib = load_library()
    Eh = E[0] if ef_per_head else E
    B, H, n, d, k, m, per_head, omega_shape = _shapes(Q, Eh, omega, phi)
    dt, dev = Q.dtype, Q.device
    code = _dtype_code(Q)
    for t, name in ((Q, "Q"), (K, "K"), (V, "V"), (out, "out"), (dOut, "dOut")):
        _check(t, name, (B, H, n, d), dt, dev)
    for t, name in ((E, "E"), (F, "F")):
        _check(t, name, (H, k, n) if ef_per_head else (k, n), dt, dev)
    gdt = torch.float32 if grad_ef_f32 else dt
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dE, dF = torch.empty(E.shape, dtype=gdt, device=dev), torch.empty(F.shape, dtype=gdt, device=dev)
    d_omega = torch.empty(omega.shape, dtype=torch.float32, device=dev) if want_d_omega else None
    plain = not (ef_per_head or grad_ef_f32 or want_d_omega)
    a = _ALGO[algo] if plain else ALGO_GENERIC
    ws = alloc_buffer(lib.flurka_workspace_bytes(B, H, n, d, k, m, code, _PHI[phi], PASS_BWD, a), dev)
    opt = FlurkaOptions(1 if ef_per_head else 0, 1 if grad_ef_f32 else 0, _ptr(d_omega))
    s = stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    st = lib.flurka_attn_bwd_ex(_ptr(Q), _ptr(K), _ptr(V), _ptr(E), _ptr(F),
                                _ptr(omega) if omega_shape is not None else None, _ptr(out), _ptr(dOut),
                                _ptr(ctx), ctx.numel(), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dE), _ptr(dF),
                                _ptr(ws), ws.numel(), B, H, n, d, k, m, per_head, code, _PHI[phi], _ALGO[algo],
                                ctypes.byref(opt), s)
    if st != OK:
        raise FlurkaError(st, "flurka_attn_bwd_ex")
    return (dQ, dK, dV, dE, dF) + ((d_omega,) if want_d_omega else ())


BASELINE_KERNEL_ATTN, BASELINE_LINFORMER = 0, 1


def baseline_supported(which, B, H, n, d, k, m, dtype, phi) -> bool:
    return bool(load_library().flurka_baseline_supported(which, B, H, n, d, k, m, dtype, _PHI[phi]))


def flurka_baseline_fwd(which, Q, K, V, E=None, F=None, omega=None, phi="performer", out=None, ctx=None,
                        workspace=None, stream=None):
    """The paper's constituents at the attention level: BASELINE_KERNEL_ATTN (E, F unused) or
    BASELINE_LINFORMER (omega unused; softmax over the projected keys).  Returns out, ctx."""
    lib = load_library()
    if Q.dim() != 4:
        raise ValueError("Q must be (B,H,n,d)")
    B, H, n, d = Q.shape
    dt, dev = Q.dtype, Q.device
    code = _dtype_code(Q)
    for t, name in ((Q, "Q"), (K, "K"), (V, "V")):
        _check(t, name, (B, H, n, d), dt, dev)
    k, m, per_head = n, d, 0
    if which == BASELINE_LINFORMER:
        k = E.shape[0]
        for t, name in ((E, "E"), (F, "F")):
            _check(t, name, (k, n), dt, dev)
        m, omega = 32, None
    elif _PHI[phi] == PHI_PERFORMER:
        m = omega.shape[1]
        per_head = 1 if (omega.shape[0] == H and H > 1) else 0
        _check(omega, "omega", (omega.shape[0], m, d), dt, dev)
    else:
        omega = None
    if out is None:
        out = torch.empty_like(Q)
    _check(out, "out", (B, H, n, d), dt, dev)
    if ctx is None:
        ctx = alloc_buffer(lib.flurka_baseline_ctx_bytes(which, B, H, n, d, k, m, code, _PHI[phi]), dev)
    if workspace is None:
        workspace = alloc_buffer(lib.flurka_baseline_workspace_bytes(which, B, H, n, d, k, m, code, _PHI[phi]), dev)
    s = stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    st = lib.flurka_baseline_fwd(which, _ptr(Q), _ptr(K), _ptr(V), _ptr(E), _ptr(F), _ptr(omega), _ptr(out),
                                 _ptr(ctx), ctx.numel() * ctx.element_size(),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 B, H, n, d, k, m, per_head, code, _PHI[phi], s)
    if st != OK:
        raise FlurkaError(st, "flurka_baseline_fwd")
    return out, ctx


STATIC_WORKSPACE_BYTES = 32 << 20       # FLURKA_STATIC_WORKSPACE_BYTES


def flurka_attn_fwd_static(Q, K, V, E, F, omega, out, ctx, phi="performer", algo="auto", stream=None):
    """flurka_attn_fwd with the scratch inside the library's device image: `out` and `ctx` come from
    the caller and nothing is allocated, here or in the library."""
    lib = load_library()
    B, H, n, d, k, m, per_head, omega_shape = _shapes(Q, E, omega, phi)
    dt, dev = Q.dtype, Q.device
    code = _dtype_code(Q)
    for t, name in ((Q, "Q"), (K, "K"), (V, "V"), (out, "out")):
        _check(t, name, (B, H, n, d), dt, dev)
    for t, name in ((E, "E"), (F, "F")):
        _check(t, name, (k, n), dt, dev)
    if omega_shape is not None:
        _check(omega, "omega", omega_shape, dt, dev)
    s = stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    st = lib.flurka_attn_fwd_static(_ptr(Q), _ptr(K), _ptr(V), _ptr(E), _ptr(F),
                                    _ptr(omega) if omega_shape is not None else None, _ptr(out),
                                    _ptr(ctx), ctx.numel() * ctx.element_size(),
                                    B, H, n, d, k, m, per_head, code, _PHI[phi], _ALGO[algo], s)
    if st != OK:
        raise FlurkaError(st, "flurka_attn_fwd_static")
    return out, ctx


def flurka_attn_bwd(Q, K, V, E, F, omega, out, dOut, ctx, phi="performer", algo="auto", workspace=None,
                    stream=None, grads=None):
    """dQ, dK, dV, dE, dF given dOut and the (out, ctx) returned by flurka_attn_fwd."""
    lib = load_library()
    B, H, n, d, k, m, per_head, omega_shape = _shapes(Q, E, omega, phi)
    dt, dev = Q.dtype, Q.device
    code = _dtype_code(Q)
    for t, name in ((Q, "Q"), (K, "K"), (V, "V"), (out, "out"), (dOut, "dOut")):
        _check(t, name, (B, H, n, d), dt, dev)
    for t, name in ((E, "E"), (F, "F")):
        _check(t, name, (k, n), dt, dev)
    if omega_shape is not None:
        _check(omega, "omega", omega_shape, dt, dev)
    if grads is None:
        grads = (torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V),
                 torch.empty_like(E), torch.empty_like(F))
    dQ, dK, dV, dE, dF = grads
    for t, name in ((dQ, "dQ"), (dK, "dK"), (dV, "dV")):
        _check(t, name, (B, H, n, d), dt, dev)
    for t, name in ((dE, "dE"), (dF, "dF")):
        _check(t, name, (k, n), dt, dev)
    wb = lib.flurka_workspace_bytes(B, H, n, d, k, m, code, _PHI[phi], PASS_BWD, _ALGO[algo])
    if workspace is None:
        workspace = alloc_buffer(wb, dev)
    s = stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    st = lib.flurka_attn_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(E), _ptr(F),
                             _ptr(omega) if omega_shape is not None else None, _ptr(out), _ptr(dOut),
                             _ptr(ctx), ctx.numel() * ctx.element_size(),
                             _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dE), _ptr(dF),
                             _ptr(workspace), workspace.numel() * workspace.element_size(),
                             B, H, n, d, k, m, per_head, code, _PHI[phi], _ALGO[algo], s)
    if st != OK:
        raise FlurkaError(st, "flurka_attn_bwd")
    return dQ, dK, dV, dE, dF
