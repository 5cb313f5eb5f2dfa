"""Thin Python binding of libfingpt_hpc.so (the C ABI in include/fingpt_hpc.h).

Argument marshalling only: every step of the layer runs in the HIP library.
PyTorch supplies device memory (tensors) and the current HIP stream, nothing else.
The library must be present: there is no fallback path, and loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

C_float = C.c_float

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfingpt_hpc.so")

FHPC_F32, FHPC_BF16 = 0, 1
FHPC_Q_INT8_PER_CHANNEL, FHPC_Q_INT4_BLOCK = 8, 4
FHPC_W_BF16 = 16          # blend and merge entry points only: dense bf16 W[K,N] in place of Wq, scales None
FHPC_W_MERGED = 17        # qlinear_lowrank_fwd/bwd only: Wq is the bf16 [K,N] weight lowrank_merge wrote for the same A, B, scaling
FHPC_OP_LOWRANK_FWD, FHPC_OP_LOWRANK_BWD, FHPC_OP_QLINEAR_FWD, FHPC_OP_QLINEAR_BWD, FHPC_OP_MERGE, FHPC_OP_DECOMPOSE = 0, 1, 2, 3, 4, 5
FHPC_PLAN_SHARED_FWD, FHPC_PLAN_SHARED_BWD, FHPC_PLAN_FFN_GATE_UP, FHPC_PLAN_FFN_DOWN_BWD = 16, 17, 18, 19

EXPORTS = [
    "lowrank_linear_fwd", "lowrank_linear_bwd", "qlinear_lowrank_fwd", "qlinear_lowrank_bwd", "qlinear_blend_fwd", "qlinear_blend_bwd", "lowrank_merge", "lowrank_decompose", "qlinear_lowrank_fwd_shared_x", "fhpc_workspace_bytes_shared_x",
    "lowrank_linear_fwd_shared_x", "lowrank_linear_bwd_shared_x", "fhpc_workspace_bytes_lowrank_shared_x",
    "lowrank_ffn_gate_up_fwd", "lowrank_ffn_down_bwd",
    "fhpc_workspace_bytes", "swiglu_fwd", "swiglu_bwd", "qweight_quantize", "qweight_unpack",
    "qweight_dequant", "fhpc_add", "fhpc_gemm_bf16", "fhpc_profile_start", "fhpc_profile_stop", "fhpc_profile_get",
    "fhpc_status_string", "fhpc_version", "fhpc_plan_slab_bytes", "qlinear_lowrank_fwd_noalloc", "fhpc_probe_mfma", "fhpc_probe_copy", "fhpc_probe_read_rows",
]

_lib = None


class QlinearWeight(C.Structure):
    """fhpc_qlinear_weight of the C header."""
    _fields_ = [("Wq", C.c_void_p), ("scales", C.c_void_p), ("A", C.c_void_p), ("B", C.c_void_p), ("Y", C.c_void_p),
                ("H_out", C.c_void_p), ("N", C.c_int64), ("scaling", C.c_float)]


class FhpcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, status_string(status)))


def load_library():
    """Load the HIP library (built in-tree by paper_2402_13533_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2402_13533_amd.build` "
            "(there is no CPU or PyTorch fallback)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i64, i32, f32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_size_t
    lib.lowrank_linear_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, vp, sz, vp]
    lib.lowrank_linear_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, vp, sz, vp]
    lib.qlinear_lowrank_fwd.argtypes = [vp, vp, vp, i32, i32, vp, vp, f32, vp, vp, i64, i64, i64, i64, vp, sz, vp]
    lib.qlinear_lowrank_bwd.argtypes = [vp, vp, vp, i32, i32, vp, vp, f32, vp, vp, vp, vp, vp,
                                        i64, i64, i64, i64, vp, sz, vp]
    lib.qlinear_blend_fwd.argtypes = lib.qlinear_lowrank_fwd.argtypes
    lib.qlinear_lowrank_fwd_noalloc.argtypes = [vp, vp, vp, i32, i32, vp, vp, f32, vp, vp, i64, i64, i64, i64, vp]
    lib.qlinear_blend_bwd.argtypes = lib.qlinear_lowrank_bwd.argtypes
    lib.lowrank_merge.argtypes = [vp, vp, i32, i32, vp, vp, f32, vp, i32, i64, i64, i64, vp, sz, vp]
    lib.lowrank_decompose.argtypes = [vp, vp, i32, vp, vp, i64, i64, i64, i64, vp, sz, vp]
    lib.qlinear_lowrank_fwd_shared_x.argtypes = [vp, C.POINTER(QlinearWeight), i32, i32, i32, i64, i64, i64, vp, sz, vp]
    lib.fhpc_workspace_bytes_shared_x.argtypes = [C.POINTER(i64), i32, i64, i64, i64, i32]
    lib.fhpc_workspace_bytes_shared_x.restype = sz
    pp = C.POINTER(vp)
    lib.lowrank_linear_fwd_shared_x.argtypes = [vp, vp, pp, pp, vp, i64, i64, i64, i64, i32, vp, sz, vp]
    lib.lowrank_linear_bwd_shared_x.argtypes = [vp, vp, pp, pp, vp, vp, vp, pp, i64, i64, i64, i64, i32, vp, sz, vp]
    lib.lowrank_ffn_gate_up_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, vp, sz, vp]
    lib.lowrank_ffn_down_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, vp, sz, vp]
    lib.fhpc_workspace_bytes_lowrank_shared_x.argtypes = [i32, i64, i64, i64, i64, i32]
    lib.fhpc_workspace_bytes_lowrank_shared_x.restype = sz
    lib.fhpc_workspace_bytes.argtypes = [i32, i64, i64, i64, i64, i32, i32]
    lib.fhpc_workspace_bytes.restype = sz
    lib.swiglu_fwd.argtypes = [vp, vp, vp, i64, i32, vp]
    lib.swiglu_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i32, vp]
    lib.qweight_quantize.argtypes = [vp, i32, i32, vp, vp, i64, i64, vp]
    lib.qweight_unpack.argtypes = [vp, i32, vp, i64, i64, vp]
    lib.qweight_dequant.argtypes = [vp, vp, i32, i32, vp, i64, i64, vp]
    lib.fhpc_add.argtypes = [vp, vp, vp, i64, i32, vp]
    lib.fhpc_gemm_bf16.argtypes = [vp, i64, i32, vp, i64, i32, vp, i64, i32, i64, i64, i64, f32, i32, i32, i32, vp]
    lib.fhpc_profile_start.argtypes = [i32]
    lib.fhpc_profile_stop.argtypes = []
    lib.fhpc_profile_get.argtypes = [i32, C.c_char_p, i32, C.POINTER(C.c_float), C.POINTER(C.c_double),
                                     C.POINTER(C.c_double)]
    lib.fhpc_plan_slab_bytes.argtypes = [i32, i64, i64, i64, i64, i32, i32, i32, i32, f32, C.POINTER(i64), C.POINTER(i64)]
    lib.fhpc_probe_mfma.argtypes = [vp, i32, i32, vp, C.POINTER(C.c_double), vp]
    lib.fhpc_probe_copy.argtypes = [vp, vp, i64, vp]
    lib.fhpc_probe_read_rows.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.fhpc_status_string.argtypes = [i32]
    lib.fhpc_status_string.restype = C.c_char_p
    lib.fhpc_version.restype = i32
    for name in EXPORTS:
        if name not in ("fhpc_workspace_bytes", "fhpc_workspace_bytes_shared_x", "fhpc_workspace_bytes_lowrank_shared_x",
                        "fhpc_status_string", "fhpc_version"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def profile_start(max_records: int = 4096) -> None:
    rc = load_library().fhpc_profile_start(max_records)
    if rc:
        raise FhpcError(rc, "fhpc_profile_start")


def profile_stop():
    """Disarm and return [(kernel name, milliseconds, flops, bytes)] for every recorded launch."""
    lib = load_library()
    n = lib.fhpc_profile_stop()
    out = []
    buf = C.create_string_buffer(64)
    ms, fl, by = C.c_float(), C.c_double(), C.c_double()
    for i in range(n):
        rc = lib.fhpc_profile_get(i, buf, 64, C.byref(ms), C.byref(fl), C.byref(by))
        if rc:
            raise FhpcError(rc, "fhpc_profile_get")
        out.append((buf.value.decode(), float(ms.value), float(fl.value), float(by.value)))
    return out


def probe_mfma(seed, workgroups: int, iters: int) -> float:
    """Enqueue the register-only matrix-core loop on the current stream; returns the launch's flop count."""
    fl = C.c_double(0.0)
    rc = load_library().fhpc_probe_mfma(_ptr(seed), workgroups, iters, None, C.byref(fl), _stream())
    if rc:
        raise FhpcError(rc, "fhpc_probe_mfma")
    return float(fl.value)


def probe_copy(src, dst) -> int:
    """Enqueue the streaming copy dst = src on the current stream; returns the bytes copied."""
    n = src.numel() * src.element_size()
    rc = load_library().fhpc_probe_copy(_ptr(src), _ptr(dst), n, _stream())
    if rc:
        raise FhpcError(rc, "fhpc_probe_copy")
    return n


def probe_read_rows(W, workgroups: int, sink) -> int:
    """Enqueue one pass over the byte matrix W ([N][row_bytes], uint8) in the weight-streaming kernels' access
    pattern and nothing else; returns the bytes read."""
    N, row_bytes = W.shape
    rc = load_library().fhpc_probe_read_rows(_ptr(W), N, row_bytes, workgroups, _ptr(sink), _stream())
    if rc:
        raise FhpcError(rc, "fhpc_probe_read_rows")
    return N * row_bytes


def status_string(status: int) -> str:
    return load_library().fhpc_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().fhpc_version())


def plan_slab_bytes(call: int, M: int, K: int, r: int, N: int, dtype: int = FHPC_BF16, qscheme: int = 0, g: int = 1,
                    outputs: int = 7, base_scale: float = 1.0):
    """Host-only test hook: (status, planned, reserved) partial-sum bytes of an entry point's launch sequence."""
    planned, reserved = C.c_int64(0), C.c_int64(0)
    rc = load_library().fhpc_plan_slab_bytes(call, M, K, r, N, dtype, qscheme, g, outputs, C_float(base_scale),
                                             C.byref(planned), C.byref(reserved))
    return int(rc), int(planned.value), int(reserved.value)


def workspace_bytes(op: int, M: int, K: int, r: int, N: int, dtype: int = FHPC_BF16, qscheme: int = 0) -> int:
    return int(load_library().fhpc_workspace_bytes(op, M, K, r, N, dtype, qscheme))


# ----------------------------------------------------------------------------- torch side

def _torch():
    import torch
    return torch


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return FHPC_F32
    if t.dtype == torch.bfloat16:
        return FHPC_BF16
    raise TypeError("dtype must be float32 or bfloat16, got %s" % t.dtype)


def _check(t, name, shape=None, dtype=None):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s has dtype %s, expected %s" % (name, t.dtype, dtype))


_workspaces = {}


def get_workspace(nbytes: int, device):
    """A cached byte tensor of at least nbytes (grown on demand), one per device and stream: calls that share a
    workspace must be ordered on one stream."""
    torch = _torch()
    key = (str(device), int(torch.cuda.current_stream(device).cuda_stream))
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        # zero once: the library keeps the workspace header (arrival counters) zero from call to call
        ws = torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def _ws(op, M, K, r, N, dtype, qscheme, device, workspace):
    need = workspace_bytes(op, M, K, r, N, dtype, qscheme)
    ws = workspace if workspace is not None else get_workspace(need, device)
    return ws, C.c_size_t(ws.numel() * ws.element_size())


def lowrank_linear_fwd(X, A, B, Y=None, H_out=None, save_H: bool = False, workspace=None):
    """Y = (X A) B.  Returns Y, or (Y, H) when save_H or H_out is given."""
    torch = _torch()
    lib = load_library()
    M, K = X.shape
    r, N = B.shape
    _check(X, "X"); _check(A, "A", (K, r), X.dtype); _check(B, "B", (r, N), X.dtype)
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    if H_out is None and save_H:
        H_out = torch.empty((M, r), dtype=X.dtype, device=X.device)
    _check(Y, "Y", (M, N), X.dtype); _check(H_out, "H_out", (M, r), X.dtype)
    dt = _dtype_code(X)
    ws, wsz = _ws(FHPC_OP_LOWRANK_FWD, M, K, r, N, dt, 0, X.device, workspace)
    rc = lib.lowrank_linear_fwd(_ptr(X), _ptr(A), _ptr(B), _ptr(Y), _ptr(H_out), M, K, r, N, dt,
                                _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, "lowrank_linear_fwd")
    return (Y, H_out) if H_out is not None else Y


def lowrank_linear_bwd(X, A, B, dY, H_saved=None, need_dX=True, need_dA=True, need_dB=True,
                       dX=None, dA=None, dB=None, workspace=None):
    """Returns (dX, dA, dB) of Y = (X A) B; dA, dB are fp32."""
    torch = _torch()
    lib = load_library()
    M, K = X.shape
    r, N = B.shape
    _check(X, "X"); _check(A, "A", (K, r), X.dtype); _check(B, "B", (r, N), X.dtype)
    _check(dY, "dY", (M, N), X.dtype); _check(H_saved, "H_saved", (M, r), X.dtype)
    if dX is None and need_dX:
        dX = torch.empty((M, K), dtype=X.dtype, device=X.device)
    if dA is None and need_dA:
        dA = torch.empty((K, r), dtype=torch.float32, device=X.device)
    if dB is None and need_dB:
        dB = torch.empty((r, N), dtype=torch.float32, device=X.device)
    _check(dX, "dX", (M, K), X.dtype); _check(dA, "dA", (K, r), torch.float32); _check(dB, "dB", (r, N), torch.float32)
    dt = _dtype_code(X)
    ws, wsz = _ws(FHPC_OP_LOWRANK_BWD, M, K, r, N, dt, 0, X.device, workspace)
    rc = lib.lowrank_linear_bwd(_ptr(X), _ptr(A), _ptr(B), _ptr(dY), _ptr(H_saved), _ptr(dX), _ptr(dA), _ptr(dB),
                                M, K, r, N, dt, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, "lowrank_linear_bwd")
    return dX, dA, dB


def _ptr_array(tensors):
    """Host array of device pointers (None entries become NULL)."""
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def _shared_ws(backward, M, K, r, N, g, device, workspace):
    torch = _torch()
    need = int(load_library().fhpc_workspace_bytes_lowrank_shared_x(int(backward), M, K, r, N, g))
    if workspace is None:
        workspace = torch.zeros(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel()


def lowrank_linear_fwd_shared_x(X, A_all, Bs, Ys=None, H_all_out=None, save_H: bool = False, workspace=None):
    """Y_i = (X A_i) B_i for the g factor pairs whose A_i sit side by side in A_all [K][g r] (bf16).
    Returns the list of Y_i, or (list, H_all) when save_H or H_all_out is given."""
    torch = _torch()
    lib = load_library()
    bf = torch.bfloat16
    M, K = X.shape
    g = len(Bs)
    r, N = Bs[0].shape
    _check(X, "X", None, bf); _check(A_all, "A_all", (K, g * r), bf)
    for B in Bs:
        _check(B, "B", (r, N), bf)
    if Ys is None:
        Ys = [torch.empty((M, N), dtype=bf, device=X.device) for _ in range(g)]
    for Y in Ys:
        _check(Y, "Y", (M, N), bf)
    if H_all_out is None and save_H:
        H_all_out = torch.empty((M, g * r), dtype=bf, device=X.device)
    _check(H_all_out, "H_all_out", (M, g * r), bf)
    ws, wsz = _shared_ws(False, M, K, r, N, g, X.device, workspace)
    rc = lib.lowrank_linear_fwd_shared_x(_ptr(X), _ptr(A_all), _ptr_array(Bs), _ptr_array(Ys), _ptr(H_all_out),
                                         M, K, r, N, g, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, "lowrank_linear_fwd_shared_x")
    return (Ys, H_all_out) if H_all_out is not None else Ys


def lowrank_ffn_gate_up_fwd(X, A_all, B_gate, B_up, G=None, U=None, Z=None, H_all_out=None, save_H: bool = False, workspace=None):
    """G = (X A_gate) B_gate, U = (X A_up) B_up, Z = SiLU(G) * U with A_all = [A_gate | A_up] (bf16).
    Returns (G, U, Z), or (G, U, Z, H_all) when save_H or H_all_out is given."""
    torch = _torch()
    lib = load_library()
    bf = torch.bfloat16
    M, K = X.shape
    r, N = B_gate.shape
    _check(X, "X", None, bf); _check(A_all, "A_all", (K, 2 * r), bf)
    _check(B_gate, "B_gate", (r, N), bf); _check(B_up, "B_up", (r, N), bf)
    G = torch.empty((M, N), dtype=bf, device=X.device) if G is None else G
    U = torch.empty((M, N), dtype=bf, device=X.device) if U is None else U
    Z = torch.empty((M, N), dtype=bf, device=X.device) if Z is None else Z
    _check(G, "G", (M, N), bf); _check(U, "U", (M, N), bf); _check(Z, "Z", (M, N), bf)
    if H_all_out is None and save_H:
        H_all_out = torch.empty((M, 2 * r), dtype=bf, device=X.device)
    _check(H_all_out, "H_all_out", (M, 2 * r), bf)
    ws, wsz = _shared_ws(False, M, K, r, N, 2, X.device, workspace)
    rc = lib.lowrank_ffn_gate_up_fwd(_ptr(X), _ptr(A_all), _ptr(B_gate), _ptr(B_up), _ptr(G), _ptr(U), _ptr(Z),
                                     _ptr(H_all_out), M, K, r, N, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, "lowrank_ffn_gate_up_fwd")
    return (G, U, Z, H_all_out) if H_all_out is not None else (G, U, Z)


def lowrank_ffn_down_bwd(Z, A, B, dY, G, U, H_saved=None, need_dA=True, need_dB=True,
                         dG=None, dU=None, dA=None, dB=None, workspace=None):
    """Backward of Y = (Z A) B with the input gradient taken through the gate Z = SiLU(G) * U.
    Returns (dG, dU, dA, dB); dA, dB are fp32."""
    torch = _torch()
    lib = load_library()
    bf = torch.bfloat16
    M, K = Z.shape
    r, N = B.shape
    _check(Z, "Z", None, bf); _check(A, "A", (K, r), bf); _check(B, "B", (r, N), bf)
    _check(dY, "dY", (M, N), bf); _check(H_saved, "H_saved", (M, r), bf)
    _check(G, "G", (M, K), bf); _check(U, "U", (M, K), bf)
    dG = torch.empty((M, K), dtype=bf, device=Z.device) if dG is None else dG
    dU = torch.empty((M, K), dtype=bf, device=Z.device) if dU is None else dU
    if dA is None and need_dA:
        dA = torch.empty((K, r), dtype=torch.float32, device=Z.device)
    if dB is None and need_dB:
        dB = torch.empty((r, N), dtype=torch.float32, device=Z.device)
    _check(dG, "dG", (M, K), bf); _check(dU, "dU", (M, K), bf)
    _check(dA, "dA", (K, r), torch.float32); _check(dB, "dB", (r, N), torch.float32)
    ws, wsz = _ws(FHPC_OP_LOWRANK_BWD, M, K, r, N, FHPC_BF16, 0, Z.device, workspace)
    rc = lib.lowrank_ffn_down_bwd(_ptr(Z), _ptr(A), _ptr(B), _ptr(dY), _ptr(H_saved), _ptr(G), _ptr(U), _ptr(dG), _ptr(dU),
                                  _ptr(dA), _ptr(dB), M, K, r, N, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, "lowrank_ffn_down_bwd")
    return dG, dU, dA, dB


def lowrank_linear_bwd_shared_x(X, A_all, Bs, dYs, H_all_saved=None, need_dX=True, need_dA=True, need_dB=True,
                                dX=None, dA_all=None, dBs=None, workspace=None):
    """Returns (dX, dA_all, [dB_i]) of the g layers of lowrank_linear_fwd_shared_x; dA_all, dB_i are fp32.
    need_dB may be a list of g flags; dX, dA_all, dBs (a list, None entries skipped) take preallocated outputs."""
    torch = _torch()
    lib = load_library()
    bf = torch.bfloat16
    M, K = X.shape
    g = len(Bs)
    r, N = Bs[0].shape
    _check(X, "X", None, bf); _check(A_all, "A_all", (K, g * r), bf); _check(H_all_saved, "H_all_saved", (M, g * r), bf)
    if len(dYs) != g:
        raise ValueError("one dY per factor pair")
    for B, dY in zip(Bs, dYs):
        _check(B, "B", (r, N), bf); _check(dY, "dY", (M, N), bf)
    flags = list(need_dB) if isinstance(need_dB, (list, tuple)) else [bool(need_dB)] * g
    if dX is None and need_dX:
        dX = torch.empty((M, K), dtype=bf, device=X.device)
    dA = dA_all
    if dA is None and need_dA:
        dA = torch.empty((K, g * r), dtype=torch.float32, device=X.device)
    if dBs is None:
        dBs = [torch.empty((r, N), dtype=torch.float32, device=X.device) if f else None for f in flags]
    flags = [b is not None for b in dBs]
    _check(dX, "dX", (M, K), bf); _check(dA, "dA_all", (K, g * r), torch.float32)
    for b in dBs:
        _check(b, "dB", (r, N), torch.float32)
    ws, wsz = _shared_ws(True, M, K, r, N, g, X.device, workspace)
    rc = lib.lowrank_linear_bwd_shared_x(_ptr(X), _ptr(A_all), _ptr_array(Bs), _ptr_array(dYs), _ptr(H_all_saved),
                                         _ptr(dX), _ptr(dA), _ptr_array(dBs) if any(flags) else None,
                                         M, K, r, N, g, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, "lowrank_linear_bwd_shared_x")
    return dX, dA, dBs


def _q_shapes(Wq, scales, qscheme, K, N, block):
    torch = _torch()
    if qscheme == FHPC_Q_INT8_PER_CHANNEL:
        _check(Wq, "Wq", (N, K), torch.int8); _check(scales, "scales", (N,), torch.float16)
    elif qscheme == FHPC_Q_INT4_BLOCK:
        _check(Wq, "Wq", (N, K // 2), torch.uint8); _check(scales, "scales", (N, K // block), torch.float16)
    elif qscheme in (FHPC_W_BF16, FHPC_W_MERGED):
        _check(Wq, "W", (K, N), torch.bfloat16)
        if scales is not None:
            raise ValueError("a dense bf16 weight has no scales")
    else:
        raise ValueError("qscheme must be 8, 4 or FHPC_W_BF16")


def qlinear_lowrank_fwd(X, Wq, scales, qscheme, A, B, scaling, block=64, Y=None, H_out=None,
                        save_H: bool = False, workspace=None, _entry="qlinear_lowrank_fwd"):
    """Y = X deq(Wq, scales) + scaling (X A) B (bf16)."""
    torch = _torch()
    lib = load_library()
    M, K = X.shape
    r, N = B.shape
    bf = torch.bfloat16
    _check(X, "X", None, bf); _check(A, "A", (K, r), bf); _check(B, "B", (r, N), bf)
    _q_shapes(Wq, scales, qscheme, K, N, block)
    if Y is None:
        Y = torch.empty((M, N), dtype=bf, device=X.device)
    if H_out is None and save_H:
        H_out = torch.empty((M, r), dtype=bf, device=X.device)
    _check(Y, "Y", (M, N), bf); _check(H_out, "H_out", (M, r), bf)
    ws, wsz = _ws(FHPC_OP_QLINEAR_FWD, M, K, r, N, FHPC_BF16, qscheme, X.device, workspace)
    rc = getattr(lib, _entry)(_ptr(X), _ptr(Wq), _ptr(scales), qscheme, block, _ptr(A), _ptr(B),
                              C.c_float(scaling), _ptr(Y), _ptr(H_out), M, K, r, N, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, _entry)
    return (Y, H_out) if H_out is not None else Y


FHPC_NOALLOC_SCRATCH_BYTES = 16 << 20


def qlinear_lowrank_fwd_noalloc(X, Wq, scales, qscheme, A, B, scaling, Y, H_out=None, block=64):
    """qlinear_lowrank_fwd without a workspace: the library's fixed scratch array serves.  Nothing is allocated here
    either, so Y (and H_out, if wanted) must be passed in."""
    torch = _torch()
    M, K = X.shape
    r, N = B.shape
    bf = torch.bfloat16
    _check(X, "X", None, bf); _check(A, "A", (K, r), bf); _check(B, "B", (r, N), bf)
    _q_shapes(Wq, scales, qscheme, K, N, block)
    _check(Y, "Y", (M, N), bf); _check(H_out, "H_out", (M, r), bf)
    rc = load_library().qlinear_lowrank_fwd_noalloc(_ptr(X), _ptr(Wq), _ptr(scales), qscheme, block, _ptr(A), _ptr(B),
                                                    C.c_float(scaling), _ptr(Y), _ptr(H_out), M, K, r, N, _stream())
    if rc:
        raise FhpcError(rc, "qlinear_lowrank_fwd_noalloc")
    return (Y, H_out) if H_out is not None else Y


def qlinear_lowrank_bwd(X, Wq, scales, qscheme, A, B, scaling, dY, block=64, H_saved=None,
                        need_dX=True, need_dA=True, need_dB=True, dX=None, dA=None, dB=None, workspace=None,
                        _entry="qlinear_lowrank_bwd"):
    """Returns (dX, dA, dB); the frozen W gets no gradient."""
    torch = _torch()
    lib = load_library()
    M, K = X.shape
    r, N = B.shape
    bf = torch.bfloat16
    _check(X, "X", None, bf); _check(A, "A", (K, r), bf); _check(B, "B", (r, N), bf)
    _check(dY, "dY", (M, N), bf); _check(H_saved, "H_saved", (M, r), bf)
    _q_shapes(Wq, scales, qscheme, K, N, block)
    if dX is None and need_dX:
        dX = torch.empty((M, K), dtype=bf, device=X.device)
    if dA is None and need_dA:
        dA = torch.empty((K, r), dtype=torch.float32, device=X.device)
    if dB is None and need_dB:
        dB = torch.empty((r, N), dtype=torch.float32, device=X.device)
    _check(dX, "dX", (M, K), bf); _check(dA, "dA", (K, r), torch.float32); _check(dB, "dB", (r, N), torch.float32)
    ws, wsz = _ws(FHPC_OP_QLINEAR_BWD, M, K, r, N, FHPC_BF16, qscheme, X.device, workspace)
    rc = getattr(lib, _entry)(_ptr(X), _ptr(Wq), _ptr(scales), qscheme, block, _ptr(A), _ptr(B),
                              C.c_float(scaling), _ptr(dY), _ptr(H_saved), _ptr(dX), _ptr(dA), _ptr(dB),
                              M, K, r, N, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, _entry)
    return dX, dA, dB


def qlinear_blend_fwd(X, Wq, scales, qscheme, A, B, alpha, **kw):
    """Y = alpha X deq(Wq, scales) + (1 - alpha) (X A) B (bf16); keywords as qlinear_lowrank_fwd."""
    return qlinear_lowrank_fwd(X, Wq, scales, qscheme, A, B, alpha, _entry="qlinear_blend_fwd", **kw)


def qlinear_blend_bwd(X, Wq, scales, qscheme, A, B, alpha, dY, **kw):
    """(dX, dA, dB) of the blend layer; keywords as qlinear_lowrank_bwd."""
    return qlinear_lowrank_bwd(X, Wq, scales, qscheme, A, B, alpha, dY, _entry="qlinear_blend_bwd", **kw)


def swiglu_fwd(G, U, Z=None):
    torch = _torch()
    _check(G, "G"); _check(U, "U", G.shape, G.dtype)
    if Z is None:
        Z = torch.empty_like(G)
    _check(Z, "Z", G.shape, G.dtype)
    rc = load_library().swiglu_fwd(_ptr(G), _ptr(U), _ptr(Z), G.numel(), _dtype_code(G), _stream())
    if rc:
        raise FhpcError(rc, "swiglu_fwd")
    return Z


def swiglu_bwd(G, U, dZ, dG=None, dU=None):
    torch = _torch()
    _check(G, "G"); _check(U, "U", G.shape, G.dtype); _check(dZ, "dZ", G.shape, G.dtype)
    if dG is None:
        dG = torch.empty_like(G)
    if dU is None:
        dU = torch.empty_like(G)
    rc = load_library().swiglu_bwd(_ptr(G), _ptr(U), _ptr(dZ), _ptr(dG), _ptr(dU), G.numel(), _dtype_code(G), _stream())
    if rc:
        raise FhpcError(rc, "swiglu_bwd")
    return dG, dU


def fhpc_add(a, b, out=None):
    torch = _torch()
    _check(a, "a"); _check(b, "b", a.shape, a.dtype)
    if out is None:
        out = torch.empty_like(a)
    rc = load_library().fhpc_add(_ptr(a), _ptr(b), _ptr(out), a.numel(), _dtype_code(a), _stream())
    if rc:
        raise FhpcError(rc, "fhpc_add")
    return out


def fhpc_gemm_bf16(A, lda, a_mode, B, ldb, b_mode, C, ldc, out_mode, M, N, K, alpha=1.0, tile=0, splits=1, dbg=0):
    """Diagnostic: one launch of the GEMM core (see the header for the argument meanings)."""
    rc = load_library().fhpc_gemm_bf16(_ptr(A), lda, a_mode, _ptr(B), ldb, b_mode, _ptr(C), ldc, out_mode,
                                       M, N, K, C_float(alpha), tile, splits, dbg, _stream())
    if rc:
        raise FhpcError(rc, "fhpc_gemm_bf16")
    return C


def qweight_quantize(W, qscheme, block=64, Wq_out=None, scales_out=None):
    """W fp32 [K,N] on the device -> (Wq, scales) in the canonical layout (into Wq_out, scales_out when given)."""
    torch = _torch()
    _check(W, "W", None, torch.float32)
    K, N = W.shape
    if qscheme == FHPC_Q_INT8_PER_CHANNEL:
        wshape, wdtype, sshape = (N, K), torch.int8, (N,)
    else:
        wshape, wdtype, sshape = (N, K // 2), torch.uint8, (N, max(K // block, 1))
    Wq = Wq_out if Wq_out is not None else torch.empty(wshape, dtype=wdtype, device=W.device)
    sc = scales_out if scales_out is not None else torch.empty(sshape, dtype=torch.float16, device=W.device)
    _check(Wq, "Wq_out", wshape, wdtype); _check(sc, "scales_out", sshape, torch.float16)
    rc = load_library().qweight_quantize(_ptr(W), qscheme, block, _ptr(Wq), _ptr(sc), K, N, _stream())
    if rc:
        raise FhpcError(rc, "qweight_quantize")
    return Wq, sc


def qlinear_lowrank_fwd_shared_x(X, weights, qscheme, block=64, save_H: bool = False, workspace=None):
    """Forward of several finetuning layers that read the same X.  weights: a list of
    (Wq, scales, A, B, scaling) tuples.  Returns the list of Y (or of (Y, H) when save_H)."""
    torch = _torch()
    lib = load_library()
    bf = torch.bfloat16
    M, K = X.shape
    _check(X, "X", None, bf)
    count = len(weights)
    arr = (QlinearWeight * count)()
    outs = []
    Ns = (C.c_int64 * count)()
    r = weights[0][2].shape[1]
    for j, (Wq, sc, A, B, scaling) in enumerate(weights):
        N = B.shape[1]
        _check(A, "A", (K, r), bf); _check(B, "B", (r, N), bf)
        _q_shapes(Wq, sc, qscheme, K, N, block)
        Y = torch.empty((M, N), dtype=bf, device=X.device)
        H = torch.empty((M, r), dtype=bf, device=X.device) if save_H else None
        arr[j] = QlinearWeight(Wq.data_ptr(), sc.data_ptr(), A.data_ptr(), B.data_ptr(), Y.data_ptr(),
                               0 if H is None else H.data_ptr(), N, float(scaling))
        Ns[j] = N
        outs.append((Y, H) if save_H else Y)
    need = int(lib.fhpc_workspace_bytes_shared_x(Ns, count, M, K, r, qscheme))
    ws = workspace if workspace is not None else get_workspace(need, X.device)
    rc = lib.qlinear_lowrank_fwd_shared_x(_ptr(X), arr, count, qscheme, block, M, K, r, _ptr(ws),
                                          C.c_size_t(ws.numel() * ws.element_size()), _stream())
    if rc:
        raise FhpcError(rc, "qlinear_lowrank_fwd_shared_x")
    return outs


def lowrank_merge(W, scales, qscheme, A, B, scaling=1.0, block=64, out_dtype=None, W_out=None, workspace=None):
    """W' [K,N] = deq(W) + scaling A B.  W: None, a bf16 [K,N] tensor (qscheme FHPC_W_BF16) or a
    quantised weight with its scales; out_dtype torch.float32 or torch.bfloat16 (default)."""
    torch = _torch()
    lib = load_library()
    K, r = A.shape
    N = B.shape[1]
    bf = torch.bfloat16
    _check(A, "A", (K, r), bf); _check(B, "B", (r, N), bf)
    if W is not None:
        _q_shapes(W, scales, qscheme, K, N, block)
    if W_out is None:
        W_out = torch.empty((K, N), dtype=out_dtype or bf, device=A.device)
    _check(W_out, "W_out", (K, N))
    need = workspace_bytes(FHPC_OP_MERGE, 1, K, r, N)
    ws = None
    if need:
        ws = workspace if workspace is not None else get_workspace(need, A.device)
    wsz = C.c_size_t(0 if ws is None else ws.numel() * ws.element_size())
    rc = lib.lowrank_merge(_ptr(W), _ptr(scales), qscheme, block, _ptr(A), _ptr(B), float(scaling), _ptr(W_out),
                           _dtype_code(W_out), K, r, N, _ptr(ws), wsz, _stream())
    if rc:
        raise FhpcError(rc, "lowrank_merge")
    return W_out


def lowrank_decompose(W, r, Omega=None, power_iters=2, seed=0, workspace=None):
    """Rank-r factor pair (A, B) of a pretrained weight W (bf16 [K,N] or a batch [L,K,N]).  Omega: the
    bf16 [N,r] random test matrix; drawn here from `seed` (standard normal) when not given."""
    torch = _torch()
    lib = load_library()
    bf = torch.bfloat16
    batched = W.dim() == 3
    L = W.shape[0] if batched else 1
    K, N = W.shape[-2], W.shape[-1]
    _check(W, "W", None, bf)
    if Omega is None:
        g = torch.Generator(device=W.device)
        g.manual_seed(seed)
        Omega = torch.randn((N, r), device=W.device, dtype=torch.float32, generator=g).to(bf)
    _check(Omega, "Omega", (N, r), bf)
    A = torch.empty((L, K, r) if batched else (K, r), dtype=bf, device=W.device)
    B = torch.empty((L, r, N) if batched else (r, N), dtype=bf, device=W.device)
    need = workspace_bytes(FHPC_OP_DECOMPOSE, 1, K, r, N)
    ws = workspace if workspace is not None else get_workspace(need, W.device)
    rc = lib.lowrank_decompose(_ptr(W), _ptr(Omega), int(power_iters), _ptr(A), _ptr(B), K, r, N, L,
                               _ptr(ws), C.c_size_t(ws.numel() * ws.element_size()), _stream())
    if rc:
        raise FhpcError(rc, "lowrank_decompose")
    return A, B


def qweight_unpack(Wq, qscheme):
    torch = _torch()
    N = Wq.shape[0]
    K = Wq.shape[1] * (2 if qscheme == FHPC_Q_INT4_BLOCK else 1)
    _check(Wq, "Wq")
    q = torch.empty((N, K), dtype=torch.int8, device=Wq.device)
    rc = load_library().qweight_unpack(_ptr(Wq), qscheme, _ptr(q), K, N, _stream())
    if rc:
        raise FhpcError(rc, "qweight_unpack")
    return q


def qweight_dequant(Wq, scales, qscheme, block=64, W_out=None):
    torch = _torch()
    N = Wq.shape[0]
    K = Wq.shape[1] * (2 if qscheme == FHPC_Q_INT4_BLOCK else 1)
    _q_shapes(Wq, scales, qscheme, K, N, block)
    out = W_out if W_out is not None else torch.empty((N, K), dtype=torch.float32, device=Wq.device)
    _check(out, "W_out", (N, K), torch.float32)
    rc = load_library().qweight_dequant(_ptr(Wq), _ptr(scales), qscheme, block, _ptr(out), K, N, _stream())
    if rc:
        raise FhpcError(rc, "qweight_dequant")
    return out
