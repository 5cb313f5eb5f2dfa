"""Python face of the CPU oracle (oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg import this
package.  It never imports the HIP library or its binding.  All arithmetic lives
in oracle.c; this file only decodes storage formats exactly into fp64 (bf16 /
fp32 bit patterns -> double) and marshals numpy arrays through ctypes.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (plain -O2, OpenMP over rows, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_f16_to_f64.restype = C.c_double
        _lib.orc_f16_to_f64.argtypes = [C.c_uint16]
        _lib.orc_f32_to_f16.restype = C.c_uint16
        _lib.orc_f32_to_f16.argtypes = [C.c_float]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _i(v) -> C.c_int64:
    return C.c_int64(int(v))


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact decode of bfloat16 bit patterns (uint16) to double."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    flat = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    f = lib().orc_f16_to_f64
    return np.array([f(int(b)) for b in flat], dtype=np.float64).reshape(np.shape(bits))


def f32_to_f16_bits(x) -> np.ndarray:
    flat = np.ascontiguousarray(x, dtype=np.float32).ravel()
    f = lib().orc_f32_to_f16
    return np.array([f(float(v)) for v in flat], dtype=np.uint16).reshape(np.shape(x))


# ---------------------------------------------------------------- low-rank layer

def lowrank_fwd(X, A, B):
    """Y = (X A) B in fp64.  Returns (Y, H)."""
    X, A, B = _d(X), _d(A), _d(B)
    M, K = X.shape
    r, N = B.shape
    assert A.shape == (K, r)
    H = np.empty((M, r))
    Y = np.empty((M, N))
    lib().orc_lowrank_fwd(_p(X), _p(A), _p(B), _p(H), _p(Y), _i(M), _i(K), _i(r), _i(N))
    return Y, H


def lowrank_bwd(X, A, B, dY):
    """Returns (dX, dA, dB) of Y = (X A) B for upstream dY, in fp64."""
    X, A, B, dY = _d(X), _d(A), _d(B), _d(dY)
    M, K = X.shape
    r, N = B.shape
    assert A.shape == (K, r) and dY.shape == (M, N)
    dX = np.empty((M, K))
    dA = np.empty((K, r))
    dB = np.empty((r, N))
    lib().orc_lowrank_bwd(_p(X), _p(A), _p(B), _p(dY), _p(dX), _p(dA), _p(dB),
                          _i(M), _i(K), _i(r), _i(N))
    return dX, dA, dB


# ---------------------------------------------------------------- quantisation

def unpack_int4(packed) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    q = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.int8)
    lib().orc_unpack_int4(_p(packed), _p(q), _i(packed.size))
    return q


def pack_int4(q) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int8)
    assert q.shape[-1] % 2 == 0
    packed = np.empty(q.shape[:-1] + (q.shape[-1] // 2,), dtype=np.uint8)
    lib().orc_pack_int4(_p(q), _p(packed), _i(packed.size))
    return packed


def quantize_int8_perchannel(W):
    """W fp32 [K,N] -> (q int8 [N,K], scales fp16 bit patterns uint16 [N])."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    q = np.empty((N, K), dtype=np.int8)
    s = np.empty((N,), dtype=np.uint16)
    lib().orc_quantize_int8_perchannel(_p(W), _p(q), _p(s), _i(K), _i(N))
    return q, s


def quantize_int4_block(W, block: int = 64):
    """W fp32 [K,N] -> (packed uint8 [N,K/2], scales fp16 bit patterns [N,K/block])."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    assert K % block == 0 and block % 2 == 0
    p = np.empty((N, K // 2), dtype=np.uint8)
    s = np.empty((N, K // block), dtype=np.uint16)
    lib().orc_quantize_int4_block(_p(W), _p(p), _p(s), _i(K), _i(N), _i(block))
    return p, s


def dequant(Wq, scales, scheme: int, block: int = 64) -> np.ndarray:
    """Exact fp64 dequantised weight Wd[K,N] from the canonical [N][...] storage."""
    scales = np.ascontiguousarray(scales, dtype=np.uint16)
    if scheme == 8:
        Wq = np.ascontiguousarray(Wq, dtype=np.int8)
        N, K = Wq.shape
    else:
        Wq = np.ascontiguousarray(Wq, dtype=np.uint8)
        N, K = Wq.shape[0], Wq.shape[1] * 2
    Wd = np.empty((K, N))
    lib().orc_dequant(_p(Wq), _p(scales), C.c_int(scheme), _i(block), _p(Wd), _i(K), _i(N))
    return Wd


# ---------------------------------------------------------------- finetuning layer

def qlinear_lowrank_fwd(X, Wd, A, B, s: float):
    """Y = X Wd + s (X A) B.  Returns (Y, H)."""
    X, Wd, A, B = _d(X), _d(Wd), _d(A), _d(B)
    M, K = X.shape
    r, N = B.shape
    assert Wd.shape == (K, N) and A.shape == (K, r)
    H = np.empty((M, r))
    Y = np.empty((M, N))
    lib().orc_qlinear_lowrank_fwd(_p(X), _p(Wd), _p(A), _p(B), C.c_double(s), _p(H), _p(Y),
                                  _i(M), _i(K), _i(r), _i(N))
    return Y, H


def qlinear_lowrank_bwd(X, Wd, A, B, s: float, dY):
    """Returns (dX, dA, dB); the frozen W gets no gradient."""
    X, Wd, A, B, dY = _d(X), _d(Wd), _d(A), _d(B), _d(dY)
    M, K = X.shape
    r, N = B.shape
    assert Wd.shape == (K, N) and A.shape == (K, r) and dY.shape == (M, N)
    dX = np.empty((M, K))
    dA = np.empty((K, r))
    dB = np.empty((r, N))
    lib().orc_qlinear_lowrank_bwd(_p(X), _p(Wd), _p(A), _p(B), C.c_double(s), _p(dY),
                                  _p(dX), _p(dA), _p(dB), _i(M), _i(K), _i(r), _i(N))
    return dX, dA, dB


# ---------------------------------------------------------------- blend layer

def blend_fwd(X, W, A, B, alpha: float):
    """Y = alpha X W + (1 - alpha) (X A) B with W[K,N] frozen.  Returns (Y, H)."""
    X, W, A, B = _d(X), _d(W), _d(A), _d(B)
    M, K = X.shape
    r, N = B.shape
    assert W.shape == (K, N) and A.shape == (K, r)
    H = np.empty((M, r))
    Y = np.empty((M, N))
    lib().orc_blend_fwd(_p(X), _p(W), _p(A), _p(B), C.c_double(alpha), _p(H), _p(Y), _i(M), _i(K), _i(r), _i(N))
    return Y, H


def blend_bwd(X, W, A, B, alpha: float, dY):
    """Returns (dX, dA, dB); the frozen W gets no gradient."""
    X, W, A, B, dY = _d(X), _d(W), _d(A), _d(B), _d(dY)
    M, K = X.shape
    r, N = B.shape
    assert W.shape == (K, N) and A.shape == (K, r) and dY.shape == (M, N)
    dX = np.empty((M, K))
    dA = np.empty((K, r))
    dB = np.empty((r, N))
    lib().orc_blend_bwd(_p(X), _p(W), _p(A), _p(B), C.c_double(alpha), _p(dY), _p(dX), _p(dA), _p(dB),
                        _i(M), _i(K), _i(r), _i(N))
    return dX, dA, dB


# ---------------------------------------------------------------- merged weight

def merge(W, A, B, s: float = 1.0):
    """W' = W + s A B (W[K,N] or None, A[K,r], B[r,N]).  Returns W'[K,N]."""
    A, B = _d(A), _d(B)
    K, r = A.shape
    N = B.shape[1]
    assert B.shape[0] == r
    Wp = np.empty((K, N))
    if W is None:
        lib().orc_merge(None, _p(A), _p(B), C.c_double(s), _p(Wp), _i(K), _i(r), _i(N))
    else:
        W = _d(W)
        assert W.shape == (K, N)
        lib().orc_merge(_p(W), _p(A), _p(B), C.c_double(s), _p(Wp), _i(K), _i(r), _i(N))
    return Wp


# ---------------------------------------------------------------- factor pair from a pretrained weight

def lowrank_factorize(W, r: int):
    """Rank-r factor pair of a pretrained weight (Sec. 4.1 item 2: W is decomposed into A[K,r] and
    B[r,N], which initialise the factorised layer).  The paper names no algorithm; the reading taken
    here is the best rank-r approximation in the Frobenius norm, i.e. the singular value
    decomposition W = U S V^T cut after the r largest singular values, with the factors balanced:
    A = U_r S_r^(1/2), B = S_r^(1/2) V_r^T.  numpy's LAPACK SVD serves as the step.
    Returns (A, B, s) with s all singular values, largest first."""
    W = _d(W)
    K, N = W.shape
    assert 1 <= r <= min(K, N)
    U, s, Vt = np.linalg.svd(W, full_matrices=False)
    root = np.sqrt(s[:r])
    return U[:, :r] * root[None, :], root[:, None] * Vt[:r, :], s


# ---------------------------------------------------------------- SiLU gate

def swiglu_fwd(G, U):
    G, U = _d(G), _d(U)
    Z = np.empty_like(G)
    lib().orc_swiglu_fwd(_p(G), _p(U), _p(Z), _i(G.size))
    return Z


def swiglu_bwd(G, U, dZ):
    G, U, dZ = _d(G), _d(U), _d(dZ)
    dG = np.empty_like(G)
    dU = np.empty_like(G)
    lib().orc_swiglu_bwd(_p(G), _p(U), _p(dZ), _p(dG), _p(dU), _i(G.size))
    return dG, dU


def rel_fro(got, ref) -> float:
    """||got - ref||_F / ||ref||_F in fp64."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return float(num / den) if den > 0 else float(num)
