"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, and validates arguments before launching anything (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

import paper_2402_13533_amd as fhpc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fingpt_hpc.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)))


def test_library_exports_every_declared_symbol():
    lib = fhpc.load_library()
    names = _declared_functions()
    assert len(names) >= 13 and "lowrank_linear_fwd" in names and "qlinear_lowrank_bwd" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(fhpc.EXPORTS) == names
    assert fhpc.version() >= 100


def test_status_strings():
    seen = {fhpc.status_string(i) for i in range(8)}
    assert len(seen) == 8 and fhpc.status_string(0) == "ok" and fhpc.status_string(99) == "unknown status"


def test_workspace_bytes_host_only():
    wb = fhpc.workspace_bytes
    assert wb(fhpc.FHPC_OP_LOWRANK_FWD, 16384, 4096, 512, 4096) >= 16384 * 512 * 2
    assert wb(fhpc.FHPC_OP_LOWRANK_BWD, 16384, 4096, 512, 4096) >= 2 * 16384 * 512 * 2
    assert wb(fhpc.FHPC_OP_QLINEAR_BWD, 4096, 4096, 8, 4096) % 256 == 0
    assert wb(fhpc.FHPC_OP_LOWRANK_FWD, 0, 4096, 512, 4096) == 0           # invalid shape
    assert wb(fhpc.FHPC_OP_LOWRANK_FWD, 16, 4100, 8, 4096) == 0            # K not a multiple of 8
    assert wb(7, 16, 64, 8, 64) == 0
    # odd rank needs padded copies of A and B
    assert wb(fhpc.FHPC_OP_LOWRANK_FWD, 64, 64, 5, 64) > wb(fhpc.FHPC_OP_LOWRANK_FWD, 64, 64, 8, 64)


def test_validation_precedes_launch():
    """Error codes for bad arguments come back without touching a device (fake, aligned,
    non-NULL addresses are never dereferenced on these paths)."""
    lib = fhpc.load_library()
    p = C.c_void_p(0x10000)
    odd = C.c_void_p(0x10004)
    nul = C.c_void_p(0)
    ws = C.c_void_p(0x20000)
    big = C.c_size_t(1 << 40)
    f = lib.lowrank_linear_fwd
    assert f(nul, p, p, p, nul, 16, 64, 8, 64, 1, ws, big, nul) == 1          # NULL X
    assert f(p, p, p, p, nul, 16, 60, 8, 64, 1, ws, big, nul) == 2            # K % 8
    assert f(p, p, p, p, nul, 0, 64, 8, 64, 1, ws, big, nul) == 2             # M < 1
    assert f(p, p, p, p, nul, 16, 64, 8, 64, 5, ws, big, nul) == 3            # dtype
    assert f(odd, p, p, p, nul, 16, 64, 8, 64, 1, ws, big, nul) == 4          # alignment
    assert f(p, p, p, p, nul, 16, 64, 8, 64, 1, nul, C.c_size_t(0), nul) == 5  # workspace
    assert f(p, p, p, p, nul, 16, 64, 8, 64, 1, ws, C.c_size_t(16), nul) == 5
    assert f(p, p, p, p, nul, 1 << 28, 4096, 8, 4096, 1, ws, big, nul) == 6    # >= 2 GiB operand
    q = lib.qlinear_lowrank_fwd
    assert q(p, p, p, 3, 64, p, p, C.c_float(1), p, nul, 16, 64, 8, 64, ws, big, nul) == 3   # scheme
    assert q(p, p, p, 4, 32, p, p, C.c_float(1), p, nul, 16, 64, 8, 64, ws, big, nul) == 6   # block
    assert q(p, p, p, 4, 64, p, p, C.c_float(1), p, nul, 16, 72, 8, 64, ws, big, nul) == 2   # K % 64
    assert q(p, nul, p, 8, 64, p, p, C.c_float(1), p, nul, 16, 64, 8, 64, ws, big, nul) == 1
    b = lib.lowrank_linear_bwd
    assert b(p, p, p, nul, nul, p, p, p, 16, 64, 8, 64, 1, ws, big, nul) == 1  # NULL dY
    assert lib.swiglu_fwd(p, p, nul, 8, 1, nul) == 1
    assert lib.swiglu_bwd(p, p, p, p, p, 8, 9, nul) == 3
    assert lib.qweight_quantize(p, 4, 48, p, p, 64, 64, nul) == 6
    assert lib.qweight_dequant(p, p, 5, 64, p, 64, 64, nul) == 3
    assert lib.fhpc_add(p, p, p, -1, 1, nul) == 2
    assert lib.fhpc_add(p, odd, p, 8, 1, nul) == 4
    assert lib.swiglu_fwd(p, p, odd, 8, 1, nul) == 4
    bl = lib.qlinear_blend_fwd
    assert bl(p, p, p, 8, 64, p, p, C.c_float(1.5), p, nul, 16, 64, 8, 64, ws, big, nul) == 2      # alpha > 1
    assert bl(p, p, p, 8, 64, p, p, C.c_float(float("nan")), p, nul, 16, 64, 8, 64, ws, big, nul) == 2
    assert bl(p, p, p, 8, 64, p, p, C.c_float(0.5), p, nul, 16, 64, 8, 64, nul, C.c_size_t(0), nul) == 5
    assert bl(p, p, nul, 16, 0, p, p, C.c_float(0.5), p, nul, 16, 64, 8, 64, nul, C.c_size_t(0), nul) == 5  # dense W: no scales needed
    assert q(p, p, nul, 16, 0, p, p, C.c_float(1), p, nul, 16, 64, 8, 64, ws, big, nul) == 3              # not for the finetuning layer
    mg = lib.lowrank_merge
    one = C.c_float(1)
    assert mg(p, p, 8, 64, nul, p, one, p, 1, 64, 8, 64, nul, C.c_size_t(0), nul) == 1            # NULL A
    assert mg(p, nul, 8, 64, p, p, one, p, 1, 64, 8, 64, nul, C.c_size_t(0), nul) == 1            # quantised W without scales
    assert mg(p, p, 8, 64, p, p, one, p, 7, 64, 8, 64, nul, C.c_size_t(0), nul) == 3              # out dtype
    assert mg(p, p, 5, 64, p, p, one, p, 1, 64, 8, 64, nul, C.c_size_t(0), nul) == 3              # scheme
    assert mg(p, p, 4, 64, p, p, one, p, 1, 72, 8, 64, nul, C.c_size_t(0), nul) == 2              # K % 64 (4-bit)
    assert mg(p, p, 8, 64, p, p, one, p, 1, 64, 8, 60, nul, C.c_size_t(0), nul) == 2              # N % 8
    assert mg(p, p, 8, 64, p, p, one, odd, 1, 64, 8, 64, nul, C.c_size_t(0), nul) == 4            # alignment
    assert mg(p, p, 8, 64, p, p, one, p, 1, 64, 5, 64, nul, C.c_size_t(0), nul) == 5              # odd rank needs a workspace
    assert mg(p, p, 8, 64, p, p, one, p, 1, 64, 5, 64, ws, C.c_size_t(64), nul) == 5
    assert mg(p, p, 8, 64, p, p, one, p, 1, 1 << 16, 8, 1 << 16, nul, C.c_size_t(0), nul) == 6    # >= 2 GiB
    sx = lib.qlinear_lowrank_fwd_shared_x
    wts = (fhpc.QlinearWeight * 2)(fhpc.QlinearWeight(0x10000, 0x10000, 0x10000, 0x10000, 0x10000, 0, 64, 1.0),
                                   fhpc.QlinearWeight(0x10000, 0x10000, 0x10000, 0x10000, 0, 0, 64, 1.0))
    assert sx(p, wts, 2, 8, 64, 4, 512, 8, ws, big, nul) == 1                                     # second weight has no Y
    assert sx(p, wts, 0, 8, 64, 4, 512, 8, ws, big, nul) == 2                                     # count
    assert sx(p, wts, 1, 5, 64, 4, 512, 8, ws, big, nul) == 3                                     # scheme
    assert sx(p, wts, 1, 8, 64, 4, 512, 8, nul, C.c_size_t(0), nul) == 5                          # workspace
    ns = (C.c_int64 * 2)(64, 128)
    assert lib.fhpc_workspace_bytes_shared_x(ns, 2, 4, 512, 8, 8) >= 4 * 192 * 4
    assert lib.fhpc_workspace_bytes_shared_x(ns, 0, 4, 512, 8, 8) == 0
    lf, lb, lw = lib.lowrank_linear_fwd_shared_x, lib.lowrank_linear_bwd_shared_x, lib.fhpc_workspace_bytes_lowrank_shared_x
    two = (C.c_void_p * 2)(0x10000, 0x10000)
    gap = (C.c_void_p * 2)(0x10000, None)
    assert lf(p, p, two, gap, nul, 256, 512, 8, 64, 2, ws, big, nul) == 1                         # second layer has no Y
    assert lf(p, p, two, two, nul, 256, 512, 8, 64, 0, ws, big, nul) == 2                         # g
    assert lf(p, p, two, two, nul, 256, 512, 8, 64, 9, ws, big, nul) == 2
    assert lf(p, p, two, two, nul, 256, 512, 12, 64, 2, ws, big, nul) == 6                        # rank not a multiple of 8
    assert lf(odd, p, two, two, nul, 256, 512, 8, 64, 2, ws, big, nul) == 4
    assert lf(p, p, two, two, nul, 256, 512, 8, 64, 2, nul, C.c_size_t(0), nul) == 5
    assert lb(p, p, two, gap, nul, p, p, two, 256, 512, 8, 64, 2, ws, big, nul) == 1              # second layer has no dY
    assert lb(p, p, two, two, nul, p, p, None, 256, 512, 8, 64, 2, nul, C.c_size_t(0), nul) == 5
    assert lw(0, 256, 512, 8, 64, 2) >= 256 * 16 * 2
    assert lw(1, 256, 512, 8, 64, 2) > lw(0, 256, 512, 8, 64, 2)
    assert lw(1, 256, 512, 12, 64, 2) == 0 and lw(1, 256, 512, 8, 64, 9) == 0
    dc = lib.lowrank_decompose
    assert dc(p, nul, 2, p, p, 64, 8, 64, 1, ws, big, nul) == 1                                   # NULL Omega
    assert dc(p, p, 2, p, p, 64, 8, 60, 1, ws, big, nul) == 2                                     # N % 8
    assert dc(p, p, 99, p, p, 64, 8, 64, 1, ws, big, nul) == 2                                    # power_iters
    assert dc(p, p, 2, p, p, 64, 8, 64, 0, ws, big, nul) == 2                                     # batch
    assert dc(p, p, 2, p, p, 64, 12, 64, 1, ws, big, nul) == 6                                    # rank not a multiple of 8
    assert dc(p, p, 2, p, p, 64, 72, 64, 1, ws, big, nul) == 6                                    # rank above min(K, N)
    assert dc(p, p, 2, odd, p, 64, 8, 64, 1, ws, big, nul) == 4
    assert dc(p, p, 2, p, p, 64, 8, 64, 1, ws, C.c_size_t(1024), nul) == 5
    assert fhpc.workspace_bytes(fhpc.FHPC_OP_DECOMPOSE, 1, 4096, 512, 4096) > 3 * 4096 * 512 * 2
    assert fhpc.workspace_bytes(fhpc.FHPC_OP_DECOMPOSE, 1, 64, 12, 64) == 0
    assert fhpc.workspace_bytes(fhpc.FHPC_OP_MERGE, 1, 64, 8, 64) == 0
    assert fhpc.workspace_bytes(fhpc.FHPC_OP_MERGE, 1, 64, 5, 64) == 16384 + 64 * 8 * 2          # the header, then a padded A


def test_ffn_gate_calls_validate_before_launch():
    lib = fhpc.load_library()
    p, odd, nul = C.c_void_p(0x10000), C.c_void_p(0x10004), C.c_void_p(0)
    ws, big = C.c_void_p(0x20000), C.c_size_t(1 << 40)
    f = lib.lowrank_ffn_gate_up_fwd
    assert f(p, p, p, p, p, p, nul, nul, 16, 64, 8, 64, ws, big, nul) == 1          # NULL Z_out
    assert f(p, p, p, p, p, p, p, nul, 16, 60, 8, 64, ws, big, nul) == 2            # K % 8
    assert f(p, p, p, p, p, p, p, nul, 16, 64, 4, 64, ws, big, nul) == 6            # r % 8: column blocks of A_all
    assert f(p, p, p, p, p, odd, p, nul, 16, 64, 8, 64, ws, big, nul) == 4          # alignment
    assert f(p, p, p, p, p, p, p, nul, 16, 64, 8, 64, ws, C.c_size_t(16), nul) == 5  # workspace
    b = lib.lowrank_ffn_down_bwd
    assert b(p, p, p, p, nul, nul, p, p, p, nul, nul, 16, 64, 8, 64, ws, big, nul) == 1   # NULL G
    assert b(p, p, p, p, nul, p, p, p, nul, nul, nul, 16, 64, 8, 64, ws, big, nul) == 1   # NULL dU_out
    assert b(p, p, p, p, nul, p, p, p, p, nul, nul, 0, 64, 8, 64, ws, big, nul) == 2      # M < 1
    assert b(p, p, p, p, nul, p, odd, p, p, nul, nul, 16, 64, 8, 64, ws, big, nul) == 4   # alignment
    assert b(p, p, p, p, nul, p, p, p, p, nul, nul, 16, 64, 8, 64, nul, C.c_size_t(0), nul) == 5


def test_read_rows_probe_validates_before_launch():
    lib = fhpc.load_library()
    p, odd, nul = C.c_void_p(0x10000), C.c_void_p(0x10004), C.c_void_p(0)
    f = lib.fhpc_probe_read_rows
    assert f(nul, 64, 256, 768, p, nul) == 1                   # NULL matrix
    assert f(p, 64, 256, 768, nul, nul) == 1                   # NULL sink
    assert f(p, 0, 256, 768, p, nul) == 2                      # no rows
    assert f(p, 64, 192, 768, p, nul) == 2                     # row_bytes % 256
    assert f(p, 1 << 20, 4096, 768, p, nul) == 2               # 2^31 bytes and more
    assert f(p, 64, 256, 0, p, nul) == 2                       # no workgroups
    assert f(odd, 64, 256, 768, p, nul) == 4                   # alignment


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros((8, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        fhpc.lowrank_linear_fwd(x, torch.zeros((64, 8), dtype=torch.bfloat16), torch.zeros((8, 64), dtype=torch.bfloat16))
