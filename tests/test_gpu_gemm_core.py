"""The bf16 matrix-core GEMM behind every entry point, launched directly through the
diagnostic entry fhpc_gemm_bf16 on every tile shape (including the eight-wave ping-pong
kernels that only large problems select by themselves), with ragged extents and K tails.
Reference: the product written out in fp64 (numpy matmul on the exactly decoded inputs)."""
import numpy as np
import pytest

from harness import TOL_BF16, Bf16, from_device

pytestmark = pytest.mark.gpu

TILES = {0: (256, 256), 1: (128, 256), 2: (256, 128), 3: (128, 128)}


def _run(a_mode, b_mode, out_mode, tile, M, N, K, splits=1, dbg=0, seed=0):
    import torch
    import paper_2402_13533_amd as fhpc
    A = Bf16.normal(1000 + seed, (M, K) if a_mode == 0 else (K, M))
    B = Bf16.normal(2000 + seed, (N, K) if b_mode == 0 else (K, N))
    Af = A.f64 if a_mode == 0 else A.f64.T
    Bf = B.f64 if b_mode == 0 else B.f64.T
    ref = Af @ Bf.T
    lda = K if a_mode == 0 else M
    ldb = K if b_mode == 0 else N
    if out_mode == 0:
        C = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    else:
        C = torch.full((splits, M, N), 7.0, dtype=torch.float32, device="cuda")
    fhpc.fhpc_gemm_bf16(A.cuda(), lda, a_mode, B.cuda(), ldb, b_mode, C, N, out_mode, M, N, K, 0.5, tile, splits, dbg)
    got = from_device(C)
    if out_mode == 1:
        # the reduction is cut in whole 64-deep steps, so fewer slices than asked for may exist;
        # slabs beyond them are left alone
        ksteps = (K + 63) // 64
        per = (ksteps + splits - 1) // splits
        used = (ksteps + per - 1) // per
        assert np.all(got[used:] == 7.0)
        got = got[:used].sum(axis=0)
    return got, 0.5 * ref


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("a_mode,b_mode", [(0, 0), (0, 1)])
@pytest.mark.parametrize("M,N,K", [(520, 776, 136), (256, 256, 64), (1000, 264, 1032), (70, 1200, 200)])
def test_bf16_output(tile, a_mode, b_mode, M, N, K):
    got, ref = _run(a_mode, b_mode, 0, tile, M, N, K, seed=tile)
    err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert err <= TOL_BF16, err


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("M,N,K,splits", [(520, 776, 1096, 1), (264, 512, 2048, 4), (1000, 264, 4000, 7)])
def test_fp32_split_output(tile, M, N, K, splits):
    """Both operands stored with the reduction index outermost (the weight-gradient products);
    every slice of the reduction writes its own slab, the slabs add up to the product."""
    got, ref = _run(1, 1, 1, tile, M, N, K, splits=splits, seed=10 + tile)
    err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert err <= 1e-5, err          # fp32 accumulation of exact bf16 products


def test_lockstep_kernels_still_reachable():
    """dbg bit 2 routes the big tiles to the lockstep kernels (kept for the quantised operands)."""
    for tile in (0, 2):
        got, ref = _run(0, 0, 0, tile, 520, 776, 200, dbg=4, seed=20)
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= TOL_BF16


@pytest.mark.parametrize("a_mode,b_mode,out_mode,splits", [(0, 0, 0, 1), (0, 1, 0, 1), (1, 1, 1, 1), (1, 1, 1, 3)])
@pytest.mark.parametrize("M,N,K", [(520, 776, 136), (256, 256, 32), (1000, 264, 1032)])
def test_four_wave_kernel(a_mode, b_mode, out_mode, splits, M, N, K):
    """dbg bit 3 selects the four-wave 256x256 kernel (one wave per SIMD, 128x128 per wave)."""
    got, ref = _run(a_mode, b_mode, out_mode, 0, M, N, K, splits=splits, dbg=8, seed=30)
    err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert err <= (TOL_BF16 if out_mode == 0 else 1e-5), err


@pytest.mark.parametrize("N,row_bytes,workgroups", [(5120, 2560, 768), (100, 256, 768), (777, 1280, 64), (64, 6912, 4096)])
def test_read_rows_probe_runs(N, row_bytes, workgroups):
    """The measurement probe that reads a byte matrix in the few-token kernels' access pattern: it returns the byte
    count, leaves its sink alone and leaves the matrix as it was (ragged row counts and every slicing case)."""
    import torch
    import paper_2402_13533_amd as fhpc
    W = torch.arange(N * row_bytes, dtype=torch.int64, device="cuda").remainder(251).to(torch.uint8).reshape(N, row_bytes)
    before = W.clone()
    sink = torch.zeros(256, dtype=torch.int32, device="cuda")
    assert fhpc.probe_read_rows(W, workgroups, sink) == N * row_bytes
    torch.cuda.synchronize()
    assert torch.equal(W, before) and int(sink.abs().sum()) == 0
