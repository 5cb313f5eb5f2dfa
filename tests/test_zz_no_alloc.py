"""The forward entry point that allocates nothing (qlinear_lowrank_fwd_noalloc: the library's fixed scratch
array in place of a caller workspace) against qlinear_lowrank_fwd on the same inputs, through the C ABI."""
import numpy as np
import pytest

import oracle
from harness import TOL_BF16, f16_bits_cuda, from_device, parity_err, qlinear_inputs

pytestmark = pytest.mark.gpu


def _case(fhpc, scheme, M, K, r, N, base):
    import torch
    W, X, A, B, _ = qlinear_inputs(7, M, K, r, N, base)
    Wq, sc = (oracle.quantize_int4_block(W, 64) if scheme == 4 else oracle.quantize_int8_perchannel(W))
    Wq_d, sc_d = torch.from_numpy(Wq).cuda(), f16_bits_cuda(sc)
    Xd, Ad, Bd = X.cuda(), A.cuda(), B.cuda()
    Y_ref, H_ref = fhpc.qlinear_lowrank_fwd(Xd, Wq_d, sc_d, scheme, Ad, Bd, 2.0, save_H=True)
    Yr, _ = oracle.qlinear_lowrank_fwd(X.f64, oracle.dequant(Wq, sc, scheme, 64), A.f64, B.f64, 2.0)
    assert parity_err(from_device(Y_ref), Yr, what="workspace entry point") <= TOL_BF16
    return (Xd, Wq_d, sc_d, scheme, Ad, Bd, 2.0), Y_ref, H_ref


@pytest.mark.parametrize("scheme", [4, 8])
@pytest.mark.parametrize("first,second", [
    ((64, 1024, 16, 1032), (16, 512, 16, 264)),      # weight-streaming route, then a smaller weight and fewer tokens
    ((300, 1024, 8, 520), (130, 256, 8, 264)),       # dequantising products, reduction cut into slices (fp32 slabs)
    ((1300, 512, 24, 520), (1152, 256, 5, 264)),     # merged-weight route (the bf16 weight lives in the scratch), padded rank
])
def test_two_calls_in_a_row_match_the_workspace_entry_point(scheme, first, second):
    import torch
    import paper_2402_13533_amd as fhpc
    for i, (M, K, r, N) in enumerate((first, second)):
        args, Y_ref, H_ref = _case(fhpc, scheme, M, K, r, N, 40 + 10 * i)
        Y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
        H = torch.full((M, r), 7.0, dtype=torch.bfloat16, device="cuda")
        fhpc.qlinear_lowrank_fwd_noalloc(*args, Y, H)
        torch.cuda.synchronize()
        # the same kernels on the same plan: the outputs agree bit for bit
        assert torch.equal(Y, Y_ref), (i, (M, K, r, N))
        assert torch.equal(H, H_ref), (i, (M, K, r, N))
        Y2 = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
        fhpc.qlinear_lowrank_fwd_noalloc(*args, Y2)                 # H not wanted
        assert torch.equal(Y2, Y_ref)


def test_sizes_beyond_the_fixed_scratch_are_refused():
    import torch
    import paper_2402_13533_amd as fhpc
    M, K, r, N = 4096, 4096, 8, 4096            # merged route: 32 MiB of bf16 weight alone
    assert fhpc.workspace_bytes(fhpc.FHPC_OP_QLINEAR_FWD, M, K, r, N, fhpc.FHPC_BF16, 8) > fhpc.FHPC_NOALLOC_SCRATCH_BYTES
    bf = torch.bfloat16
    X = torch.zeros((M, K), dtype=bf, device="cuda"); A = torch.zeros((K, r), dtype=bf, device="cuda")
    B = torch.zeros((r, N), dtype=bf, device="cuda"); Y = torch.full((M, N), 7.0, dtype=bf, device="cuda")
    Wq = torch.zeros((N, K), dtype=torch.int8, device="cuda"); sc = torch.ones((N,), dtype=torch.float16, device="cuda")
    with pytest.raises(fhpc.FhpcError) as e:
        fhpc.qlinear_lowrank_fwd_noalloc(X, Wq, sc, 8, A, B, 2.0, Y)
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())               # nothing was launched
