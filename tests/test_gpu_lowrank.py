"""GPU parity of lowrank_linear_fwd / lowrank_linear_bwd against the CPU oracle on the
same seeded inputs (element by element, relative Frobenius error per output tensor)."""
import numpy as np
import pytest

import oracle
from harness import Guarded, TOL_BF16, TOL_F32, Bf16, from_device, lowrank_inputs, sample_rows, parity_err

pytestmark = pytest.mark.gpu


def _fhpc():
    import paper_2402_13533_amd as fhpc
    return fhpc


def _check_all(tag, got, ref, tol):
    for name, g, r in zip(("Y", "dX", "dA", "dB"), got, ref):
        if g is None:
            continue
        err = parity_err(from_device(g), r, tol, "%s %s" % (tag, name))
        print("%s %s rel_fro=%.3e" % (tag, name, err), flush=True)
        assert err <= tol, (tag, name, err)


def test_config1_fp32():
    """Config 1: fp32, X 256x768, r = 32; tolerance 1e-5."""
    import torch
    fhpc = _fhpc()
    M, K, r, N = 256, 768, 32, 768
    X, A, B, dY = lowrank_inputs(1, M, K, r, N, bf16=False)
    Yr, Hr = oracle.lowrank_fwd(X, A, B)
    ref = (Yr,) + oracle.lowrank_bwd(X, A, B, dY)
    d = lambda a: torch.from_numpy(a).cuda()
    Xd, Ad, Bd, dYd = d(X), d(A), d(B), d(dY)
    Y, H = fhpc.lowrank_linear_fwd(Xd, Ad, Bd, save_H=True)
    assert parity_err(from_device(H), Hr) <= TOL_F32
    dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H)
    _check_all("c1 saved-H", (Y, dX, dA, dB), ref, TOL_F32)
    dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd)             # recompute H
    _check_all("c1 recompute", (None, dX, dA, dB), ref, TOL_F32)


@pytest.mark.parametrize("M,K,r,N", [
    (50, 136, 5, 72),        # ragged token count and rank (K and N are multiples of 8 by contract); one launch per chain: H and dH stay in LDS
    (33, 64, 64, 264),       # the largest rank that fits, a ragged row block, more columns than threads
    (17, 200, 65, 96),       # one rank beyond: two launches per chain
    (1, 8, 1, 8),
])
def test_fp32_shapes(M, K, r, N):
    """fp32 storage and arithmetic on shapes other than config 1's (tolerance 1e-5), with H saved, recomputed, and
    with outputs left out."""
    import torch
    fhpc = _fhpc()
    X, A, B, dY = lowrank_inputs(2, M, K, r, N, bf16=False)
    Yr, Hr = oracle.lowrank_fwd(X, A, B)
    ref = (Yr,) + oracle.lowrank_bwd(X, A, B, dY)
    d = lambda a: torch.from_numpy(a).cuda()
    Xd, Ad, Bd, dYd = d(X), d(A), d(B), d(dY)
    Y, H = fhpc.lowrank_linear_fwd(Xd, Ad, Bd, save_H=True)
    assert parity_err(from_device(H), Hr, TOL_F32, "H") <= TOL_F32
    Y2 = fhpc.lowrank_linear_fwd(Xd, Ad, Bd)                          # H not asked for
    assert torch.equal(Y, Y2)
    dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H)
    _check_all("f32 saved-H %s" % ((M, K, r, N),), (Y, dX, dA, dB), ref, TOL_F32)
    dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd)
    _check_all("f32 recompute %s" % ((M, K, r, N),), (None, dX, dA, dB), ref, TOL_F32)
    dX3, dA3, dB3 = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H, need_dA=False)
    assert dA3 is None and torch.equal(dX3, dX) and torch.equal(dB3, dB)


@pytest.mark.parametrize("M,K,r,N", [
    (300, 320, 64, 264),     # ragged in every dimension, several tiles
    (1, 64, 8, 72),          # a single token
    (257, 136, 5, 200),      # rank not a multiple of 8 (padded internally)
    (515, 1024, 16, 520),    # LoRA-sized rank: split reductions for H and dH
    (640, 512, 96, 1032),    # rank between tile sizes
    (1100, 768, 512, 776),   # pretraining-sized rank
    (48, 520, 40, 264),      # few tokens, small rank: dA and dB as token-deep sums in one launch
    (64, 1032, 512, 776),    # few tokens, large rank: dA and dB as tiles of outer-product sums
    (33, 328, 77, 264),      # the same with a rank that is padded (dA rows not 16-byte aligned)
    (1, 264, 130, 520),
    (4000, 2048, 512, 2056), # X A and dY B^T: 64 tiles of 256 x 128 (ragged last row), reductions cut into 4 slices on the large tiles
    (1300, 8192, 520, 264),  # X A: 6 x 3 tiles of 256 x 256 in 16 slices of 512
])
def test_bf16_shapes(M, K, r, N):
    fhpc = _fhpc()
    X, A, B, dY = lowrank_inputs(9, M, K, r, N, tensor_base=10)
    Yr, Hr = oracle.lowrank_fwd(X.f64, A.f64, B.f64)
    ref = (Yr,) + oracle.lowrank_bwd(X.f64, A.f64, B.f64, dY.f64)
    import torch
    Xd, Ad, Bd, dYd = X.cuda(), A.cuda(), B.cuda(), dY.cuda()
    # every output sits between guard regions: nothing may be written outside it
    g = Guarded()
    bf = torch.bfloat16
    Y, H = fhpc.lowrank_linear_fwd(Xd, Ad, Bd, Y=g.alloc((M, N), bf), H_out=g.alloc((M, r), bf))
    assert parity_err(from_device(H), Hr) <= TOL_BF16
    dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H, dX=g.alloc((M, K), bf),
                                         dA=g.alloc((K, r), torch.float32), dB=g.alloc((r, N), torch.float32))
    g.check("bf16 %s" % ((M, K, r, N),))
    _check_all("bf16 %s saved-H" % ((M, K, r, N),), (Y, dX, dA, dB), ref, TOL_BF16)
    Y2 = fhpc.lowrank_linear_fwd(Xd, Ad, Bd)                          # no H_out
    # (against the oracle, not bit for bit against Y: with H not asked for the products may take another route)
    assert parity_err(from_device(Y2), Yr) <= TOL_BF16
    dX2, dA2, dB2 = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd)          # recompute H
    _check_all("bf16 %s recompute" % ((M, K, r, N),), (None, dX2, dA2, dB2), ref, TOL_BF16)


@pytest.mark.parametrize("M,K,r,N", [
    (1, 4096, 512, 4096),    # one token at the pretraining configuration's layer
    (16, 1024, 128, 776),
    (32, 520, 5, 264),       # odd rank, ragged reduction
    (7, 768, 24, 72),
])
def test_bf16_few_tokens_forward(M, K, r, N):
    """At most 32 tokens: both products of the forward run as split reductions on a 32-row tile."""
    fhpc = _fhpc()
    X, A, B, _ = lowrank_inputs(9, M, K, r, N, tensor_base=30)
    Yr, Hr = oracle.lowrank_fwd(X.f64, A.f64, B.f64)
    Y, H = fhpc.lowrank_linear_fwd(X.cuda(), A.cuda(), B.cuda(), save_H=True)
    eY, eH = parity_err(from_device(Y), Yr), parity_err(from_device(H), Hr)
    print("few tokens %s: Y %.3e H %.3e" % ((M, K, r, N), eY, eH), flush=True)
    assert eY <= TOL_BF16 and eH <= TOL_BF16
    Y2 = fhpc.lowrank_linear_fwd(X.cuda(), A.cuda(), B.cuda())
    assert np.array_equal(from_device(Y2), from_device(Y))


def test_bf16_optional_outputs_and_canaries():
    """NULL outputs are skipped; nothing is written outside the output tensors."""
    import torch
    fhpc = _fhpc()
    M, K, r, N = 130, 72, 24, 88
    X, A, B, dY = lowrank_inputs(9, M, K, r, N, tensor_base=20)
    ref = oracle.lowrank_bwd(X.f64, A.f64, B.f64, dY.f64)
    Xd, Ad, Bd, dYd = X.cuda(), A.cuda(), B.cuda(), dY.cuda()
    pad = 1024
    big = torch.full((M * K + 2 * pad,), 7.0, dtype=torch.bfloat16, device="cuda")
    dX = big[pad:pad + M * K].view(M, K)
    out = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, need_dA=False, need_dB=False, dX=dX)
    assert out[1] is None and out[2] is None
    assert parity_err(from_device(dX), ref[0]) <= TOL_BF16
    assert bool((big[:pad] == 7.0).all()) and bool((big[pad + M * K:] == 7.0).all())
    _, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, need_dX=False)
    assert parity_err(from_device(dA), ref[1]) <= TOL_BF16
    assert parity_err(from_device(dB), ref[2]) <= TOL_BF16


def test_config2_full_size_sampled():
    """Config 2 at full size (16384 tokens, d = 4096, r = 512), the launch configuration the
    benchmark times.  Y and dX are checked on sampled rows (rows are independent), dA on
    sampled columns and dB on sampled rows (column j of dA / row j of dB depends only on
    column j of A / row j of B through the rank index, so the oracle evaluates the layer
    restricted to those rank indices)."""
    fhpc = _fhpc()
    M, K, r, N = 16384, 4096, 512, 4096
    for proj in range(4):                     # q, k, v, o: four independent calls
        X, A, B, dY = lowrank_inputs(2, M, K, r, N, tensor_base=10 * proj)
        Xd, Ad, Bd, dYd = X.cuda(), A.cuda(), B.cuda(), dY.cuda()
        Y, H = fhpc.lowrank_linear_fwd(Xd, Ad, Bd, save_H=True)
        dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H)
        rows = sample_rows(M, 100 + proj)
        Yr, _ = oracle.lowrank_fwd(X.rows(rows).f64, A.f64, B.f64)
        dXr, _, _ = oracle.lowrank_bwd(X.rows(rows).f64, A.f64, B.f64, dY.rows(rows).f64)
        J = np.unique(np.random.default_rng(200 + proj).integers(0, r, size=8))
        Af, Bf = A.f64, B.f64
        _, dAr, dBr = oracle.lowrank_bwd(X.f64, Af[:, J], Bf[J, :], dY.f64)
        errs = {
            "Y": parity_err(from_device(Y)[rows], Yr),
            "dX": parity_err(from_device(dX)[rows], dXr),
            "dA": parity_err(from_device(dA)[:, J], dAr),
            "dB": parity_err(from_device(dB)[J, :], dBr),
        }
        print("c2 proj %d: %s" % (proj, {k: "%.3e" % v for k, v in errs.items()}), flush=True)
        for k, v in errs.items():
            assert v <= TOL_BF16, (proj, k, v)


def test_config2_shared_x_full_size_sampled():
    """Config 2 at full size through the calls the benchmark times: q, k and v (g = 3) read one X through
    lowrank_linear_fwd/bwd_shared_x, whose wide products (X A_all 1536 wide, the input gradient over a reduction
    of 1536, dA_all 4096 x 1536) choose their own tiles and splits.  Y_i and the summed dX on sampled token rows,
    dA_all on sampled columns of every layer's block, dB_i on the same rank rows; the o projection goes through
    the single-layer calls (test_config2_full_size_sampled)."""
    fhpc = _fhpc()
    M, K, r, N, g = 16384, 4096, 512, 4096, 3
    X, As, Bs, dYs = None, [], [], []
    for i in range(g):
        Xi, A, B, dY = lowrank_inputs(2, M, K, r, N, tensor_base=40 + 10 * i)
        X = Xi if X is None else X
        As.append(A); Bs.append(B); dYs.append(dY)
    A_all = Bf16(np.concatenate([A.bits for A in As], axis=1)).cuda()
    Xd, Bd, dYd = X.cuda(), [B.cuda() for B in Bs], [dY.cuda() for dY in dYs]
    Ys, H = fhpc.lowrank_linear_fwd_shared_x(Xd, A_all, Bd, save_H=True)
    dX, dA, dBs = fhpc.lowrank_linear_bwd_shared_x(Xd, A_all, Bd, dYd, H_all_saved=H)
    rows = sample_rows(M, 300)
    Xr, Xf = X.rows(rows).f64, X.f64
    dXr = np.zeros((rows.size, K))
    H_got, dA_got = from_device(H), from_device(dA)
    for i in range(g):
        Af, Bf = As[i].f64, Bs[i].f64
        Yr, Hr = oracle.lowrank_fwd(Xr, Af, Bf)
        dx, _, _ = oracle.lowrank_bwd(Xr, Af, Bf, dYs[i].rows(rows).f64)
        dXr += dx
        J = np.unique(np.random.default_rng(310 + i).integers(0, r, size=8))
        _, dAr, dBr = oracle.lowrank_bwd(Xf, Af[:, J], Bf[J, :], dYs[i].f64)
        errs = {
            "Y%d" % i: parity_err(from_device(Ys[i])[rows], Yr, what="Y%d" % i),
            "H%d" % i: parity_err(H_got[rows][:, i * r:(i + 1) * r], Hr, what="H%d" % i),
            "dA%d" % i: parity_err(dA_got[:, i * r + J], dAr, what="dA%d" % i),
            "dB%d" % i: parity_err(from_device(dBs[i])[J, :], dBr, what="dB%d" % i),
        }
        print("c2 shared-x layer %d: %s" % (i, {k: "%.3e" % v for k, v in errs.items()}), flush=True)
        for k, v in errs.items():
            assert v <= TOL_BF16, (k, v)
    e = parity_err(from_device(dX)[rows], dXr, what="dX")
    print("c2 shared-x dX (sum of the three input gradients) %.3e" % e, flush=True)
    assert e <= TOL_BF16


@pytest.mark.parametrize("M", [1, 40, 300])
def test_bf16_rank_one_and_three(M):
    """Degenerate ranks: the pair is a single outer product (r = 1), and r = 3."""
    fhpc = _fhpc()
    for r in (1, 3):
        K, N = 264, 136
        X, A, B, dY = lowrank_inputs(9, M, K, r, N, tensor_base=50 + r)
        Yr, Hr = oracle.lowrank_fwd(X.f64, A.f64, B.f64)
        ref = (Yr,) + oracle.lowrank_bwd(X.f64, A.f64, B.f64, dY.f64)
        Xd, Ad, Bd, dYd = X.cuda(), A.cuda(), B.cuda(), dY.cuda()
        Y, H = fhpc.lowrank_linear_fwd(Xd, Ad, Bd, save_H=True)
        assert tuple(H.shape) == (M, r) and parity_err(from_device(H), Hr) <= TOL_BF16
        dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H)
        _check_all("rank %d M=%d" % (r, M), (Y, dX, dA, dB), ref, TOL_BF16)


def test_results_are_bit_reproducible_from_run_to_run():
    """The header promises it: reductions over tokens go to slabs that are added in a fixed order (no
    atomics), so two runs of the same call give the same bits, whatever ran in between."""
    import torch
    fhpc = _fhpc()
    M, K, r, N = 2100, 520, 24, 392
    X, A, B, dY = lowrank_inputs(9, M, K, r, N, tensor_base=70)
    Xd, Ad, Bd, dYd = X.cuda(), A.cuda(), B.cuda(), dY.cuda()

    def run():
        Y, H = fhpc.lowrank_linear_fwd(Xd, Ad, Bd, save_H=True)
        dX, dA, dB = fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H)
        torch.cuda.synchronize()
        return [t.clone() for t in (Y, H, dX, dA, dB)]

    first = run()
    fhpc.lowrank_linear_fwd(Xd[:77], Ad, Bd)                     # other work on the same workspace
    filler = torch.randn(1 << 22, device="cuda").sum().item()     # and on the device
    for _ in range(3):
        for a, b in zip(first, run()):
            assert torch.equal(a, b)
    assert np.isfinite(filler)


def _shared_inputs(M, K, r, N, g, base):
    """g factor pairs on one X: (X, [A_i], [B_i], [dY_i]) with the usual distributions."""
    X = None
    As, Bs, dYs = [], [], []
    for i in range(g):
        Xi, A, B, dY = lowrank_inputs(9, M, K, r, N, tensor_base=base + 4 * i)
        X = Xi if X is None else X
        As.append(A); Bs.append(B); dYs.append(dY)
    return X, As, Bs, dYs


@pytest.mark.parametrize("M,K,r,N,g", [
    (300, 320, 64, 264, 3),      # q/k/v, rank above the split threshold, ragged everywhere
    (515, 1024, 16, 520, 2),     # gate/up at a LoRA-sized rank: every narrow product splits its reduction
    (257, 136, 8, 200, 3),       # g r = 24
    (640, 512, 24, 1032, 3),     # r <= 32 < g r: dH_i split, X A_all whole
    (1100, 768, 128, 776, 2),
    (1, 64, 8, 72, 2),           # a single token
    (130, 264, 40, 136, 1),      # g = 1 is the plain layer
    (64, 264, 64, 1032, 1),      # g = 1, r > 32, N > K: dH = dY B^T of the one (dense) block splits its reduction
    (96, 128, 8, 64, 8),         # the most layers one call takes
])
def test_shared_x_factorised_layers(M, K, r, N, g):
    """lowrank_linear_fwd/bwd_shared_x against g runs of the oracle: dX is the sum of the layers' input
    gradients, dA_all and H_all hold the layers' blocks side by side."""
    import torch
    fhpc = _fhpc()
    X, As, Bs, dYs = _shared_inputs(M, K, r, N, g, base=60)
    Yr, Hr, dXr, dAr, dBr = [], [], np.zeros((M, K)), [], []
    for A, B, dY in zip(As, Bs, dYs):
        y, h = oracle.lowrank_fwd(X.f64, A.f64, B.f64)
        dx, da, db = oracle.lowrank_bwd(X.f64, A.f64, B.f64, dY.f64)
        Yr.append(y); Hr.append(h); dXr += dx; dAr.append(da); dBr.append(db)
    Hr, dAr = np.concatenate(Hr, axis=1), np.concatenate(dAr, axis=1)
    A_all = Bf16(np.concatenate([A.bits for A in As], axis=1)).cuda()
    Xd, Bd, dYd = X.cuda(), [B.cuda() for B in Bs], [dY.cuda() for dY in dYs]
    tag = "shared-x %s" % ((M, K, r, N, g),)

    def check(name, got, ref):
        err = parity_err(from_device(got), ref)
        print("%s %s rel_fro=%.3e" % (tag, name, err), flush=True)
        assert err <= TOL_BF16, (tag, name, err)

    Ys, H = fhpc.lowrank_linear_fwd_shared_x(Xd, A_all, Bd, save_H=True)
    check("H_all", H, Hr)
    for i in range(g):
        check("Y%d" % i, Ys[i], Yr[i])
    Ys2 = fhpc.lowrank_linear_fwd_shared_x(Xd, A_all, Bd)                 # H kept in the workspace
    for i in range(g):
        check("Y%d (no H_out)" % i, Ys2[i], Yr[i])
    dX, dA, dBs = fhpc.lowrank_linear_bwd_shared_x(Xd, A_all, Bd, dYd, H_all_saved=H)
    check("dX", dX, dXr); check("dA_all", dA, dAr)
    for i in range(g):
        check("dB%d" % i, dBs[i], dBr[i])
    # recomputed H; one dB left out; then weight gradients only, then the input gradient only
    flags = [i != 0 for i in range(g)]
    dX2, dA2, dBs2 = fhpc.lowrank_linear_bwd_shared_x(Xd, A_all, Bd, dYd, need_dB=flags)
    check("dX (recompute)", dX2, dXr); check("dA_all (recompute)", dA2, dAr)
    assert dBs2[0] is None
    for i in range(1, g):
        check("dB%d (recompute)" % i, dBs2[i], dBr[i])
    dX3, dA3, dBs3 = fhpc.lowrank_linear_bwd_shared_x(Xd, A_all, Bd, dYd, H_all_saved=H, need_dX=False)
    assert dX3 is None
    check("dA_all (no dX)", dA3, dAr)
    dX4, dA4, dBs4 = fhpc.lowrank_linear_bwd_shared_x(Xd, A_all, Bd, dYd, need_dA=False, need_dB=False)
    assert dA4 is None and all(b is None for b in dBs4)
    check("dX (alone)", dX4, dXr)
    torch.cuda.synchronize()


def test_shared_x_matches_the_single_layer_calls():
    """The layers' outputs and weight gradients of the shared call against those of the single-layer entry
    point on the same operands, GPU against GPU.  The wide products of the shared call may run on another
    tile shape or another split of the reduction than the narrow ones, which sums in another order, so a
    few per cent of the bf16 values differ by one ulp: the bound is a fraction of the bf16 tolerance."""
    import torch
    fhpc = _fhpc()
    M, K, r, N, g = 520, 512, 64, 264, 3
    X, As, Bs, dYs = _shared_inputs(M, K, r, N, g, base=90)
    A_all = Bf16(np.concatenate([A.bits for A in As], axis=1)).cuda()
    Xd, Bd, dYd = X.cuda(), [B.cuda() for B in Bs], [dY.cuda() for dY in dYs]
    Ys, H = fhpc.lowrank_linear_fwd_shared_x(Xd, A_all, Bd, save_H=True)
    dX, dA, dBs = fhpc.lowrank_linear_bwd_shared_x(Xd, A_all, Bd, dYd, H_all_saved=H)
    dX_sum = np.zeros((M, K))
    for i in range(g):
        Ad = As[i].cuda()
        Y1, H1 = fhpc.lowrank_linear_fwd(Xd, Ad, Bd[i], save_H=True)
        dX1, dA1, dB1 = fhpc.lowrank_linear_bwd(Xd, Ad, Bd[i], dYd[i], H_saved=H1)
        assert oracle.rel_fro(from_device(H[:, i * r:(i + 1) * r].contiguous()), from_device(H1)) <= 2e-3
        assert oracle.rel_fro(from_device(Ys[i]), from_device(Y1)) <= 2e-3
        assert oracle.rel_fro(from_device(dBs[i]), from_device(dB1)) <= 2e-3
        assert oracle.rel_fro(from_device(dA[:, i * r:(i + 1) * r].contiguous()), from_device(dA1)) <= 2e-3
        dX_sum += from_device(dX1)
    assert parity_err(from_device(dX), dX_sum) <= TOL_BF16
    torch.cuda.synchronize()
