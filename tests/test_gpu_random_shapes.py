"""Seeded random shapes through every layer entry point, each output against the oracle: token counts on
both sides of every routing threshold (16, 32, 64, 1152), reductions and widths that are not tile
multiples, ranks from 1 to beyond a tile, saved and recomputed H, all weight storages, blend factors at
the end points and inside."""
import numpy as np
import pytest

import oracle
from harness import Guarded, TOL_BF16, Bf16, f16_bits_cuda, from_device, parity_err

pytestmark = pytest.mark.gpu

TOKENS = [1, 2, 7, 16, 17, 33, 64, 65, 100, 255, 256, 300, 777, 1024, 1151, 1152, 2048, 2500]
RANKS = [1, 2, 5, 8, 16, 24, 40, 64, 72, 100, 136]
KINDS = ["lowrank", "q8", "q4", "blend8", "blend4", "dense"]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_shapes(seed):
    import torch
    import paper_2402_13533_amd as fhpc
    from paper_2402_13533_amd import synth
    rng = np.random.default_rng(9000 + seed)
    pick = lambda a: a[rng.integers(len(a))]
    for it in range(20):
        M, r, kind = int(pick(TOKENS)), int(pick(RANKS)), pick(KINDS)
        K = int(rng.integers(1, 24)) * 64
        N = int(rng.integers(1, 180)) * 8
        base = 100000 * (seed + 1) + 10 * it
        X, dY = Bf16.normal(base, (M, K), 1.0), Bf16.normal(base + 1, (M, N), 1.0)
        A = Bf16.normal(base + 2, (K, r), K ** -0.5)
        B = Bf16.normal(base + 3, (r, N), r ** -0.5 if kind == "lowrank" else 0.05)
        Xd, Ad, Bd, dYd = X.cuda(), A.cuda(), B.cuda(), dY.cuda()
        saved = bool(rng.random() < 0.5)
        tag = "%s M=%d K=%d r=%d N=%d saved_H=%s" % (kind, M, K, r, N, saved)
        # outputs between guard regions: whatever route a shape takes, nothing may be written outside them
        guard = Guarded()
        bf = torch.bfloat16
        fo = dict(Y=guard.alloc((M, N), bf), H_out=guard.alloc((M, r), bf))
        bo = dict(dX=guard.alloc((M, K), bf), dA=guard.alloc((K, r), torch.float32), dB=guard.alloc((r, N), torch.float32))
        if kind == "lowrank":
            Y, H = fhpc.lowrank_linear_fwd(Xd, Ad, Bd, **fo)
            got = (Y,) + tuple(fhpc.lowrank_linear_bwd(Xd, Ad, Bd, dYd, H_saved=H if saved else None, **bo))
            ref = (oracle.lowrank_fwd(X.f64, A.f64, B.f64)[0],) + oracle.lowrank_bwd(X.f64, A.f64, B.f64, dY.f64)
        else:
            if kind == "dense":
                W = Bf16.normal(base + 4, (K, N), K ** -0.5)
                Wd, W_dev, sc_dev, scheme = W.f64, W.cuda(), None, fhpc.FHPC_W_BF16
            else:
                scheme = 8 if kind.endswith("8") else 4
                Wf = synth.normal(base + 4, (K, N), 0.03)
                Wq, sc = oracle.quantize_int8_perchannel(Wf) if scheme == 8 else oracle.quantize_int4_block(Wf, 64)
                Wd, W_dev, sc_dev = oracle.dequant(Wq, sc, scheme, 64), torch.from_numpy(Wq).cuda(), f16_bits_cuda(sc)
            if kind in ("q8", "q4"):
                Y, H = fhpc.qlinear_lowrank_fwd(Xd, W_dev, sc_dev, scheme, Ad, Bd, 2.0, **fo)
                got = (Y,) + tuple(fhpc.qlinear_lowrank_bwd(Xd, W_dev, sc_dev, scheme, Ad, Bd, 2.0, dYd, H_saved=H if saved else None, **bo))
                ref = (oracle.qlinear_lowrank_fwd(X.f64, Wd, A.f64, B.f64, 2.0)[0],) + oracle.qlinear_lowrank_bwd(X.f64, Wd, A.f64, B.f64, 2.0, dY.f64)
            else:
                alpha = float(pick([0.0, 0.3, 0.9, 1.0]))
                tag += " alpha=%.1f" % alpha
                Y, H = fhpc.qlinear_blend_fwd(Xd, W_dev, sc_dev, scheme, Ad, Bd, alpha, **fo)
                got = (Y,) + tuple(fhpc.qlinear_blend_bwd(Xd, W_dev, sc_dev, scheme, Ad, Bd, alpha, dYd, H_saved=H if saved else None, **bo))
                ref = (oracle.blend_fwd(X.f64, Wd, A.f64, B.f64, alpha)[0],) + oracle.blend_bwd(X.f64, Wd, A.f64, B.f64, alpha, dY.f64)
        guard.check(tag)
        for name, g, rf in zip(("Y", "dX", "dA", "dB"), got, ref):
            if np.linalg.norm(rf) > 0:
                e = parity_err(from_device(g), rf)
                assert e <= TOL_BF16, (tag, name, e)
            else:
                assert not from_device(g).any(), (tag, name)          # alpha = 1: no gradient reaches the pair


@pytest.mark.parametrize("seed", [0, 1])
def test_random_shapes_shared_x(seed):
    """Seeded random shapes through lowrank_linear_fwd/bwd_shared_x (g layers on one X): every output
    against g runs of the oracle, the input gradient against their sum."""
    import paper_2402_13533_amd as fhpc
    rng = np.random.default_rng(9500 + seed)
    pick = lambda a: a[rng.integers(len(a))]
    for it in range(12):
        M = int(pick(TOKENS))
        r = int(pick([8, 16, 24, 32, 40, 64, 136]))
        g = int(pick([1, 2, 3, 4, 8]))
        K = int(rng.integers(1, 24)) * 64
        N = int(rng.integers(1, 120)) * 8
        base = 500000 * (seed + 1) + 40 * it
        saved = bool(rng.random() < 0.5)
        tag = "shared-x M=%d K=%d r=%d N=%d g=%d saved_H=%s" % (M, K, r, N, g, saved)
        X = Bf16.normal(base, (M, K), 1.0)
        As = [Bf16.normal(base + 1 + 3 * i, (K, r), K ** -0.5) for i in range(g)]
        Bs = [Bf16.normal(base + 2 + 3 * i, (r, N), r ** -0.5) for i in range(g)]
        dYs = [Bf16.normal(base + 3 + 3 * i, (M, N), 1.0) for i in range(g)]
        Xd = X.cuda()
        A_all = Bf16(np.concatenate([A.bits for A in As], axis=1)).cuda()
        Bd, dYd = [B.cuda() for B in Bs], [dY.cuda() for dY in dYs]
        Ys, H = fhpc.lowrank_linear_fwd_shared_x(Xd, A_all, Bd, save_H=True)
        dX, dA, dBs = fhpc.lowrank_linear_bwd_shared_x(Xd, A_all, Bd, dYd, H_all_saved=H if saved else None)
        dA = from_device(dA)
        dX_ref = np.zeros((M, K))
        for i in range(g):
            y = oracle.lowrank_fwd(X.f64, As[i].f64, Bs[i].f64)[0]
            dx, da, db = oracle.lowrank_bwd(X.f64, As[i].f64, Bs[i].f64, dYs[i].f64)
            dX_ref += dx
            for name, got, rf in (("Y", from_device(Ys[i]), y), ("dA", dA[:, i * r:(i + 1) * r], da), ("dB", from_device(dBs[i]), db)):
                e = parity_err(got, rf)
                assert e <= TOL_BF16, (tag, name, i, e)
        e = parity_err(from_device(dX), dX_ref)
        assert e <= TOL_BF16, (tag, "dX", e)
