"""Host-only checks of the workspace layout: over a grid of shapes, no launch of any entry point's sequence
plans more partial-sum bytes than the layout reserves for them.  (The calls refuse such a launch at run
time; this shows on the CPU that the refusal never triggers for a workspace of fhpc_workspace_bytes.)"""
import itertools

import pytest

import paper_2402_13533_amd as fhpc

Ms = [1, 16, 33, 64, 65, 130, 256, 300, 515, 1024, 1100, 1152, 2048, 4000, 4096, 16384]
KNs = [64, 136, 256, 264, 520, 1024, 1216, 2048, 4096, 5120, 11008, 13824]
RANKS = [1, 5, 8, 16, 24, 32, 40, 64, 128, 512, 1024]


def _assert_fits(call, tag, **kw):
    rc, planned, reserved = fhpc.plan_slab_bytes(call, **kw)
    assert rc == 0, (tag, kw, rc)
    assert planned <= reserved, (tag, kw, planned, reserved)
    return planned


def test_factorised_layer_slabs_fit():
    n = 0
    for M, K, N, r in itertools.product(Ms, KNs, KNs, RANKS):
        if (M + K + N + r) % 3:            # a third of the grid, spread evenly
            continue
        for outputs in (7, 1, 6, 15, 2 | 8, 4):
            _assert_fits(fhpc.FHPC_OP_LOWRANK_BWD, "lowrank_bwd", M=M, K=K, r=r, N=N, outputs=outputs)
        for outputs in (0, 1):
            _assert_fits(fhpc.FHPC_OP_LOWRANK_FWD, "lowrank_fwd", M=M, K=K, r=r, N=N, outputs=outputs)
        n += 1
    assert n > 3000


def test_shared_x_slabs_fit():
    """Includes g = 1 with r > 32 and N > K, where dH = dY B^T of the single (dense) block may take the split
    route: the shape class a fixed workspace bug lived in."""
    worst = 0
    for M, K, N, r, g in itertools.product(Ms, KNs, KNs, [8, 16, 32, 40, 64, 128, 512, 1024], [1, 2, 3, 8]):
        if (M + K + N + r + g) % 3:
            continue
        for outputs in (7, 1, 6, 15, 2 | 8, 4):
            worst = max(worst, _assert_fits(fhpc.FHPC_PLAN_SHARED_BWD, "shared_bwd", M=M, K=K, r=r, N=N, g=g, outputs=outputs))
        for outputs in (0, 1):
            _assert_fits(fhpc.FHPC_PLAN_SHARED_FWD, "shared_fwd", M=M, K=K, r=r, N=N, g=g, outputs=outputs)
    assert worst > 0
    # the two shapes the finding was reported on
    for M, K, r, N in ((64, 1024, 64, 4096), (33, 64, 40, 256)):
        rc, planned, reserved = fhpc.plan_slab_bytes(fhpc.FHPC_PLAN_SHARED_BWD, M, K, r, N, g=1)
        assert rc == 0 and 0 < planned <= reserved, (M, K, r, N, planned, reserved)


def test_ffn_gate_calls_slabs_fit():
    """lowrank_ffn_gate_up_fwd and lowrank_ffn_down_bwd: the gate in the epilogue of the large tiles, the streaming
    gate kernel elsewhere, the same workspace layouts as the calls they stand for."""
    n = 0
    for M, K, N, r in itertools.product(Ms, KNs, KNs, [8, 16, 32, 40, 64, 128, 512, 1024]):
        if (M + K + N + r) % 3:
            continue
        for outputs in (0, 1):
            _assert_fits(fhpc.FHPC_PLAN_FFN_GATE_UP, "ffn_gate_up", M=M, K=K, r=r, N=N, outputs=outputs)
        for outputs in (6, 6 | 8, 2, 4 | 8, 0):
            _assert_fits(fhpc.FHPC_PLAN_FFN_DOWN_BWD, "ffn_down_bwd", M=M, K=K, r=r, N=N, outputs=outputs)
        n += 1
    assert n > 2000


@pytest.mark.parametrize("qscheme", [fhpc.FHPC_Q_INT4_BLOCK, fhpc.FHPC_Q_INT8_PER_CHANNEL, fhpc.FHPC_W_BF16, fhpc.FHPC_W_MERGED])
def test_quantised_layer_slabs_fit(qscheme):
    for M, K, N, r in itertools.product(Ms, [64, 256, 1024, 4096, 5120, 13824], [64, 264, 1024, 4096, 5120, 13824],
                                        [1, 8, 16, 24, 40, 64, 128]):
        for base_scale in (1.0, 0.0, 0.25):
            if qscheme == fhpc.FHPC_W_MERGED and base_scale != 1.0:
                continue
            for outputs in (7, 1, 6, 15, 2 | 8, 4):
                _assert_fits(fhpc.FHPC_OP_QLINEAR_BWD, "qlinear_bwd", M=M, K=K, r=r, N=N, qscheme=qscheme,
                             outputs=outputs, base_scale=base_scale)
            for outputs in (0, 1):
                _assert_fits(fhpc.FHPC_OP_QLINEAR_FWD, "qlinear_fwd", M=M, K=K, r=r, N=N, qscheme=qscheme,
                             outputs=outputs, base_scale=base_scale)


def test_decompose_slabs_fit():
    """r close to K with N a little larger: the Gram product over K needs more slices than the one over N."""
    dims = [64, 256, 512, 1024, 1088, 1216, 2048, 4096, 4160, 8192]
    seen = 0
    for K, N in itertools.product(dims, dims):
        for r in (8, 64, 256, 512, 1024, 2048):
            if r > min(K, N):
                continue
            seen = max(seen, _assert_fits(fhpc.FHPC_OP_DECOMPOSE, "decompose", M=1, K=K, r=r, N=N))
    assert seen > 0
    rc, planned, reserved = fhpc.plan_slab_bytes(fhpc.FHPC_OP_DECOMPOSE, 1, 1024, 1024, 1216)
    assert rc == 0 and 0 < planned <= reserved
