"""Host bookkeeping pinned to the numbers the paper prints (Sec. 3.2, Sec. 4.1)."""
import os

from paper_2402_13533_amd import shapes

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "param_counts.txt")


def test_printed_parameter_counts():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for name, d_in, d_out, r, copies, dense, low, unit in rows:
        d_in, d_out, r, copies = int(d_in), int(d_out), int(r), int(copies)
        div = 1e9 if unit == "B" else 1e6
        if name == "emb_head":
            # two 32000 x 4096 matrices, each factorised through r
            got_dense = copies * shapes.dense_params(d_in, d_out)
            got_low = (d_in + d_out) * r
        else:
            got_dense = copies * shapes.dense_params(d_in, d_out)
            got_low = copies * shapes.lowrank_params(d_in, r, d_out)
        assert round(got_dense / div, 2) == float(dense), name
        assert round(got_low / div, 2) == float(low), name


def test_mults_and_compression_closed_forms():
    n, r = 4096, 512
    assert shapes.lowrank_mults_per_token(n, r, n) == 2 * n * r      # n^2 -> 2 n r
    assert shapes.compression_ratio(n, r, n) == n / (2 * r)         # Sec. 4.1
    # fwd flop = 2 * M * r * (K + N); fwd+bwd = 6 GEMMs
    assert shapes.lowrank_flops(16384, 4096, 512, 4096) == 6 * 2 * 16384 * 512 * 4096
    assert shapes.lowrank_flops(16384, 4096, 512, 4096, bwd=False) == 2 * 2 * 16384 * 512 * 4096
    assert shapes.qlinear_lowrank_flops(4096, 4096, 8, 4096) == \
        4 * 4096 ** 3 + 6 * 4096 * 8 * 8192
