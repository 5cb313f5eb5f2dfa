"""The seeded input generator: determinism, distribution, bf16 storage format."""
import numpy as np

from paper_2402_13533_amd import synth


def test_deterministic_and_seed_dependent():
    a = synth.normal(5, (33, 7))
    assert np.array_equal(a, synth.normal(5, (33, 7)))
    assert not np.array_equal(a, synth.normal(6, (33, 7)))
    # chunking does not change the stream: a prefix of a longer draw is identical
    assert np.array_equal(synth.normal(5, (10,)), synth.normal(5, (231,))[:10])
    assert synth.normal(5, (3,)).dtype == np.float32


def test_moments():
    x = synth.normal(synth.tensor_seed(2, 0), (1 << 20,), std=0.5).astype(np.float64)
    assert abs(x.mean()) < 3e-3 and abs(x.std() - 0.5) < 3e-3
    assert abs(((x / 0.5) ** 4).mean() - 3.0) < 0.05
    assert abs(np.corrcoef(x[:-1], x[1:])[0, 1]) < 5e-3


def test_bf16_rne_and_roundtrip():
    allb = np.arange(65536, dtype=np.uint16)
    f = synth.bf16_bits_to_f32(allb)
    finite = np.isfinite(f)
    assert np.array_equal(synth.f32_to_bf16_bits(f[finite]), allb[finite])
    one = np.float32(1.0)
    ulp = np.float32(2.0 ** -7)
    cases = np.array([one + ulp / 2, one + 3 * ulp / 2, one + ulp / 2 + np.float32(2.0 ** -20),
                      one + ulp / 4], dtype=np.float32)
    got = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(cases))
    assert got.tolist() == [1.0, float(one + 2 * ulp), float(one + ulp), 1.0]   # ties to even
