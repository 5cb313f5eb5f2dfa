"""Pins for the oracle's per-vector quantiser, nibble packing and dequantisation
(reading of Sec. 5.2 "Quantization").  Nothing here calls the HIP library."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quant_worked.txt")


def test_f16_decode_all_patterns_vs_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.f16_bits_to_f64(bits)
    ref = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    m = ~np.isnan(ref)
    assert np.array_equal(got[m], ref[m])
    assert np.array_equal(np.signbit(got[m]), np.signbit(ref[m]))


def test_f16_encode_vs_numpy_including_ties_and_subnormals():
    rng = np.random.default_rng(7)
    vals = [0.0, -0.0, 1.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, np.inf, -np.inf,
            2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -26, 2.0 ** -14, 2.0 ** -14 * 0.999,
            1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -20,  # ties / just above
            1.0 / 127.0, 1.0 / 7.0, 0.02 * 4 / 127]
    x = np.concatenate([np.array(vals, dtype=np.float32),
                        rng.standard_normal(4000).astype(np.float32) * 1e-3,
                        (rng.standard_normal(4000) * 10.0 ** rng.uniform(-9, 5, 4000)).astype(np.float32)])
    # every tie between adjacent halves in a binade and in the subnormal range
    h = np.arange(0x0001, 0x0420, dtype=np.uint16).view(np.float16).astype(np.float64)
    ties = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    x = np.concatenate([x, ties, -ties])
    got = oracle.f32_to_f16_bits(x)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, ref)


def test_printed_scale_values():
    assert int(oracle.f32_to_f16_bits(np.float32(1.0) / np.float32(127.0))) == 0x2008
    assert int(oracle.f32_to_f16_bits(np.float32(1.0) / np.float32(7.0))) == 0x3092
    assert float(oracle.f16_bits_to_f64(np.uint16(0x2008))) == 0.00787353515625
    assert float(oracle.f16_bits_to_f64(np.uint16(0x3092))) == 0.142822265625


def test_worked_example_golden():
    w = np.array([1.0, 0.5, 0.25, -1.0, 0.3], dtype=np.float32)
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    for scheme, hexs, *codes in rows:
        codes = np.array([int(c) for c in codes], dtype=np.int8)
        if scheme == "8":
            W = np.zeros((5, 3), dtype=np.float32); W[:, 1] = w     # channel 1 of 3
            q, s = oracle.quantize_int8_perchannel(W)
            assert s[1] == int(hexs, 16) and np.array_equal(q[1], codes)
            assert s[0] == 0 and not q[0].any() and not q[2].any()  # all-zero channels
        else:
            W = np.zeros((64, 2), dtype=np.float32); W[:5, 1] = w
            p, s = oracle.quantize_int4_block(W, 64)
            q = oracle.unpack_int4(p)
            assert s[1, 0] == int(hexs, 16) and np.array_equal(q[1, :5], codes)
            assert not q[1, 5:].any() and not q[0].any() and s[0, 0] == 0


def test_exact_power_of_two_cases_roundtrip_bit_exact():
    rng = np.random.default_rng(3)
    K, N = 96, 5
    c = rng.integers(-127, 128, size=(K, N)); c[0, :] = 127; c[1, :] = -127
    W = (c * 2.0 ** -10).astype(np.float32)
    q, s = oracle.quantize_int8_perchannel(W)
    assert np.all(s == np.float16(2.0 ** -10).view(np.uint16))
    assert np.array_equal(q, c.T.astype(np.int8))
    assert np.array_equal(oracle.dequant(q, s, 8), W.astype(np.float64))
    K, N = 128, 4
    c = rng.integers(-7, 8, size=(K, N)); c[0, :] = 7; c[64, :] = -7
    W = (c * 2.0 ** -6).astype(np.float32)
    W[64:, :] *= 4.0                                   # second block: scale 2^-4
    p, s = oracle.quantize_int4_block(W, 64)
    assert np.all(s[:, 0] == np.float16(2.0 ** -6).view(np.uint16))
    assert np.all(s[:, 1] == np.float16(2.0 ** -4).view(np.uint16))
    assert np.array_equal(oracle.unpack_int4(p), c.T.astype(np.int8))
    assert np.array_equal(oracle.dequant(p, s, 4, 64), W.astype(np.float64))


def test_ties_round_half_to_even_and_clamp():
    sf = 2.0 ** -5
    w = np.array([127 * sf, 0.5 * sf, 1.5 * sf, 2.5 * sf, -0.5 * sf, -1.5 * sf, -2.5 * sf, 3.5 * sf],
                 dtype=np.float32)
    q, s = oracle.quantize_int8_perchannel(w.reshape(-1, 1))
    assert float(oracle.f16_bits_to_f64(s[0])) == sf
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 4]
    # clamp: the fp16-rounded scale can be slightly below absmax/qmax, so the
    # extreme element may round above qmax before clamping
    w = np.array([1.0, -1.0, 0.999], dtype=np.float32)          # 1/0.00787353 = 127.0077
    q, _ = oracle.quantize_int8_perchannel(w.reshape(-1, 1))
    assert q[0].tolist() == [127, -127, 127]


def test_nibble_table_exhaustive_bruteforce():
    allb = np.arange(256, dtype=np.uint8)
    q = oracle.unpack_int4(allb.reshape(256, 1))
    for b in range(256):
        lo, hi = b & 15, b >> 4
        lo = lo - 16 if lo > 7 else lo
        hi = hi - 16 if hi > 7 else hi
        assert q[b, 0] == lo and q[b, 1] == hi
    pairs = np.array([[a, b] for a in range(-8, 8) for b in range(-8, 8)], dtype=np.int8)
    assert np.array_equal(oracle.unpack_int4(oracle.pack_int4(pairs)), pairs)
    # layout: element 0 is the LOW nibble
    assert int(oracle.pack_int4(np.array([[1, -2]], dtype=np.int8))[0, 0]) == 0xE1


@pytest.mark.parametrize("scheme", [8, 4])
def test_quantiser_invariants_random(scheme):
    rng = np.random.default_rng(11)
    K, N = 256, 24
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    W[:, 3] = 0.0
    if scheme == 8:
        q, s = oracle.quantize_int8_perchannel(W); qmax = 127
        sf = oracle.f16_bits_to_f64(s)[:, None] * np.ones((1, K))
    else:
        p, s = oracle.quantize_int4_block(W, 64); qmax = 7
        q = oracle.unpack_int4(p)
        sf = np.repeat(oracle.f16_bits_to_f64(s), 64, axis=1)
    Wd = oracle.dequant(q if scheme == 8 else p, s, scheme, 64)
    assert np.array_equal(Wd, (q.astype(np.float64) * sf).T)       # layout [N][K] -> Wd[K,N]
    assert np.abs(q).max() <= qmax and not q[3].any()
    err = np.abs(W.astype(np.float64).T - q * sf)
    unclamped = np.abs(q) < qmax
    assert np.all(err[unclamped] <= sf[unclamped] * 0.5 * (1 + 1e-6))
    # the absmax element of every non-zero vector maps to +-qmax
    vec = np.abs(q).reshape(N, -1, K if scheme == 8 else 64).max(axis=2)
    nz = np.ones_like(vec, dtype=bool); nz[3] = False
    assert np.all(vec[nz] == qmax)
    # re-quantising the dequantised weight reproduces the codes
    if scheme == 8:
        q2, s2 = oracle.quantize_int8_perchannel(Wd.astype(np.float32))
    else:
        p2, s2 = oracle.quantize_int4_block(Wd.astype(np.float32), 64)
        q2 = oracle.unpack_int4(p2)
    assert np.array_equal(q2, q) and np.array_equal(s2, s)


def test_scale_underflow_gives_zero_codes():
    W = np.full((64, 1), 1e-9, dtype=np.float32)      # absmax/127 underflows fp16 to 0
    q, s = oracle.quantize_int8_perchannel(W)
    assert s[0] == 0 and not q.any()
