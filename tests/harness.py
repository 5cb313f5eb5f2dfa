"""Shared plumbing of the GPU parity tests: seeded inputs as raw bits, their exact
fp64 decode for the oracle, and their device tensors for the HIP library.  Holds no
arithmetic of the layer."""
from __future__ import annotations

import numpy as np

from paper_2402_13533_amd import synth

TOL_BF16 = 5e-3     # relative Frobenius error, bf16 inputs with fp32 accumulation
TOL_F32 = 1e-5      # fp32 config


class Bf16:
    """A bf16 tensor held as uint16 bit patterns."""

    def __init__(self, bits: np.ndarray):
        self.bits = np.ascontiguousarray(bits, dtype=np.uint16)

    @classmethod
    def normal(cls, seed, shape, std=1.0):
        return cls(synth.normal_bf16(seed, shape, std))

    @property
    def f64(self) -> np.ndarray:
        return synth.bf16_bits_to_f32(self.bits).astype(np.float64)

    def rows(self, idx):
        return Bf16(self.bits[idx])

    def cuda(self):
        import torch
        return torch.from_numpy(self.bits.view(np.int16)).cuda().view(torch.bfloat16)


def from_device(t) -> np.ndarray:
    """Device tensor (bf16 / fp32 / integer) -> float64 (exact) or integer numpy array."""
    import torch
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).numpy().view(np.uint16)
        return synth.bf16_bits_to_f32(bits).astype(np.float64)
    if t.dtype in (torch.float32, torch.float16):
        return t.numpy().astype(np.float64)
    return t.numpy()


def parity_err(got, ref, tol=TOL_BF16, what=""):
    """Relative Frobenius error of a result against the oracle's, in fp64; also asserts, element by element,
    |got - ref| <= 2^-7 |ref| + 10 tol rms(ref): the norm alone would let a single garbage element of a large
    output through (typical element errors are a fifth of tol rms(ref), so this is some twenty deviations out),
    and that nothing is NaN or infinite."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), (what, "non-finite values")
    diff = np.abs(got - ref)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm(diff.ravel())
    rms = den / np.sqrt(max(ref.size, 1))
    over = diff - (2.0 ** -7 * np.abs(ref) + 10.0 * tol * rms)
    if over.size and over.max() > 0:
        i = np.unravel_index(int(np.argmax(over)), over.shape)
        raise AssertionError("%s: element %s off by %.3e (got %.6g, ref %.6g, bound %.3e; %d elements beyond their bound)"
                             % (what, i, diff[i], got[i], ref[i], diff[i] - over[i], int((over > 0).sum())))
    return float(num / den) if den > 0 else float(num)


def f16_bits_cuda(bits: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16)).cuda()


def sample_rows(M: int, seed: int, per_block: int = 64) -> np.ndarray:
    """Rows 0 and M-1 plus one pseudo-random row in every block of `per_block` rows."""
    rng = np.random.default_rng(seed)
    starts = np.arange(0, M, per_block)
    picks = starts + rng.integers(0, per_block, size=starts.size)
    picks = np.minimum(picks, M - 1)
    return np.unique(np.concatenate([[0, M - 1], picks]))


def lowrank_inputs(config: int, M, K, r, N, bf16=True, tensor_base=0):
    """X ~ N(0,1), A ~ N(0, var 1/K), B ~ N(0, var 1/r), dY ~ N(0,1)."""
    s = lambda i: synth.tensor_seed(config, tensor_base + i)
    gen = (lambda seed, shape, std: Bf16.normal(seed, shape, std)) if bf16 else \
        (lambda seed, shape, std: synth.normal(seed, shape, std))
    X = gen(s(0), (M, K), 1.0)
    A = gen(s(1), (K, r), K ** -0.5)
    B = gen(s(2), (r, N), r ** -0.5)
    dY = gen(s(3), (M, N), 1.0)
    return X, A, B, dY


def qlinear_inputs(config: int, M, K, r, N, tensor_base=0):
    """W ~ N(0, std 0.02) fp32; X, dY ~ N(0,1); A ~ N(0, var 1/K); B ~ N(0, std 0.01)."""
    s = lambda i: synth.tensor_seed(config, tensor_base + i)
    W = synth.normal(s(4), (K, N), 0.02)
    X = Bf16.normal(s(0), (M, K), 1.0)
    A = Bf16.normal(s(1), (K, r), K ** -0.5)
    B = Bf16.normal(s(2), (r, N), 0.01)
    dY = Bf16.normal(s(3), (M, N), 1.0)
    return W, X, A, B, dY


class Guarded:
    """Output tensors carved out of device buffers that carry 4 KiB of a fill pattern before and after the tensor:
    check() asserts that a call wrote nothing outside the outputs it was given."""
    PAD, FILL = 4096, 0xA5

    def __init__(self):
        self.items = []

    def alloc(self, shape, dtype):
        import torch
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        body = (n + 255) // 256 * 256
        buf = torch.full((2 * self.PAD + body,), self.FILL, dtype=torch.uint8, device="cuda")
        self.items.append((buf, n))
        return buf[self.PAD:self.PAD + n].view(dtype).reshape(shape)

    def check(self, what=""):
        for buf, n in self.items:
            head, tail = buf[:self.PAD], buf[self.PAD + n:]
            assert bool((head == self.FILL).all()) and bool((tail == self.FILL).all()), (what, "a call wrote outside its output")

