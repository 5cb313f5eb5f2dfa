#!/usr/bin/env python3
"""Benchmark of the factorised-layer hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM.  Default workload (config 2): forward + backward of the four
Llama-2-7B attention projections, each factorised with r = 512, on 16384 tokens in bf16.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5|c1|merge]
"""
from __future__ import annotations

import argparse
import json
import sys
import time

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM-side traffic per launch of a kernel on a workload (fetched + written bytes), from the
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in profiles/bench_c2_lowrank_gemm_kernels.txt
# (counter units scaled by a 256 MiB read + 256 MiB write kernel in the same run); None where
# not measured.  Means over the launches of a step: the q/k/v group's wide products and the o projection's
# share a kernel.  Algorithmic bytes of a 68.7 GFLOP launch of config 2 are 155-160 MB.
MEASURED_TRAFFIC_BYTES = {
    ("c2", "gemm_pp<256x128x64,a0,b1,o0>"): 335.7e6 + 33.6e6,    # H = X A (o), H_all = X A_all (q/k/v)
    ("c2", "gemm_pp<256x256x32,a0,b1,o0>"): 95.2e6 + 134.2e6,    # Y = H B
    ("c2", "gemm_pp<256x128x64,a0,b0,o0>"): 168.0e6 + 16.8e6,    # dH = dY B^T
    ("c2", "gemm_pp<256x256x32,a0,b0,o0>"): 201.0e6 + 134.2e6,   # dX = dH A^T (o), dX = dH_all A_all^T (q/k/v)
    ("c2", "gemm_pp<256x256x32,a1,b1,o1>"): 414.0e6 + 76.3e6,    # dA_all = X^T dH_all
    ("c2", "gemm_pp<256x128x64,a1,b1,o1>"): 262.4e6 + 34.6e6,    # dA = X^T dH, dB = H^T dY (4 partial-sum slabs)
    # profiles/bench_merge_c5_int4_to_bf16.txt: mean over the layer's seven weights (algorithmic 115.1 MB)
    ("merge", "merge<int4>"): 38.6e6 + 90.6e6,
    # profiles/bench_c3_ffn_kernels.txt: means over the launches of a step (they differ in shape)
    ("c3", "gemm_pp<256x256x32,a0,b1,o0>"): 451.5e6 + 191.3e6,
    ("c3", "gemm_pp<256x256x32,a0,b0,o0>"): 450.3e6 + 119.1e6,
    ("c3", "gemm_pp<256x256x32,a1,b1,o1>"): 881.0e6 + 81.8e6,
    # profiles/bench_c4_int8_qlinear_kernels.txt (algorithmic 100.7 MB: X, the merged weight, Y)
    ("c4", "gemm_pp<256x256x32,a0,b1,o0>"): 201.5e6 + 33.6e6,
    ("c4", "gemm_pp<256x256x32,a0,b0,o0>"): 201.5e6 + 33.6e6,
    # profiles/bench_c5_int4_qlinear_kernels.txt: means over the seven linears (algorithmic 132 MB read, 62 / 52 MB
    # written): the 256x128 launch order gives each XCD's L2 a panel it cannot hold
    ("c5", "gemm_pp<256x128x64,a0,b1,o0>"): 1021.9e6 + 62.3e6,
    ("c5", "gemm_pp<256x128x64,a0,b0,o0>"): 1082.4e6 + 52.1e6,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "merge", "streams"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tokens", type=int, default=0,
                    help="c2/c4/c5: override the configuration's token count (c4/c5: the weight-streaming regime is tokens <= 64, "
                         "the JSON line then quotes GB/s on the algorithmic bytes as the value to read; c2: 48 independent "
                         "layers per step below 4096 tokens)")
    ap.add_argument("--forward-only", action="store_true", help="c2/c4/c5: time the forward call alone")
    ap.add_argument("--premerged", action="store_true",
                    help="c4/c5: a step merges each weight once (lowrank_merge) and passes the merged weight to the forward "
                         "and the backward call, instead of each call merging by itself")
    ap.add_argument("--independent-x", action="store_true",
                    help="c2: four independent projections, each with its own X (default: q/k/v read one X through "
                         "lowrank_linear_fwd/bwd_shared_x, as in an attention block; o has its own input); c3: gate and up "
                         "as two single-layer calls and an add of their input gradients (default: one shared-X call)")
    ap.add_argument("--shared-x", action="store_true",
                    help="c5 with --tokens and --forward-only: the q/k/v and the gate/up projections read one X each "
                         "and go through the shared-X entry point (one call per group: qkv, o, gate+up, down); "
                         "c2, c3: the default (see --independent-x)")
    ap.add_argument("--shape", default="", help="c4/c5 only: K,N of a single frozen weight in place of the configuration's "
                                                "(large weights show the streaming kernel's rate beyond the fixed launch cost)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (removes the host's launch cost; "
                         "meant for the few-token runs, where a step is a handful of microsecond-scale kernels)")
    ap.add_argument("--recompute", action="store_true", help="backward recomputes H instead of reading the saved copy")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="after the steps, launch a plain elementwise kernel that reads 256 MiB and writes 256 MiB three "
                         "times, so that a rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE by what "
                         "the same counters read for a known amount of traffic")
    return ap.parse_args()


# ----------------------------------------------------------------------------- workloads

def randn(shape, std, dtype, gen):
    import torch
    return (torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen) * std).to(dtype)


class LowrankCall:
    """One factorised linear: preallocated tensors, fwd and bwd through the C ABI."""

    def __init__(self, fhpc, M, K, r, N, dtype, gen, recompute=False, forward_only=False):
        import torch
        self.f = fhpc
        self.forward_only = forward_only
        self.M, self.K, self.r, self.N = M, K, r, N
        self.X = randn((M, K), 1.0, dtype, gen)
        self.dY = randn((M, N), 1.0, dtype, gen)
        self.A = randn((K, r), K ** -0.5, dtype, gen)
        self.B = randn((r, N), r ** -0.5, dtype, gen)
        self.Y = torch.empty((M, N), dtype=dtype, device="cuda")
        self.H = torch.empty((M, r), dtype=dtype, device="cuda")
        self.dX = torch.empty((M, K), dtype=dtype, device="cuda")
        self.dA = torch.empty((K, r), dtype=torch.float32, device="cuda")
        self.dB = torch.empty((r, N), dtype=torch.float32, device="cuda")
        self.recompute = recompute

    def flops(self):
        from paper_2402_13533_amd import shapes
        if self.forward_only:
            return 2 * self.M * self.r * (self.K + self.N)
        return shapes.lowrank_flops(self.M, self.K, self.r, self.N)

    def io_bytes(self):
        e = self.X.element_size()
        if self.forward_only:
            return e * (self.M * self.K + self.M * self.N) + e * self.r * (self.K + self.N)
        return e * (2 * self.M * self.K + 2 * self.M * self.N) + (e + 4) * self.r * (self.K + self.N)

    def run(self):
        self.f.lowrank_linear_fwd(self.X, self.A, self.B, Y=self.Y, H_out=self.H)
        if self.forward_only:
            return
        self.f.lowrank_linear_bwd(self.X, self.A, self.B, self.dY, H_saved=None if self.recompute else self.H,
                                  dX=self.dX, dA=self.dA, dB=self.dB)


class SharedLowrankCall:
    """g factorised linears fed by one X (q/k/v) through lowrank_linear_fwd/bwd_shared_x: X A_all is one
    product and the input gradient one product over the g r columns of [dH_0 | ...]."""

    def __init__(self, fhpc, M, K, r, N, g, gen):
        import torch
        bf = torch.bfloat16
        self.f, self.lib = fhpc, fhpc.load_library()
        self.M, self.K, self.r, self.N, self.g = M, K, r, N, g
        self.X = randn((M, K), 1.0, bf, gen)
        self.A_all = randn((K, g * r), K ** -0.5, bf, gen)
        self.B = [randn((r, N), r ** -0.5, bf, gen) for _ in range(g)]
        self.dY = [randn((M, N), 1.0, bf, gen) for _ in range(g)]
        self.Y = [torch.empty((M, N), dtype=bf, device="cuda") for _ in range(g)]
        self.H = torch.empty((M, g * r), dtype=bf, device="cuda")
        self.dX = torch.empty((M, K), dtype=bf, device="cuda")
        self.dA = torch.empty((K, g * r), dtype=torch.float32, device="cuda")
        self.dB = [torch.empty((r, N), dtype=torch.float32, device="cuda") for _ in range(g)]
        need = max(self.lib.fhpc_workspace_bytes_lowrank_shared_x(b, M, K, r, N, g) for b in (0, 1))
        self.ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")

    def flops(self):
        from paper_2402_13533_amd import shapes
        return self.g * shapes.lowrank_flops(self.M, self.K, self.r, self.N)

    def io_bytes(self):
        g = self.g
        return 2 * (2 * self.M * self.K + 2 * g * self.M * self.N) + 6 * g * self.r * (self.K + self.N)

    def run(self):
        self.f.lowrank_linear_fwd_shared_x(self.X, self.A_all, self.B, Ys=self.Y, H_all_out=self.H, workspace=self.ws)
        self.f.lowrank_linear_bwd_shared_x(self.X, self.A_all, self.B, self.dY, H_all_saved=self.H, dX=self.dX,
                                           dA_all=self.dA, dBs=self.dB, workspace=self.ws)


class QlinearCall:
    def __init__(self, fhpc, M, K, r, N, scheme, gen, scaling=2.0, recompute=False, forward_only=False, premerged=False):
        import torch
        bf = torch.bfloat16
        self.f = fhpc
        self.forward_only = forward_only
        self.Wm = torch.empty((K, N), dtype=bf, device="cuda") if premerged else None
        self.M, self.K, self.r, self.N, self.scheme, self.s = M, K, r, N, scheme, scaling
        W = randn((K, N), 0.02, torch.float32, gen)
        self.Wq, self.sc = fhpc.qweight_quantize(W, scheme)       # frozen base weight, quantised on the GPU
        del W
        self.X = randn((M, K), 1.0, bf, gen)
        self.dY = randn((M, N), 1.0, bf, gen)
        self.A = randn((K, r), K ** -0.5, bf, gen)
        self.B = randn((r, N), 0.01, bf, gen)
        self.Y = torch.empty((M, N), dtype=bf, device="cuda")
        self.H = torch.empty((M, r), dtype=bf, device="cuda")
        self.dX = torch.empty((M, K), dtype=bf, device="cuda")
        self.dA = torch.empty((K, r), dtype=torch.float32, device="cuda")
        self.dB = torch.empty((r, N), dtype=torch.float32, device="cuda")
        self.recompute = recompute

    def flops(self):
        from paper_2402_13533_amd import shapes
        full = shapes.qlinear_lowrank_flops(self.M, self.K, self.r, self.N)
        if self.forward_only:
            return 2 * self.M * self.K * self.N + 2 * self.M * self.r * (self.K + self.N)
        return full

    def io_bytes(self):
        w = self.Wq.numel() * self.Wq.element_size() + 2 * self.sc.numel()
        if self.forward_only:
            return w + 2 * (self.M * self.K + self.M * self.N) + 2 * self.r * (self.K + self.N)
        return 2 * w + 2 * (2 * self.M * self.K + 2 * self.M * self.N) + 6 * self.r * (self.K + self.N)

    def run(self):
        f = self.f
        Wq, sc, scheme = self.Wq, self.sc, self.scheme
        if self.Wm is not None:
            f.lowrank_merge(self.Wq, self.sc, self.scheme, self.A, self.B, self.s, W_out=self.Wm)
            Wq, sc, scheme = self.Wm, None, f.FHPC_W_MERGED
        f.qlinear_lowrank_fwd(self.X, Wq, sc, scheme, self.A, self.B, self.s, Y=self.Y, H_out=self.H)
        if self.forward_only:
            return
        f.qlinear_lowrank_bwd(self.X, Wq, sc, scheme, self.A, self.B, self.s, self.dY,
                              H_saved=None if self.recompute else self.H, dX=self.dX, dA=self.dA, dB=self.dB)


class SharedXCall:
    """Several quantised projections of one X through qlinear_lowrank_fwd_shared_x (forward only)."""

    def __init__(self, fhpc, calls):
        self.f = fhpc
        self.calls = calls
        self.X = calls[0].X
        self.scheme = calls[0].scheme
        self.weights = [(c.Wq, c.sc, c.A, c.B, c.s) for c in calls]

    def flops(self):
        return sum(c.flops() for c in self.calls)

    def io_bytes(self):
        return sum(c.io_bytes() for c in self.calls) - 2 * self.X.numel() * (len(self.calls) - 1)

    def run(self):
        self.f.qlinear_lowrank_fwd_shared_x(self.X, self.weights, self.scheme)


class MergeCall:
    """W' = deq(Wq) + scaling A B written as bf16: the adapted weight materialised for inference."""

    def __init__(self, fhpc, K, r, N, scheme, gen, scaling=2.0):
        import torch
        bf = torch.bfloat16
        self.f = fhpc
        self.K, self.r, self.N, self.scheme, self.s = K, r, N, scheme, scaling
        W = randn((K, N), 0.02, torch.float32, gen)
        self.Wq, self.sc = fhpc.qweight_quantize(W, scheme)
        del W
        self.A = randn((K, r), K ** -0.5, bf, gen)
        self.B = randn((r, N), 0.01, bf, gen)
        self.out = torch.empty((K, N), dtype=bf, device="cuda")

    def flops(self):
        return 2 * self.K * self.N * self.r

    def io_bytes(self):
        return (self.Wq.numel() * self.Wq.element_size() + 2 * self.sc.numel() + 2 * self.K * self.N
                + 2 * self.r * (self.K + self.N))

    def run(self):
        self.f.lowrank_merge(self.Wq, self.sc, self.scheme, self.A, self.B, self.s, W_out=self.out)


class StreamCall:
    """One of the pure streaming kernels of the path (no matrix work): a closure and its algorithmic bytes."""

    def __init__(self, fn, nbytes):
        self.fn, self.nbytes = fn, nbytes

    def flops(self):
        return 0

    def io_bytes(self):
        return self.nbytes

    def run(self):
        self.fn()


def stream_calls(fhpc, gen):
    """SiLU gate forward / backward on config 3's 16384 x 11008 activations; dequantise and quantise
    on config 5's widest weight (5120 x 13824), both schemes."""
    import torch
    bf = torch.bfloat16
    n = 16384 * 11008
    G, U, dZ = (randn((16384, 11008), 1.0, bf, gen) for _ in range(3))
    Z, dG, dU = (torch.empty_like(G) for _ in range(3))
    K, N = 5120, 13824
    W = randn((K, N), 0.02, torch.float32, gen)
    calls = [StreamCall(lambda: fhpc.swiglu_fwd(G, U, Z=Z), 6 * n),
             StreamCall(lambda: fhpc.swiglu_bwd(G, U, dZ, dG=dG, dU=dU), 10 * n)]
    for scheme in (4, 8):
        Wq, sc = fhpc.qweight_quantize(W, scheme)
        out = torch.empty((N, K), dtype=torch.float32, device="cuda")
        packed = Wq.numel() * Wq.element_size() + 2 * sc.numel()
        calls.append(StreamCall(lambda Wq=Wq, sc=sc, scheme=scheme, out=out: fhpc.qweight_dequant(Wq, sc, scheme, W_out=out),
                                packed + 4 * K * N))
        calls.append(StreamCall(lambda Wq=Wq, sc=sc, scheme=scheme: fhpc.qweight_quantize(W, scheme, Wq_out=Wq, scales_out=sc),
                                4 * K * N + packed))
    return calls


class FfnCall:
    """Config 3: gate/up 4096 -> r -> 11008, SiLU gate, down 11008 -> r -> 4096, fwd + bwd."""

    def __init__(self, fhpc, M, d, r, f, gen, shared_x=False):
        import torch
        bf = torch.bfloat16
        self.fh = fhpc
        self.shared_x = shared_x
        self.M, self.d, self.r, self.f = M, d, r, f
        self.X = randn((M, d), 1.0, bf, gen)
        self.dY = randn((M, d), 1.0, bf, gen)
        self.W = [randn((d, r), d ** -0.5, bf, gen), randn((r, f), r ** -0.5, bf, gen),
                  randn((d, r), d ** -0.5, bf, gen), randn((r, f), r ** -0.5, bf, gen),
                  randn((f, r), f ** -0.5, bf, gen), randn((r, d), r ** -0.5, bf, gen)]
        if shared_x:      # gate and up factors side by side: [Ag | Au]
            Ag, Bg, Au, Bu, Ad, Bd = self.W
            self.Ws = [torch.cat([Ag, Au], dim=1).contiguous(), Bg, Bu, Ad, Bd]

    def flops(self):
        from paper_2402_13533_amd import shapes
        return 2 * shapes.lowrank_flops(self.M, self.d, self.r, self.f) + shapes.lowrank_flops(self.M, self.f, self.r, self.d)

    def io_bytes(self):
        return 2 * (4 * self.M * self.d) + 6 * 3 * self.r * (self.d + self.f)

    def run(self):
        from paper_2402_13533_amd import ffn
        if self.shared_x:
            Y, saved = ffn.ffn_fwd_shared_x(self.X, *self.Ws)
            ffn.ffn_bwd_shared_x(self.X, *self.Ws, self.dY, saved)
            return
        Y, saved = ffn.ffn_fwd(self.X, *self.W)
        ffn.ffn_bwd(self.X, *self.W, self.dY, saved)


def build_workload(name, fhpc, recompute, tokens=0, forward_only=False, shape=None, shared_x=False, premerged=False,
                   independent_x=False):
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20240213)
    bf = torch.bfloat16
    if name == "c1":
        calls = [LowrankCall(fhpc, 256, 768, 32, 768, torch.float32, gen, recompute)]
        desc = "config 1: fp32 factorised linear 256x768, r=32, fwd+bwd"
        dtype = "f32"
    elif name == "c2":
        M = tokens or 16384
        # at a reduced token count the factor pairs (8.4 MB each) would sit in the 256 MB Infinity Cache from step
        # to step: 48 independent layers then stand for the 4, so that the weights come from HBM
        copies = 4 if M >= 4096 else 48
        desc = "config 2: Llama-2-7B q/k/v/o projections factorised r=512, %d tokens, bf16, %s%s" % (
            M, "fwd" if forward_only else "fwd+bwd", "" if copies == 4 else ", %d independent layers per step" % copies)
        dtype = "bf16"
        if shared_x and (tokens or forward_only or recompute or independent_x):
            raise SystemExit("--shared-x on c2 runs the configuration's 16384 tokens, forward and backward, saved H")
        if not (tokens or forward_only or recompute or independent_x):
            # an attention block: q, k and v read the same X (their input gradients arrive summed), o its own input
            calls = [SharedLowrankCall(fhpc, M, 4096, 512, 4096, 3, gen), LowrankCall(fhpc, M, 4096, 512, 4096, bf, gen)]
            return calls, desc + ", q/k/v read one X through the shared-X call", dtype
        calls = [LowrankCall(fhpc, M, 4096, 512, 4096, bf, gen, recompute, forward_only) for _ in range(copies)]
        if independent_x:
            desc += ", four independent inputs"
        return calls, desc, dtype
    elif name == "c3":
        calls = [FfnCall(fhpc, 16384, 4096, 1024, 11008, gen, not independent_x)]
        desc = "config 3: Llama-2-7B SiLU-gated FFN factorised r=1024, 16384 tokens, bf16, fwd+bwd"
        return calls, desc + (", gate and up as single-layer calls" if independent_x else ", gate and up through the shared-X call"), "bf16"
        dtype = "bf16"
    elif name == "c4":
        M = tokens or 4096
        # four independent copies of the layer (own W, X, dY), run back to back: one copy's buffers
        # (0.17 GB) would sit in the 256 MB Infinity Cache from step to step
        K, N = shape or (4096, 4096)
        calls = [QlinearCall(fhpc, M, K, 8, N, 8, gen, 2.0, recompute, forward_only, premerged) for _ in range(1 if shape else 4)]
        desc = "config 4: int8 per-channel frozen W %dx%d + rank-8 branch, %d tokens, bf16, %s, %d buffer set(s) per step" % (
            K, N, M, "fwd" if forward_only else "fwd+bwd", len(calls))
        dtype = "bf16"
    elif name == "streams":
        calls = stream_calls(fhpc, gen)
        desc = ("streaming kernels: SiLU gate fwd/bwd on 16384x11008 bf16, dequantise and quantise of a 5120x13824 "
                "weight (int4 block-64, int8 per-channel)")
        dtype = "bf16"
    elif name == "merge":
        d, f = 5120, 13824
        shp = [(d, d)] * 4 + [(d, f), (d, f), (f, d)]
        calls = [MergeCall(fhpc, K, 16, N, 4, gen) for K, N in shp]
        desc = "merged weights of config 5's decoder layer: 7 x (int4 block-64 W + 2 A B, rank 16) -> bf16"
        dtype = "bf16"
    else:
        d, f = 5120, 13824
        shp = [shape] if shape else [(d, d)] * 4 + [(d, f), (d, f), (f, d)]
        M = tokens or 4096
        calls = [QlinearCall(fhpc, M, K, 16, N, 4, gen, 2.0, recompute, forward_only, premerged) for K, N in shp]
        desc = "config 5: %s, int4 block-64 frozen W + rank-16 branch, %d tokens, bf16, %s" % (
            "one linear %dx%d" % shape if shape else "Llama-2-13B decoder layer, 7 linears", M, "fwd" if forward_only else "fwd+bwd")
        dtype = "bf16"
    if shared_x:
        if name != "c5" or not forward_only or shape:
            raise SystemExit("--shared-x goes with --workload c5 --forward-only (c2 and c3 use their shared-X calls by default)")
        q, k, v, o, gate, up, down = calls
        calls = [SharedXCall(fhpc, [q, k, v]), o, SharedXCall(fhpc, [gate, up]), down]
        desc += ", q/k/v and gate/up through the shared-X call"
    return calls, desc, dtype


# ----------------------------------------------------------------------------- CPU baseline

def cpu_baseline(workload):
    """The fp64 oracle, as it stands, on a bounded row sample of the same workload."""
    import numpy as np
    import oracle
    from paper_2402_13533_amd import shapes, synth
    if workload in ("c1", "c2"):
        K, r, N = (768, 32, 768) if workload == "c1" else (4096, 512, 4096)
    elif workload == "c3":
        K, r, N = 4096, 1024, 11008
    elif workload == "c4":
        K, r, N = 4096, 8, 4096
    else:
        K, r, N = 5120, 16, 5120
    quant = workload in ("c4", "c5")

    def run(M):
        X = synth.normal(1, (M, K)).astype(np.float64)
        dY = synth.normal(2, (M, N)).astype(np.float64)
        A = synth.normal(3, (K, r), K ** -0.5).astype(np.float64)
        B = synth.normal(4, (r, N), r ** -0.5).astype(np.float64)
        if quant:
            Wd = synth.normal(5, (K, N), 0.02).astype(np.float64)
            t0 = time.perf_counter()
            oracle.qlinear_lowrank_fwd(X, Wd, A, B, 2.0)
            oracle.qlinear_lowrank_bwd(X, Wd, A, B, 2.0, dY)
            dt = time.perf_counter() - t0
            fl = shapes.qlinear_lowrank_flops(M, K, r, N)
        else:
            t0 = time.perf_counter()
            oracle.lowrank_fwd(X, A, B)
            oracle.lowrank_bwd(X, A, B, dY)
            dt = time.perf_counter() - t0
            fl = shapes.lowrank_flops(M, K, r, N)
        return dt, fl

    m0 = 64 if workload != "c1" else 256
    dt, fl = run(m0)                                   # calibration
    target = 15.0
    M = m0
    if workload != "c1":
        M = int(min(16384, max(m0, m0 * target / max(dt, 1e-3))))
        M = max(64, M // 64 * 64)
        dt, fl = run(M)
    return {
        "value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "fp64 oracle fwd+bwd of one linear of the workload (K=%d, r=%d, N=%d) on %d token rows, %.1f s"
                  % (K, r, N, M, dt),
    }


# ----------------------------------------------------------------------------- main

def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus %d is not supported (the layer shards over "
              "tokens with one all-reduce of dA/dB per step)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2402_13533_amd as fhpc
    fhpc.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    shape = tuple(int(v) for v in args.shape.split(",")) if args.shape else None
    calls, desc, dtype = build_workload(args.workload, fhpc, args.recompute, args.tokens, args.forward_only, shape, args.shared_x, args.premerged,
                                       args.independent_x)
    flops = sum(c.flops() for c in calls)
    io_bytes = sum(c.io_bytes() for c in calls)

    def step():
        for c in calls:
            c.run()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    timed = step
    if args.graph:
        # the library only enqueues kernels on the current stream (no allocation, no memset), so a
        # step can be captured as it is
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        timed = graph.replay
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        timed()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    tflops = flops / (ms_per_step * 1e-3) / 1e12

    # second pass over the same steps with an event pair around every GEMM launch (library hook)
    fhpc.profile_start(8192)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    recs = fhpc.profile_stop()
    agg = {}
    for name, ms, fl, by in recs:
        a = agg.setdefault(name, [0, 0.0, 0.0, 0.0])
        a[0] += 1; a[1] += ms; a[2] += fl; a[3] += by
    kernels = {n: {"launches_per_step": a[0] / args.steps, "avg_ms": a[1] / a[0], "flops_per_launch": a[2] / a[0],
                   "tflops": a[2] / a[1] / 1e9 if a[1] > 0 else None,
                   "bytes_per_launch": a[3] / a[0], "gbs": a[3] / a[1] / 1e6 if (a[1] > 0 and a[3] > 0) else None}
               for n, a in agg.items()}
    roofline = None
    if agg:
        # the kernel the roofline is quoted for: the one with the largest share of the timed kernels'
        # time (a GEMM, quoted in TFLOP/s, or a streaming kernel, quoted in GB/s on its algorithmic bytes)
        dom = max(agg, key=lambda n: agg[n][1])
        k = kernels[dom]
        share = agg[dom][1] / sum(a[1] for a in agg.values())
        if k["gbs"] is not None:
            # weight-streaming kernel: algorithmic bytes (packed weight + scales + tokens + its partial sums)
            roofline = {"kernel": dom, "bound": "hbm", "achieved": k["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": k["gbs"] / PEAK_HBM_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, dom)),
                        "avg_launch_ms": k["avg_ms"], "share_of_timed_kernels": share}
        else:
            roofline = {"kernel": dom, "bound": "mfma", "achieved": k["tflops"], "peak": PEAK_BF16_TFLOPS,
                        "unit": "TFLOP/s", "frac": k["tflops"] / PEAK_BF16_TFLOPS,
                        "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, dom)),
                        "avg_launch_ms": k["avg_ms"], "share_of_gemm_time": share}

    metric, value, unit = "fwd+bwd TFLOP/s", tflops, "TFLOP/s"
    if args.workload in ("merge", "streams"):       # streaming passes: quoted in bytes moved
        metric, value, unit = args.workload + " GB/s", io_bytes / (ms_per_step * 1e-3) / 1e9, "GB/s"
    out = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": desc, "saved_H": not args.recompute, "hip_graph": bool(args.graph),
                   "merged_once_per_step": bool(args.premerged)},
        "frac_bf16_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "io_gbs": io_bytes / (ms_per_step * 1e-3) / 1e9, "frac_hbm_peak_on_io_bytes": io_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "roofline": roofline, "kernels": kernels,
    }
    if args.pmc_calibration:
        x = torch.zeros(64 << 20, dtype=torch.float32, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline and args.workload not in ("merge", "streams"):
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
