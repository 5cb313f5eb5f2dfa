#!/usr/bin/env python3
"""Benchmark of the factorised-layer hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is
already resident in HBM.  Default workload (config 2): forward + backward of the four
Llama-2-7B attention projections, each factorised with r = 512, on 16384 tokens in bf16.
Prints ONE JSON line: the headline workload (value, roofline of its dominant kernel, CPU baseline) and, unless
--only-headline, every other configuration, the few-token sweep of the quantised layers (the metric's GB/s half)
and the measured peaks of this GPU.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5|c1|merge|streams] [--only-headline]
"""
from __future__ import annotations

import argparse
import json
import sys
import time

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
METRIC = "fwd+bwd TFLOP/s (% bf16 MFMA peak); quantised-path GB/s (% HBM peak)"


def profiled_traffic(workload, kernel):
    """HBM-side bytes per launch (fetched + written) of `kernel` on `workload`, read from the committed rocprofv3
    --pmc summary of the same command (profiles/bench_<workload>_*.txt, section "HBM-side traffic counters"), and
    the file it came from; (None, None) when no summary lists the kernel.  The bench never measures this itself:
    hardware counters need the profiler."""
    import glob
    import os
    import re
    m = re.match(r"gemm_pp<(\d+)x(\d+)x(\d+),a(\d),b(\d),o(\d)(?:,gate(\d))?>", kernel)
    if m:
        bm, bn, bk, a, b, o = (int(v) for v in m.groups()[:6])
        gate = int(m.group(7) or 0)
        # template arguments as the profiler prints them: tile, k-split flag, ring depth, operand modes, output, gate
        tail = r"(?:, 0)?>" if gate == 0 else r", %d>" % gate
        pat = re.compile(r"gemm_pp_kernel<%d, %d, %d, (?:true|false), \d+, %d, %d, %d%s" % (bm, bn, bk, a, b, o, tail))
    else:
        pat = re.compile(re.escape(kernel.split("<")[0]))
    here = os.path.dirname(os.path.abspath(__file__))
    # the summary of the plain command first (the same workload with other flags has files of its own)
    plain = {"c2": "bench_c2_lowrank_gemm_kernels.txt", "c3": "bench_c3_ffn_kernels.txt",
             "c4": "bench_c4_int8_qlinear_kernels.txt", "c5": "bench_c5_int4_qlinear_kernels.txt"}
    paths = sorted(glob.glob(os.path.join(here, "profiles", "bench_%s_*.txt" % workload)))
    first = os.path.join(here, "profiles", plain.get(workload, ""))
    if first in paths:
        paths.remove(first)
        paths.insert(0, first)
    for path in paths:
        in_table = False
        for line in open(path):
            if line.startswith("== "):
                in_table = "HBM-side traffic" in line
            elif in_table and pat.search(line):
                cols = line.split()
                try:
                    return (float(cols[-2]) + float(cols[-1])) * 1e6, os.path.relpath(path, here)
                except ValueError:
                    pass
    return None, None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "merge", "streams"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-headline", dest="all_configs", action="store_false",
                    help="time the chosen workload alone (profiler runs); by default the line also carries every other "
                         "configuration, the few-token sweep of the quantised layers and the measured peaks")
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
        self.ws = torch.zeros(max(need, 256), dtype=torch.uint8, device="cuda")      # (the header must start out zero)

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


class QlinearWeights:
    """A frozen weight quantised on the GPU and its factor pair (shared by calls at several token counts)."""

    def __init__(self, fhpc, K, r, N, scheme, gen):
        import torch
        self.K, self.r, self.N, self.scheme = K, r, N, scheme
        W = randn((K, N), 0.02, torch.float32, gen)
        self.Wq, self.sc = fhpc.qweight_quantize(W, scheme)
        del W
        self.A = randn((K, r), K ** -0.5, torch.bfloat16, gen)
        self.B = randn((r, N), 0.01, torch.bfloat16, gen)

    def packed_bytes(self):
        return self.Wq.numel() * self.Wq.element_size() + 2 * self.sc.numel()


class QlinearCall:
    def __init__(self, fhpc, M, K, r, N, scheme, gen, scaling=2.0, recompute=False, forward_only=False, premerged=False,
                 weights=None):
        import torch
        bf = torch.bfloat16
        self.f = fhpc
        self.forward_only = forward_only
        self.Wm = torch.empty((K, N), dtype=bf, device="cuda") if premerged else None
        self.M, self.K, self.r, self.N, self.scheme, self.s = M, K, r, N, scheme, scaling
        w = weights if weights is not None else QlinearWeights(fhpc, K, r, N, scheme, gen)
        self.Wq, self.sc, self.A, self.B = w.Wq, w.sc, w.A, w.B       # frozen base weight, quantised on the GPU
        self.X = randn((M, K), 1.0, bf, gen)
        self.dY = randn((M, N), 1.0, bf, gen)
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


def build_workload(name, fhpc, recompute=False, tokens=0, forward_only=False, shape=None, shared_x=False, premerged=False,
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


# ----------------------------------------------------------------------------- timing

def time_steps(step, steps, warmup, graph=False):
    """W untimed warm-up steps, then K timed steps bracketed by synchronisation; an event after every step gives
    the per-step durations.  Returns (mean, median, min) in milliseconds; the mean is first event to last."""
    import statistics
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    timed = step
    if graph:
        # the library only enqueues kernels on the current stream (no allocation, no memset), so a
        # step can be captured as it is
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        g.replay()
        torch.cuda.synchronize()
        timed = g.replay
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        timed()
        ev[i + 1].record()
    torch.cuda.synchronize()
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    return ev[0].elapsed_time(ev[steps]) / steps, statistics.median(per), min(per)


def kernel_profile(fhpc, step, steps, workload):
    """A second pass over the same steps with the library's event pair around every launch (on the launch stream):
    per-kernel averages, and the roofline object of the kernel with the largest share of the time."""
    import torch
    fhpc.profile_start(8192)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    recs = fhpc.profile_stop()
    agg = {}
    for name, ms, fl, by in recs:
        a = agg.setdefault(name, [0, 0.0, 0.0, 0.0])
        a[0] += 1; a[1] += ms; a[2] += fl; a[3] += by
    kernels = {n: {"launches_per_step": a[0] / steps, "avg_ms": a[1] / a[0], "flops_per_launch": a[2] / a[0],
                   "tflops": a[2] / a[1] / 1e9 if a[1] > 0 else None,
                   "bytes_per_launch": a[3] / a[0], "gbs": a[3] / a[1] / 1e6 if (a[1] > 0 and a[3] > 0) else None}
               for n, a in agg.items()}
    roofline = None
    if agg:
        dom = max(agg, key=lambda n: agg[n][1])
        k = kernels[dom]
        share = agg[dom][1] / sum(a[1] for a in agg.values())
        traffic, source = profiled_traffic(workload, dom)
        if k["gbs"] is not None:
            # weight-streaming kernel: algorithmic bytes (packed weight + scales + tokens + its partial sums)
            roofline = {"kernel": dom, "bound": "hbm", "achieved": k["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": k["gbs"] / PEAK_HBM_GBS, "traffic": traffic, "traffic_source": source,
                        "avg_launch_ms": k["avg_ms"], "share_of_timed_kernels": share}
        else:
            roofline = {"kernel": dom, "bound": "mfma", "achieved": k["tflops"], "peak": PEAK_BF16_TFLOPS,
                        "unit": "TFLOP/s", "frac": k["tflops"] / PEAK_BF16_TFLOPS, "traffic": traffic,
                        "traffic_source": source, "avg_launch_ms": k["avg_ms"], "share_of_gemm_time": share}
    return kernels, roofline


def measured_peaks(fhpc):
    """What this GPU delivers with no kernel design in the way: the matrix cores fed from registers (zero operands,
    and random operands, under which the chip lowers its clock) and a streaming copy / read of 1 GiB."""
    import torch
    dev = "cuda"
    out = {"bf16_mfma_tflops": {"spec": PEAK_BF16_TFLOPS}, "hbm_gbs": {"spec": PEAK_HBM_GBS}}
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    seeds = {"registers_only_zero_operands": torch.zeros(256, dtype=torch.int32, device=dev),
             "registers_only_random_operands": torch.randn(512, device=dev).to(torch.bfloat16).view(torch.int32)}
    for name, seed in seeds.items():
        best = 0.0
        for _ in range(3):
            fhpc.probe_mfma(seed, cus, 2000)                      # warm
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = fhpc.probe_mfma(seed, 4 * cus, 20000)            # about 1 ms of matrix instructions per SIMD
            e1.record()
            torch.cuda.synchronize()
            best = max(best, fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        out["bf16_mfma_tflops"][name] = best
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    best = 0.0
    for _ in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        n = fhpc.probe_copy(src, dst)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, 2 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out["hbm_gbs"]["copy_1GiB_read_plus_write"] = best
    del src, dst
    # One pass over a 4-bit weight of configuration 5 in the few-token kernels' access pattern and nothing else
    # (rows of K / 2 bytes; eight copies in turn so that the reads come from HBM; 24 passes replayed from a HIP
    # graph, as the few-token rows are timed): what the read alone costs at that size, launch included.
    sink = torch.zeros(256, dtype=torch.int32, device=dev)
    rows = {}
    for name, (K, N) in {"5120x5120": (5120, 5120), "5120x13824": (5120, 13824), "13824x5120": (13824, 5120)}.items():
        copies = [torch.empty(N, K // 2, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(8)]

        def passes():
            for i in range(24):
                fhpc.probe_read_rows(copies[i % 8], 3 * cus, sink)
        _, _, best = time_steps(passes, 5, 2, graph=True)
        n = copies[0].numel()
        rows[name] = {"weight_MB": n / 1e6, "us_per_pass": best * 1e3 / 24, "gbs": n / (best * 1e-3 / 24) / 1e9}
        del copies
    out["hbm_gbs"]["few_token_read_pattern_alone_int4_weights_of_config5"] = rows
    return out


def summarise(calls, ms_mean, ms_median, ms_min, desc, dtype):
    flops = sum(c.flops() for c in calls)
    io = sum(c.io_bytes() for c in calls)
    d = {"workload": desc, "dtype": dtype, "ms_per_step": ms_mean, "ms_per_step_median": ms_median, "ms_per_step_min": ms_min,
         "io_gbs": io / (ms_mean * 1e-3) / 1e9, "frac_hbm_peak_on_io_bytes": io / (ms_mean * 1e-3) / 1e9 / PEAK_HBM_GBS}
    if flops:
        d["tflops"] = flops / (ms_mean * 1e-3) / 1e12
        d["tflops_at_median"] = flops / (ms_median * 1e-3) / 1e12
        d["frac_bf16_mfma_peak"] = d["tflops"] / PEAK_BF16_TFLOPS
    return d


def other_configs(fhpc, headline, independent_x):
    """Every configuration beside the headline one, each timed on a few steps (they are not the quoted value)."""
    import gc
    import torch
    plan = [("c1", {}, 200, 20), ("c2", {}, 8, 2), ("c2_independent_x", {"independent_x": True}, 8, 2), ("c3", {}, 5, 2),
            ("c4", {}, 8, 2), ("c5", {}, 5, 2)]
    out = {}
    for key, kw, steps, warmup in plan:
        name = key.split("_")[0]
        if key == headline and not independent_x:
            continue
        calls, desc, dtype = build_workload(name, fhpc, False, **kw)

        def step():
            for c in calls:
                c.run()
        out[key] = summarise(calls, *time_steps(step, steps, warmup), desc, dtype)
        out[key]["steps"] = steps
        del calls, step
        gc.collect()
        torch.cuda.empty_cache()
    return out


def quantised_stream(fhpc):
    """The regime in which the quantised layers are bound by reading their packed weights: configurations 4 and 5 at
    1, 16 and 64 tokens, forward alone and forward + backward.  A step is the configuration's layer (one int8 linear;
    the seven int4 linears of a decoder layer); the steps rotate through independent copies of the weights, more than
    512 MB in all, so that the 256 MB Infinity Cache cannot serve them.  GB/s is on the algorithmic bytes
    (packed codes + scales once per pass over the weight, tokens in and out, the factor pair and its gradients)."""
    import gc
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20240214)
    d, f = 5120, 13824
    layers = {"c4": ([(4096, 4096)], 8, 8, 32), "c5": ([(d, d)] * 4 + [(d, f), (d, f), (f, d)], 16, 4, 4)}
    rows = []
    for cfg, (shapes_, r, scheme, copies) in layers.items():
        weights = [[QlinearWeights(fhpc, K, r, N, scheme, gen) for K, N in shapes_] for _ in range(copies)]
        packed = sum(w.packed_bytes() for w in weights[0]) * copies
        for M in (1, 16, 64):
            for fwd_only in (True, False):
                sets = [[QlinearCall(fhpc, M, w.K, r, w.N, scheme, gen, 2.0, False, fwd_only, weights=w) for w in ws]
                        for ws in weights]
                state = {"i": 0}

                def step():
                    for c in sets[state["i"] % copies]:
                        c.run()
                    state["i"] += 1
                io = sum(c.io_bytes() for c in sets[0])
                # eager launches from this process, then the same steps replayed from a HIP graph (one graph holds a
                # step on every copy of the weights; a serving loop would replay such a graph), which takes the
                # host's launch cost out
                for launch in ("eager", "hip_graph"):
                    if launch == "eager":
                        mean, med, mn = time_steps(step, 40, 8)
                    else:
                        def all_copies():
                            for _ in range(copies):
                                step()
                        mean, med, mn = (t / copies for t in time_steps(all_copies, 10, 2, graph=True))
                    rows.append({"config": cfg, "tokens": M, "pass": "fwd" if fwd_only else "fwd+bwd", "launch": launch,
                                 "ms_per_step": mean, "ms_per_step_median": med, "ms_per_step_min": mn, "algorithmic_bytes": io,
                                 "gbs": io / (mean * 1e-3) / 1e9, "frac_hbm_peak": io / (mean * 1e-3) / 1e9 / PEAK_HBM_GBS})
                if cfg == "c5" and fwd_only:
                    # the same forward as a decoder layer issues it: q, k and v read one X and so do gate and up, each
                    # group in one call of qlinear_lowrank_fwd_shared_x (four launches per step instead of seven)
                    shared = []
                    for cs in sets:
                        q, k, v, o, gate, up, down = cs
                        shared.append([SharedXCall(fhpc, [q, k, v]), o, SharedXCall(fhpc, [gate, up]), down])
                    sstate = {"i": 0}

                    def sstep():
                        for c in shared[sstate["i"] % copies]:
                            c.run()
                        sstate["i"] += 1

                    def sall():
                        for _ in range(copies):
                            sstep()
                    sio = sum(c.io_bytes() for c in shared[0])
                    for launch in ("eager", "hip_graph"):
                        if launch == "eager":
                            mean, med, mn = time_steps(sstep, 40, 8)
                        else:
                            mean, med, mn = (t / copies for t in time_steps(sall, 10, 2, graph=True))
                        rows.append({"config": cfg, "tokens": M, "pass": "fwd, q/k/v and gate/up through the shared-X call",
                                     "launch": launch, "ms_per_step": mean, "ms_per_step_median": med, "ms_per_step_min": mn,
                                     "algorithmic_bytes": sio, "gbs": sio / (mean * 1e-3) / 1e9,
                                     "frac_hbm_peak": sio / (mean * 1e-3) / 1e9 / PEAK_HBM_GBS})
                    del shared, sstep, sall
                del sets, step
        rows[-1]["weight_copies"] = copies
        rows[-1]["packed_weight_bytes_all_copies"] = packed
        del weights
        gc.collect()
        torch.cuda.empty_cache()
    best = max(rows, key=lambda r_: r_["gbs"])
    return {"note": "configs 4 and 5 at 1/16/64 tokens: HBM-bound regime of the quantised layers; one step = the "
                    "configuration's layer, weights rotating through > 512 MB of independent copies",
            "peak_gbs": PEAK_HBM_GBS, "best_gbs": best["gbs"], "best_frac_hbm_peak": best["frac_hbm_peak"], "rows": rows}


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

    ms_per_step, ms_median, ms_min = time_steps(step, args.steps, args.warmup, args.graph)
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    kernels, roofline = kernel_profile(fhpc, step, args.steps, args.workload)

    metric, value, unit = METRIC, tflops, "TFLOP/s"
    if args.workload in ("merge", "streams"):       # streaming passes: quoted in bytes moved
        metric, value, unit = args.workload + " GB/s", io_bytes / (ms_per_step * 1e-3) / 1e9, "GB/s"
    out = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_median": ms_median,
        "ms_per_step_min": ms_min, "higher_is_better": True,
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
    plain = not (args.tokens or args.forward_only or shape or args.shared_x or args.premerged or args.graph or args.recompute)
    if args.all_configs and plain and args.workload in ("c1", "c2", "c3", "c4", "c5"):
        # the other half of the metric and the other configurations, in the same line
        del calls
        torch.cuda.empty_cache()
        out["peaks_measured"] = measured_peaks(fhpc)
        out["configs"] = other_configs(fhpc, args.workload, args.independent_x)
        out["quantised_stream"] = quantised_stream(fhpc)
        out["quantised_path_gbs"] = out["quantised_stream"]["best_gbs"]
        out["quantised_path_frac_hbm_peak"] = out["quantised_stream"]["best_frac_hbm_peak"]
    if not args.no_cpu_baseline and args.workload not in ("merge", "streams"):
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
