#!/usr/bin/env python3
"""Benchmark of the 8-bit floating point training primitive on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input for the
ResNet-50-style 3x3 convolution layer taken as a GEMM (M=25088, N=128, K=1152):

    Q(X) -> X8                                  Q(dY * 2^12) -> E8 (+ overflow stats)
    forward GEMM  Y8  = Q(X8 . W8)              contraction K
    backward-data dX8 = Q(E8 . W8^T)            contraction N
    weight-grad   G8  = Q(X8^T . E8)            contraction M (split, summed in FP32, one rounding)
    update        W16 <- half_SR(W16 - lr * G8 / 2^12),  W8 <- Q(W16) for the next step
                  (applied by the pass that rounds G8: one call, mp8_wgrad_update_fp16_sr)

(Launched in the order Q(dY), backward-data, Q(X), forward, weight-grad + update.)
Every tensor exists once, row-major, as its producer wrote it: the GEMMs read X8 [M,K],
E8 [M,N] and W8 [K,N] in whichever orientation they need (contraction-major operands go
through transposing LDS reads), and the Q node on the weights is part of the update kernel.
`conv_step` reports the same layer run as the 3x3 convolution it stands for (implicit GEMM on
zero-padded channels-last tensors, nothing lowered): same useful flops, a ninth of the bytes.

Inputs are resident in HBM before the timed region.  Prints ONE JSON line: `value` is the
GEMM work of a step (3 * 2*M*N*K flop) divided by the time of the whole step (the steps are
replayed from a captured HIP graph unless --launch eager); `roofline` describes the kernel
that takes the largest share of the step, its duration measured with events around back-to-back
launches; `kernels` lists every kernel of the step with its own roofline; `all_configs` is a kernel-level table over the GEMM shapes
of all five configurations and the streaming kernels at 2^28 elements; `cpu_baseline` is the
CPU oracle timed on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP8_PEAK_TFLOPS = 5000.0       # MI355X dense FP8 MFMA, published
LOSS_SCALE = 2.0 ** 12
LR = 1e-3
# HBM bytes per launch read off the FETCH_SIZE and WRITE_SIZE counters for this workload, scaled
# by what the same counters read on a plain 1 GiB copy (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000);
# the runs and their raw figures are in profiles/bench_step_cfg2_hbm_traffic.txt
MEASURED_TRAFFIC_BYTES = {
    "quantize_X_gemm_fwd": 149119098, "quantize_dY": 16142647, "gemm_bwd_data": 33493089,
    "gemm_wgrad_update": 51595802,
    # with --separate-quantize (measured before the two were fused)
    "quantize_X": 144555139, "gemm_fwd": 33417730,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--launch", choices=("graph", "eager"), default="graph",
                    help="how the timed steps are launched: replay of a captured HIP graph "
                         "(default) or one Python call per kernel")
    ap.add_argument("--separate-update", action="store_true",
                    help="weight gradient and master-weight update as two calls (mp8_gemm_fp8, "
                         "mp8_sgd_update_fp16_sr) instead of one mp8_wgrad_update_fp16_sr")
    ap.add_argument("--separate-quantize", action="store_true",
                    help="activations quantised by a call of their own (mp8_quantize_e5m2, "
                         "mp8_gemm_fp8) instead of inside the forward GEMM (mp8_quantize_gemm_fwd_fp8)")
    ap.add_argument("--two-streams", action="store_true",
                    help="error path (Q(dY), backward data) on a second stream beside the activation path")
    ap.add_argument("--batch-quantize", action="store_true",
                    help="run the two Q nodes of the step as one mp8_quantize_e5m2_batch launch")
    ap.add_argument("--kernel-reps", type=int, default=50,
                    help="back-to-back launches per graph in the per-kernel timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-conv-step", action="store_true",
                    help="skip the implicit-GEMM convolution form of the same layer")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time the vendor library's GEMM (torch._scaled_mm, e5m2 in and out) beside every "
                         "GEMM row of the all_configs table, for context")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the kernel-level table over the GEMM shapes of all configurations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device-to-device copy of 1 GiB ten times (the "
                         "known-size kernel that scales the HBM traffic counters), then exit")
    return ap.parse_args()


class StatsRing:
    """Every step accumulates its overflow statistics into a slot of its own (16 bytes); the
    slots are cleared together, by one small fill kernel (no memset node, so the steps can be
    captured), each time the ring wraps around: one clearing launch per `size` steps instead of
    one per step.  The host reads a step's slot at its leisure (the loss scaler needs the count
    only before the next update of the scale)."""

    def __init__(self, torch, size=10):
        self.slots = torch.zeros((size, 4), dtype=torch.int32, device="cuda")
        self.size, self.index = size, -1

    def resize(self, size):
        """Start over with `size` slots (the next step is the first of a ring period)."""
        self.slots = self.slots.new_zeros((size, 4))
        self.size, self.index = size, -1

    def advance(self):
        self.index += 1
        if self.index % self.size == 0:
            self.slots.zero_()

    def current(self):
        return self.slots[max(self.index, 0) % self.size]


class Workload:
    """Device buffers and launch closures for the configs[1] layer."""

    def __init__(self, mp8, torch, lay, batch_quantize=False, fused_update=False, fused_quantize=False,
                 two_streams=False):
        self.mp8, self.torch = mp8, torch
        M, N, K = lay.M, lay.N, lay.K
        self.M, self.N, self.K = M, N, K
        dev = "cuda"
        u8 = torch.uint8
        self.X = torch.from_numpy(lay.X).to(dev)
        self.W = torch.from_numpy(lay.W).to(dev)
        self.dY = torch.from_numpy(lay.dY).to(dev)
        self.W16 = torch.from_numpy(lay.W.astype(np.float16)).to(dev)
        self.X8 = torch.empty((M, K), dtype=u8, device=dev)
        self.W8 = torch.empty((K, N), dtype=u8, device=dev)
        self.E8 = torch.empty((M, N), dtype=u8, device=dev)
        self.Y8 = torch.empty((M, N), dtype=u8, device=dev)
        self.dX8 = torch.empty((M, K), dtype=u8, device=dev)
        self.G8 = torch.empty((K, N), dtype=u8, device=dev)
        self.ring = StatsRing(torch)
        ws = max(mp8.gemm_fp8_workspace_bytes(op, M, N, K) for op in (mp8.FWD, mp8.BWD_DATA, mp8.WGRAD))
        self.ws = torch.empty(max(ws, 16), dtype=u8, device=dev)
        self.step_no = 0
        mp8_ = mp8
        # Every GEMM reads the row-major tensors as their producers wrote them; no transposed
        # copy of anything exists.  The 8-bit weights of a step are written by the previous
        # step's update (its w8_out), i.e. the Q node on the weights is fused into the update.
        self.kernels = [
            # name, closure, algorithmic bytes, flops, bound
            ("quantize_X", lambda: mp8_.quantize_e5m2(self.X, self.X8), 5 * M * K, 0, "hbm"),
            ("quantize_dY", lambda: mp8_.quantize_e5m2(self.dY, self.E8, scale=LOSS_SCALE,
                                                       stats=self.stats), 5 * M * N, 0, "hbm"),
            ("gemm_fwd", lambda: mp8_.gemm_fp8(mp8_.FWD, M, N, K, self.X8, self.W8, out8=self.Y8,
                                               workspace=self.ws, flags=mp8_.FLAG_B_CONTRACTION_MAJOR),
             M * K + K * N + M * N, 2 * M * N * K, "mfma"),
            ("gemm_bwd_data", lambda: mp8_.gemm_fp8(mp8_.BWD_DATA, M, N, K, self.E8, self.W8,
                                                    out8=self.dX8, workspace=self.ws),
             M * N + K * N + M * K, 2 * M * N * K, "mfma"),
            ("gemm_wgrad", lambda: mp8_.gemm_fp8(mp8_.WGRAD, M, N, K, self.X8, self.E8, out8=self.G8,
                                                 workspace=self.ws, flags=mp8_.FLAG_CONTRACTION_MAJOR),
             M * K + M * N + K * N, 2 * M * N * K, "mfma"),
            ("sgd_update", self._update, 6 * K * N, 0, "hbm"),
        ]
        if fused_update:
            # Figure 1b in one call: the pass that rounds the weight gradient also updates the
            # master weights and writes the next step's 8-bit weights
            self.kernels[-2:] = [("gemm_wgrad_update", self._wgrad_update,
                                  M * K + M * N + K * N + 6 * K * N, 2 * M * N * K, "mfma")]
        if fused_quantize and not batch_quantize:
            # Figure 1a's Q node on the activations inside the forward GEMM: X is read once, rounded,
            # written as X8 for the weight gradient and multiplied from the codes in LDS
            fwd = ("quantize_X_gemm_fwd", lambda: mp8_.quantize_gemm_fwd_fp8(
                M, N, K, self.X, self.X8, self.W8, out8=self.Y8, workspace=self.ws),
                5 * M * K + K * N + M * N, 2 * M * N * K, "hbm")
            self.kernels = [k for k in self.kernels if k[0] not in ("quantize_X", "gemm_fwd")]
            self.kernels.insert(1, fwd)
        if batch_quantize:
            # both Q nodes of the step in one launch (measured: no faster inside the step)
            self.kernels[:2] = [("quantize_X_dY", lambda: mp8_.quantize_e5m2_batch([
                dict(src=self.X, dst=self.X8),
                dict(src=self.dY, dst=self.E8, scale=LOSS_SCALE, stats=self.stats)]),
                5 * M * K + 5 * M * N, 0, "hbm")]
        if not batch_quantize:
            # error path first, then the activation path: the forward GEMM and the weight gradient
            # find X8 freshly written (measured 0.7 us per step against the order of the list above)
            by_name = {k[0]: k for k in self.kernels}
            order = ["quantize_dY", "gemm_bwd_data", "quantize_X", "gemm_fwd", "quantize_X_gemm_fwd"]
            order = [n for n in order if n in by_name]
            self.kernels = [by_name[n] for n in order] + [k for k in self.kernels if k[0] not in order]
        # the weights of the first step: Q(W16), outside the timed region
        mp8_.quantize_e5m2(self.W16.view(K, N), self.W8)
        self.side = torch.cuda.Stream() if two_streams else None

    def _wgrad_update(self):
        self.step_no += 1
        mp8 = self.mp8
        mp8.wgrad_update_fp16_sr(self.M, self.N, self.K, self.X8, self.E8, self.W16, LR, 1.0 / LOSS_SCALE,
                                 g8_out=self.G8, flags=mp8.FLAG_CONTRACTION_MAJOR, w_round=mp8.SR,
                                 w_seed=0x1905_1233_4000_0002, w_offset=self.step_no,
                                 skip_if_nonzero=self.stats[1:2], w8_out=self.W8, workspace=self.ws)

    def _update(self):
        # every step draws from its own Philox offset; the overflow count of the error tensor
        # (left in stats by quantize_dY) makes the kernel skip the step without a host round
        # trip; the new master weights are also written as the next step's 8-bit weights
        self.step_no += 1
        self.mp8.sgd_update_fp16_sr(self.W16, self.G8, LR, 1.0 / LOSS_SCALE, round=self.mp8.SR,
                                    seed=0x1905_1233_4000_0002, offset=self.step_no,
                                    skip_if_nonzero=self.stats[1:2], w8_out=self.W8)

    @property
    def stats(self):
        return self.ring.current()

    def step(self):
        self.ring.advance()
        if self.side is None:
            for _, fn, _, _, _ in self.kernels:
                fn()
            return
        # the error path beside the activation path; both need the previous step's weights, the
        # weight gradient needs both
        torch = self.torch
        main = torch.cuda.current_stream()
        error_path = [k for k in self.kernels if k[0] in ("quantize_dY", "gemm_bwd_data")]
        rest = [k for k in self.kernels if k not in error_path]
        self.side.wait_stream(main)
        with torch.cuda.stream(self.side):
            for _, fn, _, _, _ in error_path:
                fn()
        for _, fn, _, _, _ in rest[:-1]:
            fn()
        main.wait_stream(self.side)
        rest[-1][1]()


class ConvWorkload:
    """The same layer as the 3x3 convolution it stands for (batch 32, 28x28, 128 -> 128 channels),
    run as an implicit GEMM: activations and errors live channels-last on the zero-padded pixel
    grid ([28800, 128] instead of the lowered [25088, 1152]); a filter tap is a row shift of the
    operand, so nothing is lowered and nothing is transposed."""

    def __init__(self, mp8, torch, lay):
        self.mp8, self.torch = mp8, torch
        B, H, W, C = 32, 28, 28, 128
        self.dims = (B, H, W, C, C)
        dev, u8 = "cuda", torch.uint8
        P = mp8.conv_prows(B, H, W)
        n = B * (H + 2) * (W + 2)
        from paper_1905_12334_amd import workloads

        def padded(x):      # [B,H,W,C] host FP32 -> [P, C] device FP32 with zero padding
            xp = np.zeros((B, H + 2, W + 2, C), np.float32)
            xp[:, 1:-1, 1:-1] = x
            out = torch.zeros((P, C), dtype=torch.float32, device=dev)
            out[:n] = torch.from_numpy(xp.reshape(-1, C)).to(dev)
            return out
        self.X = padded(workloads.relu_normal(2, 10, (B, H, W, C)))
        self.dY = padded(workloads.normal(2, 12, (B, H, W, C), 1e-4))
        w = workloads.normal(2, 11, (3, 3, C, C), float(np.sqrt(2.0 / (9 * C))))
        self.W16 = torch.from_numpy(w.astype(np.float16).reshape(-1)).to(dev)
        self.X8, self.E8 = mp8.conv_buffer(P, C, W), mp8.conv_buffer(P, C, W)
        self.W8 = torch.empty((9 * C, C), dtype=u8, device=dev)
        self.Y8 = torch.empty((P, C), dtype=u8, device=dev)
        self.dX8 = torch.empty((P, C), dtype=u8, device=dev)
        self.G8 = torch.empty((9 * C, C), dtype=u8, device=dev)
        self.ring = StatsRing(torch)
        ws = max(mp8.conv3x3_fp8_workspace_bytes(op, *self.dims) for op in (mp8.FWD, mp8.BWD_DATA, mp8.WGRAD))
        self.ws = torch.empty(max(ws, 16), dtype=u8, device=dev)
        self.step_no = 0
        flops = 2 * B * H * W * 9 * C * C
        conv = lambda op, a, b, out: mp8.conv3x3_fp8(op, *self.dims, a, b, out8=out, workspace=self.ws)
        self.kernels = [
            ("quantize_X", lambda: mp8.quantize_e5m2(self.X, self.X8), 5 * P * C, 0, "hbm"),
            ("quantize_dY", lambda: mp8.quantize_e5m2(self.dY, self.E8, scale=LOSS_SCALE, stats=self.stats),
             5 * P * C, 0, "hbm"),
            ("conv_fwd", lambda: conv(mp8.FWD, self.X8, self.W8, self.Y8), 2 * P * C + 9 * C * C, flops, "mfma"),
            ("conv_bwd_data", lambda: conv(mp8.BWD_DATA, self.E8, self.W8, self.dX8),
             2 * P * C + 9 * C * C, flops, "mfma"),
            # weight gradient, its rounding and the master-weight update in one call
            ("conv_wgrad_update", self._wgrad_update, 2 * P * C + 9 * C * C + 6 * 9 * C * C, flops, "mfma"),
        ]
        mp8.quantize_e5m2(self.W16.view(9 * C, C), self.W8)

    def _wgrad_update(self):
        self.step_no += 1
        mp8 = self.mp8
        mp8.conv3x3_wgrad_update_fp16_sr(*self.dims, self.X8, self.E8, self.W16, LR, 1.0 / LOSS_SCALE,
                                         g8_out=self.G8, w_round=mp8.SR, w_seed=0x1905_1233_4000_0003,
                                         w_offset=self.step_no, skip_if_nonzero=self.stats[1:2],
                                         w8_out=self.W8, workspace=self.ws)

    @property
    def stats(self):
        return self.ring.current()

    def step(self):
        self.ring.advance()
        for _, fn, _, _, _ in self.kernels:
            fn()


def kernel_table(kernels, times_ms, traffic=None):
    out = []
    for (name, _, nbytes, flops, bound), ms in zip(kernels, times_ms):
        if bound == "mfma":
            achieved, peak, unit = flops / (ms * 1e-3) / 1e12, FP8_PEAK_TFLOPS, "TFLOP/s"
        else:
            achieved, peak, unit = nbytes / (ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        out.append({"kernel": name, "bound": bound, "us": ms * 1e3, "achieved": achieved,
                    "peak": peak, "unit": unit, "frac": achieved / peak,
                    "alg_bytes": nbytes, "flops": flops,
                    "hbm_gbs": nbytes / (ms * 1e-3) / 1e9,
                    "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "traffic": (traffic or {}).get(name)})
    return out


def time_steps(torch, wl, steps, launch):
    """Times exactly `steps` steps between two events on the current stream; returns ms/step."""
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if launch == "eager":
        torch.cuda.synchronize()
        s.record()
        for _ in range(steps):
            wl.step()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / steps
    per_graph = max(d for d in range(1, 11) if steps % d == 0)
    wl.ring.resize(per_graph)          # one graph = one period of the statistics ring
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(per_graph):
            wl.step()
    graph.replay()
    torch.cuda.synchronize()
    s.record()
    for _ in range(steps // per_graph):
        graph.replay()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / steps


def time_kernels(torch, wl, reps):
    """Average duration of every kernel of the step: each one is captured `reps` times back to
    back in a HIP graph of its own and the replay is timed with events on the replay stream, so
    the figure is device time per launch (launch gaps of about a microsecond included), free of
    host launch cost.  Returns ms per launch."""
    out = []
    for _, fn, _, _, _ in wl.kernels:
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(reps):
                fn()
        graph.replay()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        graph.replay()
        graph.replay()
        e.record()
        torch.cuda.synchronize()
        out.append(s.elapsed_time(e) / (2 * reps))
    return out


def graph_time_us(torch, fn, reps=20):
    """Device time per call of fn, from a captured graph of `reps` back-to-back calls."""
    fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(reps):
            fn()
    graph.replay()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    graph.replay()
    graph.replay()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / (2 * reps) * 1e3


def all_configs_report(mp8, torch, vendor_gemm=False):
    """Kernel-level throughput on the GEMM shapes of every workload configuration (plus two large
    shapes that show what the main loop reaches when nothing else binds) and on the streaming
    kernels at a size far beyond the caches.  Operands are the codes of standard-normal values (the
    Q node's own output): the time of an MFMA-bound GEMM depends on its operand values, because the
    chip lowers its clock under the power the matrix cores draw, so low-entropy operands would
    flatter the large shapes (their rows with all-zero operands show the rate at which the loop can
    issue, not a rate any training tensor sees).  Parity on these shapes is the business of the
    tests, not of this table."""
    dev = "cuda"
    rows = []

    def codes(r, c, zeros=False):
        if zeros:
            return torch.zeros((r, c), dtype=torch.uint8, device=dev)
        out = torch.empty((r, c), dtype=torch.uint8, device=dev)
        mp8.quantize_e5m2(torch.empty((r, c), dtype=torch.float32, device=dev).normal_(), out)
        torch.cuda.synchronize()
        return out
    gemms = [("configs[0] fwd", mp8.FWD, 256, 256, 256, mp8.RNE),
             ("configs[1] fwd", mp8.FWD, 25088, 128, 1152, mp8.RNE),
             ("configs[1] bwd_data", mp8.BWD_DATA, 25088, 128, 1152, mp8.RNE),
             ("configs[1] wgrad", mp8.WGRAD, 25088, 128, 1152, mp8.RNE),
             ("configs[2] ffn1 fwd", mp8.FWD, 4096, 2048, 512, mp8.RNE),
             ("configs[2] ffn1 bwd_data", mp8.BWD_DATA, 4096, 2048, 512, mp8.RNE),
             ("configs[2] ffn1 wgrad", mp8.WGRAD, 4096, 2048, 512, mp8.RNE),
             ("configs[2] ffn2 fwd", mp8.FWD, 4096, 512, 2048, mp8.RNE),
             ("configs[2] ffn2 bwd_data", mp8.BWD_DATA, 4096, 512, 2048, mp8.RNE),
             ("configs[2] ffn2 wgrad", mp8.WGRAD, 4096, 512, 2048, mp8.RNE),
             ("configs[3] fwd (one timestep)", mp8.FWD, 128, 4096, 2048, mp8.RNE),
             ("configs[3] bwd_data (one timestep)", mp8.BWD_DATA, 128, 4096, 2048, mp8.RNE),
             ("configs[3] wgrad (50 timesteps stacked)", mp8.WGRAD, 6400, 4096, 2048, mp8.RNE),
             ("configs[4] wgrad, SR epilogue", mp8.WGRAD, 16384, 4096, 1024, mp8.SR),
             ("large 4096x4096x16384 fwd", mp8.FWD, 4096, 4096, 16384, mp8.RNE),
             ("large 8192^3 fwd", mp8.FWD, 8192, 8192, 8192, mp8.RNE),
             ("large 4096x4096x16384 fwd, all-zero operands", mp8.FWD, 4096, 4096, 16384, mp8.RNE),
             ("large 8192^3 fwd, all-zero operands", mp8.FWD, 8192, 8192, 8192, mp8.RNE)]
    for name, op, M, N, K, rnd in gemms:
        r, c, kc = {mp8.FWD: (M, N, K), mp8.BWD_DATA: (M, K, N), mp8.WGRAD: (K, N, M)}[op]
        a, b = codes(r, kc, "all-zero" in name), codes(c, kc, "all-zero" in name)
        out = torch.empty((r, c), dtype=torch.uint8, device=dev)
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(op, M, N, K), 16), dtype=torch.uint8, device=dev)
        us = graph_time_us(torch, lambda: mp8.gemm_fp8(op, M, N, K, a, b, out8=out, round=rnd, seed=5,
                                                       offset=1, workspace=ws))
        flops, nbytes = 2.0 * M * N * K, r * kc + c * kc + r * c
        rows.append({"kernel": "gemm_fp8", "case": name, "us": us, "tflops": flops / us / 1e6,
                     "frac_mfma_peak": flops / us / 1e6 / FP8_PEAK_TFLOPS,
                     "alg_gbs": nbytes / us / 1e3, "flop_per_byte": flops / nbytes})
        if vendor_gemm and hasattr(torch, "float8_e5m2") and hasattr(torch, "_scaled_mm"):
            # context, not a target: the vendor library's GEMM on the same codes, same box, same minute
            try:
                one = torch.ones((), device=dev)
                af, bf = a.view(torch.float8_e5m2), b.view(torch.float8_e5m2).t()
                vendor = lambda: torch._scaled_mm(af, bf, scale_a=one, scale_b=one, out_dtype=torch.float8_e5m2)
                for _ in range(3):  # lets the library pick its kernel and workspace before the capture
                    vendor()
                torch.cuda.synchronize()
                vus = graph_time_us(torch, vendor)
                rows.append({"kernel": "torch._scaled_mm (vendor library, for context)", "case": name, "us": vus,
                             "tflops": flops / vus / 1e6, "frac_mfma_peak": flops / vus / 1e6 / FP8_PEAK_TFLOPS})
            except Exception as exc:  # the table does not depend on it
                torch.cuda.synchronize()
                rows.append({"kernel": "torch._scaled_mm (vendor library, for context)", "case": name,
                             "error": repr(exc)[:200]})
        del a, b, out, ws
    # configs[3] weight gradient the naive way: one call per timestep accumulating into an FP32
    # tensor (acc_mode 2), 50 calls for what the stacked contraction above does in one
    M, N, K = 128, 4096, 2048
    a, b = codes(K, M), codes(N, M)
    acc = torch.zeros((K, N), dtype=torch.float32, device=dev)
    out = torch.empty((K, N), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device=dev)
    us = graph_time_us(torch, lambda: mp8.gemm_fp8(mp8.WGRAD, M, N, K, a, b, out8=out, acc=acc, acc_mode=2,
                                                   workspace=ws), 10)
    rows.append({"kernel": "gemm_fp8", "case": "configs[3] wgrad, one timestep accumulated in FP32 "
                 "(acc_mode 2); x50 for all timesteps", "us": us, "tflops": 2.0 * M * N * K / us / 1e6,
                 "frac_mfma_peak": 2.0 * M * N * K / us / 1e6 / FP8_PEAK_TFLOPS,
                 "alg_gbs": (K * M + N * M + 9 * K * N) / us / 1e3,
                 "flop_per_byte": 2.0 * M * N * K / (K * M + N * M + 9 * K * N)})
    del a, b, acc, out, ws
    # configs[4] as a whole: weight gradient from the row-major X8 [tokens, 1024] and E8 [tokens, 4096],
    # rounded stochastically to 8 bits, then the FP16 master-weight step with stochastic rounding
    # (mp8_wgrad_update_fp16_sr; lr 1e-3, loss scale 2^14)
    M, N, K = 16384, 4096, 1024
    x8, e8 = codes(M, K), codes(M, N)
    w16 = torch.empty(K * N, dtype=torch.float16, device=dev).normal_(0, 0.02)
    g8 = torch.empty(K * N, dtype=torch.uint8, device=dev)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device=dev)
    us = graph_time_us(torch, lambda: mp8.wgrad_update_fp16_sr(
        M, N, K, x8, e8, w16, 1e-3, 2.0 ** -14, g8_out=g8, g_round=mp8.SR, flags=mp8.FLAG_CONTRACTION_MAJOR,
        g_seed=5, g_offset=1, w_round=mp8.SR, w_seed=6, w_offset=1, workspace=ws), 10)
    rows.append({"kernel": "wgrad_update_fp16_sr", "case": "configs[4] wgrad (SR) + FP16 SR update, row-major operands",
                 "us": us, "tflops": 2.0 * M * N * K / us / 1e6,
                 "frac_mfma_peak": 2.0 * M * N * K / us / 1e6 / FP8_PEAK_TFLOPS,
                 "alg_gbs": (M * K + M * N + 6 * K * N) / us / 1e3,
                 "flop_per_byte": 2.0 * M * N * K / (M * K + M * N + 6 * K * N)})
    del x8, e8, w16, g8, ws
    n = 1 << 28
    src = torch.empty((1 << 14, 1 << 14), dtype=torch.float32, device=dev).normal_()
    d8 = torch.empty((1 << 14, 1 << 14), dtype=torch.uint8, device=dev)
    for rnd, rn in ((mp8.RNE, "RNE"), (mp8.SR, "SR")):
        us = graph_time_us(torch, lambda: mp8.quantize_e5m2(src, d8, round=rnd, seed=1, offset=2), 5)
        rows.append({"kernel": "quantize_e5m2", "case": f"2^28 elements, {rn}", "us": us,
                     "alg_gbs": 5.0 * n / us / 1e3, "frac_hbm_peak": 5.0 * n / us / 1e3 / HBM_PEAK_GBS})
    w16 = torch.empty(n, dtype=torch.float16, device=dev).normal_(0, 0.02)
    g8 = d8.view(-1)
    for rnd, rn in ((mp8.RNE, "RNE"), (mp8.SR, "SR")):
        us = graph_time_us(torch, lambda: mp8.sgd_update_fp16_sr(w16, g8, LR, 1.0 / LOSS_SCALE, round=rnd,
                                                                 seed=1, offset=3), 5)
        rows.append({"kernel": "sgd_update_fp16_sr", "case": f"2^28 elements, {rn}", "us": us,
                     "alg_gbs": 5.0 * n / us / 1e3, "frac_hbm_peak": 5.0 * n / us / 1e3 / HBM_PEAK_GBS})
    # many small tensors (the weights of eight layers of configs[1]): eight launches or one
    small = [torch.empty(1152 * 128, dtype=torch.float32, device=dev).normal_(0, 0.04) for _ in range(8)]
    small8 = [torch.empty(1152 * 128, dtype=torch.uint8, device=dev) for _ in range(8)]
    us = graph_time_us(torch, lambda: [mp8.quantize_e5m2(x.view(1, -1), y) for x, y in zip(small, small8)], 5)
    rows.append({"kernel": "quantize_e5m2", "case": "8 tensors of 147456 elements, 8 launches", "us": us,
                 "alg_gbs": 5.0 * 8 * 147456 / us / 1e3, "frac_hbm_peak": 5.0 * 8 * 147456 / us / 1e3 / HBM_PEAK_GBS})
    us = graph_time_us(torch, lambda: mp8.quantize_e5m2_batch([dict(src=x, dst=y) for x, y in zip(small, small8)]), 5)
    rows.append({"kernel": "quantize_e5m2_batch", "case": "8 tensors of 147456 elements, 1 launch", "us": us,
                 "alg_gbs": 5.0 * 8 * 147456 / us / 1e3, "frac_hbm_peak": 5.0 * 8 * 147456 / us / 1e3 / HBM_PEAK_GBS})
    del small, small8
    # optimizers with FP32 state: 13 (momentum) and 21 (ADAM) bytes per element
    nm = 1 << 27
    st0 = torch.zeros(nm, dtype=torch.float32, device=dev)
    st1 = torch.zeros(nm, dtype=torch.float32, device=dev)
    us = graph_time_us(torch, lambda: mp8.sgd_momentum_fp16_sr(w16[:nm], st0, g8[:nm], LR, 1.0 / LOSS_SCALE,
                                                               0.9, 1e-4, round=mp8.SR, seed=1, offset=4), 5)
    rows.append({"kernel": "sgd_momentum_fp16_sr", "case": "2^27 elements, SR", "us": us,
                 "alg_gbs": 13.0 * nm / us / 1e3, "frac_hbm_peak": 13.0 * nm / us / 1e3 / HBM_PEAK_GBS})
    us = graph_time_us(torch, lambda: mp8.adam_fp16_sr(w16[:nm], st0, st1, g8[:nm], LR, 1.0 / LOSS_SCALE, 10,
                                                       weight_decay=1e-4, round=mp8.SR, seed=1, offset=5), 5)
    rows.append({"kernel": "adam_fp16_sr", "case": "2^27 elements, SR", "us": us,
                 "alg_gbs": 21.0 * nm / us / 1e3, "frac_hbm_peak": 21.0 * nm / us / 1e3 / HBM_PEAK_GBS})
    del src, d8, w16, st0, st1
    x = torch.empty((100352, 1152), dtype=torch.float32, device=dev).normal_()
    q, qt = torch.empty((100352, 1152), dtype=torch.uint8, device=dev), torch.empty((1152, 100352), dtype=torch.uint8, device=dev)
    us = graph_time_us(torch, lambda: mp8.quantize_e5m2(x, q, qt), 5)
    rows.append({"kernel": "quantize_e5m2", "case": "with transposed copy, 100352x1152 (4x configs[1] X), RNE",
                 "us": us, "alg_gbs": 6.0 * x.numel() / us / 1e3,
                 "frac_hbm_peak": 6.0 * x.numel() / us / 1e3 / HBM_PEAK_GBS})
    return rows


def calibrate_copy(torch):
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 256)
    dst = torch.empty_like(src)
    for _ in range(10):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibrate_copy": {"bytes_read": n, "bytes_written": n, "launches": 10}}))


def cpu_baseline(lay):
    """The CPU oracle, as it stands, on full steps of the same workload (about 10-20 s)."""
    import oracle
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    w16 = lay.W.astype(np.float16).view(np.uint16).reshape(-1)

    def one_step():
        X8, X8t = oracle.quantize_e5m2(lay.X, want_t=True)
        W8, W8t = oracle.quantize_e5m2(lay.W, want_t=True)
        E8, E8t = oracle.quantize_e5m2(lay.dY, scale=LOSS_SCALE, want_t=True)
        tq = time.perf_counter()
        fwd, _ = oracle.gemm_ref(X8, W8t, want_abs=False)
        bwd, _ = oracle.gemm_ref(E8, W8, want_abs=False)
        wg, _ = oracle.gemm_ref(X8t, E8t, want_abs=False)
        tg = time.perf_counter()
        oracle.round_ref_e5m2(fwd)
        oracle.round_ref_e5m2(bwd)
        G8 = oracle.round_ref_e5m2(wg)
        oracle.sgd_update_fp16(w16, G8.reshape(-1), LR, 1.0 / LOSS_SCALE, mode=oracle.SR, seed=1,
                               offset=1)
        return tg - tq

    t0 = time.perf_counter()
    gemm_s = [one_step()]
    first = time.perf_counter() - t0
    reps = max(1, min(25, int(15.0 / max(first, 1e-3))))
    for _ in range(reps - 1):
        gemm_s.append(one_step())
    total = time.perf_counter() - t0
    step_s = total / reps
    flops = 3 * 2.0 * lay.M * lay.N * lay.K
    return {
        "value": flops / step_s / 1e12,
        "unit": "TFLOP/s",
        "cores": threads,
        "kind": "oracle",
        "sample": (f"{reps} full step(s) of the same workload (all three GEMMs over every output "
                   f"row, quantize, update), {total:.1f} s of CPU work; GEMMs alone "
                   f"{flops / (sum(gemm_s) / reps) / 1e9:.1f} GFLOP/s"),
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no collectives, no sharding "
              "are part of it)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_1905_12334_amd as mp8
    from paper_1905_12334_amd import workloads
    mp8.lib()   # raises if the HIP library is not built: there is no fallback

    if args.calibrate_copy:
        calibrate_copy(torch)
        return

    props = torch.cuda.get_device_properties(0)
    lay = workloads.config2()
    wl = Workload(mp8, torch, lay, batch_quantize=args.batch_quantize, fused_update=not args.separate_update,
                  fused_quantize=not args.separate_quantize, two_streams=args.two_streams)
    for _ in range(args.warmup):
        wl.step()
    ms_per_step = time_steps(torch, wl, args.steps, args.launch)
    nonfinite = mp8.read_stats(wl.stats)[1]

    gemm_flops = 3 * 2.0 * lay.M * lay.N * lay.K
    value = gemm_flops / (ms_per_step * 1e-3) / 1e12

    kernels = kernel_table(wl.kernels, time_kernels(torch, wl, args.kernel_reps), MEASURED_TRAFFIC_BYTES)
    dom = max(kernels, key=lambda k: k["us"])
    roofline = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"],
                "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"],
                "traffic": MEASURED_TRAFFIC_BYTES.get(dom["kernel"])}
    gemm_us = sum(k["us"] for k in kernels if k["flops"] > 0)  # incl. a quantize fused into a GEMM

    out = {
        "metric": "FP8 GEMM TFLOP/s (E5M2 in, FP32 acc, FP8 out) and % of MFMA FP8 peak",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8_e5m2 x fp8_e5m2 -> f32",
        "data": "synthetic",
        "config": {"workload": "configs[1]: ResNet-50-style 3x3 conv as GEMM, M=25088 N=128 K=1152, "
                               "quantize X and dY + fwd + bwd_data + wgrad + FP16 SR update emitting the next 8-bit weights, loss scale 2^12",
                   "M": lay.M, "N": lay.N, "K": lay.K, "launch": args.launch},
        "pct_of_fp8_peak_whole_step": 100.0 * value / FP8_PEAK_TFLOPS,
        "gemm_only_tflops": gemm_flops / (gemm_us * 1e-6) / 1e12,
        "overflow_count_last_step": nonfinite,
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "max_clock_mhz": getattr(props, "clock_rate", 0) / 1e3 or None,
                   "memory_gib": round(props.total_memory / 2 ** 30, 1)},
        "roofline": roofline,
        "kernels": kernels,
    }
    del wl
    torch.cuda.empty_cache()
    if not args.no_conv_step:
        # the same layer without the lowering: 3x3 convolution as an implicit GEMM
        try:
            cw = ConvWorkload(mp8, torch, lay)
            for _ in range(args.warmup):
                cw.step()
            conv_ms = time_steps(torch, cw, args.steps, args.launch)
            out["conv_step"] = {
                "workload": "the configs[1] layer as an implicit-GEMM 3x3 convolution on zero-padded "
                            "channels-last tensors (no lowered operand): quantize X and dY, conv "
                            "fwd + bwd_data + wgrad, FP16 SR update emitting the next 8-bit weights",
                "ms_per_step": conv_ms,
                "value": gemm_flops / (conv_ms * 1e-3) / 1e12,
                "unit": "TFLOP/s (useful flops of the unpadded layer, 3 * 2*M*N*K)",
                "overflow_count_last_step": mp8.read_stats(cw.stats)[1],
                "kernels": kernel_table(cw.kernels, time_kernels(torch, cw, args.kernel_reps)),
            }
            del cw
            torch.cuda.empty_cache()
        except Exception as exc:
            out["conv_step"] = {"error": repr(exc)}
    if not args.no_all_configs:
        try:
            out["all_configs"] = all_configs_report(mp8, torch, args.vendor_gemm)
        except Exception as exc:  # the table is extra evidence; the line above it stands on its own
            out["all_configs"] = {"error": repr(exc)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(lay)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
