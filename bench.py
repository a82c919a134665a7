#!/usr/bin/env python3
"""Benchmark of the 8-bit floating point training primitive on one MI355X.

The headline workload is the largest configuration that fits one GPU, configs[4]: the
Transformer-big weight gradient and master-weight update over 16384 tokens
(X [16384, 1024], dY [16384, 4096], W [1024, 4096]).  One "step" is one pass of the whole hot
path over one batch of synthetic input:

    Q(X) -> X8                                   FP32 -> (1,5,2), RNE
    Q(dY * 2^14) -> E8 (+ overflow statistics)   the loss scale applied by the Q node
    weight-grad  G8  = Q_SR(X8^T . E8)           contraction over the tokens, FP32 accumulation
                                                 on the matrix cores, ONE stochastic rounding
    update       W16 <- half_SR(W16 - lr * G8 / 2^14),  W8 <- Q(W16) for the next step
                 (skipped on the device if the statistics hold an overflow)

Every tensor exists once, row-major, as its producer wrote it: the GEMM reads X8 [tokens, 1024]
and E8 [tokens, 4096] contraction-major through transposing LDS reads.  Inputs are resident in
HBM before the timed region; by default the steps rotate over several input sets so that no
step finds its FP32 inputs in the 256 MB memory-side cache (`--warm` replays one set).

Prints ONE JSON line: `value` is the GEMM work of a step (2*M*N*K flop) divided by the time of
the whole step (steps are replayed from a captured HIP graph unless --launch eager); `roofline`
describes the kernel that takes the largest share of the step (its duration measured with events
around back-to-back launches on the launch stream); `kernels` lists every kernel of the step with
its own roofline, warm (same buffers every launch) and cold (buffers rotating through more than
twice the cache); `configs1_step` and `conv_step` are the configs[1] layer (three GEMMs, as a
lowered GEMM and as the 3x3 convolution it stands for) timed the same way; `all_configs` is a
kernel-level table over the GEMM shapes of all five configurations, the streaming kernels at
sizes far beyond the caches and plain copies of matching read:write ratio; `cpu_baseline` is the
CPU oracle timed on this host on a bounded sample of the headline workload.
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
LOSS_SCALE = 2.0 ** 12         # configs[1]
LR = 1e-3
CACHE_BYTES = 256 << 20        # memory-side cache; "cold" rotates through more than twice that
PROFILE_TRAFFIC = os.path.join(ROOT, "profiles", "bench_step_cfg5_hbm_traffic.txt")


def profiled_traffic():
    """HBM bytes per launch of the step's kernels as the FETCH_SIZE / WRITE_SIZE counters gave them
    in the profiling runs kept under profiles/ (NOT measured in this run: counters need a run of
    their own).  The summary file carries one line `TRAFFIC_BYTES {json}`."""
    try:
        for line in open(PROFILE_TRAFFIC):
            if line.startswith("TRAFFIC_BYTES "):
                return json.loads(line[len("TRAFFIC_BYTES "):])
    except (OSError, ValueError):
        pass
    return {}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=420)
    ap.add_argument("--warmup", type=int, default=28)
    ap.add_argument("--warm", action="store_true",
                    help="every step works on the same input buffers (what fits stays in the 256 MB cache); "
                         "default: the steps rotate over input sets (--cold)")
    ap.add_argument("--cold", action="store_true", help="the default, spelled out: inputs rotate over sets")
    ap.add_argument("--no-configs1-step", action="store_true",
                    help="skip the configs[1] layer (three GEMMs per step, lowered form)")
    ap.add_argument("--cpu-seconds", type=float, default=8.0,
                    help="CPU time budget of each of the two oracle baselines (1 thread, all threads)")
    ap.add_argument("--launch", choices=("graph", "eager"), default="graph",
                    help="how the timed steps are launched: replay of a captured HIP graph "
                         "(default) or one Python call per kernel")
    ap.add_argument("--separate-update", action="store_true",
                    help="weight gradient and master-weight update as two calls (mp8_gemm_fp8, "
                         "mp8_sgd_update_fp16_sr) instead of one mp8_wgrad_update_fp16_sr (both workloads)")
    ap.add_argument("--separate-quantize", action="store_true",
                    help="configs[1] step: activations quantised by a call of their own (mp8_quantize_e5m2, "
                         "mp8_gemm_fp8) instead of inside the forward GEMM (mp8_quantize_gemm_fwd_fp8)")
    ap.add_argument("--two-streams", action="store_true",
                    help="configs[1] step: error path (Q(dY), backward data) on a second stream beside the activation path")
    ap.add_argument("--batch-quantize", action="store_true",
                    help="configs[1] step: run its two Q nodes as one mp8_quantize_e5m2_batch launch")
    ap.add_argument("--kernel-reps", type=int, default=50,
                    help="back-to-back launches per graph in the per-kernel timing")
    ap.add_argument("--steps-only", action="store_true",
                    help="headline workload only, and of it only whole steps (the timed ones and the ones with an "
                         "event between consecutive kernels): no stand-alone per-kernel loops, no clock sampling -- the "
                         "run to put under a tracer, whose per-kernel averages are then in-step durations")
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


class Cfg5Workload:
    """configs[4]: Transformer-big weight gradient and master-weight update over 16384 tokens.

    A launch closure takes the index i of the step (or of the launch, when a kernel is timed on
    its own) and works on buffer set i modulo the number of sets: one set in warm mode; in cold
    mode enough sets that a buffer comes round again only after more than twice the 256 MB cache
    has passed through.  The master weights of the step are one tensor (a training loop updates
    the same weights every step); only the stand-alone timing of the update kernel rotates them."""

    SEED_G, SEED_W = 0x1905_1233_4000_0004, 0x1905_1233_4000_0005

    def __init__(self, mp8, torch, lay, cold=True, fused_update=True):
        self.mp8, self.torch, self.cold = mp8, torch, cold
        M, N, K = lay.M, lay.N, lay.K            # tokens, d_out, d_in
        self.M, self.N, self.K = M, N, K
        self.scale, self.lr = float(lay.loss_scale), float(lay.extra["lr"])
        dev, u8, f32 = "cuda", torch.uint8, torch.float32

        def sets(nbytes_per_set):
            return max(2, -(-2 * CACHE_BYTES // nbytes_per_set) + 1) if cold else 1
        x0, e0 = torch.from_numpy(lay.X).to(dev), torch.from_numpy(lay.dY).to(dev)
        n_gemm = sets(M * K + M * N)              # what the GEMM reads per launch
        n_x = sets(5 * M * K)
        n_e = sets(5 * M * N)
        n_u = sets(6 * K * N)
        # FP32 inputs: the seeded tensors, and copies of them with rows rolled (same values, other
        # addresses) -- the statistics and the operand value distribution stay those of the workload
        self.X = [x0] + [x0.roll(i, 0).contiguous() for i in range(1, n_x)]
        self.dY = [e0] + [e0.roll(i, 0).contiguous() for i in range(1, n_e)]
        self.X8 = [torch.empty((M, K), dtype=u8, device=dev) for _ in range(max(n_gemm, n_x))]
        self.E8 = [torch.empty((M, N), dtype=u8, device=dev) for _ in range(max(n_gemm, n_e))]
        w16 = torch.from_numpy(lay.W.astype(np.float16)).to(dev).reshape(-1)
        self.W16 = [w16] + [w16.clone() for _ in range(1, n_u)]
        self.G8 = [torch.empty(K * N, dtype=u8, device=dev) for _ in range(n_u)]
        self.W8 = [torch.empty(K * N, dtype=u8, device=dev) for _ in range(n_u)]
        self.ring = StatsRing(torch)
        self.ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), K * N, 16), dtype=u8, device=dev)
        self.fused_update = fused_update
        self.step_no = 0
        self.plan = mp8.gemm_fp8_plan(mp8.WGRAD, M, N, K, mp8.FLAG_CONTRACTION_MAJOR)
        pick = lambda lst, i: lst[i % len(lst)]
        self.kernels = [
            # name, closure(i), algorithmic bytes, flops, bound
            ("quantize_X", lambda i: mp8.quantize_e5m2(pick(self.X, i), pick(self.X8, i)), 5 * M * K, 0, "hbm"),
            ("quantize_dY", lambda i: mp8.quantize_e5m2(pick(self.dY, i), pick(self.E8, i), scale=self.scale,
                                                        stats=self.stats), 5 * M * N, 0, "hbm"),
            ("gemm_wgrad_sr", lambda i: mp8.gemm_fp8(mp8.WGRAD, M, N, K, pick(self.X8, i), pick(self.E8, i),
                                                     out8=pick(self.G8, i), round=mp8.SR, seed=self.SEED_G,
                                                     offset=self.step_no, workspace=self.ws,
                                                     flags=mp8.FLAG_CONTRACTION_MAJOR),
             M * K + M * N + K * N, 2 * M * N * K, "mfma"),
            ("sgd_update_sr", lambda i: mp8.sgd_update_fp16_sr(pick(self.W16, i), pick(self.G8, i), self.lr,
                                                               1.0 / self.scale, round=mp8.SR, seed=self.SEED_W,
                                                               offset=self.step_no, skip_if_nonzero=self.stats[1:2],
                                                               w8_out=pick(self.W8, i)), 6 * K * N, 0, "hbm"),
        ]
        for i in range(len(self.X8)):            # every 8-bit operand set holds real codes from the start
            self.kernels[0][1](i)
        for i in range(len(self.E8)):
            self.kernels[1][1](i)
        torch.cuda.synchronize()

    @property
    def stats(self):
        return self.ring.current()

    def step(self):
        """One pass of the hot path.  The weight gradient and the update go through ONE call of the
        library (mp8_wgrad_update_fp16_sr) unless --separate-update; for this shape, whose
        contraction is not split, that call launches the GEMM with its rounding epilogue and the
        update kernel, i.e. the same two kernels as the two calls of the table."""
        self.ring.advance()
        i = self.step_no
        self.step_no += 1
        mp8 = self.mp8
        self.kernels[0][1](i)
        self.kernels[1][1](i)
        if not self.fused_update:
            self.kernels[2][1](i)
            mp8.sgd_update_fp16_sr(self.W16[0], self.G8[i % len(self.G8)], self.lr, 1.0 / self.scale, round=mp8.SR,
                                   seed=self.SEED_W, offset=i, skip_if_nonzero=self.stats[1:2], w8_out=self.W8[0])
            return
        mp8.wgrad_update_fp16_sr(self.M, self.N, self.K, self.X8[i % len(self.X8)], self.E8[i % len(self.E8)],
                                 self.W16[0], self.lr, 1.0 / self.scale, g8_out=self.G8[i % len(self.G8)],
                                 g_round=mp8.SR, flags=mp8.FLAG_CONTRACTION_MAJOR, g_seed=self.SEED_G, g_offset=i,
                                 w_round=mp8.SR, w_seed=self.SEED_W, w_offset=i, skip_if_nonzero=self.stats[1:2],
                                 w8_out=self.W8[0], workspace=self.ws)


class Cfg2Workload:
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
            ("quantize_X", lambda i=0: mp8_.quantize_e5m2(self.X, self.X8), 5 * M * K, 0, "hbm"),
            ("quantize_dY", lambda i=0: mp8_.quantize_e5m2(self.dY, self.E8, scale=LOSS_SCALE,
                                                       stats=self.stats), 5 * M * N, 0, "hbm"),
            ("gemm_fwd", lambda i=0: mp8_.gemm_fp8(mp8_.FWD, M, N, K, self.X8, self.W8, out8=self.Y8,
                                               workspace=self.ws, flags=mp8_.FLAG_B_CONTRACTION_MAJOR),
             M * K + K * N + M * N, 2 * M * N * K, "mfma"),
            ("gemm_bwd_data", lambda i=0: mp8_.gemm_fp8(mp8_.BWD_DATA, M, N, K, self.E8, self.W8,
                                                    out8=self.dX8, workspace=self.ws),
             M * N + K * N + M * K, 2 * M * N * K, "mfma"),
            ("gemm_wgrad", lambda i=0: mp8_.gemm_fp8(mp8_.WGRAD, M, N, K, self.X8, self.E8, out8=self.G8,
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
            fwd = ("quantize_X_gemm_fwd", lambda i=0: mp8_.quantize_gemm_fwd_fp8(
                M, N, K, self.X, self.X8, self.W8, out8=self.Y8, workspace=self.ws),
                5 * M * K + K * N + M * N, 2 * M * N * K, "hbm")
            self.kernels = [k for k in self.kernels if k[0] not in ("quantize_X", "gemm_fwd")]
            self.kernels.insert(1, fwd)
        if batch_quantize:
            # both Q nodes of the step in one launch (measured: no faster inside the step)
            self.kernels[:2] = [("quantize_X_dY", lambda i=0: mp8_.quantize_e5m2_batch([
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

    def _wgrad_update(self, i=0):
        self.step_no += 1
        mp8 = self.mp8
        mp8.wgrad_update_fp16_sr(self.M, self.N, self.K, self.X8, self.E8, self.W16, LR, 1.0 / LOSS_SCALE,
                                 g8_out=self.G8, flags=mp8.FLAG_CONTRACTION_MAJOR, w_round=mp8.SR,
                                 w_seed=0x1905_1233_4000_0002, w_offset=self.step_no,
                                 skip_if_nonzero=self.stats[1:2], w8_out=self.W8, workspace=self.ws)

    def _update(self, i=0):
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

    def __init__(self, mp8, torch, lay, shape=(32, 28, 28, 128)):
        self.mp8, self.torch = mp8, torch
        B, H, W, C = shape
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
            ("quantize_X", lambda i=0: mp8.quantize_e5m2(self.X, self.X8), 5 * P * C, 0, "hbm"),
            ("quantize_dY", lambda i=0: mp8.quantize_e5m2(self.dY, self.E8, scale=LOSS_SCALE, stats=self.stats),
             5 * P * C, 0, "hbm"),
            ("conv_fwd", lambda i=0: conv(mp8.FWD, self.X8, self.W8, self.Y8), 2 * P * C + 9 * C * C, flops, "mfma"),
            ("conv_bwd_data", lambda i=0: conv(mp8.BWD_DATA, self.E8, self.W8, self.dX8),
             2 * P * C + 9 * C * C, flops, "mfma"),
            # weight gradient, its rounding and the master-weight update in one call
            ("conv_wgrad_update", self._wgrad_update, 2 * P * C + 9 * C * C + 6 * 9 * C * C, flops, "mfma"),
        ]
        mp8.quantize_e5m2(self.W16.view(9 * C, C), self.W8)

    def _wgrad_update(self, i=0):
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


def kernel_table(kernels, times_ms, traffic=None, cold_ms=None, in_step_ms=None):
    """One row per kernel.  `us` / `achieved` / `frac` come from back-to-back launches on the same
    buffers (warm); `us_cold` / `achieved_cold` / `frac_cold`, where measured, from launches that
    rotate through buffer sets of more than twice the 256 MB cache; `us_in_step` / `achieved_in_step`
    / `frac_in_step`, where measured, from events between the kernels of whole steps (each kernel
    finds in the caches what the kernel before it left there, as in training).  Without the
    stand-alone loops (`times_ms` None) the in-step figures stand in for `us` / `achieved` / `frac`."""
    out = []
    if times_ms is None:
        times_ms = in_step_ms
    for j, ((name, _, nbytes, flops, bound), ms) in enumerate(zip(kernels, times_ms)):
        def rate(t_ms):
            if bound == "mfma":
                return flops / (t_ms * 1e-3) / 1e12, FP8_PEAK_TFLOPS, "TFLOP/s"
            return nbytes / (t_ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        achieved, peak, unit = rate(ms)
        row = {"kernel": name, "bound": bound, "us": ms * 1e3, "achieved": achieved,
               "peak": peak, "unit": unit, "frac": achieved / peak,
               "alg_bytes": nbytes, "flops": flops,
               "hbm_gbs": nbytes / (ms * 1e-3) / 1e9,
               "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "traffic": (traffic or {}).get(name)}
        if cold_ms is not None:
            ac, _, _ = rate(cold_ms[j])
            row.update({"us_cold": cold_ms[j] * 1e3, "achieved_cold": ac, "frac_cold": ac / peak,
                        "hbm_gbs_cold": nbytes / (cold_ms[j] * 1e-3) / 1e9})
        if in_step_ms is not None:
            ai, _, _ = rate(in_step_ms[j])
            row.update({"us_in_step": in_step_ms[j] * 1e3, "achieved_in_step": ai, "frac_in_step": ai / peak})
        out.append(row)
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
    per_graph = max(d for d in range(1, 15) if steps % d == 0)
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


def time_kernels(torch, wl, reps, rotate=False):
    """Average duration of every kernel of the step: each one is captured `reps` times back to
    back in a HIP graph of its own and the replay is timed with events on the replay stream (the
    stream the kernels are launched on), so the figure is device time per launch (launch gaps of
    about a microsecond included), free of host launch cost.  rotate: launch j works on buffer set
    j (cold); else every launch on set 0 (warm).  Returns ms per launch."""
    out = []
    for _, fn, _, _, _ in wl.kernels:
        fn(0)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for j in range(reps):
                fn(j if rotate else 0)
        graph.replay()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        graph.replay()
        graph.replay()
        e.record()
        torch.cuda.synchronize()
        out.append(s.elapsed_time(e) / (2 * reps))
    return out


def time_kernels_in_step(torch, wl, steps):
    """Average duration of every kernel INSIDE the step: `steps` whole steps are launched one
    call per kernel with ONE event between consecutive kernels (on the stream the kernels run on);
    a kernel's figure is the time from the event before it to the event after it.  The host stays
    ahead of the device (a step is four launches and five event records against about 150 us of
    device time), so the interval is the kernel plus the gap in which the device picks up the next
    command (1-2 us; a tracer's per-kernel average of the same launches is shorter by that much).
    The steps continue the workload's own sequence (input sets, statistics ring, Philox offsets).
    Returns ms per launch, in the order of wl.kernels."""
    n = len(wl.kernels)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(n + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    for t in range(steps):
        wl.ring.advance()
        i = wl.step_no
        wl.step_no += 1
        ev[t][0].record()
        for j, (_, fn, _, _, _) in enumerate(wl.kernels):
            fn(i)
            ev[t][j + 1].record()
    torch.cuda.synchronize()
    return [sum(ev[t][j].elapsed_time(ev[t][j + 1]) for t in range(steps)) / steps for j in range(n)]


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
    # configs[3] as the recurrence it is: 50 dependent forward GEMMs, the hidden state of step t+1
    # being the cell's output of step t.  The cell itself is harness code (half-precision torch ops
    # on two gate slices, then the library's Q node), timed with the chain and named as such.
    M, N, K, H, T = 128, 4096, 2048, 1024, 50
    w8 = codes(N, K)
    a_t = [codes(M, K) for _ in range(2)]              # [x_t, h_{t-1}]; the h half is overwritten per step
    y8 = torch.empty((M, N), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, M, N, K), 16), dtype=torch.uint8, device=dev)

    def recurrence(with_cell):
        def run():
            for t in range(T):
                cur, nxt = a_t[t & 1], a_t[(t + 1) & 1]
                mp8.gemm_fp8(mp8.FWD, M, N, K, cur, w8, out8=y8, workspace=ws)
                if with_cell:
                    y = (y8.to(torch.int16) << 8).view(torch.float16)
                    h = torch.tanh(y[:, 2 * H:3 * H]) * torch.sigmoid(y[:, 3 * H:])
                    hq = torch.empty((M, H), dtype=torch.uint8, device=dev)
                    mp8.quantize_e5m2(h.contiguous(), hq)
                    nxt[:, H:].copy_(hq)
        return run
    for with_cell, label in ((False, "50 forward GEMMs back to back in one graph"),
                             (True, "50 dependent steps in one graph: forward GEMM, cell stand-in (harness: half-precision "
                                    "tanh * sigmoid in torch, 5 small kernels), Q node, copy into the next step's operand")):
        us = graph_time_us(torch, recurrence(with_cell), 1) / T
        rows.append({"kernel": "gemm_fp8 (recurrence)", "case": "configs[3] " + label + ", per timestep", "us": us,
                     "tflops": 2.0 * M * N * K / us / 1e6, "frac_mfma_peak": 2.0 * M * N * K / us / 1e6 / FP8_PEAK_TFLOPS})
    del w8, a_t, y8, ws
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
    # plain movement of bytes in the streaming kernels' access pattern and read:write ratio: what
    # the memory system gives a kernel of that shape, next to which the rows above are read
    pdst = torch.empty(n, dtype=torch.float32, device=dev)
    for ratio, what in ((4, "4 bytes read per byte written (the Q node's ratio)"), (1, "1:1 (plain copy)")):
        us = graph_time_us(torch, lambda: mp8.stream_probe(src, pdst, ratio), 5)
        moved = 4.0 * n * (1 + 1.0 / ratio)
        rows.append({"kernel": "stream_probe (bytes only, no arithmetic)", "case": f"2^30 bytes read, {what}", "us": us,
                     "alg_gbs": moved / us / 1e3, "frac_hbm_peak": moved / us / 1e3 / HBM_PEAK_GBS})
    del pdst
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


def _omp():
    """The OpenMP runtime the oracle library is linked against (thread control and count)."""
    import ctypes
    for name in ("libgomp.so.1", "libomp.so", "libiomp5.so"):
        try:
            return ctypes.CDLL(name)
        except OSError:
            continue
    return None


def cpu_baseline(lay, seconds=8.0):
    """The CPU oracle, as it stands, on a bounded sample of the headline workload, once with one
    thread and once with all the threads OpenMP gives it.  Sample: the two Q nodes over the whole
    tensors (they are cheap), the weight gradient's double-precision reference, its stochastic
    rounding and the master-weight update over the first R of the K = 1024 output rows, R chosen
    from a short trial so that the leg takes about `seconds`.  The time of a whole step is the
    Q nodes' time plus K / R times the rest; `value` = 2*M*N*K flop / that time."""
    import oracle
    omp = _omp()
    M, N, K = lay.M, lay.N, lay.K
    scale, lr = float(lay.loss_scale), float(lay.extra["lr"])
    w16 = lay.W.astype(np.float16).view(np.uint16)
    all_threads = int(omp.omp_get_max_threads()) if omp is not None else int(os.environ.get("OMP_NUM_THREADS", 1))
    legs = []
    for threads in ((1, all_threads) if omp is not None and all_threads > 1 else (all_threads,)):
        if omp is not None:
            omp.omp_set_num_threads(threads)
        t0 = time.perf_counter()
        X8 = oracle.quantize_e5m2(lay.X)[0]                        # [M, K]
        E8 = oracle.quantize_e5m2(lay.dY, scale=scale)[0]          # [M, N]
        tq = time.perf_counter() - t0
        a, b = np.ascontiguousarray(X8.T), np.ascontiguousarray(E8.T)   # [K, M], [N, M] (a re-layout, untimed)

        def rows_leg(R):
            t1 = time.perf_counter()
            ref, _ = oracle.gemm_ref(a, b, row_idx=np.arange(R), want_abs=False)
            tg = time.perf_counter() - t1
            g8 = oracle.quantize_e5m2(ref.astype(np.float32), mode=oracle.SR, seed=1, offset=1)[0]
            oracle.sgd_update_fp16(w16[:R].reshape(-1), g8.reshape(-1), lr, 1.0 / scale, mode=oracle.SR, seed=2, offset=1)
            return time.perf_counter() - t1, tg
        trial = min(K, 4 * threads)
        t_trial, _ = rows_leg(trial)                 # also warms the thread pool up
        R = int(max(trial, min(K, trial * (seconds - tq) / max(t_trial, 1e-4))))
        t_rows, t_gemm = rows_leg(R)
        step_s = tq + t_rows * (K / R)
        legs.append({"threads": threads, "value": 2.0 * M * N * K / step_s / 1e12, "rows": R,
                     "quantize_s": tq, "rows_s": t_rows,
                     "gemm_gflops": 2.0 * R * N * M / max(t_gemm, 1e-9) / 1e9})
    if omp is not None:
        omp.omp_set_num_threads(all_threads)
    best = legs[-1]
    return {
        "value": best["value"],
        "unit": "TFLOP/s",
        "cores": best["threads"],
        "kind": "oracle",
        "sample": (f"both Q nodes over the whole tensors ({best['quantize_s']:.2f} s) + reference weight gradient, SR "
                   f"rounding and FP16 SR update of {best['rows']} of the {K} output rows ({best['rows_s']:.2f} s, "
                   f"GEMM reference alone {best['gemm_gflops']:.1f} GFLOP/s), scaled to a whole step"),
        "one_thread": ({"value": legs[0]["value"], "rows": legs[0]["rows"], "gemm_gflops": legs[0]["gemm_gflops"]}
                       if len(legs) > 1 else None),
        "host_cpus": os.cpu_count(),
    }


def device_clock_sample(torch, fn, seconds=1.0):
    """Shader clock and socket power while `fn` (an enqueue of GPU work) keeps the GPU busy for
    about `seconds`, polled in-process through the amdsmi library from a side thread; None where the
    library is missing or refuses."""
    import threading
    try:
        import amdsmi
        amdsmi.amdsmi_init()
        handle = amdsmi.amdsmi_get_processor_handles()[0]
    except Exception:
        return None
    samples, stop = [], threading.Event()

    def poll():
        while not stop.is_set():
            try:
                clk = amdsmi.amdsmi_get_clock_info(handle, amdsmi.AmdSmiClkType.GFX)
                pw = amdsmi.amdsmi_get_power_info(handle)
                power = pw.get("current_socket_power")
                if not isinstance(power, (int, float)):
                    power = pw.get("average_socket_power")
                samples.append((clk.get("clk"), power if isinstance(power, (int, float)) else None))
            except Exception:
                return
            time.sleep(0.02)
    th = threading.Thread(target=poll, daemon=True)
    try:
        t_end = time.perf_counter() + seconds
        for _ in range(50):                     # the GPU is busy before the first sample
            fn()
        th.start()
        while time.perf_counter() < t_end:
            for _ in range(50):
                fn()
            torch.cuda.synchronize()
    finally:
        stop.set()
        if th.is_alive():
            th.join(timeout=2)
        torch.cuda.synchronize()
        try:
            amdsmi.amdsmi_shut_down()
        except Exception:
            pass
    clk = [c for c, _ in samples if isinstance(c, (int, float)) and c > 0]
    pw = [p_ for _, p_ in samples if p_]
    if not clk and not pw:
        return None
    return {"samples": len(samples), "sclk_mhz_mean": sum(clk) / len(clk) if clk else None,
            "sclk_mhz_min": min(clk) if clk else None, "sclk_mhz_max": max(clk) if clk else None,
            "power_w_mean": sum(pw) / len(pw) if pw else None}


def timed_workload(torch, wl, args, traffic=None, rotate=False, in_step=False):
    """Warm-up, the timed steps, and the per-kernel table of one workload."""
    for _ in range(args.warmup):
        wl.step()
    ms = time_steps(torch, wl, args.steps, args.launch)
    inside = time_kernels_in_step(torch, wl, min(args.steps, 140)) if in_step else None
    if args.steps_only and in_step:
        return ms, kernel_table(wl.kernels, None, traffic, None, inside)
    warm = time_kernels(torch, wl, args.kernel_reps)
    cold = time_kernels(torch, wl, args.kernel_reps, rotate=True) if rotate else None
    return ms, kernel_table(wl.kernels, warm, traffic, cold, inside)


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
    cold = not args.warm
    lay = workloads.config5()
    traffic = profiled_traffic()
    wl = Cfg5Workload(mp8, torch, lay, cold=cold, fused_update=not args.separate_update)
    if args.steps_only:
        args.no_configs1_step = args.no_all_configs = args.no_cpu_baseline = True
    ms_per_step, kernels = timed_workload(torch, wl, args, traffic, rotate=cold, in_step=True)
    nonfinite = mp8.read_stats(wl.stats)[1]
    gemm_flops = 2.0 * lay.M * lay.N * lay.K
    value = gemm_flops / (ms_per_step * 1e-3) / 1e12
    # the dominant kernel and its rate are those of the timed region: durations inside the step
    dom = max(kernels, key=lambda k: k["us_in_step"])
    sfx = "_cold" if cold else ""
    roofline = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved_in_step"],
                "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac_in_step"],
                "us": dom["us_in_step"],
                "timing": "events before and after the kernel inside whole steps whose FP32 inputs rotate over sets; "
                          "its 8-bit operands are what the two Q nodes of the same step have just written"
                          if cold else "events before and after the kernel inside whole steps on one input set",
                "us_alone_warm": dom.get("us") if not args.steps_only else None,
                "us_alone_cold": dom.get("us_cold"),
                "frac_alone_cold": dom.get("frac_cold"),
                "plan": list(wl.plan),
                "traffic": traffic.get(dom["kernel"]),
                "traffic_source": "profiles/bench_step_cfg5_hbm_traffic.txt (counter runs of this command, not this run)"
                                  if traffic.get(dom["kernel"]) else None}
    gemm = next(k for k in kernels if k["kernel"] == "gemm_wgrad_sr")
    clocks = None if args.steps_only else device_clock_sample(torch, lambda: wl.kernels[2][1](0))
    if clocks and clocks.get("sclk_mhz_mean") and roofline["bound"] == "mfma":
        # the same rate against the matrix-core peak at the clock the chip actually held under this
        # kernel (256 CUs x 4 SIMDs x 2048 flop per clock x sampled clock) beside the datasheet's 2.4 GHz
        at_clock = 256 * 4 * 2048 * clocks["sclk_mhz_mean"] * 1e6 / 1e12
        roofline["peak_at_sampled_clock"] = at_clock
        roofline["frac_at_sampled_clock"] = roofline["achieved"] / at_clock
        roofline["sampled_clock_mhz"] = clocks["sclk_mhz_mean"]

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
        "config": {"workload": "configs[4]: Transformer-big weight gradient + update, 16384 tokens, W 1024x4096: "
                               "quantize X and dY*2^14 (RNE, overflow statistics), wgrad GEMM 1024x4096 over 16384 "
                               "with FP32 accumulation and ONE stochastic rounding to E5M2 (Philox), FP16 master-weight "
                               "SGD step lr=1e-3 with stochastic rounding, emitting the next 8-bit weights",
                   "M": lay.M, "N": lay.N, "K": lay.K, "launch": args.launch,
                   "inputs": "rotate over sets (no step finds its FP32 inputs in the 256 MB cache)" if cold
                             else "one set, replayed"},
        "pct_of_fp8_peak_whole_step": 100.0 * value / FP8_PEAK_TFLOPS,
        "gemm_only_tflops": gemm["achieved_in_step"],
        "gemm_only_pct_of_fp8_peak": 100.0 * gemm["frac_in_step"],
        "overflow_count_last_step": nonfinite,
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "max_clock_mhz": getattr(props, "clock_rate", 0) / 1e3 or None,
                   "memory_gib": round(props.total_memory / 2 ** 30, 1),
                   "during_gemm": clocks},
        "roofline": roofline,
        "kernels": kernels,
    }
    del wl
    torch.cuda.empty_cache()
    if not args.no_configs1_step:
        # configs[1]: the layer with all three GEMMs per step (lowered form), as timed before
        try:
            lay2 = workloads.config2()
            w2 = Cfg2Workload(mp8, torch, lay2, batch_quantize=args.batch_quantize, fused_update=not args.separate_update,
                              fused_quantize=not args.separate_quantize, two_streams=args.two_streams)
            ms2, k2 = timed_workload(torch, w2, args)
            flops2 = 3 * 2.0 * lay2.M * lay2.N * lay2.K
            out["configs1_step"] = {
                "workload": "configs[1]: ResNet-50-style 3x3 conv as GEMM, M=25088 N=128 K=1152: quantize X and dY, "
                            "fwd + bwd_data + wgrad, FP16 SR update emitting the next 8-bit weights, loss scale 2^12 "
                            "(one input set, replayed)",
                "ms_per_step": ms2, "value": flops2 / (ms2 * 1e-3) / 1e12, "unit": "TFLOP/s (3 * 2*M*N*K per step)",
                "overflow_count_last_step": mp8.read_stats(w2.stats)[1], "kernels": k2}
            del w2
            torch.cuda.empty_cache()
            if not args.no_conv_step:
                # the same layer without the lowering: 3x3 convolution as an implicit GEMM
                cw = ConvWorkload(mp8, torch, lay2)
                msc, kc_ = timed_workload(torch, cw, args)
                out["conv_step"] = {
                    "workload": "the configs[1] layer as an implicit-GEMM 3x3 convolution on zero-padded "
                                "channels-last tensors (no lowered operand): quantize X and dY, conv "
                                "fwd + bwd_data + wgrad, FP16 SR update emitting the next 8-bit weights",
                    "ms_per_step": msc, "value": flops2 / (msc * 1e-3) / 1e12,
                    "unit": "TFLOP/s (useful flops of the unpadded layer, 3 * 2*M*N*K)",
                    "overflow_count_last_step": mp8.read_stats(cw.stats)[1], "kernels": kc_}
                del cw
                torch.cuda.empty_cache()
                # the first stage of the residual networks: 64 channels at four times the pixels (a stage
                # of the contraction spans two filter taps, the last stage is half a stage)
                cw = ConvWorkload(mp8, torch, lay2, shape=(32, 56, 56, 64))
                msc, kc_ = timed_workload(torch, cw, args)
                flops64 = 3 * 2.0 * 32 * 56 * 56 * 9 * 64 * 64
                out["conv64_step"] = {
                    "workload": "a 3x3 convolution of the 64-channel stage (batch 32, 56x56, 64 -> 64 channels) as an "
                                "implicit GEMM: quantize X and dY, conv fwd + bwd_data + wgrad, FP16 SR update "
                                "emitting the next 8-bit weights",
                    "ms_per_step": msc, "value": flops64 / (msc * 1e-3) / 1e12,
                    "unit": "TFLOP/s (useful flops of the unpadded layer, 3 * 2*B*H*W*9*Cin*Cout)",
                    "overflow_count_last_step": mp8.read_stats(cw.stats)[1], "kernels": kc_}
                del cw
                torch.cuda.empty_cache()
        except Exception as exc:  # extra evidence; the headline stands on its own
            out["configs1_step"] = out.get("configs1_step") or {"error": repr(exc)}
            out.setdefault("conv_step", {"error": repr(exc)})
    if not args.no_all_configs:
        try:
            out["all_configs"] = all_configs_report(mp8, torch, args.vendor_gemm)
        except Exception as exc:  # the table is extra evidence; the line above it stands on its own
            out["all_configs"] = {"error": repr(exc)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(lay, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
