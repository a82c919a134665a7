"""GPU parity at the full sizes of the five workload configurations, through the C ABI with the
automatic kernel choice (the launch configuration the benchmark times).

Quantisation, rounding and the update are compared with the oracle over whole tensors, bit for
bit.  GEMM accumulators are compared with the double reference on sampled output rows (each
output element is an independent dot product) that include the first and last row and rows on
both sides of tile boundaries; the 8-bit outputs are compared with the oracle's rounding of the
GPU's own accumulator over the whole tensor."""
import numpy as np
import pytest

import oracle
from paper_1905_12334_amd import workloads
from gpu_util import gpu, host, check_outputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mp8():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1905_12334_amd as m
    m.lib()
    return m


def sample_rows(rows, n, seed):
    fixed = [0, 1, 63, 64, 127, 128, 255, 256, rows - 257, rows - 129, rows - 65, rows - 2, rows - 1]
    fixed = [r for r in fixed if 0 <= r < rows]
    rnd = np.random.default_rng(seed).integers(0, rows, max(n - len(fixed), 0)).tolist()
    return np.array(sorted(set(fixed + rnd)), dtype=np.int64)


def quantize_both(mp8, x, scale=1.0, with_stats=False, **kw):
    """Q(x*scale) with transposed copy on the GPU, checked against the oracle; device tensors."""
    import torch
    rows, cols = x.shape
    d = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
    dt = torch.empty((cols, rows), dtype=torch.uint8, device="cuda")
    st = mp8.new_stats() if with_stats else None
    mp8.quantize_e5m2(gpu(x), d, dt, scale=scale, stats=st, **kw)
    torch.cuda.synchronize()
    ost = oracle.Stats()
    want, want_t = oracle.quantize_e5m2(x, scale=scale, want_t=True, stats=ost,
                                        mode=kw.get("round", oracle.RNE), seed=kw.get("seed", 0),
                                        offset=kw.get("offset", 0))
    assert np.array_equal(host(d), want), "quantize: row-major copy differs from the oracle"
    assert np.array_equal(host(dt), want_t), "quantize: transposed copy differs from the oracle"
    if with_stats:
        assert mp8.read_stats(st) == ost.as_tuple()
    return d, dt, want, want_t, (ost.as_tuple() if with_stats else None)


def gemm_checked(mp8, op, dims, a_dev, b_dev, a8, b8, nsample=40, alpha=1.0, mode=oracle.RNE,
                 seed=0, offset=0, acc_in=None, acc_mode=1, flags=0):
    """One GEMM as the benchmark calls it (8-bit output only, automatic plan), and again with the
    FP32 accumulator exposed; both must give the same codes; the accumulator is checked against
    the double reference on sampled rows.  a8 / b8 are the host operands in the plain layout
    ([rows, kc] and [cols, kc]); with the contraction-major flag the device tensors are their
    transposes.  Returns (acc as device tensor, out8 as host array)."""
    import torch
    M, N, K = dims
    rows, kc = a8.shape
    cols = b8.shape[0]
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(op, M, N, K), 16), dtype=torch.uint8, device="cuda")
    out_a = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
    out_b = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
    acc = torch.zeros((rows, cols), dtype=torch.float32, device="cuda")
    if acc_in is not None:
        acc.copy_(acc_in)
    kw = dict(alpha=alpha, round=mode, seed=seed, offset=offset, workspace=ws, flags=flags)
    if acc_mode == 1:
        mp8.gemm_fp8(op, M, N, K, a_dev, b_dev, out8=out_a, **kw)
    mp8.gemm_fp8(op, M, N, K, a_dev, b_dev, out8=out_b, acc=acc, acc_mode=acc_mode, **kw)
    torch.cuda.synchronize()
    acc_h, out_h = host(acc), host(out_b)
    if acc_mode == 1:
        assert np.array_equal(host(out_a), out_h), "fused and two-pass epilogues disagree"
    # whole tensor: codes = oracle rounding of the GPU's own accumulator
    want, _ = oracle.quantize_e5m2(acc_h, scale=alpha, mode=mode, seed=seed, offset=offset)
    assert np.array_equal(out_h, want), "out8 != oracle rounding of the GPU accumulator"
    if acc_mode == 1 and nsample > 0:
        idx = sample_rows(rows, nsample, rows + cols)
        ref, absref = oracle.gemm_ref(a8, b8, row_idx=idx)
        check_outputs(acc_h[idx], out_h[idx], ref, absref, kc, alpha=alpha, mode=mode, seed=seed,
                      offset=offset, first_index=idx * cols)
    return acc, out_h


def test_config2_resnet_conv_layer_full_step(mp8):
    """configs[1]: quantize, the three GEMMs and the update, at M=25088 N=128 K=1152."""
    import torch
    lay = workloads.config2()
    M, N, K = lay.M, lay.N, lay.K
    X8d, X8td, X8, X8t, _ = quantize_both(mp8, lay.X)
    W8d, W8td, W8, W8t, _ = quantize_both(mp8, lay.W)
    E8d, E8td, E8, E8t, est = quantize_both(mp8, lay.dY, scale=lay.loss_scale, with_stats=True)
    assert est[1] == 0                                     # no overflow at loss scale 2^12
    gemm_checked(mp8, mp8.FWD, (M, N, K), X8d, W8td, X8, W8t)
    gemm_checked(mp8, mp8.BWD_DATA, (M, N, K), E8d, W8d, E8, W8)
    _, G8 = gemm_checked(mp8, mp8.WGRAD, (M, N, K), X8td, E8td, X8t, E8t, nsample=96)
    # the same weight gradient straight from the row-major X8 and E8 (what the benchmark runs)
    _, G8b = gemm_checked(mp8, mp8.WGRAD, (M, N, K), X8d, E8d, X8t, E8t, nsample=96,
                          flags=mp8.FLAG_CONTRACTION_MAJOR)
    assert np.abs(G8.astype(np.int32) - G8b.astype(np.int32)).max() <= 1   # different slicing only
    # the update takes the oracle's weight gradient (the rounded double reference), on both sides
    G8o = oracle.round_ref_e5m2(oracle.gemm_ref(X8t, E8t, want_abs=False)[0])
    w16 = lay.W.astype(np.float16).view(np.uint16).reshape(-1)
    wd = gpu(w16.view(np.int16))
    mp8.sgd_update_fp16_sr(wd, gpu(G8o.reshape(-1)), 1e-3, 1.0 / lay.loss_scale, round=mp8.SR,
                           seed=77, offset=1)
    torch.cuda.synchronize()
    want, _ = oracle.sgd_update_fp16(w16, G8o.reshape(-1), 1e-3, 1.0 / lay.loss_scale,
                                     mode=oracle.SR, seed=77, offset=1)
    assert np.array_equal(host(wd).view(np.uint16), want)


def test_config3_transformer_ffn_with_dynamic_scale_floor(mp8):
    """configs[2]: both FFN layers, all three GEMMs each; the error tensors are quantised at the
    scaler's floor 2^10, and the overflow count drives the host scaler."""
    for lay in workloads.config3():
        M, N, K = lay.M, lay.N, lay.K
        X8d, X8td, X8, X8t, _ = quantize_both(mp8, lay.X)
        W8d, W8td, W8, W8t, _ = quantize_both(mp8, lay.W)
        E8d, E8td, E8, E8t, est = quantize_both(mp8, lay.dY, scale=lay.loss_scale, with_stats=True)
        sc = mp8.scaler_new(2.0 ** 10, 2.0 ** 10, 4)
        assert est[1] == 0 and mp8.scaler_update(sc, est[1]) == 0 and sc.scale == 2.0 ** 10
        gemm_checked(mp8, mp8.FWD, (M, N, K), X8d, W8td, X8, W8t)
        gemm_checked(mp8, mp8.BWD_DATA, (M, N, K), E8d, W8d, E8, W8)
        gemm_checked(mp8, mp8.WGRAD, (M, N, K), X8td, E8td, X8t, E8t)
        # without loss scaling nearly all of these errors vanish in the 8-bit format (Section 3.1)
        z = oracle.Stats()
        oracle.quantize_e5m2(lay.dY[:256], stats=z)
        assert z.as_tuple()[2] > 0.5 * lay.dY[:256].size and est[2] < 0.1 * lay.dY.size


def cell_stub(y8, hidden):
    """Harness code, not part of the method: a stand-in for the LSTM cell non-linearity in half
    precision -- h = tanh(g) * sigmoid(o) on two of the four gate slices -- rounded to 8 bits by
    the oracle.  Computed on the host from the oracle's 8-bit gate outputs."""
    y = (y8.astype(np.uint16) << 8).view(np.float16).astype(np.float32)
    g, o = y[:, 2 * hidden:3 * hidden], y[:, 3 * hidden:]
    h = (np.tanh(g) * (1.0 / (1.0 + np.exp(-o)))).astype(np.float16).astype(np.float32)
    return oracle.quantize_e5m2(h)[0]


def test_config4_gnmt_lstm_gates_chained_timesteps(mp8):
    """configs[3]: 50 dependent forward GEMMs (h_t feeds step t+1), 50 backward-data GEMMs, and
    the weight gradient accumulated over all timesteps two ways -- one contraction over the
    stacked steps, and FP32 accumulation across per-step calls -- both rounded once."""
    import torch
    lay = workloads.config4()
    B, N, K, T, H = lay.M, lay.N, lay.K, lay.extra["steps"], lay.extra["hidden"]
    W8d, W8td, W8, W8t, _ = quantize_both(mp8, lay.W)
    E8d, E8td, E8, E8t, _ = quantize_both(mp8, lay.dY, scale=lay.loss_scale, with_stats=True)
    x8_all = oracle.quantize_e5m2(lay.X.reshape(T * B, H))[0].reshape(T, B, H)
    h8 = oracle.quantize_e5m2(lay.extra["h0"])[0]
    xh_steps = []
    for t in range(T):
        # the recurrence runs through the oracle (no value computed by the GPU is ever an input
        # of the oracle): the GPU gets the same [x_t; h_t] and must reproduce the step
        xh = np.ascontiguousarray(np.concatenate([x8_all[t], h8], axis=1))      # [B, 2H]
        xh_steps.append(xh)
        ref, absref = oracle.gemm_ref(xh, W8t)
        y8_ref = oracle.round_ref_e5m2(ref)
        acc, y8 = gemm_checked(mp8, mp8.FWD, (B, N, K), gpu(xh), W8td, xh, W8t, nsample=0)
        check_outputs(host(acc), y8, ref, absref, K)
        assert np.mean(y8 != y8_ref) < 0.01          # the few differences are single codes (checked above)
        h8 = cell_stub(y8_ref, H)
    for t in reversed(range(T)):
        e_t = np.ascontiguousarray(E8[t * B:(t + 1) * B])
        gemm_checked(mp8, mp8.BWD_DATA, (B, N, K), E8d[t * B:(t + 1) * B], W8d, e_t, W8,
                     nsample=6 if t % 10 else 20)
    # weight gradient: one contraction of length T*B over the stacked timesteps
    xh_all = np.concatenate(xh_steps, axis=0)                                   # [T*B, 2H]
    a8 = np.ascontiguousarray(xh_all.T)                                         # [K, T*B]
    acc1, out1 = gemm_checked(mp8, mp8.WGRAD, (T * B, N, K), gpu(a8), E8td, a8, E8t, nsample=24)
    # the same sum accumulated in FP32 across per-step calls, rounded after the last one
    acc = torch.zeros((K, N), dtype=torch.float32, device="cuda")
    for t in range(T):
        a_t = np.ascontiguousarray(xh_steps[t].T)                               # [K, B]
        b_t = np.ascontiguousarray(E8t[:, t * B:(t + 1) * B])                   # [N, B]
        acc, out2 = gemm_checked(mp8, mp8.WGRAD, (B, N, K), gpu(a_t), gpu(b_t), a_t, b_t,
                                 acc_in=acc, acc_mode=2)
    idx = sample_rows(K, 24, 4)
    ref, absref = oracle.gemm_ref(a8, E8t, row_idx=idx)
    check_outputs(host(acc)[idx], out2[idx], ref, absref, T * B)
    # both accumulation orders round to codes at most one apart wherever the sum is well conditioned
    from gpu_util import signed_rank
    well = np.abs(ref) >= absref / np.sqrt(float(T * B))
    assert np.abs(signed_rank(out1[idx]) - signed_rank(out2[idx]))[well].max() <= 1


def test_config5_transformer_big_wgrad_sr_and_update(mp8):
    """configs[4]: weight gradient over 16384 tokens with a stochastic-rounding epilogue, then
    the FP16 master-weight SGD step with stochastic rounding."""
    import torch
    lay = workloads.config5()
    M, N, K = lay.M, lay.N, lay.K
    seed, lr = lay.extra["seed"], lay.extra["lr"]
    X8d, X8td, X8, X8t, _ = quantize_both(mp8, lay.X)
    E8d, E8td, E8, E8t, est = quantize_both(mp8, lay.dY, scale=lay.loss_scale, with_stats=True)
    assert est[1] == 0
    gemm_checked(mp8, mp8.WGRAD, (M, N, K), X8td, E8td, X8t, E8t, nsample=20,
                 mode=oracle.SR, seed=seed, offset=11)
    gemm_checked(mp8, mp8.WGRAD, (M, N, K), X8d, E8d, X8t, E8t, nsample=20, mode=oracle.SR,
                 seed=seed, offset=11, flags=mp8.FLAG_CONTRACTION_MAJOR)
    # the update takes the oracle's weight gradient (its double reference over all rows, rounded
    # to FP32 and then stochastically to 8 bits with the same stream), on both sides
    ref_all, _ = oracle.gemm_ref(X8t, E8t, want_abs=False)
    G8 = oracle.quantize_e5m2(ref_all.astype(np.float32), mode=oracle.SR, seed=seed, offset=11)[0]
    w16 = lay.W.astype(np.float16).view(np.uint16).reshape(-1)
    for rnd in (oracle.SR, oracle.RNE):
        wd = gpu(w16.view(np.int16))
        st = mp8.new_stats()
        mp8.sgd_update_fp16_sr(wd, gpu(G8.reshape(-1)), lr, 1.0 / lay.loss_scale, round=rnd,
                               seed=seed, offset=12, stats=st)
        torch.cuda.synchronize()
        want, _ = oracle.sgd_update_fp16(w16, G8.reshape(-1), lr, 1.0 / lay.loss_scale, mode=rnd,
                                         seed=seed, offset=12)
        got = host(wd).view(np.uint16)
        assert np.array_equal(got, want)
        # the updates are far below half a spacing of most half-precision weights: stochastic
        # rounding carries them out on average, nearest-even rounding loses most (Section 3.2)
        dec16 = lambda c: c.view(np.float16).astype(np.float64)
        g = (G8.reshape(-1).astype(np.uint16) << 8).view(np.float16).astype(np.float64) / lay.loss_scale
        u = -lr * g
        carried = float(np.sum(np.sign(u) * (dec16(got) - dec16(w16))) / np.sum(np.abs(u)))
        assert (0.95 < carried < 1.05) if rnd == oracle.SR else (carried < 0.6), (rnd, carried)


def test_degenerate_sizes(mp8):
    import torch
    u8 = lambda *s: torch.zeros(s, dtype=torch.uint8, device="cuda")
    # empty outputs: nothing is launched, nothing is touched
    mp8.gemm_fp8(mp8.FWD, 0, 128, 128, u8(0, 128), u8(128, 128), out8=u8(0, 128))
    mp8.gemm_fp8(mp8.FWD, 128, 0, 128, u8(128, 128), u8(0, 128), out8=u8(128, 0))
    mp8.sgd_update_fp16_sr(torch.zeros(0, dtype=torch.int16, device="cuda"), u8(0), 1e-3, 1.0)
    # empty contraction: the sum over nothing is +0
    out = torch.full((16, 16), 0xAA, dtype=torch.uint8, device="cuda")
    acc = torch.full((16, 16), 5.0, dtype=torch.float32, device="cuda")
    mp8.gemm_fp8(mp8.FWD, 16, 16, 0, u8(16, 0), u8(16, 0), out8=out, acc=acc, acc_mode=1)
    torch.cuda.synchronize()
    assert int(out.max()) == 0 and float(acc.abs().max()) == 0.0
    # a single element, and a single row times a long contraction
    a8 = workloads.random_e5m2_codes(1, (1, 4096))
    b8 = workloads.random_e5m2_codes(2, (1, 4096))
    a8, b8 = (a8 & 0x83) | 0x38, (b8 & 0x83) | 0x38
    o1 = torch.zeros((1, 1), dtype=torch.uint8, device="cuda")
    a1 = torch.zeros((1, 1), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, 1, 1, 4096), 16), dtype=torch.uint8, device="cuda")
    mp8.gemm_fp8(mp8.FWD, 1, 1, 4096, gpu(a8), gpu(b8), out8=o1, acc=a1, acc_mode=1, workspace=ws)
    torch.cuda.synchronize()
    ref, absref = oracle.gemm_ref(a8, b8)
    check_outputs(host(a1), host(o1), ref, absref, 4096)
