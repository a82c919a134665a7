"""GPU parity: the GEMMs that quantise their own FP32 operand (mp8_quantize_gemm_fwd_fp8) against
the oracle's chain quantize -> GEMM, and against the two separate calls on the GPU."""
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


def activations(rng, shape, specials):
    """FP32 values over five binades (the matrix cores align the products of a group to the
    largest one, so the accumulator tolerance is stated for operands of moderate range);
    optionally a few NaN / Inf / zero / tiny / overflowing values, which the caller's row mask
    keeps out of the tolerance check."""
    x = (rng.standard_normal(shape) * np.exp2(rng.integers(-3, 2, shape))).astype(np.float32)
    if specials:
        flat = x.reshape(-1)
        idx = rng.choice(flat.size, size=min(40, flat.size), replace=False)
        flat[idx] = np.resize(np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-30, 30720.0, 28672.0,
                                        32768.0, -30719.9], dtype=np.float32), idx.size)
    return x


def moderate_rows(codes):
    """Rows whose codes are all finite and below 128 in magnitude."""
    return np.flatnonzero(((codes >> 2) & 31).max(axis=1) <= 21)


def check_rounding_of_gpu_accumulator(acc, out8, alpha, mode, flags, seed, offset):
    """out8 is the oracle's rounding of alpha * acc, element by element (any rows, any values)."""
    if mode == oracle.RNE:
        want, _ = oracle.quantize_e5m2(acc, scale=alpha, mode=oracle.RNE, flags=flags)
    else:
        want, _ = oracle.quantize_e5m2(acc, scale=alpha, mode=oracle.SR, flags=flags, seed=seed, offset=offset)
    assert np.array_equal(out8, want), "out8 != oracle rounding of the GPU accumulator"


def finite_codes(rng, shape, emax=17):
    """Random 8-bit codes of moderate range: exponent field 12 .. emax."""
    e = rng.integers(12, emax + 1, shape)
    return ((rng.integers(0, 2, shape) << 7) | (e << 2) | rng.integers(0, 4, shape)).astype(np.uint8)


def run_fused(mp8, x, w8, want_acc=True, ldw=None, **kw):
    """(x8, acc, out8, x_stats, stats) of one fused call, with guard bytes behind every output."""
    import torch
    M, K = x.shape
    N = w8.shape[1]
    x8buf = torch.full((M * K + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    obuf = torch.full((M * N + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    accbuf = torch.full((M * N + 16,), 7.0, dtype=torch.float32, device="cuda")
    xs, st = mp8.new_stats(), mp8.new_stats()
    with_x_stats = kw.pop("with_x_stats", True)
    with_stats = kw.pop("with_stats", True)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, M, N, K), 16), dtype=torch.uint8, device="cuda")
    wdev = gpu(w8)
    mp8.quantize_gemm_fwd_fp8(M, N, K, gpu(x), x8buf[: M * K], wdev, out8=obuf[: M * N],
                              acc=accbuf[: M * N] if want_acc else None, acc_mode=1 if want_acc else 0,
                              x_stats=xs if with_x_stats else None, stats=st if with_stats else None,
                              workspace=ws, ldw=ldw, **kw)
    torch.cuda.synchronize()
    assert bool((x8buf[M * K:] == 0xAA).all()), "write past the end of x8_out"
    assert bool((obuf[M * N:] == 0xAA).all()), "write past the end of out8"
    assert bool((accbuf[M * N:] == 7.0).all()), "write past the end of acc"
    return (host(x8buf[: M * K]).reshape(M, K), host(accbuf[: M * N]).reshape(M, N),
            host(obuf[: M * N]).reshape(M, N), mp8.read_stats(xs), mp8.read_stats(st))


def separate_calls(mp8, x, w8, x_kw, g_kw):
    """The two calls the fused one stands for: (x8, out8, x_stats, stats)."""
    import torch
    M, K = x.shape
    N = w8.shape[1]
    x8 = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
    out = torch.zeros((M, N), dtype=torch.uint8, device="cuda")
    xs, st = mp8.new_stats(), mp8.new_stats()
    mp8.quantize_e5m2(gpu(x), x8, stats=xs, **x_kw)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, M, N, K), 16), dtype=torch.uint8, device="cuda")
    flags = g_kw.pop("flags", 0) | mp8.FLAG_B_CONTRACTION_MAJOR
    mp8.gemm_fp8(mp8.FWD, M, N, K, x8, gpu(w8), out8=out, stats=st, workspace=ws, flags=flags, **g_kw)
    torch.cuda.synchronize()
    return host(x8), host(out), mp8.read_stats(xs), mp8.read_stats(st)


@pytest.mark.parametrize("shape", [(64, 128, 128), (1, 16, 128), (200, 128, 1152), (333, 48, 384),
                                   (129, 112, 256), (64, 128, 1280)])
def test_fused_forward_plain_rounding(mp8, shape):
    """RNE on both sides, no statistics (the kernel variant a training step uses) and the
    variant with the FP32 result: codes of x bit for bit the oracle's, the accumulator within
    tolerance of the double product of those codes, the output the oracle's rounding of it."""
    M, N, K = shape
    rng = np.random.default_rng(1000 + M + N + K)
    x = activations(rng, (M, K), specials=False)
    w8 = finite_codes(rng, (K, N))
    want8, _ = oracle.quantize_e5m2(x, scale=0.5)
    ref, absref = oracle.gemm_ref(want8, np.ascontiguousarray(w8.T))
    x8, acc, out8, _, _ = run_fused(mp8, x, w8, x_scale=0.5, with_x_stats=False, with_stats=False)
    assert np.array_equal(x8, want8), "x8_out differs from the oracle's quantize"
    check_outputs(acc, out8, ref, absref, K)
    # without the FP32 result: the lean kernel; its codes must be the same
    x8b, _, out8b, _, _ = run_fused(mp8, x, w8, want_acc=False, x_scale=0.5, with_x_stats=False,
                                    with_stats=False)
    assert np.array_equal(x8b, want8) and np.array_equal(out8b, out8)
    s8, sout, _, _ = separate_calls(mp8, x, w8, dict(scale=0.5), {})
    assert np.array_equal(s8, x8) and np.array_equal(sout, out8), "fused differs from the two calls"


@pytest.mark.parametrize("shape", [(150, 128, 384), (70, 32, 256)])
def test_fused_forward_stochastic_rounding_saturation_statistics(mp8, shape):
    """Every option at once: SR of the activations with their own stream, saturation, NaN / Inf /
    zero inputs, statistics of both tensors, alpha, SR of the output."""
    M, N, K = shape
    rng = np.random.default_rng(77 + M)
    x = activations(rng, (M, K), specials=True)
    w8 = finite_codes(rng, (K, N), emax=17)
    for x_flags, x_mode in ((0, oracle.SR), (1, oracle.SR), (1, oracle.RNE)):
        ost = oracle.Stats()
        want8, _ = oracle.quantize_e5m2(x, scale=2.0, mode=x_mode, flags=x_flags, seed=11, offset=5, stats=ost)
        ref, absref = oracle.gemm_ref(want8, np.ascontiguousarray(w8.T))
        kw = dict(x_scale=2.0, x_round=x_mode, x_flags=x_flags, x_seed=11, x_offset=5)
        x8, acc, out8, xst, st = run_fused(mp8, x, w8, alpha=0.25, round=mp8.SR, seed=3, offset=9, flags=1, **kw)
        assert np.array_equal(x8, want8), "x8_out differs from the oracle's quantize"
        assert xst == ost.as_tuple(), "statistics of x differ from the oracle's"
        check_rounding_of_gpu_accumulator(acc, out8, 0.25, oracle.SR, 1, 3, 9)
        assert np.array_equal(np.isnan(acc), np.isnan(ref)) and np.array_equal(np.isinf(acc), np.isinf(ref))
        rows = moderate_rows(want8)
        assert rows.size > M // 2
        check_outputs(acc[rows], out8[rows], ref[rows], absref[rows], K, alpha=0.25, mode=oracle.SR, flags=1,
                      seed=3, offset=9, first_index=rows * N)
        s8, sout, sxst, sst = separate_calls(
            mp8, x, w8, dict(scale=2.0, round=x_mode, flags=x_flags, seed=11, offset=5),
            dict(alpha=0.25, round=mp8.SR, seed=3, offset=9, flags=1))
        assert np.array_equal(s8, x8) and np.array_equal(sout, out8)
        assert sxst == xst and sst == st, "statistics differ from the two calls'"


def test_fused_forward_row_stride_of_the_weights_and_other_shapes(mp8):
    """A weight matrix that is a column block of a wider one (row stride > N) goes through the
    fused kernel; more than 128 columns, or a contraction that is not a multiple of 128, run as
    the two calls: the same results either way."""
    rng = np.random.default_rng(5)
    for (M, N, K, ldw) in ((96, 64, 256, 160), (40, 256, 256, None), (50, 64, 200, None), (0, 64, 128, None)):
        x = activations(rng, (M, K), specials=False)
        wide = finite_codes(rng, (K, ldw or N))
        w8 = wide[:, :N]
        if M == 0:
            run_fused(mp8, x, np.ascontiguousarray(w8))
            continue
        want8, _ = oracle.quantize_e5m2(x)
        ref, absref = oracle.gemm_ref(want8, np.ascontiguousarray(w8.T))
        import torch
        x8 = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
        out = torch.zeros((M, N), dtype=torch.uint8, device="cuda")
        acc = torch.zeros((M, N), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, M, N, K), 16), dtype=torch.uint8, device="cuda")
        mp8.quantize_gemm_fwd_fp8(M, N, K, gpu(x), x8, gpu(wide), out8=out, acc=acc, acc_mode=1,
                                  workspace=ws, ldw=ldw)
        torch.cuda.synchronize()
        assert np.array_equal(host(x8), want8)
        check_outputs(host(acc), host(out), ref, absref, K)


def test_fused_forward_full_size_layer(mp8):
    """configs[1] at full size, as the benchmark launches it: every code of x against the oracle,
    the output against the two separate calls (all of it) and against the oracle on sampled rows."""
    import torch
    lay = workloads.config2()
    M, N, K = lay.M, lay.N, lay.K
    w8, _ = oracle.quantize_e5m2(lay.W)
    want8, _ = oracle.quantize_e5m2(lay.X)
    xd, wd = gpu(lay.X), gpu(w8)
    x8 = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
    out = torch.zeros((M, N), dtype=torch.uint8, device="cuda")
    mp8.quantize_gemm_fwd_fp8(M, N, K, xd, x8, wd, out8=out)
    torch.cuda.synchronize()
    assert np.array_equal(host(x8), want8), "x8_out differs from the oracle's quantize"
    s8, sout, _, _ = separate_calls(mp8, lay.X, w8, {}, {})
    assert np.array_equal(sout, host(out)), "fused differs from the two calls"
    rows = np.random.default_rng(9).choice(M, size=64, replace=False)
    rows = np.concatenate([rows, [0, M - 1]])
    acc = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    mp8.quantize_gemm_fwd_fp8(M, N, K, xd, x8, wd, out8=out, acc=acc, acc_mode=1)
    torch.cuda.synchronize()
    ref, absref = oracle.gemm_ref(want8, np.ascontiguousarray(w8.T), row_idx=rows)
    check_outputs(host(acc)[rows], host(out)[rows], ref, absref, K)
    assert np.array_equal(host(out), sout)



def test_fused_forward_many_rows_every_option(mp8):
    """Enough rows for the kernel variant with 128 rows per workgroup, a ragged last workgroup, and
    every option at once (SR of the activations, saturation, special values, statistics of both
    tensors, alpha, SR of the output, FP32 result); then the lean variant on the same data."""
    from gpu_util import acc_tolerance_ok
    M, N, K = 128 * 128 + 37, 48, 256
    rng = np.random.default_rng(4242)
    x = activations(rng, (M, K), specials=True)
    w8 = finite_codes(rng, (K, N))
    ost = oracle.Stats()
    want8, _ = oracle.quantize_e5m2(x, scale=2.0, mode=oracle.SR, flags=1, seed=31, offset=2, stats=ost)
    ref, absref = oracle.gemm_ref(want8, np.ascontiguousarray(w8.T))
    x8, acc, out8, xst, st = run_fused(mp8, x, w8, x_scale=2.0, x_round=mp8.SR, x_flags=1, x_seed=31,
                                       x_offset=2, alpha=0.5, round=mp8.SR, seed=8, offset=1, flags=1)
    assert np.array_equal(x8, want8), "x8_out differs from the oracle's quantize"
    assert xst == ost.as_tuple(), "statistics of x differ from the oracle's"
    check_rounding_of_gpu_accumulator(acc, out8, 0.5, oracle.SR, 1, 8, 1)
    assert np.array_equal(np.isnan(acc), np.isnan(ref)) and np.array_equal(np.isinf(acc), np.isinf(ref))
    rows = moderate_rows(want8)
    ok, worst, _ = acc_tolerance_ok(acc[rows], ref[rows], absref[rows], K)
    assert ok, f"accumulator outside tolerance (worst ratio {worst})"
    s8, sout, sxst, sst = separate_calls(mp8, x, w8, dict(scale=2.0, round=mp8.SR, flags=1, seed=31, offset=2),
                                         dict(alpha=0.5, round=mp8.SR, seed=8, offset=1, flags=1))
    assert np.array_equal(s8, x8) and np.array_equal(sout, out8) and sxst == xst and sst == st
    # RNE, no statistics, no FP32 result
    xp = activations(rng, (M, K), specials=False)
    wantp, _ = oracle.quantize_e5m2(xp)
    x8p, _, out8p, _, _ = run_fused(mp8, xp, w8, want_acc=False, with_x_stats=False, with_stats=False)
    assert np.array_equal(x8p, wantp)
    _, accp, out8q, _, _ = run_fused(mp8, xp, w8, with_x_stats=False, with_stats=False)
    assert np.array_equal(out8q, out8p)
    refp, absrefp = oracle.gemm_ref(wantp, np.ascontiguousarray(w8.T))
    check_outputs(accp, out8p, refp, absrefp, K)


def test_fused_forward_rejects_bad_arguments_and_enqueues_nothing(mp8):
    """Null or misaligned tensors, a weight row stride below N, bad enums: a status, and the outputs
    stay as they were."""
    import torch
    M, N, K = 64, 64, 128
    x = torch.ones((M, K), dtype=torch.float32, device="cuda")
    w8 = torch.full((K, N), 0x3C, dtype=torch.uint8, device="cuda")
    x8 = torch.full((M * K + 16,), 0xAA, dtype=torch.uint8, device="cuda")
    out = torch.full((M * N + 16,), 0xAA, dtype=torch.uint8, device="cuda")
    good = dict(out8=out[: M * N])
    bad_calls = [
        lambda: mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[: M * K], w8, ldw=N - 16, **good),       # row stride < N
        lambda: mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[1: M * K + 1], w8, **good),               # misaligned x8_out
        lambda: mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[: M * K], w8, out8=out[1: M * N + 1]),    # misaligned out8
        lambda: mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[: M * K], w8, x_round=7, **good),         # bad rounding mode
        lambda: mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[: M * K], w8, round=-1, **good),
        lambda: mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[: M * K], w8, acc_mode=1, **good),        # acc_mode without acc
        lambda: mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[: M * K], w8, acc_mode=3, **good),
    ]
    for call in bad_calls:
        with pytest.raises(mp8.Mp8Error):
            call()
    torch.cuda.synchronize()
    assert bool((x8 == 0xAA).all()) and bool((out == 0xAA).all()), "a rejected call wrote something"
    # and the same call with good arguments works: 1.0 * 1.0 summed over K = 128
    mp8.quantize_gemm_fwd_fp8(M, N, K, x, x8[: M * K], w8, **good)
    torch.cuda.synchronize()
    assert bool((x8[: M * K] == 0x3C).all()) and bool((out[: M * N] == oracle.e5m2_encode(128.0)).all())
