"""GPU parity: mp8_sgd_update_fp16_sr against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import oracle
from paper_1905_12334_amd import workloads
from gpu_util import gpu, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mp8():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1905_12334_amd as m
    m.lib()
    return m


def _run(mp8, w16, g8, lr, inv, rnd, seed=0, offset=0, skip=None, want_w8=False):
    import torch
    w = gpu(w16.view(np.int16))
    g = gpu(g8)
    w8 = torch.zeros(w16.size, dtype=torch.uint8, device="cuda") if want_w8 else None
    sk = None if skip is None else torch.tensor([skip], dtype=torch.int32, device="cuda")
    stats = mp8.new_stats()
    mp8.sgd_update_fp16_sr(w, g, lr, inv, round=rnd, seed=seed, offset=offset, skip_if_nonzero=sk,
                           w8_out=w8, stats=stats)
    torch.cuda.synchronize()
    return host(w).view(np.uint16), (host(w8) if want_w8 else None), mp8.read_stats(stats)


@pytest.mark.parametrize("n", [1, 15, 16, 17, 4099, 1 << 20])
@pytest.mark.parametrize("rnd", [oracle.RNE, oracle.SR])
def test_update_random_values_all_sizes(mp8, n, rnd):
    rng = np.random.default_rng(n)
    w16 = (rng.standard_normal(n) * np.exp2(rng.integers(-26, 2, n))).astype(np.float16).view(np.uint16)
    g8 = workloads.random_e5m2_codes(n + 1, (n,), finite_only=False)
    lr, inv = 0.05, 1.0 / 512
    got, got8, gst = _run(mp8, w16, g8, lr, inv, rnd, seed=11, offset=n, want_w8=True)
    st = oracle.Stats()
    want, want8 = oracle.sgd_update_fp16(w16, g8, lr, inv, mode=rnd, seed=11, offset=n, want_w8=True,
                                         stats=st)
    assert np.array_equal(got, want)
    assert np.array_equal(got8, want8)
    assert gst[1] == st.nonfinite


def test_update_all_half_patterns(mp8):
    w16 = np.arange(65536, dtype=np.uint16)
    for code in (0x00, 0x3C, 0xBC, 0x01, 0x7B, 0xFB, 0x44):
        g8 = np.full(65536, code, dtype=np.uint8)
        for rnd in (oracle.RNE, oracle.SR):
            got, _, _ = _run(mp8, w16, g8, 1e-3, 1.0, rnd, seed=3, offset=code)
            want, _ = oracle.sgd_update_fp16(w16, g8, 1e-3, 1.0, mode=rnd, seed=3, offset=code)
            assert np.array_equal(got, want), (code, rnd)


@pytest.mark.parametrize("lr,inv", [(1e-3, 1.0 / 4096), (0.25, 1.0), (7.0, 1.0 / 3)])
def test_update_every_weight_and_gradient_code_pair(mp8, lr, inv):
    """All 65536 half-precision weights x all 256 gradient codes (2^24 pairs), both rounding
    modes, with the 8-bit copy of the new weights."""
    w16 = np.tile(np.arange(65536, dtype=np.uint16), 256)
    g8 = np.repeat(np.arange(256, dtype=np.uint8), 65536)
    for rnd in (oracle.RNE, oracle.SR):
        got, got8, gst = _run(mp8, w16, g8, lr, inv, rnd, seed=99, offset=5, want_w8=True)
        st = oracle.Stats()
        want, want8 = oracle.sgd_update_fp16(w16, g8, lr, inv, mode=rnd, seed=99, offset=5,
                                             want_w8=True, stats=st)
        assert np.array_equal(got, want), (lr, rnd)
        assert np.array_equal(got8, want8), (lr, rnd)
        assert gst[1] == st.nonfinite == 8 * 65536


def test_update_transformer_big_magnitudes_and_skip(mp8):
    lay = workloads.config5(tokens=8, d_in=256, d_out=512)
    w16 = lay.W.astype(np.float16).view(np.uint16).reshape(-1)
    n = w16.size
    g = (np.random.default_rng(5).standard_normal(n) * 1e-5 * lay.loss_scale).astype(np.float32)
    g8, _ = oracle.quantize_e5m2(g.reshape(1, -1))
    g8 = g8.reshape(-1)
    lr, inv = lay.extra["lr"], 1.0 / lay.loss_scale
    seed = lay.extra["seed"]
    rne, _, _ = _run(mp8, w16, g8, lr, inv, oracle.RNE)
    want_rne, _ = oracle.sgd_update_fp16(w16, g8, lr, inv, mode=oracle.RNE)
    assert np.array_equal(rne, want_rne)
    assert (rne == w16).mean() > 0.999                # RNE stalls at these magnitudes
    sr, _, _ = _run(mp8, w16, g8, lr, inv, oracle.SR, seed=seed, offset=1)
    want, _ = oracle.sgd_update_fp16(w16, g8, lr, inv, mode=oracle.SR, seed=seed, offset=1)
    assert np.array_equal(sr, want) and not np.array_equal(sr, w16)
    # device-side skip flag: weights untouched, non-finite gradients still counted
    g_bad = g8.copy()
    g_bad[7] = 0x7C
    skipped, _, st = _run(mp8, w16, g_bad, lr, inv, oracle.SR, seed=seed, offset=1, skip=1)
    assert np.array_equal(skipped, w16) and st[1] == 1
    ran, _, _ = _run(mp8, w16, g8, lr, inv, oracle.SR, seed=seed, offset=1, skip=0)
    assert np.array_equal(ran, want)


@pytest.mark.parametrize("n", [1, 7, 511, 1579, 4099, 1 << 20])
@pytest.mark.parametrize("rnd", [oracle.RNE, oracle.SR])
def test_momentum_update_matches_oracle_over_several_steps(mp8, n, rnd):
    """Momentum SGD with L2 regularisation: weights, FP32 velocity and the 8-bit weight copy
    bit-exact against the oracle over three chained steps."""
    import torch
    rng = np.random.default_rng(n + rnd)
    w16 = (rng.standard_normal(n) * np.exp2(rng.integers(-20, 1, n))).astype(np.float16).view(np.uint16)
    vel = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    lr, inv, mu, wd = 0.05, 1.0 / 1024, 0.9, 1e-4
    wd_dev, vd = gpu(w16.view(np.int16)), gpu(vel)
    w8d = torch.zeros(n, dtype=torch.uint8, device="cuda")
    ow, ov = w16, vel
    for step in range(3):
        g8 = workloads.random_e5m2_codes(100 * step + n % 97, (n,), finite_only=(step != 1))
        st = mp8.new_stats()
        mp8.sgd_momentum_fp16_sr(wd_dev, vd, gpu(g8), lr, inv, mu, wd, round=rnd, seed=5, offset=step,
                                 w8_out=w8d, stats=st)
        torch.cuda.synchronize()
        ost = oracle.Stats()
        ow, ov, o8 = oracle.sgd_momentum_fp16(ow, ov, g8, lr, inv, mu, wd, mode=rnd, seed=5, offset=step,
                                              want_w8=True, stats=ost)
        assert np.array_equal(host(wd_dev).view(np.uint16), ow), step
        gv = host(vd)                      # bit-exact except for the payload of NaNs
        ok = ~np.isnan(ov)
        assert np.array_equal(np.isnan(gv), ~ok) and np.array_equal(gv[ok].view(np.uint32), ov[ok].view(np.uint32)), step
        assert np.array_equal(host(w8d), o8), step
        assert mp8.read_stats(st)[1] == ost.nonfinite


def test_momentum_update_skip_and_reduction_to_plain_update(mp8):
    import torch
    n = 50000
    rng = np.random.default_rng(12)
    w16 = (rng.standard_normal(n) * 0.02).astype(np.float16).view(np.uint16)
    g8 = workloads.random_e5m2_codes(13, (n,))
    a = gpu(w16.view(np.int16))
    b = gpu(w16.view(np.int16))
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    mp8.sgd_update_fp16_sr(a, gpu(g8), 1e-2, 1 / 64.0, round=mp8.SR, seed=1, offset=2)
    mp8.sgd_momentum_fp16_sr(b, v, gpu(g8), 1e-2, 1 / 64.0, 0.0, 0.0, round=mp8.SR, seed=1, offset=2)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    # a skipped step touches neither weights nor velocity
    flag = torch.ones(1, dtype=torch.int32, device="cuda")
    v0, b0 = v.clone(), b.clone()
    mp8.sgd_momentum_fp16_sr(b, v, gpu(g8), 1e-2, 1 / 64.0, 0.9, 0.0, skip_if_nonzero=flag)
    torch.cuda.synchronize()
    assert torch.equal(b, b0) and torch.equal(v, v0)


def _same_f32(got, want):
    """Bit-exact FP32 arrays except for the payload of NaNs."""
    ok = ~np.isnan(want)
    return np.array_equal(np.isnan(got), ~ok) and np.array_equal(got[ok].view(np.uint32), want[ok].view(np.uint32))


@pytest.mark.parametrize("n", [1, 7, 511, 1579, 4099, 1 << 20])
@pytest.mark.parametrize("rnd", [oracle.RNE, oracle.SR])
def test_adam_update_matches_oracle_over_several_steps(mp8, n, rnd):
    """ADAM with L2 regularisation: weights, both FP32 moments and the 8-bit weight copy bit-exact
    against the oracle over four chained steps (division and square root included); the second
    step's gradients contain Inf / NaN codes."""
    import torch
    rng = np.random.default_rng(3 * n + rnd)
    w16 = (rng.standard_normal(n) * np.exp2(rng.integers(-20, 1, n))).astype(np.float16).view(np.uint16)
    m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v0 = (rng.random(n) * 1e-5).astype(np.float32)
    v0[::7] = 0.0                                      # sqrt(0) + eps in the denominator
    lr, inv, b1, b2, eps, wd = 1e-3, 1.0 / 4096, 0.9, 0.999, 1e-8, 1e-4
    wdev, md, vd = gpu(w16.view(np.int16)), gpu(m0), gpu(v0)
    w8d = torch.zeros(n, dtype=torch.uint8, device="cuda")
    ow, om, ov = w16, m0, v0
    for step in range(1, 5):
        g8 = workloads.random_e5m2_codes(100 * step + n % 89, (n,), finite_only=(step != 2))
        st = mp8.new_stats()
        mp8.adam_fp16_sr(wdev, md, vd, gpu(g8), lr, inv, step, beta1=b1, beta2=b2, eps=eps, weight_decay=wd,
                         round=rnd, seed=8, offset=step, w8_out=w8d, stats=st)
        torch.cuda.synchronize()
        ost = oracle.Stats()
        ow, om, ov, o8 = oracle.adam_fp16(ow, om, ov, g8, lr, inv, step, beta1=b1, beta2=b2, eps=eps,
                                          weight_decay=wd, mode=rnd, seed=8, offset=step, want_w8=True, stats=ost)
        assert _same_f32(host(md), om) and _same_f32(host(vd), ov), step
        assert np.array_equal(host(wdev).view(np.uint16), ow), step
        assert np.array_equal(host(w8d), o8), step
        assert mp8.read_stats(st)[1] == ost.nonfinite


def test_adam_update_wide_range_of_moments_skip_and_errors(mp8):
    """Moments and gradients across the whole FP32 / 8-bit range (denormal second moments, huge
    first moments, eps = 0 with zero denominators): still bit for bit; the skip flag; bad steps."""
    import torch
    n = 1 << 16
    rng = np.random.default_rng(77)
    w16 = rng.integers(0, 1 << 16, n).astype(np.uint16)          # every class of half, NaN and Inf too
    m0 = (rng.standard_normal(n) * np.exp2(rng.integers(-140, 100, n).astype(np.float64))).astype(np.float32)
    v0 = np.exp2(rng.integers(-149, 120, n).astype(np.float64)).astype(np.float32)
    g8 = rng.integers(0, 256, n).astype(np.uint8)
    for eps, step in ((0.0, 1), (1e-8, 1000)):
        wdev, md, vd = gpu(w16.view(np.int16)), gpu(m0), gpu(v0)
        mp8.adam_fp16_sr(wdev, md, vd, gpu(g8), 0.01, 1.0 / 128, step, eps=eps, round=mp8.RNE)
        torch.cuda.synchronize()
        ow, om, ov, _ = oracle.adam_fp16(w16, m0, v0, g8, 0.01, 1.0 / 128, step, eps=eps, mode=oracle.RNE)
        assert _same_f32(host(md), om) and _same_f32(host(vd), ov)
        assert np.array_equal(host(wdev).view(np.uint16), ow)
    flag = torch.ones(1, dtype=torch.int32, device="cuda")
    w_before, m_before = wdev.clone(), md.clone()
    mp8.adam_fp16_sr(wdev, md, vd, gpu(g8), 0.01, 1.0, 3, skip_if_nonzero=flag)
    torch.cuda.synchronize()
    assert torch.equal(wdev.view(torch.int16), w_before.view(torch.int16)) and torch.equal(md.view(torch.int32), m_before.view(torch.int32))
    with pytest.raises(mp8.Mp8Error):
        mp8.adam_fp16_sr(wdev, md, vd, gpu(g8), 0.01, 1.0, 0)


@pytest.mark.parametrize("layout", ["row-major", "contraction-major"])
def test_weight_gradient_and_update_in_one_call_against_the_oracle_chain(mp8, layout):
    """mp8_wgrad_update_fp16_sr = GEMM, one rounding to 8 bits, update of the half master
    weights.  Operands whose sums are exact in FP32 make the accumulator equal the oracle's
    reference, so the whole chain -- gradient codes, new master weights, new 8-bit weights -- is
    compared with the oracle's own chain bit for bit: split and unsplit contractions, a ragged
    column count (per-element path), RNE and SR for both roundings, the skip flag."""
    import torch
    from test_gpu_gemm import exact_sum_codes
    rng = np.random.default_rng(17)
    for (M, N, K) in ((1024, 64, 256), (4736, 128, 384), (512, 50, 128), (8192, 64, 64)):
        if layout == "contraction-major" and N % 16:
            continue                                    # that layout wants rows and columns in 16s
        xt, et = exact_sum_codes(rng, (K, M)), exact_sum_codes(rng, (N, M))      # X^T [K, M], dY^T [N, M]
        if M == 8192:                                   # keep the sums exact: three of four terms are zero
            xt[:, rng.random(M) < 0.75] = 0
            assert mp8.gemm_fp8_plan(mp8.WGRAD, M, N, K, 0 if layout == "row-major" else mp8.FLAG_CONTRACTION_MAJOR)[1] > 1
        ref, _ = oracle.gemm_ref(xt, et, want_abs=False)                          # dW [K, N], exact
        w16 = (rng.standard_normal(K * N) * 0.05).astype(np.float16).view(np.uint16)
        alpha, lr, inv = 2.0 ** -9, 0.05, 1.0 / 64
        if layout == "row-major":
            a, b, flags = gpu(xt), gpu(et), 0
        else:
            a, b, flags = gpu(np.ascontiguousarray(xt.T)), gpu(np.ascontiguousarray(et.T)), mp8.FLAG_CONTRACTION_MAJOR
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
        for g_round, w_round, skip in ((oracle.RNE, oracle.SR, 0), (oracle.SR, oracle.RNE, 0), (oracle.RNE, oracle.SR, 3)):
            want_g = oracle.quantize_e5m2(ref.astype(np.float32), scale=alpha, mode=g_round, seed=21, offset=22)[0]
            want_w, want_w8 = oracle.sgd_update_fp16(w16, want_g.reshape(-1), lr, inv, mode=w_round, seed=23, offset=24,
                                                     skip=skip or None, want_w8=True)
            wd = gpu(w16.view(np.int16))
            g8 = torch.full((K * N + 64,), 0xAA, dtype=torch.uint8, device="cuda")
            w8 = torch.full((K * N + 64,), 0x55, dtype=torch.uint8, device="cuda")
            flag = torch.full((1,), skip, dtype=torch.int32, device="cuda")
            st = mp8.new_stats()
            mp8.wgrad_update_fp16_sr(M, N, K, a, b, wd, lr, inv, g8_out=g8[: K * N], alpha=alpha, g_round=g_round,
                                     flags=flags, g_seed=21, g_offset=22, stats=st, w_round=w_round, w_seed=23,
                                     w_offset=24, skip_if_nonzero=flag, w8_out=w8[: K * N], workspace=ws)
            torch.cuda.synchronize()
            assert np.array_equal(host(g8[: K * N]).reshape(K, N), want_g), (M, N, K, g_round)
            assert bool((g8[K * N:] == 0xAA).all()) and bool((w8[K * N:] == 0x55).all())
            assert np.array_equal(host(wd).view(np.uint16), want_w), (M, N, K, w_round, skip)
            if skip:
                assert bool((w8[: K * N] == 0x55).all())           # a skipped step writes no weights
            else:
                assert np.array_equal(host(w8[: K * N]), want_w8), (M, N, K, w_round)
            # the same without keeping the gradient codes
            wd2 = gpu(w16.view(np.int16))
            mp8.wgrad_update_fp16_sr(M, N, K, a, b, wd2, lr, inv, alpha=alpha, g_round=g_round, flags=flags,
                                     g_seed=21, g_offset=22, w_round=w_round, w_seed=23, w_offset=24,
                                     skip_if_nonzero=flag, workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(wd2, wd)


@pytest.mark.parametrize("layout", ["row-major", "contraction-major"])
def test_weight_gradient_and_update_on_the_one_tile_per_cu_plan(mp8, layout):
    """The weight gradient with its SGD step on the plan of the Transformer-big shape class (one
    128x128 tile per CU, a long unsplit contraction, every wave a quarter of it).  Exact-sum operands (nine in ten contraction positions zero) make the chain the
    oracle's: gradient codes (stochastic rounding), master weights (stochastic rounding), 8-bit
    weights, bit for bit; a set skip flag leaves the weights alone; the statistics count the
    gradient's Inf codes."""
    import torch
    from test_gpu_gemm import exact_sum_codes
    rng = np.random.default_rng(53)
    M, N, K = 8192, 3072, 1024
    flags = 0 if layout == "row-major" else mp8.FLAG_CONTRACTION_MAJOR
    assert mp8.gemm_fp8_plan(mp8.WGRAD, M, N, K, flags) == ("128x128x128p", 1)
    xt, et = exact_sum_codes(rng, (K, M)), exact_sum_codes(rng, (N, M))
    xt[:, rng.random(M) < 0.9] = 0
    ref, _ = oracle.gemm_ref(xt, et, want_abs=False)
    w16 = (rng.standard_normal(K * N) * 0.05).astype(np.float16).view(np.uint16)
    lr, inv = 0.05, 1.0 / 64
    a, b = (gpu(xt), gpu(et)) if layout == "row-major" else (gpu(np.ascontiguousarray(xt.T)), gpu(np.ascontiguousarray(et.T)))
    for alpha, skip in ((2.0 ** -9, 0), (2.0 ** -9, 5), (2.0 ** 6, 0)):
        want_g = oracle.quantize_e5m2(ref.astype(np.float32), scale=alpha, mode=oracle.SR, seed=21, offset=22)[0]
        want_w, want_w8 = oracle.sgd_update_fp16(w16, want_g.reshape(-1), lr, inv, mode=oracle.SR, seed=23, offset=24,
                                                 skip=skip or None, want_w8=True)
        for keep_codes in (True, False):
            wd = gpu(w16.view(np.int16))
            g8 = torch.full((K * N + 64,), 0xAA, dtype=torch.uint8, device="cuda")
            w8 = torch.full((K * N + 64,), 0x55, dtype=torch.uint8, device="cuda")
            flag = torch.full((1,), skip, dtype=torch.int32, device="cuda")
            st = mp8.new_stats()
            ws = None if keep_codes else torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), K * N),
                                                     dtype=torch.uint8, device="cuda")
            mp8.wgrad_update_fp16_sr(M, N, K, a, b, wd, lr, inv, g8_out=g8[: K * N] if keep_codes else None, alpha=alpha,
                                     g_round=oracle.SR, flags=flags, g_seed=21, g_offset=22, stats=st, w_round=oracle.SR,
                                     w_seed=23, w_offset=24, skip_if_nonzero=flag, w8_out=w8[: K * N], workspace=ws)
            torch.cuda.synchronize()
            if keep_codes:
                assert np.array_equal(host(g8[: K * N]).reshape(K, N), want_g), (alpha, skip)
            assert bool((g8[K * N:] == 0xAA).all()) and bool((w8[K * N:] == 0x55).all())
            assert np.array_equal(host(wd).view(np.uint16), want_w), (alpha, skip)
            assert mp8.read_stats(st)[1] == int(np.count_nonzero((want_g & 0x7C) == 0x7C))
            if skip:
                assert bool((w8[: K * N] == 0x55).all())
            else:
                assert np.array_equal(host(w8[: K * N]), want_w8), (alpha, skip)


def test_fused_update_with_the_skip_flag_inside_the_statistics_of_the_same_call(mp8):
    """Section 3.1's back-off skips a step whose gradients overflowed.  When the skip flag is the
    Inf/NaN count of the statistics that the very same call accumulates into, the count is only
    final once the whole gradient has been rounded: an overflowing gradient must leave every master
    weight untouched (not a part of them), a clean one must update all of them -- on a split
    contraction (whose finishing pass would otherwise carry the update) and on an unsplit one, for
    the three optimizer rules.  Without g8_out there is nowhere to keep the codes between the two
    launches: rejected."""
    import torch
    from test_gpu_gemm import exact_sum_codes
    rng = np.random.default_rng(41)
    for (M, N, K) in ((8192, 64, 64), (1024, 64, 256)):
        xt, et = exact_sum_codes(rng, (K, M)), exact_sum_codes(rng, (N, M))
        if M == 8192:
            xt[:, rng.random(M) < 0.75] = 0
            assert mp8.gemm_fp8_plan(mp8.WGRAD, M, N, K, 0)[1] > 1
        ref, _ = oracle.gemm_ref(xt, et, want_abs=False)
        a, b = gpu(xt), gpu(et)
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
        w16 = (rng.standard_normal(K * N) * 0.05).astype(np.float16).view(np.uint16)
        lr, inv = 0.05, 1.0 / 64
        for alpha in (2.0 ** 20, 2.0 ** -9):          # every sum overflows / none does
            want_g = oracle.quantize_e5m2(ref.astype(np.float32), scale=alpha)[0]
            overflow = int(np.count_nonzero((want_g & 0x7C) == 0x7C))
            assert (overflow > 0) == (alpha > 1)
            want_w, want_w8 = oracle.sgd_update_fp16(w16, want_g.reshape(-1), lr, inv, mode=oracle.SR, seed=23, offset=24,
                                                     skip=overflow or None, want_w8=True)
            if overflow:
                assert np.array_equal(want_w, w16)
            for rule in ("sgd", "momentum", "adam"):
                wd = gpu(w16.view(np.int16))
                g8 = torch.full((K * N,), 0xAA, dtype=torch.uint8, device="cuda")
                w8 = torch.full((K * N,), 0x55, dtype=torch.uint8, device="cuda")
                st = mp8.new_stats()
                flag = st[1:2]                                   # the nonfinite word of the same struct
                common = dict(g8_out=g8, alpha=alpha, stats=st, w_round=oracle.SR, w_seed=23, w_offset=24,
                              skip_if_nonzero=flag, w8_out=w8, workspace=ws)
                if rule == "sgd":
                    mp8.wgrad_update_fp16_sr(M, N, K, a, b, wd, lr, inv, **common)
                elif rule == "momentum":
                    vel = torch.zeros(K * N, dtype=torch.float32, device="cuda")
                    mp8.wgrad_momentum_fp16_sr(M, N, K, a, b, wd, vel, lr, inv, 0.0, 0.0, **common)
                else:
                    m1 = torch.zeros(K * N, dtype=torch.float32, device="cuda")
                    m2 = torch.zeros(K * N, dtype=torch.float32, device="cuda")
                    mp8.wgrad_adam_fp16_sr(M, N, K, a, b, wd, m1, m2, lr, inv, 1, **common)
                torch.cuda.synchronize()
                assert np.array_equal(host(g8).reshape(K, N), want_g), (M, rule)
                assert mp8.read_stats(st)[1] == overflow
                got = host(wd).view(np.uint16)
                if overflow:
                    assert np.array_equal(got, w16), (M, rule, "an overflowed step must not touch any weight")
                    assert bool((w8 == 0x55).all())
                    if rule == "adam":
                        assert not bool(m1.any()) and not bool(m2.any())
                elif rule != "adam":                             # momentum 0, decay 0 = the plain update
                    assert np.array_equal(got, want_w), (M, rule)
                    assert np.array_equal(host(w8), want_w8)
                else:
                    assert not np.array_equal(got, w16)
        if M == 8192:
            st = mp8.new_stats()
            with pytest.raises(mp8.Mp8Error):
                mp8.wgrad_update_fp16_sr(M, N, K, a, b, gpu(w16.view(np.int16)), lr, inv, stats=st,
                                         skip_if_nonzero=st[1:2], workspace=ws)


@pytest.mark.parametrize("layout", ["row-major", "contraction-major"])
def test_weight_gradient_and_momentum_update_in_one_call_against_the_oracle_chain(mp8, layout):
    """mp8_wgrad_momentum_fp16_sr over two consecutive steps (the velocity carries over) on exact-sum
    operands: gradient codes, master weights, velocity and 8-bit weights bit for bit the oracle's
    chain GEMM -> one rounding -> momentum update with L2 regularisation; split and unsplit
    contractions, a ragged column count, RNE and SR, the skip flag."""
    import torch
    from test_gpu_gemm import exact_sum_codes
    rng = np.random.default_rng(29)
    for (M, N, K) in ((1024, 64, 256), (512, 50, 128), (8192, 64, 64)):
        if layout == "contraction-major" and N % 16:
            continue
        xt, et = exact_sum_codes(rng, (K, M)), exact_sum_codes(rng, (N, M))
        if M == 8192:
            xt[:, rng.random(M) < 0.75] = 0
        ref, _ = oracle.gemm_ref(xt, et, want_abs=False)
        alpha, lr, inv, mu, wd_ = 2.0 ** -9, 0.05, 1.0 / 64, 0.9, 1e-3
        if layout == "row-major":
            a, b, flags = gpu(xt), gpu(et), 0
        else:
            a, b, flags = gpu(np.ascontiguousarray(xt.T)), gpu(np.ascontiguousarray(et.T)), mp8.FLAG_CONTRACTION_MAJOR
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
        for g_round, w_round, skip in ((oracle.RNE, oracle.SR, 0), (oracle.SR, oracle.RNE, 0), (oracle.RNE, oracle.SR, 2)):
            w_ref = (rng.standard_normal(K * N) * 0.05).astype(np.float16).view(np.uint16)
            v_ref = (rng.standard_normal(K * N) * 0.01).astype(np.float32)
            wdev, vdev = gpu(w_ref.view(np.int16)), gpu(v_ref)
            g8 = torch.full((K * N + 64,), 0xAA, dtype=torch.uint8, device="cuda")
            w8 = torch.full((K * N + 64,), 0x55, dtype=torch.uint8, device="cuda")
            flag = torch.full((1,), skip, dtype=torch.int32, device="cuda")
            for step in (1, 2):
                want_g = oracle.quantize_e5m2(ref.astype(np.float32), scale=alpha, mode=g_round, seed=31, offset=step)[0]
                w_ref, v_ref, want_w8 = oracle.sgd_momentum_fp16(w_ref, v_ref, want_g.reshape(-1), lr, inv, mu, wd_,
                                                                 mode=w_round, seed=33, offset=step,
                                                                 skip=skip or None, want_w8=True)
                mp8.wgrad_momentum_fp16_sr(M, N, K, a, b, wdev, vdev, lr, inv, mu, wd_, g8_out=g8[: K * N],
                                           alpha=alpha, g_round=g_round, flags=flags, g_seed=31, g_offset=step,
                                           w_round=w_round, w_seed=33, w_offset=step, skip_if_nonzero=flag,
                                           w8_out=w8[: K * N], workspace=ws)
                torch.cuda.synchronize()
                assert np.array_equal(host(g8[: K * N]).reshape(K, N), want_g), (M, N, K, g_round, step)
                assert np.array_equal(host(wdev).view(np.uint16), w_ref), (M, N, K, w_round, skip, step)
                assert np.array_equal(host(vdev).view(np.uint32), v_ref.view(np.uint32)), (M, N, K, skip, step)
                if skip:
                    assert bool((w8[: K * N] == 0x55).all())
                else:
                    assert np.array_equal(host(w8[: K * N]), want_w8)
            assert bool((g8[K * N:] == 0xAA).all()) and bool((w8[K * N:] == 0x55).all())
    # and on random operands: the one call equals the two calls it stands for
    M, N, K = 4736, 128, 384
    x8 = workloads.random_e5m2_codes(5, (M, K)) & 0xBF
    e8 = workloads.random_e5m2_codes(6, (M, N)) & 0xBF
    a, b = gpu(x8), gpu(e8)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
    w0 = (rng.standard_normal(K * N) * 0.05).astype(np.float16).view(np.int16)
    v0 = (rng.standard_normal(K * N) * 0.01).astype(np.float32)
    w1, v1, g1, q1 = gpu(w0), gpu(v0), torch.zeros(K * N, dtype=torch.uint8, device="cuda"), torch.zeros(K * N, dtype=torch.uint8, device="cuda")
    mp8.wgrad_momentum_fp16_sr(M, N, K, a, b, w1, v1, 0.01, 1 / 16, 0.9, 5e-4, g8_out=g1, flags=mp8.FLAG_CONTRACTION_MAJOR,
                               w_seed=3, w_offset=4, w8_out=q1, workspace=ws)
    w2, v2, g2, q2 = gpu(w0), gpu(v0), torch.zeros((K, N), dtype=torch.uint8, device="cuda"), torch.zeros(K * N, dtype=torch.uint8, device="cuda")
    mp8.gemm_fp8(mp8.WGRAD, M, N, K, a, b, out8=g2, flags=mp8.FLAG_CONTRACTION_MAJOR, workspace=ws)
    mp8.sgd_momentum_fp16_sr(w2, v2, g2.view(-1), 0.01, 1 / 16, 0.9, 5e-4, round=mp8.SR, seed=3, offset=4, w8_out=q2)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2.view(-1)) and torch.equal(w1, w2) and torch.equal(v1.view(torch.int32), v2.view(torch.int32))
    assert torch.equal(q1, q2)


def test_weight_gradient_and_adam_update_in_one_call_against_the_oracle_chain(mp8):
    """mp8_wgrad_adam_fp16_sr over two consecutive steps (moments and bias corrections carry over)
    on exact-sum operands: gradient codes, master weights, both moments and the 8-bit weights bit
    for bit the oracle's chain GEMM -> one rounding -> ADAM; split and unsplit contractions, a
    ragged column count, SR and RNE, the skip flag; then the one call against the two calls on
    random operands."""
    import torch
    from test_gpu_gemm import exact_sum_codes
    rng = np.random.default_rng(41)
    for (M, N, K) in ((1024, 64, 256), (512, 50, 128), (8192, 64, 64)):
        xt, et = exact_sum_codes(rng, (K, M)), exact_sum_codes(rng, (N, M))
        if M == 8192:
            xt[:, rng.random(M) < 0.75] = 0
        ref, _ = oracle.gemm_ref(xt, et, want_abs=False)
        alpha, lr, inv, wd_ = 2.0 ** -9, 0.01, 1.0 / 64, 1e-3
        a, b = gpu(xt), gpu(et)
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
        for w_round, skip in ((oracle.SR, 0), (oracle.RNE, 0), (oracle.SR, 5)):
            w_ref = (rng.standard_normal(K * N) * 0.05).astype(np.float16).view(np.uint16)
            m_ref = (rng.standard_normal(K * N) * 0.01).astype(np.float32)
            v_ref = (rng.random(K * N) * 1e-3).astype(np.float32)
            wdev, mdev, vdev = gpu(w_ref.view(np.int16)), gpu(m_ref), gpu(v_ref)
            g8 = torch.full((K * N + 64,), 0xAA, dtype=torch.uint8, device="cuda")
            w8 = torch.full((K * N + 64,), 0x55, dtype=torch.uint8, device="cuda")
            flag = torch.full((1,), skip, dtype=torch.int32, device="cuda")
            want_g = oracle.quantize_e5m2(ref.astype(np.float32), scale=alpha)[0]
            for step in (1, 2):
                w_ref, m_ref, v_ref, want_w8 = oracle.adam_fp16(w_ref, m_ref, v_ref, want_g.reshape(-1), lr, inv, step,
                                                                weight_decay=wd_, mode=w_round, seed=43, offset=step,
                                                                skip=skip or None, want_w8=True)
                mp8.wgrad_adam_fp16_sr(M, N, K, a, b, wdev, mdev, vdev, lr, inv, step, weight_decay=wd_,
                                       g8_out=g8[: K * N], alpha=alpha, w_round=w_round, w_seed=43, w_offset=step,
                                       skip_if_nonzero=flag, w8_out=w8[: K * N], workspace=ws)
                torch.cuda.synchronize()
                assert np.array_equal(host(g8[: K * N]).reshape(K, N), want_g), (M, N, K, step)
                assert np.array_equal(host(wdev).view(np.uint16), w_ref), (M, N, K, w_round, skip, step)
                assert np.array_equal(host(mdev).view(np.uint32), m_ref.view(np.uint32)), (M, N, K, skip, step)
                assert np.array_equal(host(vdev).view(np.uint32), v_ref.view(np.uint32)), (M, N, K, skip, step)
                if skip:
                    assert bool((w8[: K * N] == 0x55).all())
                else:
                    assert np.array_equal(host(w8[: K * N]), want_w8)
            assert bool((g8[K * N:] == 0xAA).all()) and bool((w8[K * N:] == 0x55).all())
    M, N, K = 4736, 128, 384
    a, b = gpu(workloads.random_e5m2_codes(7, (M, K)) & 0xBF), gpu(workloads.random_e5m2_codes(8, (M, N)) & 0xBF)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
    w0 = (rng.standard_normal(K * N) * 0.05).astype(np.float16).view(np.int16)
    m0 = (rng.standard_normal(K * N) * 0.01).astype(np.float32)
    v0 = (rng.random(K * N) * 1e-3).astype(np.float32)
    w1, m1, v1 = gpu(w0), gpu(m0), gpu(v0)
    g1, q1 = torch.zeros(K * N, dtype=torch.uint8, device="cuda"), torch.zeros(K * N, dtype=torch.uint8, device="cuda")
    mp8.wgrad_adam_fp16_sr(M, N, K, a, b, w1, m1, v1, 1e-3, 1 / 16, 3, g8_out=g1, flags=mp8.FLAG_CONTRACTION_MAJOR,
                           w_seed=3, w_offset=4, w8_out=q1, workspace=ws)
    w2, m2, v2 = gpu(w0), gpu(m0), gpu(v0)
    g2, q2 = torch.zeros((K, N), dtype=torch.uint8, device="cuda"), torch.zeros(K * N, dtype=torch.uint8, device="cuda")
    mp8.gemm_fp8(mp8.WGRAD, M, N, K, a, b, out8=g2, flags=mp8.FLAG_CONTRACTION_MAJOR, workspace=ws)
    mp8.adam_fp16_sr(w2, m2, v2, g2.view(-1), 1e-3, 1 / 16, 3, round=mp8.SR, seed=3, offset=4, w8_out=q2)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2.view(-1)) and torch.equal(w1, w2) and torch.equal(q1, q2)
    assert torch.equal(m1.view(torch.int32), m2.view(torch.int32)) and torch.equal(v1.view(torch.int32), v2.view(torch.int32))
