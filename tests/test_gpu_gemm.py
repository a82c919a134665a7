"""GPU parity: mp8_gemm_fp8 (all three training GEMMs, RNE and SR epilogue, split
contraction, ragged shapes) against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_1905_12334_amd import workloads
from gpu_util import gpu, host, check_outputs, acc_tolerance_ok, signed_rank

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mp8():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1905_12334_amd as m
    m.lib()
    return m


def run_gemm(mp8, a8, b8, op=None, dims=None, want_t=False, acc_in=None, acc_mode=1, **kw):
    """out[r,c] = sum_j a8[r,j] b8[c,j] through the C ABI; returns (acc, out8, out8_t, stats)."""
    import torch
    rows, kc = a8.shape
    cols = b8.shape[0]
    if op is None:
        op, dims = mp8.FWD, (rows, cols, kc)
    M, N, K = dims
    a, b = gpu(a8), gpu(b8)
    acc = torch.full((rows * cols + 16,), 7.0, dtype=torch.float32, device="cuda")
    if acc_in is not None:
        acc[: rows * cols] = gpu(acc_in).reshape(-1)
    obuf = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    out8 = obuf[: rows * cols]
    out8_t = torch.full((rows * cols,), 0xAA, dtype=torch.uint8, device="cuda") if want_t else None
    tile, split = kw.pop("tile_config", 0), kw.pop("split_k", 0)
    wsb = mp8.gemm_fp8_workspace_bytes(op, M, N, K, tile, split)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    stats = mp8.new_stats()
    mp8.gemm_fp8(op, M, N, K, a, b, out8=out8, out8_t=out8_t, acc=acc[: rows * cols],
                 acc_mode=acc_mode, stats=stats, workspace=ws, tile_config=tile, split_k=split, **kw)
    torch.cuda.synchronize()
    assert bool((obuf[rows * cols:] == 0xAA).all()), "write past the end of out8"
    assert bool((acc[rows * cols:] == 7.0).all()), "write past the end of acc"
    res = (host(acc[: rows * cols]).reshape(rows, cols), host(out8).reshape(rows, cols),
           host(out8_t).reshape(cols, rows) if want_t else None, mp8.read_stats(stats))
    if acc_mode == 1:
        # the same call without FP32 / transposed outputs takes the fused epilogue (when the
        # contraction is not split): its codes and statistics must be identical; once with
        # statistics, once without (two different kernels)
        for with_stats in (True, False):
            o2 = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
            st2 = mp8.new_stats() if with_stats else None
            mp8.gemm_fp8(op, M, N, K, a, b, out8=o2[: rows * cols], stats=st2, workspace=ws,
                         tile_config=tile, split_k=split, **kw)
            torch.cuda.synchronize()
            assert bool((o2[rows * cols:] == 0xAA).all()), "fused: write past the end of out8"
            assert np.array_equal(host(o2[: rows * cols]).reshape(rows, cols), res[1]), "fused out8 differs"
            if with_stats:
                assert mp8.read_stats(st2) == res[3], "fused statistics differ"
    return res


def exact_sum_codes(rng, shape):
    """Codes of {1,1.25,1.5,1.75} * 2^{0..3}, both signs: sums of up to 1024 products of two such
    values are integers/16 below 2^24, hence exact in FP32 in any order."""
    e = rng.integers(15, 19, shape)
    m = rng.integers(0, 4, shape)
    s = rng.integers(0, 2, shape)
    return ((s << 7) | (e << 2) | m).astype(np.uint8)


@pytest.mark.parametrize("kpos", [0, 37, 127, 200])
def test_exhaustive_product_table(mp8, kpos):
    """All 256 x 256 code pairs through the matrix cores: one non-zero contraction position,
    so the FP32 accumulator must be exactly value(a) * value(b), with IEEE Inf/NaN classes."""
    a8 = np.zeros((256, 256), np.uint8)
    b8 = np.zeros((256, 256), np.uint8)
    a8[:, kpos] = np.arange(256)
    b8[:, kpos] = np.arange(256)
    acc, out8, _, _ = run_gemm(mp8, a8, b8)
    ref, _ = oracle.gemm_ref(a8, b8, want_abs=False)
    assert np.array_equal(np.isnan(acc), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(acc[ok].astype(np.float64), ref[ok])
    assert np.array_equal(np.signbit(acc[ok]), np.signbit(ref[ok]))
    want8, _ = oracle.quantize_e5m2(acc)
    assert np.array_equal(out8, want8)


def test_exact_sums_every_tile_config_and_split(mp8):
    rng = np.random.default_rng(10)
    rows, cols, kc = 320, 288, 1024        # ragged against every tile shape
    a8, b8 = exact_sum_codes(rng, (rows, kc)), exact_sum_codes(rng, (cols, kc))
    ref, _ = oracle.gemm_ref(a8, b8, want_abs=False)
    want8 = oracle.round_ref_e5m2(ref)
    ntiles = len(mp8.gemm_tile_configs())
    for tile in range(0, ntiles + 1):
        if tile > 0 and mp8.gemm_fp8_plan(mp8.FWD, rows, cols, kc, 0, tile)[0] is None:
            with pytest.raises(mp8.Mp8Error):       # a kernel for short contractions only
                run_gemm(mp8, a8, b8, tile_config=tile)
            continue
        for split in (0, 1, 2, 3, 8):
            acc, out8, out8_t, _ = run_gemm(mp8, a8, b8, want_t=True, tile_config=tile, split_k=split)
            assert np.array_equal(acc.astype(np.float64), ref), (tile, split)
            assert np.array_equal(out8, want8), (tile, split)
            assert np.array_equal(out8_t, want8.T), (tile, split)


def test_static_lds_of_every_kernel_is_what_its_tile_implies(mp8):
    """The number of workgroups a CU holds hangs on the LDS a kernel allocates: a ring of S
    stages of (BM + BN) x 128 bytes and nothing else (a private array that the compiler moved
    to LDS once cost a third of the speed of the split kernels without failing any test)."""
    for i, name in enumerate(mp8.gemm_tile_configs(), start=1):
        for epi in range(3):
            got = mp8.gemm_tile_config_lds_bytes(i, epi)
            if name.endswith("k"):          # all stages in dynamic LDS; statistics need 1 KB
                assert 0 <= got <= 1024, (name, epi, got)
            elif name.endswith("p"):        # one stage per wave, or four half tiles of FP32 for the reduction
                assert 4 * 64 * 132 * 4 <= got <= 4 * 64 * 132 * 4 + 1024, (name, epi, got)
            elif name.endswith("w"):        # a two-stage ring of (BM + BN) x 128 bytes per wave
                bm, bn = (int(x) for x in name.split("x")[:2])
                ring = 4 * 2 * (bm + bn) * 128
                assert ring <= got <= ring + 1024, (name, epi, got)
            else:
                bm, bn, rest = name.split("x")
                stages = int(rest.split("s")[1])
                ring = stages * (int(bm) + int(bn)) * 128
                # (the FP32 row bands of the largest tile's epilogue need 4 KB more than its ring)
                assert ring <= got <= ring + 4096 + 1024, (name, epi, got)   # + statistics


@pytest.mark.parametrize("kc", [128, 256])
def test_short_contraction_every_tile_config(mp8, kc):
    """Contractions of one or two 128-byte stages, where a dedicated kernel exists: every tile
    configuration gives the exact sums, on row and column counts ragged against every tile, with
    the fused and the two-pass epilogue, RNE and SR, statistics and saturation."""
    rng = np.random.default_rng(kc)
    names = mp8.gemm_tile_configs()
    for rows, cols in ((320, 288), (130, 200), (1, 16)):
        a8, b8 = exact_sum_codes(rng, (rows, kc)), exact_sum_codes(rng, (cols, kc))
        ref, _ = oracle.gemm_ref(a8, b8, want_abs=False)
        want8 = oracle.round_ref_e5m2(ref)
        used = set()
        for tile in range(0, len(names) + 1):
            used.add(mp8.gemm_fp8_plan(mp8.FWD, rows, cols, kc, 0, tile)[0])
            acc, out8, out8_t, _ = run_gemm(mp8, a8, b8, want_t=True, tile_config=tile)
            assert np.array_equal(acc.astype(np.float64), ref), (tile, rows, cols)
            assert np.array_equal(out8, want8), (tile, rows, cols)
            assert np.array_equal(out8_t, want8.T), (tile, rows, cols)
        assert used >= set(names)               # every kernel, the short-contraction one included
    # the dedicated kernel with everything its epilogue carries (large alpha: overflows)
    short = 1 + [n.endswith("k") for n in names].index(True)
    a8 = workloads.random_e5m2_codes(kc, (300, kc))
    b8 = workloads.random_e5m2_codes(kc + 1, (272, kc))
    a8, b8 = (a8 & 0x83) | 0x3C, (b8 & 0x83) | 0x3C
    ref, absref = oracle.gemm_ref(a8, b8)
    for mode, flags, alpha in ((oracle.RNE, 0, 1.0), (oracle.SR, 0, 0.37), (oracle.SR, oracle.FLAG_SATURATE, 3000.0),
                               (oracle.RNE, 0, 3000.0)):
        acc, out8, _, st = run_gemm(mp8, a8, b8, tile_config=short, round=mode, flags=flags, alpha=alpha,
                                    seed=11, offset=5)
        check_outputs(acc, out8, ref, absref, kc, mode=mode, seed=11, offset=5, alpha=alpha, flags=flags)
        ost = oracle.Stats()
        oracle.quantize_e5m2(acc, scale=alpha, mode=mode, seed=11, offset=5, flags=flags, stats=ost)
        assert st == ost.as_tuple(), (mode, flags, alpha)


def test_short_contraction_automatic_choice_full_size(mp8):
    """A backward-data GEMM of the shape the planner gives to the short-contraction kernel
    (2048 x 1536 outputs, contraction 128), checked element by element."""
    rows, cols, kc = 2048, 1536, 128
    assert mp8.gemm_fp8_plan(mp8.BWD_DATA, rows, kc, cols)[0].endswith("k")
    a8 = workloads.random_e5m2_codes(31, (rows, kc))
    b8 = workloads.random_e5m2_codes(32, (cols, kc))
    a8, b8 = (a8 & 0x83) | 0x38, (b8 & 0x83) | 0x38
    acc, out8, _, _ = run_gemm(mp8, a8, b8, op=mp8.BWD_DATA, dims=(rows, kc, cols))
    ref, absref = oracle.gemm_ref(a8, b8)
    check_outputs(acc, out8, ref, absref, kc)


@pytest.mark.parametrize("rows,cols,kc,alpha", [(160 * 128 + 37, 1152, 128, 1.0), (161 * 128, 384, 256, 0.25),
                                                (25088, 1152, 128, 1.0), (160 * 128 + 1, 384, 128, 1.0)])
def test_short_contraction_many_row_blocks(mp8, rows, cols, kc, alpha):
    """Short contraction over many blocks of 128 rows and whole 128-column tiles (the
    backward-data GEMM of configs[1] is the third case): exact-sum operands, every output byte
    against the oracle, with a ragged and a full last row block; the fused RNE epilogue and the
    path with an FP32 output (finishing pass) must give the same codes."""
    import torch
    rng = np.random.default_rng(rows + cols + kc)
    a8, b8 = exact_sum_codes(rng, (rows, kc)), exact_sum_codes(rng, (cols, kc))
    ref, _ = oracle.gemm_ref(a8, b8, want_abs=False)
    want8 = oracle.round_ref_e5m2(ref, alpha=alpha)
    a, b = gpu(a8), gpu(b8)
    obuf = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    for _ in range(2):          # twice: the second call finds the caches warm
        mp8.gemm_fp8(mp8.FWD, rows, cols, kc, a, b, out8=obuf[: rows * cols].view(rows, cols), alpha=alpha)
    torch.cuda.synchronize()
    assert bool((obuf[rows * cols:] == 0xAA).all()), "write past the end of out8"
    assert np.array_equal(host(obuf[: rows * cols]).reshape(rows, cols), want8)
    acc, out8, _, _ = run_gemm(mp8, a8, b8, alpha=alpha)
    assert np.array_equal(acc.astype(np.float64), ref)
    assert np.array_equal(out8, want8)


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (17, 33, 100), (64, 64, 128), (100, 36, 256),
                                   (257, 130, 384), (31, 515, 128), (130, 70, 130)])
def test_ragged_shapes_identity_and_onehot(mp8, shape):
    rows, cols, kc = shape
    rng = np.random.default_rng(rows * 7 + cols)
    a8 = workloads.random_e5m2_codes(rows + 1, (rows, kc))
    sel = rng.integers(0, kc, cols)
    b8 = np.zeros((cols, kc), np.uint8)
    b8[np.arange(cols), sel] = 0x3C                     # 1.0: out[r,c] = a[r, sel[c]]
    acc, out8, out8_t, _ = run_gemm(mp8, a8, b8, want_t=True)
    ref, _ = oracle.gemm_ref(a8, b8, want_abs=False)
    assert np.array_equal(acc.astype(np.float64), ref)
    want8, _ = oracle.quantize_e5m2(acc)
    assert np.array_equal(out8, want8) and np.array_equal(out8_t, want8.T)
    # random operands on the same ragged shape
    b8 = workloads.random_e5m2_codes(cols + 2, (cols, kc))
    a8 = (a8 & 0x83) | 0x38 | (a8 & 0x0C) >> 2 << 2    # exponents 14..15: no overflow
    b8 = (b8 & 0x83) | 0x38 | (b8 & 0x0C) >> 2 << 2
    acc, out8, _, _ = run_gemm(mp8, a8, b8)
    ref, absref = oracle.gemm_ref(a8, b8)
    check_outputs(acc, out8, ref, absref, kc)


def _layer_operands(lay):
    """8-bit operands of one layer as the library wants them (all from the oracle's Q)."""
    X8, X8t = oracle.quantize_e5m2(lay.X, want_t=True)
    W8, W8t = oracle.quantize_e5m2(lay.W, want_t=True)
    E8, E8t = oracle.quantize_e5m2(lay.dY, scale=lay.loss_scale, want_t=True)
    return X8, X8t, W8, W8t, E8, E8t


def test_config1_square_256(mp8):
    lay = workloads.config1()
    X8, _, _, W8t, _, _ = _layer_operands(lay)
    acc, out8, _, st = run_gemm(mp8, X8, W8t, op=mp8.FWD, dims=(256, 256, 256))
    ref, absref = oracle.gemm_ref(X8, W8t)
    check_outputs(acc, out8, ref, absref, 256)
    ost = oracle.Stats()
    oracle.quantize_e5m2(acc, stats=ost)
    assert st == ost.as_tuple()
    # the reference itself agrees with a float64 matmul of independently decoded operands
    dec = lambda c: (c.astype(np.uint16) << 8).view(np.float16).astype(np.float64)
    assert np.allclose(ref, dec(X8) @ dec(W8t).T, rtol=1e-12, atol=1e-12)


def test_three_training_gemms_small_layer(mp8):
    lay = workloads.config2(batch=1, hw=16, cin=128, cout=64)     # M=256, K=1152, N=64
    M, N, K = lay.M, lay.N, lay.K
    X8, X8t, W8, W8t, E8, E8t = _layer_operands(lay)
    # forward: contraction K
    acc, out8, _, _ = run_gemm(mp8, X8, W8t, op=mp8.FWD, dims=(M, N, K))
    ref, absref = oracle.gemm_ref(X8, W8t)
    check_outputs(acc, out8, ref, absref, K)
    # backward data: contraction N; equals forward GEMM on explicitly transposed inputs
    acc, out8, _, _ = run_gemm(mp8, E8, W8, op=mp8.BWD_DATA, dims=(M, N, K))
    ref, absref = oracle.gemm_ref(E8, W8)
    assert acc.shape == (M, K)
    check_outputs(acc, out8, ref, absref, N)
    # weight gradient: contraction M, un-scaled in the epilogue via alpha
    alpha = 1.0 / 64
    acc, out8, _, _ = run_gemm(mp8, X8t, E8t, op=mp8.WGRAD, dims=(M, N, K), alpha=alpha)
    ref, absref = oracle.gemm_ref(X8t, E8t)
    assert acc.shape == (K, N)
    check_outputs(acc, out8, ref, absref, M, alpha=alpha)


def test_sr_epilogue_matches_oracle_stream(mp8):
    lay = workloads.config5(tokens=512, d_in=128, d_out=192)
    X8, X8t, _, _, E8, E8t = _layer_operands(lay)
    seed, offset = lay.extra["seed"], 17
    for split in (1, 4):
        acc, out8, out8_t, st = run_gemm(mp8, X8t, E8t, op=mp8.WGRAD, dims=(lay.M, lay.N, lay.K),
                                         round=oracle.SR, seed=seed, offset=offset, want_t=True,
                                         split_k=split)
        ref, absref = oracle.gemm_ref(X8t, E8t)
        check_outputs(acc, out8, ref, absref, lay.M, mode=oracle.SR, seed=seed, offset=offset)
        assert np.array_equal(out8_t, out8.T)
        # bracket of the reference: toward-zero code or the next one (+-1 for accumulator error)
        lo = np.vectorize(lambda v: oracle.e5m2_encode(v, oracle.SR, 0))(ref).astype(np.uint8)
        d = signed_rank(out8) - signed_rank(lo)
        away = np.where(signed_rank(lo) < 0, -d, d)
        well = np.abs(ref) >= absref / np.sqrt(float(lay.M))      # well-conditioned sums only
        assert away[well].min() >= -1 and away[well].max() <= 2
    # a ragged column count takes the per-element stream path
    a8 = workloads.random_e5m2_codes(1, (70, 256))
    b8 = workloads.random_e5m2_codes(2, (50, 256))
    a8, b8 = (a8 & 0x83) | 0x3C, (b8 & 0x83) | 0x3C
    acc, out8, _, _ = run_gemm(mp8, a8, b8, round=oracle.SR, seed=5, offset=6)
    ref, absref = oracle.gemm_ref(a8, b8)
    check_outputs(acc, out8, ref, absref, 256, mode=oracle.SR, seed=5, offset=6)


def test_accumulate_across_calls_equals_stacked_contraction(mp8):
    """GNMT-style weight gradient: per-timestep GEMMs accumulated in FP32 (acc_mode 2) and one
    GEMM over the stacked timesteps must both match the one double reference; rounding to 8 bits
    happens once, after the last step."""
    steps, batch, kdim, ndim = 4, 128, 64, 96
    rng = np.random.default_rng(4)
    xs = [workloads.random_e5m2_codes(100 + t, (kdim, batch)) for t in range(steps)]   # X_t^T [K, B]
    es = [workloads.random_e5m2_codes(200 + t, (ndim, batch)) for t in range(steps)]   # dY_t^T [N, B]
    xs = [(x & 0x83) | 0x38 for x in xs]
    es = [(e & 0x83) | 0x34 for e in es]
    a_stack, b_stack = np.concatenate(xs, axis=1), np.concatenate(es, axis=1)
    ref, absref = oracle.gemm_ref(a_stack, b_stack)
    acc1, out1, _, _ = run_gemm(mp8, a_stack, b_stack, op=mp8.WGRAD, dims=(steps * batch, ndim, kdim))
    check_outputs(acc1, out1, ref, absref, steps * batch)
    acc = np.zeros((kdim, ndim), np.float32)
    for t in range(steps):
        acc, out2, _, _ = run_gemm(mp8, xs[t], es[t], op=mp8.WGRAD, dims=(batch, ndim, kdim),
                                   acc_in=acc, acc_mode=2)
    check_outputs(acc, out2, ref, absref, steps * batch)


def test_alpha_saturate_stats_nonfinite_and_determinism(mp8):
    rng = np.random.default_rng(6)
    a8 = workloads.random_e5m2_codes(7, (256, 512))
    b8 = workloads.random_e5m2_codes(8, (128, 512))
    a8, b8 = (a8 & 0x83) | 0x58, (b8 & 0x83) | 0x58         # values ~ 2^7: sums overflow 57344
    acc, out8, _, st = run_gemm(mp8, a8, b8)
    ost = oracle.Stats()
    want, _ = oracle.quantize_e5m2(acc, stats=ost)
    assert np.array_equal(out8, want) and st == ost.as_tuple() and st[1] > 0
    acc_s, out_s, _, st_s = run_gemm(mp8, a8, b8, flags=oracle.FLAG_SATURATE)
    want_s, _ = oracle.quantize_e5m2(acc_s, flags=oracle.FLAG_SATURATE)
    assert np.array_equal(out_s, want_s) and st_s[1] == 0
    # Inf / NaN operand codes propagate as IEEE says
    a8[0, 0], b8[0, 0], b8[1, 0] = 0x7C, 0x00, 0x3C
    acc_n, out_n, _, _ = run_gemm(mp8, a8, b8)
    ref, _ = oracle.gemm_ref(a8, b8, want_abs=False)
    assert np.isnan(acc_n[0, 0]) and np.isnan(ref[0, 0]) and out_n[0, 0] == 0x7F
    assert np.isinf(acc_n[0, 1]) and acc_n[0, 1] == ref[0, 1]
    # bit-reproducible, including the split path
    for split in (1, 4):
        r1 = run_gemm(mp8, a8, b8, split_k=split, round=oracle.SR, seed=1, offset=2)
        r2 = run_gemm(mp8, a8, b8, split_k=split, round=oracle.SR, seed=1, offset=2)
        assert np.array_equal(r1[0], r2[0], equal_nan=True) and np.array_equal(r1[1], r2[1])
    # out8 only (no accumulator requested), as the benchmark calls it
    import torch
    o = torch.empty(256 * 128, dtype=torch.uint8, device="cuda")
    mp8.gemm_fp8(mp8.FWD, 256, 128, 512, gpu(a8), gpu(b8), out8=o)
    torch.cuda.synchronize()
    assert np.array_equal(host(o).reshape(256, 128), out_n)
    # leading dimensions larger than the contraction length (operands are column windows)
    big_a = workloads.random_e5m2_codes(9, (64, 640))
    big_b = workloads.random_e5m2_codes(10, (64, 768))
    big_a, big_b = (big_a & 0x83) | 0x38, (big_b & 0x83) | 0x38
    accl = torch.empty(64 * 64, dtype=torch.float32, device="cuda")
    mp8.gemm_fp8(mp8.FWD, 64, 64, 256, gpu(big_a).reshape(-1)[128:], gpu(big_b).reshape(-1)[256:],
                 acc=accl, acc_mode=1, lda=640, ldb=768)
    torch.cuda.synchronize()
    ref, _ = oracle.gemm_ref(big_a[:, 128:384], big_b[:, 256:512], want_abs=False)
    assert np.array_equal(host(accl).reshape(64, 64).astype(np.float64), ref)


def run_gemm_tn(mp8, a_km, b_km, **kw):
    """out[r,c] = sum_j a_km[j,r] b_km[j,c] with contraction-major operands; returns (acc, out8)."""
    import torch
    kc, rows = a_km.shape
    cols = b_km.shape[1]
    tile, split = kw.pop("tile_config", 0), kw.pop("split_k", 0)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, rows, cols, kc, tile, split), 16),
                     dtype=torch.uint8, device="cuda")
    acc = torch.full((rows * cols + 16,), 7.0, dtype=torch.float32, device="cuda")
    obuf = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    flags = kw.pop("flags", 0) | mp8.FLAG_CONTRACTION_MAJOR
    mp8.gemm_fp8(mp8.FWD, rows, cols, kc, gpu(a_km), gpu(b_km), out8=obuf[: rows * cols],
                 acc=acc[: rows * cols], acc_mode=1, workspace=ws, flags=flags, tile_config=tile,
                 split_k=split, **kw)
    o2 = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    mp8.gemm_fp8(mp8.FWD, rows, cols, kc, gpu(a_km), gpu(b_km), out8=o2[: rows * cols], workspace=ws,
                 flags=flags, tile_config=tile, split_k=split, **kw)
    torch.cuda.synchronize()
    assert bool((obuf[rows * cols:] == 0xAA).all()) and bool((o2[rows * cols:] == 0xAA).all())
    assert bool((acc[rows * cols:] == 7.0).all())
    out8 = host(obuf[: rows * cols]).reshape(rows, cols)
    assert np.array_equal(host(o2[: rows * cols]).reshape(rows, cols), out8), "fused out8 differs"
    return host(acc[: rows * cols]).reshape(rows, cols), out8


def test_contraction_major_operands_exact_sums_every_capable_tile(mp8):
    """Operands stored [contraction, rows]: the kernel's transposing LDS reads must deliver the
    same sums as the plain layout; exact-sum codes make any mix-up of indices visible."""
    rng = np.random.default_rng(21)
    rows, cols, kc = 320, 288, 1024                   # ragged against 128- and 256-row tiles
    a_km, b_km = exact_sum_codes(rng, (kc, rows)), exact_sum_codes(rng, (kc, cols))
    ref, _ = oracle.gemm_ref(np.ascontiguousarray(a_km.T), np.ascontiguousarray(b_km.T), want_abs=False)
    want8 = oracle.round_ref_e5m2(ref)
    names = mp8.gemm_tile_configs()
    tried = 0
    for tile in range(0, len(names) + 1):
        for split in (0, 1, 3):
            try:
                acc, out8 = run_gemm_tn(mp8, a_km, b_km, tile_config=tile, split_k=split)
            except mp8.Mp8Error:
                assert tile > 0              # a tile shape without contraction-major kernels
                continue
            tried += 1
            assert np.array_equal(acc.astype(np.float64), ref), (tile, split)
            assert np.array_equal(out8, want8), (tile, split)
    assert tried >= 9


@pytest.mark.parametrize("shape", [(128, 128, 128), (144, 16, 256), (400, 272, 384), (70, 50, 256),
                                   (64, 64, 100)])
def test_contraction_major_operands_random(mp8, shape):
    rows, cols, kc = shape                            # the last two take the any-shape kernel
    a_km = (workloads.random_e5m2_codes(rows, (kc, rows)) & 0x83) | 0x38
    b_km = (workloads.random_e5m2_codes(cols + 7, (kc, cols)) & 0x83) | 0x38
    acc, out8 = run_gemm_tn(mp8, a_km, b_km, round=oracle.SR, seed=4, offset=9)
    ref, absref = oracle.gemm_ref(np.ascontiguousarray(a_km.T), np.ascontiguousarray(b_km.T))
    check_outputs(acc, out8, ref, absref, kc, mode=oracle.SR, seed=4, offset=9)


def test_wave_split_kernel_all_epilogues_and_uneven_slices(mp8):
    """The kernel that divides the contraction among the waves of a workgroup: a contraction of
    37 stages (uneven over four waves and over the slices), rows and columns ragged against its
    64x64 tile, every epilogue it carries -- FP32 accumulator out and accumulate-into, RNE and SR,
    saturation, statistics -- against the oracle; and the planner's own choice of it."""
    import torch
    names = mp8.gemm_tile_configs()
    wk = 1 + [n.endswith("w") for n in names].index(True)
    rows, cols, kc = 208, 144, 128 * 37
    a_km = (workloads.random_e5m2_codes(41, (kc, rows)) & 0x83) | 0x38
    b_km = (workloads.random_e5m2_codes(42, (kc, cols)) & 0x83) | 0x38
    ref, absref = oracle.gemm_ref(np.ascontiguousarray(a_km.T), np.ascontiguousarray(b_km.T))
    a, b = gpu(a_km), gpu(b_km)
    flags = mp8.FLAG_CONTRACTION_MAJOR
    for split in (0, 1, 2, 5):
        tile = 0 if split == 0 else wk
        assert mp8.gemm_fp8_plan(mp8.FWD, rows, cols, kc, flags, tile, split)[0] == names[wk - 1]
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, rows, cols, kc, tile, split), 16),
                         dtype=torch.uint8, device="cuda")
        for mode, fl, alpha in ((oracle.RNE, 0, 1.0), (oracle.SR, 0, 0.01), (oracle.SR, oracle.FLAG_SATURATE, 40.0),
                                (oracle.RNE, 0, 40.0)):
            acc = torch.full((rows * cols + 16,), 7.0, dtype=torch.float32, device="cuda")
            obuf = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
            st = mp8.new_stats()
            mp8.gemm_fp8(mp8.FWD, rows, cols, kc, a, b, out8=obuf[: rows * cols], acc=acc[: rows * cols], acc_mode=1,
                         alpha=alpha, round=mode, flags=flags | fl, seed=3, offset=8, stats=st, workspace=ws,
                         tile_config=tile, split_k=split)
            # the same without the FP32 output: the epilogue runs inside the kernel when unsplit
            o2 = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
            st2 = mp8.new_stats()
            mp8.gemm_fp8(mp8.FWD, rows, cols, kc, a, b, out8=o2[: rows * cols], alpha=alpha, round=mode,
                         flags=flags | fl, seed=3, offset=8, stats=st2, workspace=ws, tile_config=tile, split_k=split)
            torch.cuda.synchronize()
            assert bool((obuf[rows * cols:] == 0xAA).all()) and bool((o2[rows * cols:] == 0xAA).all())
            assert bool((acc[rows * cols:] == 7.0).all())
            acc_h, out8 = host(acc[: rows * cols]).reshape(rows, cols), host(obuf[: rows * cols]).reshape(rows, cols)
            check_outputs(acc_h, out8, ref, absref, kc, mode=mode, seed=3, offset=8, alpha=alpha, flags=fl)
            assert np.array_equal(host(o2[: rows * cols]).reshape(rows, cols), out8), (split, mode, fl)
            ost = oracle.Stats()
            oracle.quantize_e5m2(acc_h, scale=alpha, mode=mode, seed=3, offset=8, flags=fl, stats=ost)
            assert mp8.read_stats(st) == ost.as_tuple() == mp8.read_stats(st2), (split, mode, fl)
        # accumulate into an FP32 buffer across two calls (acc_mode 2): twice the sum
        acc2 = torch.zeros(rows * cols, dtype=torch.float32, device="cuda")
        for _ in range(2):
            mp8.gemm_fp8(mp8.FWD, rows, cols, kc, a, b, acc=acc2, acc_mode=2, flags=flags, workspace=ws,
                         tile_config=tile, split_k=split)
        torch.cuda.synchronize()
        ok, worst, _ = acc_tolerance_ok(host(acc2).reshape(rows, cols) / 2, ref, absref, kc)
        assert ok, worst


def test_small_wave_split_tiles_every_epilogue_and_their_automatic_choice(mp8):
    """The 32x64 and 32x32 tiles of the kernel that divides the contraction among the waves (for
    outputs with so few 64x64 tiles that most CUs would idle, e.g. the per-timestep GEMMs of the
    LSTM configuration): rows and columns ragged against the tile, 19 stages (uneven over four
    waves and over slices), RNE and SR, saturation, statistics, FP32 output, row-major operands
    and -- for the 32x64 tile -- b contraction-major; then the planner's own choice."""
    names = mp8.gemm_tile_configs()
    rows, cols, kc = 100, 208, 128 * 19
    a8 = workloads.random_e5m2_codes(51, (rows, kc))
    b8 = workloads.random_e5m2_codes(52, (cols, kc))
    a8, b8 = (a8 & 0x83) | 0x38, (b8 & 0x83) | 0x38
    ref, absref = oracle.gemm_ref(a8, b8)
    for name in ("32x64x128w", "32x32x128w"):
        tile = 1 + names.index(name)
        for split in (1, 3):
            assert mp8.gemm_fp8_plan(mp8.FWD, rows, cols, kc, 0, tile, split) == (name, split)
            for mode, fl, alpha in ((oracle.RNE, 0, 1.0), (oracle.SR, 0, 0.01), (oracle.SR, oracle.FLAG_SATURATE, 40.0)):
                acc, out8, out8_t, st = run_gemm(mp8, a8, b8, want_t=True, tile_config=tile, split_k=split,
                                                 alpha=alpha, round=mode, flags=fl, seed=6, offset=2)
                check_outputs(acc, out8, ref, absref, kc, mode=mode, seed=6, offset=2, alpha=alpha, flags=fl)
                assert np.array_equal(out8_t, out8.T), (name, split, mode)
                ost = oracle.Stats()
                oracle.quantize_e5m2(acc, scale=alpha, mode=mode, seed=6, offset=2, flags=fl, stats=ost)
                assert st == ost.as_tuple(), (name, split, mode, fl)
    # b contraction-major (the forward GEMM from row-major weights) on the 32x64 tile
    import torch
    b_km = np.ascontiguousarray(b8.T)
    tile = 1 + names.index("32x64x128w")
    acc = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
    out = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, rows, cols, kc, tile, 1), 16), dtype=torch.uint8,
                     device="cuda")
    mp8.gemm_fp8(mp8.FWD, rows, cols, kc, gpu(a8), gpu(b_km), out8=out, acc=acc, acc_mode=1, round=oracle.SR, seed=6,
                 offset=2, flags=mp8.FLAG_B_CONTRACTION_MAJOR, workspace=ws, tile_config=tile, split_k=1)
    torch.cuda.synchronize()
    check_outputs(host(acc), host(out), ref, absref, kc, mode=oracle.SR, seed=6, offset=2)
    # no contraction-major b for the 32-column tile: no plan, and the call is refused
    t32 = 1 + names.index("32x32x128w")
    assert mp8.gemm_fp8_plan(mp8.FWD, rows, cols, kc, mp8.FLAG_B_CONTRACTION_MAJOR, t32)[0] is None
    with pytest.raises(mp8.Mp8Error):
        mp8.gemm_fp8(mp8.FWD, rows, cols, kc, gpu(a8), gpu(b_km), out8=out, flags=mp8.FLAG_B_CONTRACTION_MAJOR,
                     workspace=ws, tile_config=t32)
    # the per-timestep GEMMs of the LSTM configuration (128 rows): few tiles, contraction too
    # short to split
    assert mp8.gemm_fp8_plan(mp8.BWD_DATA, 128, 4096, 2048) == ("32x32x128w", 1)
    assert mp8.gemm_fp8_plan(mp8.FWD, 128, 4096, 2048) == ("32x64x128w", 1)
    assert mp8.gemm_fp8_plan(mp8.FWD, 128, 4096, 2048, mp8.FLAG_B_CONTRACTION_MAJOR) == ("32x64x128w", 1)
    lay_a = workloads.random_e5m2_codes(53, (128, 4096))
    lay_b = workloads.random_e5m2_codes(54, (2048, 4096))
    lay_a, lay_b = (lay_a & 0x8F) | 0x30, (lay_b & 0x8F) | 0x30
    r2, ar2 = oracle.gemm_ref(lay_a, lay_b)
    acc, out8, _, _ = run_gemm(mp8, lay_a, lay_b, op=mp8.BWD_DATA, dims=(128, 4096, 2048))
    check_outputs(acc, out8, r2, ar2, 4096)


def test_weight_gradient_from_row_major_activations_and_errors(mp8):
    """The weight gradient straight from X8 [M, K] and dY8 [M, N] as the Q node writes them
    equals the one computed from the transposed copies."""
    import torch
    lay = workloads.config2(batch=2, hw=16, cin=128, cout=128)       # M=512, K=1152, N=128
    X8, X8t, _, _, E8, E8t = _layer_operands(lay)
    M, N, K = lay.M, lay.N, lay.K
    acc_t, out_t, _, _ = run_gemm(mp8, X8t, E8t, op=mp8.WGRAD, dims=(M, N, K))
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
    acc = torch.zeros((K, N), dtype=torch.float32, device="cuda")
    out = torch.zeros((K, N), dtype=torch.uint8, device="cuda")
    mp8.gemm_fp8(mp8.WGRAD, M, N, K, gpu(X8), gpu(E8), out8=out, acc=acc, acc_mode=1, workspace=ws,
                 flags=mp8.FLAG_CONTRACTION_MAJOR)
    torch.cuda.synchronize()
    ref, absref = oracle.gemm_ref(X8t, E8t)
    check_outputs(host(acc), host(out), ref, absref, M)
    # both layouts feed the matrix cores the same products in the same order
    assert np.array_equal(host(acc), acc_t) and np.array_equal(host(out), out_t)


def test_forward_from_row_major_weights(mp8):
    """The forward GEMM reading W8 [K, N] (b contraction-major) gives exactly what it gives from
    the transposed copy W8^T [N, K]; ragged row count, exact and random operands."""
    import torch
    lay = workloads.config2(batch=1, hw=17, cin=128, cout=128)        # M=289, K=1152, N=128
    X8, _, W8, W8t, _, _ = _layer_operands(lay)
    M, N, K = lay.M, lay.N, lay.K
    acc_t, out_t, _, _ = run_gemm(mp8, X8, W8t, op=mp8.FWD, dims=(M, N, K))
    for split in (0, 3):
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, M, N, K, 0, split), 16),
                         dtype=torch.uint8, device="cuda")
        acc = torch.zeros((M, N), dtype=torch.float32, device="cuda")
        out = torch.zeros((M, N), dtype=torch.uint8, device="cuda")
        mp8.gemm_fp8(mp8.FWD, M, N, K, gpu(X8), gpu(W8), out8=out, acc=acc, acc_mode=1, workspace=ws,
                     flags=mp8.FLAG_B_CONTRACTION_MAJOR, split_k=split)
        torch.cuda.synchronize()
        ref, absref = oracle.gemm_ref(X8, W8t)
        check_outputs(host(acc), host(out), ref, absref, K)
        if split == 0:
            assert np.array_equal(host(out), out_t)
    # only a contraction-major: no kernel is built for it, and the call says so
    with pytest.raises(mp8.Mp8Error):
        mp8.gemm_fp8(mp8.FWD, 128, 128, 128, gpu(X8[:128, :128].copy()), gpu(W8t[:, :128].copy()),
                     out8=torch.zeros((128, 128), dtype=torch.uint8, device="cuda"),
                     flags=mp8.FLAG_A_CONTRACTION_MAJOR)


def test_random_shapes_layouts_and_leading_dimensions(mp8):
    """Seeded random shapes through whatever kernel the planner picks: rows and columns from 1
    to 700 (some around 2000), contractions of 1 to 48 stages (and some that are not multiples of 128), the three
    operand layouts, leading dimensions larger than needed -- FP32 accumulator within tolerance,
    8-bit output equal to the oracle's rounding of it, nothing written out of bounds."""
    import torch
    rng = np.random.default_rng(20260)
    kernels = set()
    for case in range(48):
        layout = (0, 0, mp8.FLAG_B_CONTRACTION_MAJOR, mp8.FLAG_CONTRACTION_MAJOR)[case % 4]
        step = 16 if layout else 1
        rows = int(rng.integers(1, 700 // step + 1)) * step
        cols = int(rng.integers(1, 700 // step + 1)) * step
        if layout == mp8.FLAG_B_CONTRACTION_MAJOR:
            rows = int(rng.integers(1, 701))              # only b is contraction-major: any row count
        kc = int(rng.integers(1, 49)) * 128 if case % 8 else int(rng.integers(1, 300))
        if case % 6 == 5:                                 # enough 128x128 tiles for the large-tile kernels
            rows, cols, kc = 16 * int(rng.integers(100, 150)), 16 * int(rng.integers(100, 150)), 128 * int(rng.integers(1, 5))
        a_km, b_km = bool(layout & mp8.FLAG_A_CONTRACTION_MAJOR), bool(layout & mp8.FLAG_B_CONTRACTION_MAJOR)
        pad_a, pad_b = 16 * int(rng.integers(0, 3)), 16 * int(rng.integers(0, 3))
        a_rm = (workloads.random_e5m2_codes(1000 + case, (rows, kc)) & 0x83) | 0x38     # logical [rows, kc]
        b_rm = (workloads.random_e5m2_codes(2000 + case, (cols, kc)) & 0x83) | 0x38
        ref, absref = oracle.gemm_ref(a_rm, b_rm)

        def stored(x_rm, km, pad):
            """The operand as the call wants it: [n, kc] or [kc, n] with a padded leading dimension."""
            x = np.ascontiguousarray(x_rm.T) if km else x_rm
            buf = np.full((x.shape[0], x.shape[1] + pad), 0x7E, np.uint8)   # NaN codes in the padding
            buf[:, : x.shape[1]] = x
            return gpu(buf), x.shape[1] + pad

        a, lda = stored(a_rm, a_km, pad_a)
        b, ldb = stored(b_rm, b_km, pad_b)
        kernels.add(mp8.gemm_fp8_plan(mp8.FWD, rows, cols, kc, layout))
        ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, rows, cols, kc), 16), dtype=torch.uint8, device="cuda")
        acc = torch.full((rows * cols + 16,), 7.0, dtype=torch.float32, device="cuda")
        o1 = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
        o2 = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
        mp8.gemm_fp8(mp8.FWD, rows, cols, kc, a, b, out8=o1[: rows * cols], acc=acc[: rows * cols], acc_mode=1,
                     flags=layout, workspace=ws, lda=lda, ldb=ldb)
        mp8.gemm_fp8(mp8.FWD, rows, cols, kc, a, b, out8=o2[: rows * cols], flags=layout, workspace=ws, lda=lda, ldb=ldb)
        torch.cuda.synchronize()
        what = (case, rows, cols, kc, layout, lda, ldb)
        assert bool((o1[rows * cols:] == 0xAA).all()) and bool((o2[rows * cols:] == 0xAA).all()), what
        assert bool((acc[rows * cols:] == 7.0).all()), what
        out8 = host(o1[: rows * cols]).reshape(rows, cols)
        check_outputs(host(acc[: rows * cols]).reshape(rows, cols), out8, ref, absref, kc)
        assert np.array_equal(host(o2[: rows * cols]).reshape(rows, cols), out8), what
    assert len({k[0] for k in kernels}) >= 5        # the cases reach most kernels, the any-shape one too
