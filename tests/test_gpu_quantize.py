"""GPU parity: mp8_quantize_e5m2 and mp8_sr_bits against the CPU oracle, bit for bit."""
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


def _run(mp8, x, want_t=False, with_stats=True, **kw):
    import torch
    src = gpu(x)
    buf = torch.full((x.size + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    dst = buf[: x.size].view(x.shape)       # 64 canary bytes behind the output
    dst_t = torch.empty((x.shape[1], x.shape[0]), dtype=torch.uint8, device="cuda") if want_t else None
    stats = mp8.new_stats() if with_stats else None
    mp8.quantize_e5m2(src, dst, dst_t, stats=stats, **kw)
    torch.cuda.synchronize()
    assert bool((buf[x.size:] == 0xAA).all()), "write past the end of dst"
    return host(dst), (host(dst_t) if want_t else None), (mp8.read_stats(stats) if with_stats else None)


def _oracle(x, want_t=False, **kw):
    st = oracle.Stats()
    mode = kw.pop("round", oracle.RNE)
    q, qt = oracle.quantize_e5m2(x, mode=mode, want_t=want_t, stats=st, **kw)
    return q, qt, st.as_tuple()


def test_sr_bits_stream_matches_oracle(mp8):
    import torch
    n = 100_003
    out = torch.empty(n, dtype=torch.int16, device="cuda")
    seed, offset = 0xDEADBEEFCAFEF00D, 0x0123456789ABCDEF
    mp8.sr_bits(out, seed, offset)
    got = host(out).view(np.uint16)
    idx = np.concatenate([np.arange(0, 4096), np.arange(n - 4096, n)])
    want = np.array([oracle.sr_bits(seed, offset, int(i)) for i in idx], dtype=np.uint16)
    assert np.array_equal(got[idx], want)
    assert abs(got.astype(np.float64).mean() / 65536 - 0.5) < 0.01


def test_all_codes_roundtrip_and_edge_values(mp8):
    codes = np.arange(256, dtype=np.uint16)
    vals = (codes << 8).astype(np.uint16).view(np.float16).astype(np.float32)
    edge = np.array([61440.0, np.nextafter(np.float32(61440), np.float32(0)), 65536.0, 1e30,
                     -61440.0, 2.0 ** -17, np.nextafter(np.float32(2.0 ** -17), np.float32(1)),
                     1.5 * 2.0 ** -16, 2.5 * 2.0 ** -16, -0.0, 0.0, np.inf, -np.inf, np.nan,
                     1e-45, -1e-45, 1.1754942e-38, 1.125, 1.375, 1.625, 57344.0, 3.0e-5],
                    dtype=np.float32)
    # all midpoints between adjacent finite codes, and their FP32 neighbours
    fin = vals[:0x7C].astype(np.float64)
    mids = ((fin[:-1] + fin[1:]) / 2).astype(np.float32)
    around = np.concatenate([mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9))])
    x = np.concatenate([vals, edge, around, -around]).astype(np.float32)
    x = np.concatenate([x, np.zeros((-x.size) % 16 + 5, np.float32)]).reshape(1, -1)
    for rnd in (oracle.RNE, oracle.SR):
        for flags in (0, oracle.FLAG_SATURATE):
            got, _, gst = _run(mp8, x, round=rnd, flags=flags, seed=9, offset=4)
            want, _, wst = _oracle(x, round=rnd, flags=flags, seed=9, offset=4)
            assert np.array_equal(got, want), (rnd, flags, np.nonzero(got != want))
            assert gst == wst


@pytest.mark.parametrize("rnd", [oracle.RNE, oracle.SR])
def test_random_bit_patterns_4m(mp8, rnd):
    x = workloads.random_f32_bit_patterns(77, 1 << 22).reshape(2048, 2048)
    got, got_t, gst = _run(mp8, x, want_t=True, round=rnd, seed=1234, offset=99)
    want, want_t, wst = _oracle(x, want_t=True, round=rnd, seed=1234, offset=99)
    assert np.array_equal(got, want)
    assert np.array_equal(got_t, want_t)
    assert gst == wst


@pytest.mark.parametrize("shape", [(1, 1), (1, 15), (3, 17), (64, 64), (65, 130), (257, 48),
                                   (1000, 3), (5, 1031), (128, 1152)])
@pytest.mark.parametrize("rnd", [oracle.RNE, oracle.SR])
def test_ragged_shapes_scale_transpose_stats(mp8, shape, rnd):
    rng = np.random.default_rng(shape[0] * 1000 + shape[1])
    x = (rng.standard_normal(shape) * np.exp2(rng.integers(-22, 4, shape))).astype(np.float32)
    for want_t in (False, True):
        got, got_t, gst = _run(mp8, x, want_t=want_t, scale=4096.0, round=rnd, seed=5, offset=8)
        want, want_t_arr, wst = _oracle(x, want_t=want_t, scale=4096.0, round=rnd, seed=5, offset=8)
        assert np.array_equal(got, want)
        if want_t:
            assert np.array_equal(got_t, want_t_arr)
        assert gst == wst


@pytest.mark.parametrize("shape,with_stats", [
    ((100, 36), True),        # a handful of 64x64 tiles, ragged in both directions
    ((1100, 1284), True),     # 128x128 tiles with ragged edges, grid-strided stats variant
    ((1100, 1284), False),
    ((4096, 4100), False),    # about a thousand tiles: persistent blocks prefetching across tiles
    ((4096, 4100), True),
    ((16384, 6148), False),   # several rounds of tiles, narrow: one tile per block
    ((8192, 8196), True),     # wide and tall: super-tiled block order, capped grid
    ((8192, 8196), False),
])
def test_transposed_copy_on_every_launch_path(mp8, shape, with_stats):
    x = workloads.random_f32_bit_patterns(shape[0] + shape[1], shape[0] * shape[1]).reshape(shape)
    x[3, 5] = np.float32(3.0e-5)
    rnd = oracle.SR if shape[1] % 8 else oracle.RNE
    got, got_t, gst = _run(mp8, x, want_t=True, with_stats=with_stats, round=rnd, seed=21, offset=6)
    want, want_t, wst = _oracle(x, want_t=True, round=rnd, seed=21, offset=6)
    assert np.array_equal(got, want)
    assert np.array_equal(got_t, want_t)
    if with_stats:
        assert gst == wst


@pytest.mark.parametrize("quarter", [0, 1, 2, 3])
def test_every_fp32_bit_pattern_rne(mp8, quarter):
    """All 2^32 FP32 inputs (a quarter per case, 2^26 at a time), nearest-even rounding with
    statistics: the hardware conversion path, its NaN detour and the counters against the oracle."""
    import torch
    n = 1 << 26
    dst = torch.empty((1 << 13, 1 << 13), dtype=torch.uint8, device="cuda")
    for chunk in range(16 * quarter, 16 * quarter + 16):
        x = np.arange(chunk * n, (chunk + 1) * n, dtype=np.uint64).astype(np.uint32).view(np.float32)
        x = x.reshape(1 << 13, 1 << 13)
        st = mp8.new_stats()
        mp8.quantize_e5m2(gpu(x), dst, stats=st)
        torch.cuda.synchronize()
        ost = oracle.Stats()
        want, _ = oracle.quantize_e5m2(x, stats=ost)
        assert np.array_equal(host(dst), want), f"chunk {chunk}"
        assert mp8.read_stats(st) == ost.as_tuple(), f"chunk {chunk}"


def test_every_16th_fp32_bit_pattern_sr_and_saturating(mp8):
    """2^28 FP32 inputs spread over the whole range with stochastic rounding (Philox bits by
    element index), and the same inputs in the saturating mode under both rounding rules."""
    import torch
    n = 1 << 26
    dst = torch.empty((1 << 13, 1 << 13), dtype=torch.uint8, device="cuda")
    for chunk in range(4):
        x = ((np.arange(chunk * n, (chunk + 1) * n, dtype=np.uint64) * 16 + 5) & 0xFFFFFFFF)
        x = x.astype(np.uint32).view(np.float32).reshape(1 << 13, 1 << 13)
        xd = gpu(x)
        for kw in (dict(round=oracle.SR, seed=0xABCDEF + chunk, offset=chunk),
                   dict(round=oracle.RNE, flags=oracle.FLAG_SATURATE),
                   dict(round=oracle.SR, flags=oracle.FLAG_SATURATE, seed=77, offset=chunk)):
            mp8.quantize_e5m2(xd, dst, **kw)
            torch.cuda.synchronize()
            want, _ = oracle.quantize_e5m2(x, mode=kw.get("round"), flags=kw.get("flags", 0),
                                           seed=kw.get("seed", 0), offset=kw.get("offset", 0))
            assert np.array_equal(host(dst), want), (chunk, kw)


def test_half_precision_source(mp8):
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((130, 96)) * np.exp2(rng.integers(-18, 12, (130, 96)))).astype(np.float16)
    for rnd in (oracle.RNE, oracle.SR):
        for want_t in (False, True):
            got, got_t, gst = _run(mp8, x, want_t=want_t, scale=0.5, round=rnd, seed=2, offset=1)
            want, wt, wst = _oracle(x, want_t=want_t, scale=0.5, round=rnd, seed=2, offset=1)
            assert np.array_equal(got, want) and gst == wst
            if want_t:
                assert np.array_equal(got_t, wt)


def test_config_tensors_and_loss_scale_effect(mp8):
    lay = workloads.config2(batch=4)                      # dY: 3136 x 128, errors N(0, 1e-4)
    got, got_t, gst = _run(mp8, lay.dY, want_t=True, scale=lay.loss_scale)
    want, want_t, wst = _oracle(lay.dY, want_t=True, scale=lay.loss_scale)
    assert np.array_equal(got, want) and np.array_equal(got_t, want_t) and gst == wst
    unscaled, _, st1 = _run(mp8, lay.dY * np.float32(0.1))
    assert st1[2] > 0.5 * lay.dY.size          # most small errors vanish without loss scaling
    assert gst[2] < 0.05 * lay.dY.size
    lay5 = workloads.config5(tokens=512)
    for rnd in (oracle.RNE, oracle.SR):
        got, _, gst = _run(mp8, lay5.dY, scale=lay5.loss_scale, round=rnd, seed=lay5.extra["seed"], offset=3)
        want, _, wst = _oracle(lay5.dY, scale=lay5.loss_scale, round=rnd, seed=lay5.extra["seed"], offset=3)
        assert np.array_equal(got, want) and gst == wst


def test_no_stats_and_empty_and_determinism(mp8):
    import torch
    x = workloads.normal(9, 0, (300, 200))
    a, _, _ = _run(mp8, x, with_stats=False, round=oracle.SR, seed=3, offset=3)
    b, _, _ = _run(mp8, x, with_stats=False, round=oracle.SR, seed=3, offset=3)
    c, _, _ = _run(mp8, x, with_stats=False, round=oracle.SR, seed=3, offset=4)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    want, _, _ = _oracle(x, round=oracle.SR, seed=3, offset=3)
    assert np.array_equal(a, want)
    e = torch.empty((0, 16), dtype=torch.float32, device="cuda")
    mp8.quantize_e5m2(e, torch.empty((0, 16), dtype=torch.uint8, device="cuda"))
    # overflow is counted, and saturation removes it
    big = np.full((4, 32), 7e4, np.float32)
    _, _, st = _run(mp8, big)
    assert st[1] == 128
    _, _, st = _run(mp8, big, flags=oracle.FLAG_SATURATE)
    assert st[1] == 0


def test_batched_quantize_equals_separate_calls_and_the_oracle(mp8):
    """Several Q nodes in one launch: FP32 and half sources, RNE and SR, saturation, statistics
    (two items share one statistics struct), sizes from 1 element to millions with ragged tails,
    an empty item -- each item bit for bit what the oracle gives for it alone."""
    import torch
    rng = np.random.default_rng(91)
    specs = [  # n, half source, scale, round, flags, seed, offset, statistics slot
        (3 * 1000 * 1000 + 3, False, 4096.0, oracle.RNE, 0, 0, 0, 0),
        (1, False, 1.0, oracle.SR, 0, 5, 6, None),
        (40961, True, 0.5, oracle.SR, oracle.FLAG_SATURATE, 7, 8, 1),
        (0, False, 1.0, oracle.RNE, 0, 0, 0, None),
        (8 * 1000 * 1000, False, 1.0, oracle.RNE, 0, 0, 0, None),
        (123457, False, 3.0e4, oracle.RNE, oracle.FLAG_SATURATE, 0, 0, 1),
        (77, True, 1.0, oracle.RNE, 0, 0, 0, None),
        (65536, False, 1e-3, oracle.SR, 0, 9, 10, None),
    ]
    stats = [mp8.new_stats(), mp8.new_stats()]
    ostats = [oracle.Stats(), oracle.Stats()]
    items, hosts, outs = [], [], []
    for n, half, scale, rnd, fl, seed, off, slot in specs:
        x = (rng.standard_normal(n) * np.exp2(rng.integers(-18, 17, n))).astype(np.float16 if half else np.float32)
        if n > 100:
            x[5], x[17], x[33] = np.inf, np.nan, -np.inf
        hosts.append(x)
        o = torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")
        outs.append(o)
        items.append(dict(src=gpu(x), dst=o[:n], scale=scale, round=rnd, flags=fl, seed=seed, offset=off,
                          stats=None if slot is None else stats[slot]))
    mp8.quantize_e5m2_batch(items)
    torch.cuda.synchronize()
    for (n, half, scale, rnd, fl, seed, off, slot), x, o in zip(specs, hosts, outs):
        assert bool((o[n:] == 0xAA).all()), "write past the end of an item"
        if n == 0:
            continue
        want, _ = oracle.quantize_e5m2(x.reshape(1, -1), scale=scale, mode=rnd, flags=fl, seed=seed, offset=off,
                                       stats=None if slot is None else ostats[slot])
        assert np.array_equal(host(o[:n]), want.reshape(-1)), (n, half, rnd, fl)
    for s, os_ in zip(stats, ostats):
        assert mp8.read_stats(s) == os_.as_tuple()
    # one item is the plain call; too many items or a bad round are refused before any launch
    o1 = torch.empty(specs[0][0], dtype=torch.uint8, device="cuda")
    mp8.quantize_e5m2(gpu(hosts[0]).view(1, -1), o1, scale=specs[0][2])
    torch.cuda.synchronize()
    assert torch.equal(o1, outs[0][: specs[0][0]])
    with pytest.raises(mp8.Mp8Error):
        mp8.quantize_e5m2_batch(items + [items[0]])
    with pytest.raises(mp8.Mp8Error):
        mp8.quantize_e5m2_batch([dict(items[1], round=7)])
