"""GPU parity at sizes whose element indices or byte offsets do not fit 32 bits: tensors of more
than 2^32 elements through the Q node, the random stream and the update; GEMM operands, outputs
and contractions beyond 2^32 bytes.  The tensors live on the GPU only (tens of GB); the oracle
computes sampled elements or rows -- the head, the ragged tail, both sides of offset 2^32 and
random positions."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

TWO32 = 1 << 32


@pytest.fixture(scope="module")
def mp8():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1905_12334_amd as m
    m.lib()
    return m


def sample_indices(n, seed):
    rng = np.random.default_rng(seed)
    parts = [np.arange(0, 2048), np.arange(n - 2048, n), np.arange(TWO32 - 1024, min(TWO32 + 1024, n)),
             rng.integers(0, n, 20000)]
    return np.unique(np.concatenate(parts).astype(np.int64))


def take(t, idx):
    import torch
    return t.reshape(-1)[torch.from_numpy(idx).cuda()].cpu().numpy()


def oracle_sr_codes(x, idx, seed, offset):
    """Element by element: the code of x[i] with the random halfword of stream position idx[i]."""
    return np.array([oracle.e5m2_encode(float(v), oracle.SR, oracle.sr_bits(seed, offset, int(i)))
                     for v, i in zip(x, idx)], dtype=np.uint8)


def test_quantize_flat_beyond_2_32_elements(mp8):
    import torch
    n = TWO32 + 3 * 4096 + 3            # three elements in the ragged tail
    x = torch.empty((1, n), dtype=torch.float32, device="cuda").normal_()
    x.mul_(torch.empty((1, n), dtype=torch.float32, device="cuda").uniform_(0.0, 8.0).exp2_())
    idx = sample_indices(n, 1)
    xs = take(x, idx)
    d = torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    seed, offset = 0x5EED_0000_1234, 9
    mp8.quantize_e5m2(x, d[:n], round=mp8.SR, seed=seed, offset=offset)
    torch.cuda.synchronize()
    assert bool((d[n:] == 0xAA).all()), "write past the end of dst"
    assert np.array_equal(take(d[:n], idx), oracle_sr_codes(xs, idx, seed, offset))
    # the variant that gathers statistics (other block shape, grid-stride loop): same codes everywhere
    d2 = torch.empty(n, dtype=torch.uint8, device="cuda")
    st = mp8.new_stats()
    mp8.quantize_e5m2(x, d2, round=mp8.SR, seed=seed, offset=offset, stats=st)
    torch.cuda.synchronize()
    assert bool(torch.equal(d2, d[:n]))
    # round to nearest even, against the oracle's array routine on the sampled values
    mp8.quantize_e5m2(x, d[:n], round=mp8.RNE)
    torch.cuda.synchronize()
    assert np.array_equal(take(d[:n], idx), oracle.quantize_e5m2(xs.reshape(1, -1))[0].reshape(-1))


def test_quantize_with_transposed_copy_beyond_2_32_elements(mp8):
    import torch
    rows, cols = 65536 + 4, 65536 + 8   # ragged against the 128 x 128 tiles
    n = rows * cols
    assert n > TWO32
    x = torch.empty((rows, cols), dtype=torch.float32, device="cuda").normal_()
    idx = sample_indices(n, 2)
    xs = take(x, idx)
    d = torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    dt = torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    seed, offset = 77, 3
    mp8.quantize_e5m2(x, d[:n].view(rows, cols), dt[:n].view(cols, rows), round=mp8.SR, seed=seed, offset=offset)
    torch.cuda.synchronize()
    assert bool((d[n:] == 0xAA).all()) and bool((dt[n:] == 0xAA).all()), "write past the end"
    want = oracle_sr_codes(xs, idx, seed, offset)
    assert np.array_equal(take(d[:n], idx), want)
    r, c = idx // cols, idx % cols
    assert np.array_equal(take(dt[:n], c * rows + r), want)
    del x
    assert bool(torch.equal(dt[:n].view(cols, rows).t(), d[:n].view(rows, cols))), "copies differ somewhere"


def test_random_stream_beyond_2_32_elements(mp8):
    import torch
    n = TWO32 + 1000
    out = torch.empty(n, dtype=torch.int16, device="cuda")
    seed, offset = 0xABCDEF, 1 << 40
    mp8.sr_bits(out, seed, offset)
    torch.cuda.synchronize()
    idx = sample_indices(n, 3)
    got = take(out, idx).view(np.uint16)
    assert got.tolist() == [oracle.sr_bits(seed, offset, int(i)) for i in idx]


def test_update_beyond_2_32_elements(mp8):
    import torch
    n = TWO32 + 8 * 777 + 5             # five elements in the ragged tail
    w = torch.empty(n, dtype=torch.float16, device="cuda").normal_(0, 0.05)
    g = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 256)
    g = torch.where((g & 0x7C) == 0x7C, g & 0xBF, g)          # finite codes only
    idx = sample_indices(n, 4)
    ws, gs = take(w.view(torch.int16), idx).view(np.uint16), take(g, idx)
    mp8.sgd_update_fp16_sr(w.view(torch.int16), g, 0.02, 1.0 / 1024, round=mp8.RNE)
    torch.cuda.synchronize()
    want, _ = oracle.sgd_update_fp16(ws, gs, 0.02, 1.0 / 1024, mode=oracle.RNE)
    assert np.array_equal(take(w.view(torch.int16), idx).view(np.uint16), want)


def exact_codes_on_gpu(shape, exps, seed):
    """Random E5M2 codes of +-{1, 1.25, 1.5, 1.75} * 2^e, e drawn from `exps` (biased exponent
    fields), generated on the GPU: sums of products of such values stay exactly representable
    in FP32, so accumulators must equal the double-precision reference bit for bit."""
    import torch
    g = torch.Generator(device="cuda").manual_seed(seed)
    c = torch.randint(0, 256, shape, dtype=torch.uint8, device="cuda", generator=g)
    e = torch.tensor(exps, dtype=torch.uint8, device="cuda")[((c >> 2) & 3).long() % len(exps)]
    return (c & 0x83) | (e << 2)


def row_samples(M, row_bytes, seed):
    cross = TWO32 // row_bytes                  # the row in which byte offset 2^32 falls
    rng = np.random.default_rng(seed)
    return np.unique(np.concatenate([np.arange(0, 64), np.arange(M - 140, M), np.arange(cross - 40, cross + 40),
                                     rng.integers(0, M, 64)]).astype(np.int64))


def test_tall_layer_operands_beyond_2_32_bytes(mp8):
    """A layer with so many rows (batch x pixels) that activations, their codes and the
    backward-data output each exceed 2^32 bytes: the forward GEMM that quantises its
    activations, the plain forward GEMM and the backward-data GEMM (fused epilogue, and the
    two-pass path with an FP32 output), on sampled rows against the oracle."""
    import torch
    M, N, K = (1 << 22) + 77, 128, 1152
    rng = np.random.default_rng(8)
    w8 = ((rng.integers(0, 2, (K, N)) << 7) | (rng.integers(15, 19, (K, N)) << 2) | rng.integers(0, 4, (K, N))).astype(np.uint8)
    w8t = np.ascontiguousarray(w8.T)
    W8, W8t = torch.from_numpy(w8).cuda(), torch.from_numpy(w8t).cuda()
    x8_codes = exact_codes_on_gpu((M, K), [15, 16, 17, 18], 11)
    X = x8_codes.view(torch.float8_e5m2).to(torch.float32)     # the values of those codes, as FP32 activations
    del x8_codes
    rows = row_samples(M, K, 5)
    rows_d = torch.from_numpy(rows).cuda()
    ox8 = oracle.quantize_e5m2(X[rows_d].cpu().numpy())[0]
    ref, _ = oracle.gemm_ref(ox8, w8t, want_abs=False)
    want8 = oracle.round_ref_e5m2(ref)

    def buf(n):
        return torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")

    X8, Y8, Y8b = buf(M * K), buf(M * N), buf(M * N)
    acc = torch.empty((M, N), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.FWD, M, N, K), 16), dtype=torch.uint8, device="cuda")
    mp8.quantize_gemm_fwd_fp8(M, N, K, X, X8[: M * K].view(M, K), W8, out8=Y8[: M * N].view(M, N), workspace=ws)
    mp8.quantize_gemm_fwd_fp8(M, N, K, X, X8[: M * K].view(M, K), W8, out8=Y8b[: M * N].view(M, N), acc=acc,
                              acc_mode=1, workspace=ws)
    torch.cuda.synchronize()
    for b in (X8, Y8, Y8b):
        assert bool((b[-64:] == 0xAA).all()), "write past the end"
    assert np.array_equal(X8[: M * K].view(M, K)[rows_d].cpu().numpy(), ox8)
    assert np.array_equal(acc[rows_d].cpu().numpy().astype(np.float64), ref)
    assert np.array_equal(Y8[: M * N].view(M, N)[rows_d].cpu().numpy(), want8)
    assert bool(torch.equal(Y8, Y8b))
    del X
    # the plain forward GEMM from the codes
    Y8b.fill_(0xAA)
    acc.zero_()
    mp8.gemm_fp8(mp8.FWD, M, N, K, X8[: M * K].view(M, K), W8t, out8=Y8b[: M * N].view(M, N), acc=acc, acc_mode=1,
                 workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(acc[rows_d].cpu().numpy().astype(np.float64), ref)
    assert bool(torch.equal(Y8, Y8b))
    del acc, Y8, Y8b
    # backward data: errors [M, N] . weights [K, N] -> [M, K], more than 2^32 output bytes
    E8 = exact_codes_on_gpu((M, N), [15, 16, 17, 18], 12)
    ref2, _ = oracle.gemm_ref(E8[rows_d].cpu().numpy(), w8, want_abs=False)
    want2 = oracle.round_ref_e5m2(ref2)
    D8, D8b = X8, buf(M * K)                      # reuse the activations' buffer (canary intact)
    mp8.gemm_fp8(mp8.BWD_DATA, M, N, K, E8, W8, out8=D8[: M * K].view(M, K))
    acc2 = torch.empty((M, K), dtype=torch.float32, device="cuda")
    mp8.gemm_fp8(mp8.BWD_DATA, M, N, K, E8, W8, out8=D8b[: M * K].view(M, K), acc=acc2, acc_mode=1)
    torch.cuda.synchronize()
    assert bool((D8[-64:] == 0xAA).all()) and bool((D8b[-64:] == 0xAA).all()), "write past the end"
    assert np.array_equal(D8[: M * K].view(M, K)[rows_d].cpu().numpy(), want2)
    assert np.array_equal(acc2[rows_d].cpu().numpy().astype(np.float64), ref2)
    assert bool(torch.equal(D8, D8b))


def test_weight_gradient_over_a_contraction_beyond_2_32_bytes(mp8):
    """The weight gradient of the same tall layer: a contraction over 2^22 + 384 rows read from
    the row-major activations (more than 2^32 bytes) and errors, split into slices and summed by
    the finishing pass; sampled output rows against the oracle's exact sums."""
    import torch
    M, N, K = (1 << 22) + 384, 128, 1152
    X8 = exact_codes_on_gpu((M, K), [15, 16], 21)
    E8 = exact_codes_on_gpu((M, N), [15, 16], 22)
    ks = np.array([0, 1, 63, 64, 577, 1150, 1151])
    a_rows = np.ascontiguousarray(X8[:, torch.from_numpy(ks).cuda()].t().cpu().numpy())      # [7, M]
    e8t = np.ascontiguousarray(E8.t().cpu().numpy())                                          # [N, M]
    ref, _ = oracle.gemm_ref(a_rows, e8t, want_abs=False)
    assert np.max(np.abs(ref)) < 2.0 ** 20          # every partial sum far inside FP32's exact range
    g8 = torch.full((K * N + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    acc = torch.empty((K, N), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K), 16), dtype=torch.uint8, device="cuda")
    alpha = 2.0 ** -6
    mp8.gemm_fp8(mp8.WGRAD, M, N, K, X8, E8, out8=g8[: K * N].view(K, N), acc=acc, acc_mode=1, alpha=alpha,
                 flags=mp8.FLAG_CONTRACTION_MAJOR, workspace=ws)
    torch.cuda.synchronize()
    assert bool((g8[-64:] == 0xAA).all()), "write past the end"
    assert np.array_equal(acc.cpu().numpy()[ks].astype(np.float64), ref)
    assert np.array_equal(g8[: K * N].view(K, N).cpu().numpy()[ks], oracle.round_ref_e5m2(ref, alpha=alpha))


def test_output_beyond_2_32_elements_with_stochastic_rounding(mp8):
    """An output of more than 2^32 elements (short contraction): the stochastic epilogue draws
    the random halfword of each element's row-major index, also beyond 2^32; FP32 output and
    fused epilogue; sampled rows against the oracle, element by element."""
    import torch
    R = 65536 + 64
    kc = 128
    assert R * R > TWO32
    a8, b8 = exact_codes_on_gpu((R, kc), [15, 16, 17, 18], 31), exact_codes_on_gpu((R, kc), [15, 16, 17, 18], 32)
    rows = np.array([0, 1, TWO32 // R, TWO32 // R + 1, R - 1])
    rows_d = torch.from_numpy(rows).cuda()
    ref, _ = oracle.gemm_ref(a8[rows_d].cpu().numpy(), b8.cpu().numpy(), want_abs=False)
    seed, offset, alpha = 99, 5, 2.0 ** -7
    want = np.array([[oracle.e5m2_encode(float(np.float32(v) * np.float32(alpha)), oracle.SR,
                                         oracle.sr_bits(seed, offset, int(r) * R + c)) for c, v in enumerate(line)]
                     for r, line in zip(rows, ref)], dtype=np.uint8)
    out = torch.full((R * R + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    mp8.gemm_fp8(mp8.FWD, R, R, kc, a8, b8, out8=out[: R * R].view(R, R), alpha=alpha, round=mp8.SR, seed=seed,
                 offset=offset)
    torch.cuda.synchronize()
    assert bool((out[-64:] == 0xAA).all()), "write past the end"
    assert np.array_equal(out[: R * R].view(R, R)[rows_d].cpu().numpy(), want)
    # the two-pass path (FP32 output, finishing kernel) gives the same codes everywhere
    out2 = torch.full((R * R + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    acc = torch.empty((R, R), dtype=torch.float32, device="cuda")
    mp8.gemm_fp8(mp8.FWD, R, R, kc, a8, b8, out8=out2[: R * R].view(R, R), acc=acc, acc_mode=1, alpha=alpha,
                 round=mp8.SR, seed=seed, offset=offset)
    torch.cuda.synchronize()
    assert np.array_equal(acc[rows_d].cpu().numpy().astype(np.float64), ref)
    assert bool(torch.equal(out, out2))


def test_optimizers_with_state_beyond_2_32_elements(mp8):
    """Momentum SGD and ADAM (FP32 state arrays of more than 2^34 bytes) on sampled elements."""
    import torch
    n = TWO32 + 8 * 321 + 3
    idx = sample_indices(n, 6)
    g = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 256)
    g = torch.where((g & 0x7C) == 0x7C, g & 0xBF, g)
    gs = take(g, idx)
    w = torch.empty(n, dtype=torch.float16, device="cuda").normal_(0, 0.05)
    vel = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0, 0.01)
    ws, vs = take(w.view(torch.int16), idx).view(np.uint16), take(vel, idx)
    mp8.sgd_momentum_fp16_sr(w.view(torch.int16), vel, g, 0.02, 1.0 / 1024, 0.9, weight_decay=1e-4, round=mp8.RNE)
    torch.cuda.synchronize()
    ow, ov, _ = oracle.sgd_momentum_fp16(ws, vs, gs, 0.02, 1.0 / 1024, 0.9, weight_decay=1e-4, mode=oracle.RNE)
    assert np.array_equal(take(w.view(torch.int16), idx).view(np.uint16), ow)
    assert np.array_equal(take(vel, idx).view(np.uint32), ov.view(np.uint32))
    # ADAM, third step, on the weights as they are now; the velocity array serves as first moment
    m, v = vel, torch.empty(n, dtype=torch.float32, device="cuda").uniform_(0.0, 1e-4)
    ws, ms, vs = take(w.view(torch.int16), idx).view(np.uint16), take(m, idx), take(v, idx)
    mp8.adam_fp16_sr(w.view(torch.int16), m, v, g, 1e-3, 1.0 / 1024, 3, round=mp8.RNE)
    torch.cuda.synchronize()
    ow, om, ov, _ = oracle.adam_fp16(ws, ms, vs, gs, 1e-3, 1.0 / 1024, 3, mode=oracle.RNE)
    assert np.array_equal(take(w.view(torch.int16), idx).view(np.uint16), ow)
    assert np.array_equal(take(m, idx).view(np.uint32), om.view(np.uint32))
    assert np.array_equal(take(v, idx).view(np.uint32), ov.view(np.uint32))
