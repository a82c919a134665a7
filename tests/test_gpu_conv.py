"""GPU parity: mp8_conv3x3_fp8 (implicit GEMM on zero-padded channels-last tensors) against the
oracle's direct convolution references."""
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


def to_padded(mp8, x):
    """[B,H,W,C] host codes -> device [prows, C] view on the padded grid (zero padding, guards)."""
    import torch
    B, H, W, C = x.shape
    prows = mp8.conv_prows(B, H, W)
    xp = np.zeros((B, H + 2, W + 2, C), np.uint8)
    xp[:, 1:-1, 1:-1] = x
    buf = mp8.conv_buffer(prows, C, W)
    buf[: B * (H + 2) * (W + 2)] = torch.from_numpy(xp.reshape(-1, C)).cuda()
    return buf


def interior(arr, B, H, W):
    """[prows, C] host array on the padded grid -> [B,H,W,C] interior, and the padding rows."""
    C = arr.shape[1]
    n = B * (H + 2) * (W + 2)
    grid = arr[:n].reshape(B, H + 2, W + 2, C)
    mask = np.ones((B, H + 2, W + 2), bool)
    mask[:, 1:-1, 1:-1] = False
    pad_rows = np.concatenate([grid[mask].reshape(-1, C), arr[n:]], axis=0)
    return grid[:, 1:-1, 1:-1], pad_rows


def run_conv(mp8, op, dims, a_dev, b_dev, want_acc=True, **kw):
    import torch
    B, H, W, Ci, Co = dims
    prows = mp8.conv_prows(B, H, W)
    shape = {mp8.FWD: (prows, Co), mp8.BWD_DATA: (prows, Ci), mp8.WGRAD: (9 * Ci, Co)}[op]
    ws = torch.empty(max(mp8.conv3x3_fp8_workspace_bytes(op, B, H, W, Ci, Co), 16), dtype=torch.uint8, device="cuda")
    out = torch.full(shape, 0xAA, dtype=torch.uint8, device="cuda")
    acc = torch.zeros(shape, dtype=torch.float32, device="cuda") if want_acc else None
    st = mp8.new_stats()
    mp8.conv3x3_fp8(op, B, H, W, Ci, Co, a_dev, b_dev, out8=out, acc=acc, acc_mode=1 if want_acc else 0,
                    stats=st, workspace=ws, **kw)
    torch.cuda.synchronize()
    return (host(acc) if want_acc else None), host(out), mp8.read_stats(st)


def exact_codes(rng, shape):
    """{1,1.25,1.5,1.75} * 2^{0..3}, both signs: sums of a few thousand products stay exact in FP32."""
    e, m, s = rng.integers(15, 19, shape), rng.integers(0, 4, shape), rng.integers(0, 2, shape)
    return ((s << 7) | (e << 2) | m).astype(np.uint8)


@pytest.mark.parametrize("dims", [(2, 6, 5, 128, 128), (1, 9, 14, 128, 256), (3, 4, 4, 256, 128),
                                  (2, 6, 5, 64, 64), (1, 9, 14, 64, 128), (3, 4, 4, 128, 64), (2, 5, 7, 192, 64),
                                  (1, 3, 3, 64, 320)])
def test_conv_exact_sums_all_three_operations(mp8, dims):
    """Exactly representable sums: the FP32 accumulators must equal the direct convolution bit for
    bit on every interior pixel, padding rows of the outputs must be zero codes.  Channel counts
    that are odd multiples of 64 (the first stage of the residual networks of Section 4) make a
    stage of the contraction span two taps, and its last stage half a stage."""
    B, H, W, Ci, Co = dims
    rng = np.random.default_rng(sum(dims))
    x, w, e = exact_codes(rng, (B, H, W, Ci)), exact_codes(rng, (3, 3, Ci, Co)), exact_codes(rng, (B, H, W, Co))
    xd, ed, wd = to_padded(mp8, x), to_padded(mp8, e), gpu(w)
    for op, a_dev, b_dev, name, a_h, b_h in ((mp8.FWD, xd, wd, "fwd", x, w), (mp8.BWD_DATA, ed, wd, "bwd_data", e, w)):
        ref, _ = oracle.conv3x3_ref(name, a_h, b_h, want_abs=False)
        acc, out8, _ = run_conv(mp8, op, dims, a_dev, b_dev)
        acc_i, _ = interior(acc, B, H, W)
        out_i, out_pad = interior(out8, B, H, W)
        assert np.array_equal(acc_i.astype(np.float64), ref), name
        assert np.array_equal(out_i, oracle.round_ref_e5m2(ref)), name
        assert not out_pad.any(), name + ": padding rows must be zero codes"
        # the fused epilogue (no FP32 output requested) gives the same codes
        _, out_b, _ = run_conv(mp8, op, dims, a_dev, b_dev, want_acc=False)
        assert np.array_equal(out_b, out8), name
    ref, _ = oracle.conv3x3_ref("wgrad", x, e, want_abs=False)
    alpha = 1.0 / 32
    acc, out8, _ = run_conv(mp8, mp8.WGRAD, dims, xd, ed, alpha=alpha)
    assert np.array_equal(acc.reshape(3, 3, Ci, Co).astype(np.float64), ref)
    assert np.array_equal(out8.reshape(3, 3, Ci, Co), oracle.round_ref_e5m2(ref, alpha=alpha))


@pytest.mark.parametrize("channels", [(128, 128), (64, 64), (192, 64)])
def test_conv_weight_gradient_and_update_in_one_call(mp8, channels):
    """mp8_conv3x3_wgrad_update_fp16_sr against the oracle's chain (direct convolution weight
    gradient -> one rounding -> FP16 update) on exact-sum operands: gradient codes, new master
    weights and their 8-bit copies bit for bit."""
    import torch
    B, H, W, (Ci, Co) = 2, 6, 5, channels
    rng = np.random.default_rng(77)
    x, e = exact_codes(rng, (B, H, W, Ci)), exact_codes(rng, (B, H, W, Co))
    ref, _ = oracle.conv3x3_ref("wgrad", x, e, want_abs=False)
    w16 = (rng.standard_normal(9 * Ci * Co) * 0.05).astype(np.float16).view(np.uint16)
    alpha, lr, inv = 1.0 / 32, 0.05, 1.0 / 16
    want_g = oracle.round_ref_e5m2(ref, alpha=alpha).reshape(-1)
    want_w, want_w8 = oracle.sgd_update_fp16(w16, want_g, lr, inv, mode=oracle.SR, seed=5, offset=6, want_w8=True)
    xd, ed = to_padded(mp8, x), to_padded(mp8, e)
    ws = torch.empty(max(mp8.conv3x3_fp8_workspace_bytes(mp8.WGRAD, B, H, W, Ci, Co), 16), dtype=torch.uint8, device="cuda")
    wd = gpu(w16.view(np.int16))
    g8 = torch.full((9 * Ci * Co,), 0xAA, dtype=torch.uint8, device="cuda")
    w8 = torch.full((9 * Ci * Co,), 0x55, dtype=torch.uint8, device="cuda")
    mp8.conv3x3_wgrad_update_fp16_sr(B, H, W, Ci, Co, xd, ed, wd, lr, inv, g8_out=g8, alpha=alpha, w_round=mp8.SR,
                                     w_seed=5, w_offset=6, w8_out=w8, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(g8), want_g)
    assert np.array_equal(host(wd).view(np.uint16), want_w) and np.array_equal(host(w8), want_w8)


@pytest.mark.parametrize("channels", [(128, 128), (64, 128)])
def test_conv_weight_gradient_and_momentum_update_in_one_call(mp8, channels):
    """mp8_conv3x3_wgrad_momentum_fp16_sr against the oracle's chain (direct convolution weight
    gradient -> one rounding -> momentum update with L2 regularisation) on exact-sum operands, two
    steps in a row: gradient codes, master weights, velocity and 8-bit weights bit for bit."""
    import torch
    B, H, W, (Ci, Co) = 2, 6, 5, channels
    rng = np.random.default_rng(78)
    x, e = exact_codes(rng, (B, H, W, Ci)), exact_codes(rng, (B, H, W, Co))
    ref, _ = oracle.conv3x3_ref("wgrad", x, e, want_abs=False)
    w_ref = (rng.standard_normal(9 * Ci * Co) * 0.05).astype(np.float16).view(np.uint16)
    v_ref = (rng.standard_normal(9 * Ci * Co) * 0.01).astype(np.float32)
    alpha, lr, inv, mu, wd_ = 1.0 / 32, 0.05, 1.0 / 16, 0.9, 1e-3
    want_g = oracle.round_ref_e5m2(ref, alpha=alpha).reshape(-1)
    xd, ed = to_padded(mp8, x), to_padded(mp8, e)
    ws = torch.empty(max(mp8.conv3x3_fp8_workspace_bytes(mp8.WGRAD, B, H, W, Ci, Co), 16), dtype=torch.uint8, device="cuda")
    wdev, vdev = gpu(w_ref.view(np.int16)), gpu(v_ref)
    g8 = torch.full((9 * Ci * Co,), 0xAA, dtype=torch.uint8, device="cuda")
    w8 = torch.full((9 * Ci * Co,), 0x55, dtype=torch.uint8, device="cuda")
    for step in (1, 2):
        w_ref, v_ref, want_w8 = oracle.sgd_momentum_fp16(w_ref, v_ref, want_g, lr, inv, mu, wd_, mode=oracle.SR,
                                                         seed=5, offset=step, want_w8=True)
        mp8.conv3x3_wgrad_momentum_fp16_sr(B, H, W, Ci, Co, xd, ed, wdev, vdev, lr, inv, mu, wd_, g8_out=g8,
                                           alpha=alpha, w_round=mp8.SR, w_seed=5, w_offset=step, w8_out=w8,
                                           workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(host(g8), want_g)
        assert np.array_equal(host(wdev).view(np.uint16), w_ref) and np.array_equal(host(w8), want_w8)
        assert np.array_equal(host(vdev).view(np.uint32), v_ref.view(np.uint32))


@pytest.mark.parametrize("channels", [(128, 128), (64, 64), (64, 192)])
def test_conv_random_operands_sr_epilogue_and_statistics(mp8, channels):
    B, H, W, (Ci, Co) = 2, 7, 9, channels
    dims = (B, H, W, Ci, Co)
    x = (workloads.random_e5m2_codes(1, (B, H, W, Ci)) & 0x83) | 0x38
    w = (workloads.random_e5m2_codes(2, (3, 3, Ci, Co)) & 0x83) | 0x34
    e = (workloads.random_e5m2_codes(3, (B, H, W, Co)) & 0x83) | 0x3C
    x[0, 0, 0, :5] = 0                                   # a few zero activations
    xd, ed, wd = to_padded(mp8, x), to_padded(mp8, e), gpu(w)
    prows = mp8.conv_prows(B, H, W)
    for op, a_dev, b_dev, name, a_h, b_h, kc, cols in ((mp8.FWD, xd, wd, "fwd", x, w, 9 * Ci, Co),
                                                       (mp8.BWD_DATA, ed, wd, "bwd_data", e, w, 9 * Co, Ci)):
        ref, absref = oracle.conv3x3_ref(name, a_h, b_h)
        acc, out8, st = run_conv(mp8, op, dims, a_dev, b_dev, round=oracle.SR, seed=8, offset=3)
        acc_i, _ = interior(acc, B, H, W)
        out_i, out_pad = interior(out8, B, H, W)
        assert not out_pad.any()
        # the SR stream is indexed by the position in the padded output matrix
        grid = np.arange(B * (H + 2) * (W + 2)).reshape(B, H + 2, W + 2)[:, 1:-1, 1:-1].reshape(-1)
        check_outputs(acc_i.reshape(-1, cols), out_i.reshape(-1, cols), ref.reshape(-1, cols),
                      absref.reshape(-1, cols), kc, mode=oracle.SR, seed=8, offset=3,
                      first_index=grid * cols)
        ost = oracle.Stats()
        oracle.quantize_e5m2(acc_i.reshape(-1, cols), stats=ost)
        assert st[0] == ost.as_tuple()[0] and st[1] == ost.as_tuple()[1]   # padding rows stay out
    ref, absref = oracle.conv3x3_ref("wgrad", x, e)
    acc, out8, _ = run_conv(mp8, mp8.WGRAD, dims, xd, ed)
    check_outputs(acc, out8, ref.reshape(9 * Ci, Co), absref.reshape(9 * Ci, Co), B * H * W)


def test_conv_config2_layer_full_size(mp8):
    """configs[1] as the convolution it stands for: batch 32, 28x28, 128 -> 128 channels."""
    import torch
    B, H, W, C = 32, 28, 28, 128
    dims = (B, H, W, C, C)
    x32 = workloads.relu_normal(2, 10, (B, H, W, C))
    w32 = workloads.normal(2, 11, (3, 3, C, C), float(np.sqrt(2.0 / (9 * C))))
    e32 = workloads.normal(2, 12, (B, H, W, C), 1e-4)
    x = oracle.quantize_e5m2(x32.reshape(-1, C))[0].reshape(B, H, W, C)
    w = oracle.quantize_e5m2(w32.reshape(-1, C))[0].reshape(3, 3, C, C)
    e = oracle.quantize_e5m2(e32.reshape(-1, C), scale=2.0 ** 12)[0].reshape(B, H, W, C)
    xd, ed, wd = to_padded(mp8, x), to_padded(mp8, e), gpu(w)
    for op, a_dev, b_dev, name, a_h, b_h in ((mp8.FWD, xd, wd, "fwd", x, w), (mp8.BWD_DATA, ed, wd, "bwd_data", e, w)):
        ref, absref = oracle.conv3x3_ref(name, a_h, b_h)
        acc, out8, _ = run_conv(mp8, op, dims, a_dev, b_dev)
        acc_i, _ = interior(acc, B, H, W)
        out_i, out_pad = interior(out8, B, H, W)
        assert not out_pad.any()
        check_outputs(acc_i.reshape(-1, C), out_i.reshape(-1, C), ref.reshape(-1, C), absref.reshape(-1, C), 9 * C)
    ref, absref = oracle.conv3x3_ref("wgrad", x, e)
    acc, out8, _ = run_conv(mp8, mp8.WGRAD, dims, xd, ed)
    check_outputs(acc, out8, ref.reshape(9 * C, C), absref.reshape(9 * C, C), B * H * W)


def test_conv_argument_checks(mp8):
    import torch
    u8 = lambda *s: torch.zeros(s, dtype=torch.uint8, device="cuda")
    with pytest.raises(mp8.Mp8Error):                      # channels not a multiple of 64
        mp8.conv3x3_fp8(mp8.FWD, 1, 4, 4, 32, 128, mp8.conv_buffer(128, 32, 4), u8(3, 3, 32, 128), out8=u8(128, 128))
    with pytest.raises(mp8.Mp8Error):                      # no guard rows around the shifted operand
        mp8.conv3x3_fp8(mp8.FWD, 1, 4, 4, 128, 128, u8(128, 128), u8(3, 3, 128, 128), out8=u8(128, 128))
