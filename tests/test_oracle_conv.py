"""Pins for the oracle's 3x3 convolution references (no GPU): a library routine (torch conv2d
and its autograd in float64), the lowered-GEMM identity against the already pinned GEMM
reference, and shift / identity kernels whose results are known in closed form."""
import numpy as np
import pytest
import torch

import oracle
from paper_1905_12334_amd import workloads


def dec(c):
    return (c.astype(np.uint16) << 8).view(np.float16).astype(np.float64)


def finite_codes(seed, shape):
    return workloads.random_e5m2_codes(seed, shape, finite_only=True)


@pytest.mark.parametrize("dims", [(1, 3, 3, 4, 5), (2, 5, 7, 8, 12), (3, 1, 4, 16, 8), (1, 6, 1, 3, 3)])
def test_conv_refs_match_torch_conv2d_and_autograd(dims):
    B, H, W, Ci, Co = dims
    x, w, e = finite_codes(1, (B, H, W, Ci)), finite_codes(2, (3, 3, Ci, Co)), finite_codes(3, (B, H, W, Co))
    # keep magnitudes moderate so float64 sums of either order agree to rounding
    x, w, e = (x & 0x83) | 0x38, (w & 0x83) | 0x34, (e & 0x83) | 0x3C
    xt = torch.tensor(dec(x)).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.tensor(dec(w)).permute(3, 2, 0, 1).contiguous().requires_grad_(True)
    y = torch.nn.functional.conv2d(xt, wt, padding=1)
    (y * torch.tensor(dec(e)).permute(0, 3, 1, 2)).sum().backward()
    fwd, fabs = oracle.conv3x3_ref("fwd", x, w)
    bwd, _ = oracle.conv3x3_ref("bwd_data", e, w)
    wg, _ = oracle.conv3x3_ref("wgrad", x, e)
    assert np.allclose(fwd, y.detach().permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(bwd, xt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(wg, wt.grad.permute(2, 3, 1, 0).numpy(), rtol=1e-12, atol=1e-12)
    assert np.all(fabs >= np.abs(fwd))


def im2col(x):
    """[B,H,W,C] codes -> [B*H*W, 9*C] with zero codes outside the image, column (r, s, c)."""
    B, H, W, C = x.shape
    xp = np.zeros((B, H + 2, W + 2, C), np.uint8)
    xp[:, 1:-1, 1:-1] = x
    cols = [xp[:, r:r + H, s:s + W] for r in range(3) for s in range(3)]
    return np.ascontiguousarray(np.concatenate(cols, axis=3).reshape(B * H * W, 9 * C))


def test_conv_fwd_equals_gemm_on_lowered_operand_bit_for_bit():
    """The convolution is the GEMM of the lowered operand: same products in the same order
    (zeros added where the window leaves the image), so the two double results are identical --
    this ties the new reference to the GEMM reference and its pins."""
    B, H, W, Ci, Co = 2, 6, 5, 16, 24
    x, w = finite_codes(11, (B, H, W, Ci)), finite_codes(12, (3, 3, Ci, Co))
    fwd, fabs = oracle.conv3x3_ref("fwd", x, w)
    bt = np.ascontiguousarray(w.reshape(9 * Ci, Co).T)
    ref, absref = oracle.gemm_ref(im2col(x), bt)
    assert np.array_equal(fwd.reshape(-1, Co), ref) and np.array_equal(fabs.reshape(-1, Co), absref)
    # weight gradient: contraction over pixels of lowered activations and errors
    e = finite_codes(13, (B, H, W, Co))
    wg, _ = oracle.conv3x3_ref("wgrad", x, e)
    at = np.ascontiguousarray(im2col(x).T)
    et = np.ascontiguousarray(e.reshape(-1, Co).T)
    ref, _ = oracle.gemm_ref(at, et, want_abs=False)
    assert np.allclose(wg.reshape(9 * Ci, Co), ref, rtol=1e-13, atol=0)   # zeros skipped vs added: same sums


@pytest.mark.parametrize("tap", range(9))
def test_single_tap_identity_kernel_shifts_the_image(tap):
    B, H, W, C = 2, 4, 5, 6
    r, s = divmod(tap, 3)
    x = finite_codes(20 + tap, (B, H, W, C))
    w = np.zeros((3, 3, C, C), np.uint8)
    w[r, s, np.arange(C), np.arange(C)] = 0x3C                          # 1.0 on the diagonal
    fwd, _ = oracle.conv3x3_ref("fwd", x, w)
    want = np.zeros((B, H, W, C))
    xd = dec(x)
    for h in range(H):
        for ww in range(W):
            hh, w2 = h + r - 1, ww + s - 1
            if 0 <= hh < H and 0 <= w2 < W:
                want[:, h, ww] = xd[:, hh, w2]
    assert np.array_equal(fwd, want)
    # backward data with the same kernel shifts the other way
    bwd, _ = oracle.conv3x3_ref("bwd_data", x, w)
    want = np.zeros((B, H, W, C))
    for h in range(H):
        for ww in range(W):
            hh, w2 = h - r + 1, ww - s + 1
            if 0 <= hh < H and 0 <= w2 < W:
                want[:, h, ww] = xd[:, hh, w2]
    assert np.array_equal(bwd, want)
