"""GPU system test: a two-layer network trained end to end through the C ABI, every tensor of
every GEMM in the 8-bit format, FP16 master weights (Section 3, Figure 1).  It checks the
qualitative claims of Sections 3.1 and 3.2 on synthetic data (the paper's datasets are not
available): without loss scaling the back-propagated errors vanish in the 8-bit format and
training does not move; with it the same run converges; and with small updates nearest-even
rounding of the master weights loses progress that stochastic rounding keeps.

The non-linearity, the loss and its gradient are a few torch calls (plumbing around the
library); quantisation, all GEMMs and the weight updates are the library's kernels."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mp8():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1905_12334_amd as m
    m.lib()
    return m


def train(mp8, loss_scale, rnd, lr, target_scale=1.0, steps=300, M=2048, D=256, Hd=256, O=128):
    """Teacher-student regression y = relu(x W1) W2; returns (losses, share of error elements
    that the Q node flushed to zero)."""
    import torch
    dev, u8 = "cuda", torch.uint8
    g = torch.Generator(device="cpu").manual_seed(0)
    X = torch.randn(M, D, generator=g).to(dev)
    Wt1 = (torch.randn(D, Hd, generator=g) / D ** 0.5).to(dev)
    Wt2 = (torch.randn(Hd, O, generator=g) / Hd ** 0.5).to(dev)
    T = target_scale * (torch.relu(X @ Wt1) @ Wt2)
    W1 = (torch.randn(D, Hd, generator=g) * (2 / D) ** 0.5).half().to(dev).contiguous()
    W2 = (target_scale * torch.randn(Hd, O, generator=g) * (1 / Hd) ** 0.5).half().to(dev).contiguous()
    X8, W1_8, W2_8 = (torch.empty(s, dtype=u8, device=dev) for s in ((M, D), (D, Hd), (Hd, O)))
    mp8.quantize_e5m2(X, X8)
    mp8.quantize_e5m2(W1, W1_8)
    mp8.quantize_e5m2(W2, W2_8)
    H8, E8, dH8 = (torch.empty(s, dtype=u8, device=dev) for s in ((M, Hd), (M, O), (M, Hd)))
    G1, G2 = torch.empty((D, Hd), dtype=u8, device=dev), torch.empty((Hd, O), dtype=u8, device=dev)
    Y = torch.empty((M, O), dtype=torch.float32, device=dev)
    ws = torch.empty(64 << 20, dtype=u8, device=dev)
    stats = mp8.new_stats()
    both, b_only = mp8.FLAG_CONTRACTION_MAJOR, mp8.FLAG_B_CONTRACTION_MAJOR
    losses, flushed = [], 0
    for it in range(steps):
        mp8.gemm_fp8(mp8.FWD, M, Hd, D, X8, W1_8, out8=H8, workspace=ws, flags=b_only)
        H8r = torch.where((H8 & 0x80) != 0, torch.zeros_like(H8), H8)          # ReLU on the codes
        mp8.gemm_fp8(mp8.FWD, M, O, Hd, H8r, W2_8, acc=Y, acc_mode=1, workspace=ws, flags=b_only)
        diff = Y - T
        losses.append(float((diff * diff).mean()))
        stats.zero_()
        mp8.quantize_e5m2((2.0 / (M * O)) * diff, E8, scale=loss_scale, stats=stats)
        flushed += mp8.read_stats(stats)[2]
        mp8.gemm_fp8(mp8.BWD_DATA, M, O, Hd, E8, W2_8, out8=dH8, workspace=ws)
        dH8m = torch.where(H8r == 0, torch.zeros_like(dH8), dH8)
        mp8.gemm_fp8(mp8.WGRAD, M, O, Hd, H8r, E8, out8=G2, workspace=ws, flags=both)
        mp8.gemm_fp8(mp8.WGRAD, M, Hd, D, X8, dH8m, out8=G1, workspace=ws, flags=both)
        mp8.sgd_update_fp16_sr(W1, G1, lr, 1.0 / loss_scale, round=rnd, seed=11, offset=2 * it, w8_out=W1_8)
        mp8.sgd_update_fp16_sr(W2, G2, lr, 1.0 / loss_scale, round=rnd, seed=11, offset=2 * it + 1, w8_out=W2_8)
    return losses, flushed / (steps * M * O)


def test_loss_scaling_decides_between_no_training_and_convergence(mp8):
    """Section 3.1: errors of magnitude ~1e-7 are below the smallest 8-bit subnormal; unscaled,
    every one of them is flushed to zero and nothing is learned, with a loss scale of 2^16 the
    same run converges."""
    flat, share = train(mp8, 1.0, mp8.SR, 0.5, target_scale=0.05)
    assert share > 0.99 and flat[-1] == flat[0]
    good, share = train(mp8, 2.0 ** 16, mp8.SR, 0.5, target_scale=0.05)
    assert share < 0.01 and good[-1] < 0.25 * good[0]


def test_training_converges_and_is_reproducible(mp8):
    a, _ = train(mp8, 2.0 ** 16, mp8.SR, 0.5)
    b, _ = train(mp8, 2.0 ** 16, mp8.SR, 0.5)
    assert a[-1] < 0.2 * a[0]
    assert a == b                      # same seeds, same Philox offsets: bit-identical runs


def test_stochastic_rounding_of_master_weights_keeps_small_updates(mp8):
    """Section 3.2: with a small learning rate most updates are below half a spacing of the
    FP16 master weights; nearest-even rounding drops them, stochastic rounding carries them
    out on average, and the loss falls faster."""
    sr, _ = train(mp8, 2.0 ** 16, mp8.SR, 0.002)
    rne, _ = train(mp8, 2.0 ** 16, mp8.RNE, 0.002)
    assert sr[-1] < 0.97 * rne[-1] < rne[0]
