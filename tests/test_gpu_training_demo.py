"""GPU system tests: small networks trained end to end through the C ABI, every tensor of every
8-bit GEMM in the 8-bit format, FP16 master weights (Section 3, Figure 1).  They check the
qualitative claims of Sections 3.1 and 3.2 on synthetic data (the paper's datasets are not
available): without loss scaling the back-propagated errors vanish in the 8-bit format and
training does not move; with it the same run converges; with small updates nearest-even
rounding of the master weights loses progress that stochastic rounding keeps; the back-off
scaler driven by the kernels' own overflow counts halves, skips, grows and respects a minimum
that is raised during the run, step by step like the oracle's scaler; stochastic rounding at the
activation and error Q nodes keeps training where nearest-even rounding flushes the errors; and
the first and the last layer may stay in FP16 around the 8-bit layers (Section 4).

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


# --- the policy layer of Sections 3.1, 3.2 and 4 around the kernels -----------------------------

def codes_as_fp16(codes):
    """An 8-bit (1,5,2) code is the upper byte of the FP16 number of the same value."""
    import torch
    return (codes.to(torch.int16) << 8).view(torch.float16)


class PolicyRun:
    """A four-layer network y = relu(relu(relu(x W0) W1) W2) W3 trained as Section 4 sets its networks
    up: the first and the last layer stay in FP16 (torch half matmuls: they are outside the 8-bit
    path), the two layers between them are the library's 8-bit GEMMs with FP16 master weights.
    Every Q node on an activation or an error rounds with `act_round`; the master-weight update
    rounds stochastically.  The loss scale comes from the library's host-side scaler, driven by
    the Inf/NaN count that the kernels of the backward pass leave on the device, and an oracle
    scaler is fed the same counts; the two must agree after every step."""

    def __init__(self, mp8, act_round, scale, floor, growth_interval, lr=0.5, lr_ends=0.5 / 64, target_scale=1.0,
                 M=2048, D=128, Hd=256, O=128, seed=0):
        import torch
        import oracle
        self.mp8, self.oracle, self.torch = mp8, oracle, torch
        self.act_round, self.lr, self.lr_ends = act_round, lr, lr_ends
        self.M, self.D, self.Hd, self.O = M, D, Hd, O
        dev, u8 = "cuda", torch.uint8
        g = torch.Generator(device="cpu").manual_seed(seed)
        rn = lambda *s: torch.randn(*s, generator=g)
        self.X = rn(M, D).half().to(dev)
        teacher = [rn(D, Hd) / D ** 0.5, rn(Hd, Hd) * (2 / Hd) ** 0.5, rn(Hd, Hd) * (2 / Hd) ** 0.5, rn(Hd, O) / Hd ** 0.5]
        t = self.X.float().cpu()
        for i, w in enumerate(teacher):
            t = t @ w
            if i < 3:
                t = torch.relu(t)
        self.T = (target_scale * t).to(dev)
        # the FP16 layers start at the teacher's values and take a smaller learning rate, so that
        # what the loss shows is what the 8-bit layers between them learn
        self.W0 = teacher[0].half().to(dev)
        self.W1 = (rn(Hd, Hd) * (2 / Hd) ** 0.5).half().to(dev).contiguous()
        self.W2 = (rn(Hd, Hd) * (2 / Hd) ** 0.5).half().to(dev).contiguous()
        self.W3 = (target_scale * teacher[3]).half().to(dev)
        self.W1_8, self.W2_8 = (torch.empty((Hd, Hd), dtype=u8, device=dev) for _ in range(2))
        mp8.quantize_e5m2(self.W1, self.W1_8)
        mp8.quantize_e5m2(self.W2, self.W2_8)
        self.A0_8, self.H1_8, self.H2_8, self.E2_8, self.E1_8, self.E0_8 = (
            torch.empty((M, Hd), dtype=u8, device=dev) for _ in range(6))
        self.G1, self.G2 = (torch.empty((Hd, Hd), dtype=u8, device=dev) for _ in range(2))
        self.ws = torch.empty(64 << 20, dtype=u8, device=dev)
        self.stats = mp8.new_stats()
        self.scaler = mp8.scaler_new(scale, floor, growth_interval)
        self.orc_scaler = oracle.scaler_new(scale, floor, growth_interval)
        self.it = 0
        self.losses, self.scales, self.skips, self.flushed = [], [], [], []

    def set_floor(self, floor):
        self.mp8.scaler_set_floor(self.scaler, floor)
        self.oracle.scaler_set_floor(self.orc_scaler, floor)
        assert self.scaler.scale == self.orc_scaler.scale

    def step(self):
        mp8, torch = self.mp8, self.torch
        M, Hd, O = self.M, self.Hd, self.O
        b_only, both = mp8.FLAG_B_CONTRACTION_MAJOR, mp8.FLAG_CONTRACTION_MAJOR
        rnd, it, st, ws = self.act_round, self.it, self.stats, self.ws
        S = float(self.scaler.scale)
        zero8 = torch.zeros((), dtype=torch.uint8, device="cuda")
        relu8 = lambda c: torch.where((c & 0x80) != 0, zero8, c)
        # forward: FP16 first layer, Q node, two 8-bit layers, FP16 last layer
        A0 = torch.relu(self.X @ self.W0)
        mp8.quantize_e5m2(A0, self.A0_8, round=rnd, seed=31, offset=8 * it)
        mp8.gemm_fp8(mp8.FWD, M, Hd, Hd, self.A0_8, self.W1_8, out8=self.H1_8, round=rnd, seed=31, offset=8 * it + 1,
                     workspace=ws, flags=b_only)
        H1r = relu8(self.H1_8)
        mp8.gemm_fp8(mp8.FWD, M, Hd, Hd, H1r, self.W2_8, out8=self.H2_8, round=rnd, seed=31, offset=8 * it + 2,
                     workspace=ws, flags=b_only)
        H2r = relu8(self.H2_8)
        H2f = codes_as_fp16(H2r)
        Y = (H2f @ self.W3).float()
        diff = Y - self.T
        self.losses.append(float((diff * diff).mean()))
        # backward: the scaled error enters in FP16 (last layer), then through the Q nodes
        dY = ((2.0 * S / (M * O)) * diff).half()
        dW3 = H2f.t() @ dY
        dH2 = dY @ self.W3.t()
        st.zero_()
        mp8.quantize_e5m2(dH2, self.E2_8, round=rnd, seed=31, offset=8 * it + 3, stats=st)
        self.flushed.append(mp8.read_stats(st)[2] / (M * Hd))
        E2m = torch.where(H2r == 0, zero8, self.E2_8)
        mp8.gemm_fp8(mp8.WGRAD, M, Hd, Hd, H1r, E2m, out8=self.G2, round=rnd, seed=31, offset=8 * it + 4, stats=st,
                     workspace=ws, flags=both)
        mp8.gemm_fp8(mp8.BWD_DATA, M, Hd, Hd, E2m, self.W2_8, out8=self.E1_8, round=rnd, seed=31, offset=8 * it + 5,
                     stats=st, workspace=ws)
        E1m = torch.where(H1r == 0, zero8, self.E1_8)
        mp8.gemm_fp8(mp8.WGRAD, M, Hd, Hd, self.A0_8, E1m, out8=self.G1, round=rnd, seed=31, offset=8 * it + 6, stats=st,
                     workspace=ws, flags=both)
        mp8.gemm_fp8(mp8.BWD_DATA, M, Hd, Hd, E1m, self.W1_8, out8=self.E0_8, round=rnd, seed=31, offset=8 * it + 7,
                     stats=st, workspace=ws)
        dA0 = torch.where(A0 > 0, codes_as_fp16(self.E0_8), torch.zeros((), dtype=torch.float16, device="cuda"))
        dW0 = self.X.t() @ dA0
        # the FP16 layers' gradients count towards the overflow decision like every other tensor
        st[1] += ((~torch.isfinite(dW3)).sum() + (~torch.isfinite(dW0)).sum()).to(torch.int32)
        # updates: the kernels read the skip decision from the device counter; the host reads the
        # same counter for the scaler
        before = (self.W1.clone(), self.W2.clone(), self.W1_8.clone(), self.W2_8.clone())
        flag = st[1:2]
        mp8.sgd_update_fp16_sr(self.W1, self.G1, self.lr, 1.0 / S, round=mp8.SR, seed=37, offset=2 * it,
                               skip_if_nonzero=flag, w8_out=self.W1_8)
        mp8.sgd_update_fp16_sr(self.W2, self.G2, self.lr, 1.0 / S, round=mp8.SR, seed=37, offset=2 * it + 1,
                               skip_if_nonzero=flag, w8_out=self.W2_8)
        nonfinite = mp8.read_stats(st)[1]
        skip = mp8.scaler_update(self.scaler, nonfinite)
        want = self.oracle.scaler_update(self.orc_scaler, nonfinite)
        assert skip == want == int(nonfinite != 0), (it, nonfinite, skip, want)
        assert self.scaler.scale == self.orc_scaler.scale and self.scaler.good_steps == self.orc_scaler.good_steps, it
        assert self.scaler.scale >= self.scaler.floor
        if skip:
            after = (self.W1, self.W2, self.W1_8, self.W2_8)
            assert all(torch.equal(x, y) for x, y in zip(before, after)), f"step {it} was to be skipped"
        else:
            self.W0 -= ((self.lr_ends / S) * dW0.float()).half()
            self.W3 -= ((self.lr_ends / S) * dW3.float()).half()
        self.scales.append(S)
        self.skips.append(skip)
        self.it += 1
        return skip


def test_dynamic_loss_scale_backs_off_skips_grows_and_keeps_above_a_raised_minimum(mp8):
    """Section 3.1's back-off scaling: a scale that starts far too large overflows the 8-bit
    errors and gradients; every such step is skipped (the update kernels read the overflow count
    on the device and leave weights and 8-bit weights alone) and halves the scale; after a run of
    clean steps the scale doubles, until it overflows again.  Mid-run the minimum is raised to a
    scale the run has shown to be clean; from then on no back-off goes below it.  PolicyRun.step
    compares every decision, the scale and the clean-step count with the oracle's scaler."""
    r = PolicyRun(mp8, mp8.SR, 2.0 ** 30, 1.0, 20)
    for _ in range(140):
        r.step()
    first_clean = r.skips.index(0)
    assert first_clean >= 5 and all(r.skips[:first_clean])              # the forced overflow at the start
    assert r.scales[first_clean] == 2.0 ** (30 - first_clean)
    grown = [i for i in range(1, len(r.scales)) if r.scales[i] > r.scales[i - 1]]
    assert len(grown) >= 3
    assert any(s and i > grown[0] for i, s in enumerate(r.skips)), "no overflow after the scale had grown"
    floor = min(r.scales[-40:])
    r.set_floor(floor)
    for _ in range(100):
        r.step()
    assert min(r.scales[140:]) >= floor
    assert sum(r.skips[140:]) >= 1, "the raised minimum was never reached from above"
    assert r.losses[-1] < 0.4 * r.losses[0]


def test_raising_the_minimum_scale_brings_flushed_errors_back(mp8):
    """Section 3.1: with too small a scale the errors round to zero in the 8-bit format (nearest
    rounding here, the cleanest case) and the 8-bit layers stop learning; raising the scaler's
    minimum lifts the scale at once, the errors survive, and the loss falls faster than in the
    same run without the raise."""
    raised = PolicyRun(mp8, mp8.RNE, 1.0, 1.0, 100000)
    left = PolicyRun(mp8, mp8.RNE, 1.0, 1.0, 100000)
    for _ in range(60):
        raised.step()
        left.step()
    assert raised.losses == left.losses
    raised.set_floor(2.0 ** 14)
    for _ in range(180):
        raised.step()
        left.step()
    assert set(raised.scales[:60]) == {1.0} and set(raised.scales[60:]) == {2.0 ** 14}
    assert min(raised.flushed[:60]) > 0.8 and max(raised.flushed[60:]) < 0.01
    assert min(left.flushed) > 0.8
    assert sum(raised.skips) == 0
    assert raised.losses[-1] < 0.85 * left.losses[-1]


def test_stochastic_rounding_at_the_q_nodes_survives_an_underscaled_error(mp8):
    """Section 3.2: stochastic rounding at the activation and error Q nodes is unbiased, so errors
    below half the smallest 8-bit subnormal still arrive on average and training proceeds as with
    a generous scale; nearest rounding flushes them and the run falls behind.  With a generous
    scale the two roundings train alike."""
    final = {}
    for name, rnd, scale in (("sr-small", mp8.SR, 0.5), ("rne-small", mp8.RNE, 0.5),
                             ("sr-large", mp8.SR, 2.0 ** 14), ("rne-large", mp8.RNE, 2.0 ** 14)):
        r = PolicyRun(mp8, rnd, scale, scale, 100000)
        for _ in range(200):
            r.step()
        assert sum(r.skips) == 0
        final[name] = r.losses[-1]
    assert final["sr-small"] < 0.7 * final["rne-small"]
    assert abs(final["sr-small"] - final["sr-large"]) < 0.1 * final["sr-large"]
    assert abs(final["rne-large"] - final["sr-large"]) < 0.1 * final["sr-large"]
