"""Pins for the oracle's Philox stream, GEMM reference, master-weight update and loss
scaler (CPU only).  Expected values: published Philox known answers (tests/golden), exact
integer / rational arithmetic, numpy float64 matmul and numpy float16 conversions."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_1905_12334_amd import workloads


# ---- Philox --------------------------------------------------------------------------

def test_philox_known_answers(golden_dir):
    n = 0
    with open(f"{golden_dir}/philox4x32_10_kat.txt") as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(t, 16) for t in line.split()]
            out = oracle.philox4x32_10(w[0:4], w[4:6])
            assert [int(v) for v in out] == w[6:10]
            n += 1
    assert n == 3


def test_sr_stream_layout():
    seed, offset = 0x0123456789ABCDEF, 0xFEDCBA9876543210
    for i in (0, 1, 7, 8, 9, 1023, 2 ** 35 + 5, 2 ** 40 - 1):
        blk = i >> 3
        ctr = [blk & 0xFFFFFFFF, blk >> 32, offset & 0xFFFFFFFF, offset >> 32]
        key = [seed & 0xFFFFFFFF, seed >> 32]
        w = oracle.philox4x32_10(ctr, key)
        halves = []
        for word in w:
            halves += [int(word) & 0xFFFF, int(word) >> 16]
        assert oracle.sr_bits(seed, offset, i) == halves[i & 7]
    # different offsets / seeds give different streams
    a = [oracle.sr_bits(1, 0, i) for i in range(64)]
    assert a != [oracle.sr_bits(1, 1, i) for i in range(64)]
    assert a != [oracle.sr_bits(2, 0, i) for i in range(64)]


def test_sr_stream_is_uniform():
    r = np.array([oracle.sr_bits(42, 3, i) for i in range(200_000)], dtype=np.float64)
    assert abs(r.mean() / 65536 - 0.5) < 4 * (1 / np.sqrt(12 * r.size))
    hist = np.bincount((r.astype(np.int64) >> 12), minlength=16)
    chi2 = ((hist - r.size / 16) ** 2 / (r.size / 16)).sum()
    assert chi2 < 45.0   # 15 dof, p ~ 1e-4


# ---- GEMM reference -------------------------------------------------------------------

def _decode_np(codes):
    return (codes.astype(np.uint16) << 8).view(np.float16).astype(np.float64)


def test_gemm_ref_vs_numpy_float64_matmul():
    a = workloads.random_e5m2_codes(1, (37, 160))
    b = workloads.random_e5m2_codes(2, (53, 160))
    a[:, :] = (a & 0x83) | ((a & 0x7C) % 0x30 + 0x20) & 0x7C | (a & 0x03)  # moderate exponents
    b[:, :] = (b & 0x83) | ((b & 0x7C) % 0x30 + 0x20) & 0x7C | (b & 0x03)
    ref, absref = oracle.gemm_ref(a, b)
    A, B = _decode_np(a), _decode_np(b)
    want = A @ B.T
    wabs = np.abs(A) @ np.abs(B).T
    assert ref.shape == (37, 53)
    assert np.all(np.abs(ref - want) <= 1e-13 * wabs)
    assert np.allclose(absref, wabs, rtol=1e-13, atol=0)


def test_gemm_ref_exact_sum_inputs_bit_equal_any_order():
    # values {1,1.25,1.5,1.75} * 2^{0..3}, both signs: every partial sum is an integer
    # multiple of 2^-4 far below 2^53, so order cannot matter and numpy must agree exactly
    rng = np.random.default_rng(3)
    def codes(shape):
        e = rng.integers(15, 19, shape)
        m = rng.integers(0, 4, shape)
        s = rng.integers(0, 2, shape)
        return ((s << 7) | (e << 2) | m).astype(np.uint8)
    a, b = codes((19, 256)), codes((23, 256))
    ref, _ = oracle.gemm_ref(a, b)
    assert np.array_equal(ref, _decode_np(a) @ _decode_np(b).T)
    perm = rng.permutation(256)
    ref2, _ = oracle.gemm_ref(np.ascontiguousarray(a[:, perm]), np.ascontiguousarray(b[:, perm]))
    assert np.array_equal(ref, ref2)
    ex, bad = oracle.gemm_exact(a, b)
    assert bad == 0
    assert all(Fraction(ex[r][c], 2 ** 32) == Fraction(ref[r, c]) for r in range(19) for c in range(23))


def test_gemm_exact_vs_rational_bruteforce_full_range():
    a = workloads.random_e5m2_codes(4, (5, 24))
    b = workloads.random_e5m2_codes(5, (6, 24))
    ex, bad = oracle.gemm_exact(a, b)
    assert bad == 0
    A, B = _decode_np(a), _decode_np(b)
    ref, _ = oracle.gemm_ref(a, b)
    for r in range(5):
        for c in range(6):
            s = sum(Fraction(A[r, j]) * Fraction(B[c, j]) for j in range(24))
            assert Fraction(ex[r][c], 2 ** 32) == s
            assert abs(Fraction(ref[r, c]) - s) <= Fraction(1, 2 ** 45) * sum(
                abs(Fraction(A[r, j]) * Fraction(B[c, j])) for j in range(24))


def test_gemm_row_subset_strides_and_structure():
    a = workloads.random_e5m2_codes(6, (40, 96))
    b = workloads.random_e5m2_codes(7, (24, 96))
    full, fabs_ = oracle.gemm_ref(a, b)
    idx = np.array([39, 0, 17, 17, 5])
    sub, sabs = oracle.gemm_ref(a, b, row_idx=idx)
    assert np.array_equal(sub, full[idx]) and np.array_equal(sabs, fabs_[idx])
    # leading dimension larger than the contraction length
    big = workloads.random_e5m2_codes(8, (40, 200))
    v, _ = oracle.gemm_ref(big[:, 8:104], b)
    w, _ = oracle.gemm_ref(np.ascontiguousarray(big[:, 8:104]), b)
    assert np.array_equal(v, w)
    # one-hot B picks out columns of A: ref[r,c] = a[r, sel[c]]
    sel = np.array([3, 95, 0, 50])
    onehot = np.zeros((4, 96), dtype=np.uint8)
    onehot[np.arange(4), sel] = 0x3C
    p, _ = oracle.gemm_ref(a, onehot)
    assert np.array_equal(p, _decode_np(a)[:, sel])
    # swapping operands transposes the result (catches a transposed / swapped operand)
    t, _ = oracle.gemm_ref(b, a)
    assert np.array_equal(t, full.T)
    # IEEE propagation of Inf / NaN codes
    a2 = a.copy()
    a2[0, 0] = 0x7C
    b2 = b.copy()
    b2[1, 0] = 0x00
    b2[2, 0] = 0x3C
    b2[3, 0] = 0xBC
    z, _ = oracle.gemm_ref(a2, b2)
    assert np.isnan(z[0, 1]) and z[0, 2] == np.inf and z[0, 3] == -np.inf


def test_round_ref():
    ref = np.array([1.0, 1.125, 1.1250001, -61440.0, 3e-6, 1e-5], dtype=np.float64)
    out = oracle.round_ref_e5m2(ref)
    assert list(out) == [0x3C, 0x3C, 0x3D, 0xFC, 0x00, 0x01]
    assert list(oracle.round_ref_e5m2(ref, alpha=2.0 ** -12)[:2]) == [0x0C, 0x0C]


# ---- master-weight update -------------------------------------------------------------

def _f32_fma_exact(lr, g, w):
    """Correctly rounded FP32 of w - lr*g from exact rational arithmetic."""
    t = Fraction(float(w)) - Fraction(float(lr)) * Fraction(float(g))
    c = np.float32(float(t))           # within one FP32 ulp of t
    cands = [c, np.nextafter(c, np.float32(-np.inf)), np.nextafter(c, np.float32(np.inf))]
    def key(v):
        return (abs(Fraction(float(v)) - t), int(np.array([v]).view(np.uint32)[0]) & 1)
    return min(cands, key=key)


def test_update_rne_vs_exact_rational_and_numpy_half():
    rng = np.random.default_rng(31)
    n = 3000
    w16 = (rng.standard_normal(n) * 0.05).astype(np.float16)
    g8 = workloads.random_e5m2_codes(32, (n,))
    lr, inv = np.float32(0.37), np.float32(1.0 / 1024)
    new, w8 = oracle.sgd_update_fp16(w16.view(np.uint16), g8, lr, inv, mode=oracle.RNE, want_w8=True)
    gval = (_decode_np(g8).astype(np.float32) * inv).astype(np.float32)
    for i in range(n):
        wn = _f32_fma_exact(lr, gval[i], np.float32(w16[i]))
        with np.errstate(over="ignore"):
            want = int(np.array([wn]).astype(np.float16).view(np.uint16)[0])
        assert int(new[i]) == want, i
    # the 8-bit copy is the RNE quantisation of the stored half weight
    import torch
    want8 = torch.from_numpy(new.view(np.float16).astype(np.float32)).to(torch.float8_e5m2).view(
        torch.uint8).numpy()
    assert np.array_equal(w8, want8)


def test_update_identities_and_skip():
    rng = np.random.default_rng(33)
    n = 4096
    w16 = (rng.standard_normal(n) * 0.02).astype(np.float16).view(np.uint16)
    g8 = workloads.random_e5m2_codes(34, (n,))
    for mode in (oracle.RNE, oracle.SR):
        same, _ = oracle.sgd_update_fp16(w16, g8, 0.0, 1.0, mode=mode, seed=5, offset=6)
        assert np.array_equal(same, w16)              # lr = 0: exactly representable, never moves
        skipped, _ = oracle.sgd_update_fp16(w16, g8, 0.1, 1.0, mode=mode, skip=1)
        assert np.array_equal(skipped, w16)
        notskipped, _ = oracle.sgd_update_fp16(w16, g8, 0.1, 1.0, mode=mode, skip=0)
        assert not np.array_equal(notskipped, w16)
    st = oracle.Stats()
    g_bad = g8.copy()
    g_bad[5] = 0x7C
    g_bad[9] = 0xFE
    oracle.sgd_update_fp16(w16, g_bad, 0.1, 1.0, stats=st, skip=1)
    assert st.nonfinite == 2


def test_update_sr_bracket_and_unbiased_where_rne_stalls():
    # magnitudes of the Transformer-big update: |w| ~ 0.02 (half spacing 1.5e-5),
    # lr * g ~ 1e-3 * 1e-5, far below half a spacing
    lay = workloads.config5(tokens=8, d_in=64, d_out=128)
    w16 = lay.W.astype(np.float16).view(np.uint16).reshape(-1)
    n = w16.size
    g = (np.random.default_rng(35).standard_normal(n) * 1e-5 * lay.loss_scale).astype(np.float32)
    g8, _ = oracle.quantize_e5m2(g.reshape(1, -1))
    g8 = g8.reshape(-1)
    lr, inv = 1e-3, 1.0 / lay.loss_scale
    rne, _ = oracle.sgd_update_fp16(w16, g8, lr, inv, mode=oracle.RNE)
    assert np.array_equal(rne, w16)                    # every weight stalls under RNE
    w = w16.view(np.float16).astype(np.float64)
    exact = w - np.float64(np.float32(lr)) * (_decode_np(g8) * inv)
    trials = 400
    acc = np.zeros(n)
    for t in range(trials):
        sr, _ = oracle.sgd_update_fp16(w16, g8, lr, inv, mode=oracle.SR, seed=77, offset=t)
        v = sr.view(np.float16).astype(np.float64)
        acc += v
        spacing = np.maximum(np.abs(np.spacing(w16.view(np.float16))).astype(np.float64), 0)
        assert np.all(np.abs(v - exact) <= spacing * 1.0000001)
    mean_move = acc / trials - w
    step = exact - w
    spacing = np.abs(np.spacing(w16.view(np.float16))).astype(np.float64)
    # E[move] = step for every weight; project on the step's direction and sum: the
    # variance of each Bernoulli move is at most |step| * spacing / trials
    got = (mean_move * np.sign(step)).sum()
    want = np.abs(step).sum()
    sigma = np.sqrt((np.abs(step) * spacing).sum() / trials)
    assert want > 20 * sigma                 # the test has power: the signal is visible
    assert abs(got - want) < 5 * sigma


# ---- loss scaler ----------------------------------------------------------------------

def test_scaler_traces():
    s = oracle.scaler_new(2.0 ** 15, 2.0 ** 10, 3)
    trace = []
    for nf in (0, 0, 0, 0, 1, 0, 7, 0, 0, 0):
        skip = oracle.scaler_update(s, nf)
        trace.append((skip, s.scale))
    assert trace == [(0, 2.0 ** 15), (0, 2.0 ** 15), (0, 2.0 ** 16), (0, 2.0 ** 16), (1, 2.0 ** 15),
                     (0, 2.0 ** 15), (1, 2.0 ** 14), (0, 2.0 ** 14), (0, 2.0 ** 14), (0, 2.0 ** 15)]
    # never below the floor, and raising the floor lifts the scale (Section 3.1's schedule:
    # minimum 8K, later 32K)
    s = oracle.scaler_new(4096.0, 1024.0, 1000)
    for _ in range(10):
        assert oracle.scaler_update(s, 1) == 1
    assert s.scale == 1024.0
    oracle.scaler_set_floor(s, 8192.0)
    assert s.scale == 8192.0
    oracle.scaler_update(s, 3)
    assert s.scale == 8192.0
    oracle.scaler_set_floor(s, 32768.0)
    assert s.scale == 32768.0 and s.floor == 32768.0
    # growth stops at 2^32 (hand trace: 2^30 doubles twice, then stays); an overflow still halves;
    # a floor above the limit is respected and not grown further
    s = oracle.scaler_new(2.0 ** 30, 1.0, 1)
    assert [oracle.scaler_update(s, 0) or s.scale for _ in range(4)] == [2.0 ** 31, 2.0 ** 32, 2.0 ** 32, 2.0 ** 32]
    assert oracle.scaler_update(s, 5) == 1 and s.scale == 2.0 ** 31
    s = oracle.scaler_new(3.0 * 2.0 ** 30, 1.0, 1)      # 1.5 * 2^31 doubles past the limit: clamped
    oracle.scaler_update(s, 0)
    assert s.scale == 2.0 ** 32
    s = oracle.scaler_new(1.0, 1.0, 1)
    oracle.scaler_set_floor(s, 2.0 ** 40)
    oracle.scaler_update(s, 0)
    assert s.scale == 2.0 ** 40
    oracle.scaler_update(s, 1)
    assert s.scale == 2.0 ** 40


def test_overflow_injection_drives_scaler():
    lay = workloads.config3(tokens=16, d_model=32, d_ff=64)[0]
    st = oracle.Stats()
    e = lay.dY.copy()
    e[3, 4] = np.inf
    oracle.quantize_e5m2(e, scale=lay.loss_scale, stats=st)
    s = oracle.scaler_new(2.0 ** 12, 2.0 ** 10, 2000)
    assert st.nonfinite == 1 and oracle.scaler_update(s, st.nonfinite) == 1 and s.scale == 2.0 ** 11


# --- momentum optimizer on the master weights (Figure 1b, Eq. 1) ------------------------------

def test_momentum_update_reduces_to_plain_update_and_closed_forms():
    rng = np.random.default_rng(5)
    n = 4096
    w16 = (rng.standard_normal(n) * 0.05).astype(np.float16).view(np.uint16)
    g8 = workloads.random_e5m2_codes(6, (n,), finite_only=False)
    vel = np.zeros(n, np.float32)
    # momentum 0, no decay: the plain update, bit for bit, under both rounding modes
    for mode in (oracle.RNE, oracle.SR):
        a, _ = oracle.sgd_update_fp16(w16, g8, 0.01, 1 / 256.0, mode=mode, seed=3, offset=4)
        b, v, _ = oracle.sgd_momentum_fp16(w16, vel, g8, 0.01, 1 / 256.0, 0.0, 0.0, mode=mode, seed=3, offset=4)
        assert np.array_equal(a, b)
        gf = ((g8.astype(np.uint16) << 8).view(np.float16).astype(np.float32) * np.float32(1 / 256.0))
        assert np.array_equal(v, gf, equal_nan=True)                       # velocity = gradient
    # constant gradient 1.0, momentum 1/2: v_t = 2 - 2^(1-t) exactly; lr = 2^-6 keeps every
    # weight on the half-precision grid, so t steps from w = 1 give 1 - 2^-6 * sum_{k<=t} v_k exactly
    w = np.array([0x3C00], np.uint16)                                       # 1.0
    v = np.zeros(1, np.float32)
    g = np.array([0x3C], np.uint8)
    want_w = 1.0
    for t in range(1, 6):
        w, v, _ = oracle.sgd_momentum_fp16(w, v, g, 2.0 ** -6, 1.0, 0.5, 0.0, mode=oracle.RNE)
        assert v[0] == 2.0 - 2.0 ** (1 - t)
        want_w -= 2.0 ** -6 * v[0]
        assert oracle.fp16_decode(int(w[0])) == want_w
    # regularisation alone: zero gradient, decay d, lr: w' = w - lr*d*w = w * (1 - lr*d)
    w = np.array([0x4000], np.uint16)                                       # 2.0
    w2, v2, _ = oracle.sgd_momentum_fp16(w, np.zeros(1, np.float32), np.zeros(1, np.uint8), 0.25, 1.0, 0.0,
                                         0.5, mode=oracle.RNE)
    assert v2[0] == 1.0 and oracle.fp16_decode(int(w2[0])) == 2.0 * (1 - 0.25 * 0.5)
    # the skip flag leaves weights and velocity untouched, non-finite gradient codes are counted
    st = oracle.Stats()
    g_bad = np.array([0x7C, 0x3C, 0xFF], np.uint8)
    w3 = np.array([0x3C00, 0x3C00, 0x3C00], np.uint16)
    w4, v4, _ = oracle.sgd_momentum_fp16(w3, np.ones(3, np.float32), g_bad, 0.1, 1.0, 0.9, 0.0, skip=1, stats=st)
    assert np.array_equal(w4, w3) and np.array_equal(v4, np.ones(3, np.float32)) and st.nonfinite == 2


def test_momentum_update_against_float32_numpy():
    """numpy float32 arithmetic with the fused multiply-adds written as exact double products
    (a double holds the product of two floats exactly) rounded once to float32."""
    rng = np.random.default_rng(8)
    n = 20000
    w16 = (rng.standard_normal(n) * 0.1).astype(np.float16).view(np.uint16)
    g8 = workloads.random_e5m2_codes(9, (n,))
    vel = (rng.standard_normal(n) * 0.01).astype(np.float32)
    lr, inv, mu, wd = np.float32(0.05), np.float32(1 / 1024.0), np.float32(0.9), np.float32(1e-4)
    got_w, got_v, _ = oracle.sgd_momentum_fp16(w16, vel, g8, lr, inv, mu, wd, mode=oracle.RNE)
    fma = lambda a, b, c: (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)
    w = w16.view(np.float16).astype(np.float32)
    g0 = ((g8.astype(np.uint16) << 8).view(np.float16).astype(np.float32) * inv).astype(np.float32)
    g = fma(np.full(n, wd), w, g0)
    v = fma(np.full(n, mu), vel, g)
    wn = fma(np.full(n, -lr), v, w)
    # the double-then-float rounding of the emulation differs from a true fused operation only on
    # rare double-rounding ties: allow a handful of last-bit differences in the velocity
    assert np.mean(got_v.view(np.uint32) != v.view(np.uint32)) < 1e-3
    same = got_v.view(np.uint32) == v.view(np.uint32)
    assert np.array_equal(got_w[same], wn.astype(np.float16).view(np.uint16)[same])


# --- ADAM on the master weights (Section 4 names the optimizer; published algorithm) ----------

def _half_grid_error(w16_codes, ref):
    """|value(code) - ref| in units of the half-precision spacing at ref."""
    got = np.asarray(w16_codes, np.uint16).view(np.float16).astype(np.float64)
    spacing = np.maximum(np.spacing(np.abs(ref).astype(np.float16)).astype(np.float64), 2.0 ** -24)
    return np.abs(got - ref) / spacing


def test_adam_closed_forms_and_special_cases():
    f16 = lambda x: np.array([x], np.float16).view(np.uint16)
    z = np.zeros(1, np.float32)
    one = np.array([0x3C], np.uint8)                                         # gradient 1.0
    # first step from zero moments: mhat = g and vhat = g^2 whatever the betas, so the step is
    # lr * g / (|g| + eps) -- the sign of the gradient times lr (the textbook property of ADAM)
    for g8, sign in ((0x3C, 1.0), (0xBC, -1.0), (0x30, 1.0), (0xC4, -1.0), (0x54, 1.0)):
        w, m, v, _ = oracle.adam_fp16(f16(1.0), z, z, np.array([g8], np.uint8), 2.0 ** -5, 1.0, 1,
                                      beta1=0.5, beta2=0.75, eps=0.0, mode=oracle.RNE)
        assert oracle.fp16_decode(int(w[0])) == 1.0 - sign * 2.0 ** -5
        gval = oracle.e5m2_decode(g8)
        assert m[0] == 0.5 * gval and v[0] == 0.25 * gval * gval            # (1-b1) g, (1-b2) g^2
    # constant gradient: mhat = g and vhat = g^2 at EVERY step (the bias corrections undo the
    # geometric sums exactly for these dyadic betas), so t steps move the weight by t * lr
    w, m, v = f16(1.0), z, z
    for t in range(1, 7):
        w, m, v, _ = oracle.adam_fp16(w, m, v, one, 2.0 ** -6, 1.0, t, beta1=0.5, beta2=0.5, eps=0.0,
                                      mode=oracle.RNE)
        assert m[0] == 1.0 - 0.5 ** t and v[0] == 1.0 - 0.5 ** t
        assert oracle.fp16_decode(int(w[0])) == 1.0 - t * 2.0 ** -6
    # eps enters the denominator: g = 1, eps = 1 -> step lr / 2
    w, _, _, _ = oracle.adam_fp16(f16(1.0), z, z, one, 2.0 ** -4, 1.0, 1, beta1=0.5, beta2=0.5, eps=1.0,
                                  mode=oracle.RNE)
    assert oracle.fp16_decode(int(w[0])) == 1.0 - 2.0 ** -5
    # the loss scale is divided out before the moments: g8 = 4.0 with inv_loss_scale 1/4 is g = 1
    w, m, _, _ = oracle.adam_fp16(f16(1.0), z, z, np.array([0x44], np.uint8), 2.0 ** -4, 0.25, 1, beta1=0.5,
                                  beta2=0.5, eps=1.0, mode=oracle.RNE)
    assert oracle.fp16_decode(int(w[0])) == 1.0 - 2.0 ** -5 and m[0] == 0.5
    # zero gradient, zero moments, eps > 0: nothing moves (0 / (0 + eps) = 0)
    w, m, v, _ = oracle.adam_fp16(f16(0.75), z, z, np.zeros(1, np.uint8), 0.1, 1.0, 3, eps=1e-8)
    assert oracle.fp16_decode(int(w[0])) == 0.75 and m[0] == 0 and v[0] == 0
    # regularisation alone (Eq. 1): the gradient is weight_decay * w; first step, eps = 0:
    # w' = w - lr * sign(w)
    w, m, _, _ = oracle.adam_fp16(f16(-2.0), z, z, np.zeros(1, np.uint8), 2.0 ** -3, 1.0, 1, beta1=0.5,
                                  beta2=0.5, eps=0.0, weight_decay=0.5, mode=oracle.RNE)
    assert oracle.fp16_decode(int(w[0])) == -2.0 + 2.0 ** -3 and m[0] == 0.5 * (0.5 * -2.0)
    # skip flag: nothing changes, non-finite gradient codes are still counted
    st = oracle.Stats()
    w3 = np.array([0x3C00, 0x3C00, 0x3C00], np.uint16)
    w4, m4, v4, _ = oracle.adam_fp16(w3, np.ones(3, np.float32), np.ones(3, np.float32),
                                     np.array([0x7C, 0x3C, 0xFF], np.uint8), 0.1, 1.0, 2, skip=1, stats=st)
    assert np.array_equal(w4, w3) and np.all(m4 == 1) and np.all(v4 == 1) and st.nonfinite == 2
    # stochastic rounding of the new weight: r16 = 0 truncates toward zero (offset chosen freely:
    # the expected value over many offsets is the FP32 result)
    g = np.full(4096, 0x3C, np.uint8)
    w0 = np.full(4096, 0x3C00, np.uint16)
    zz = np.zeros(4096, np.float32)
    ws, _, _, _ = oracle.adam_fp16(w0, zz, zz, g, 2.0 ** -13, 1.0, 1, beta1=0.5, beta2=0.5, eps=0.0,
                                   mode=oracle.SR, seed=7, offset=9)
    vals = ws.view(np.float16).astype(np.float64)                            # 1 - 2^-13: between 1-2^-11 and 1
    assert set(np.unique(vals)) == {1.0 - 2.0 ** -11, 1.0}
    assert abs(vals.mean() - (1.0 - 2.0 ** -13)) < 3 * 2.0 ** -11 * 0.5 / np.sqrt(4096) * 2


def test_adam_against_float64_numpy_and_torch():
    rng = np.random.default_rng(12)
    n = 20000
    w16 = (rng.standard_normal(n) * 0.1).astype(np.float16).view(np.uint16)
    g8 = workloads.random_e5m2_codes(13, (n,))
    g8 = (g8 & 0x83) | 0x48                               # |g8| in [32, 56]: un-scaled gradients ~ 0.04
    m0 = (rng.standard_normal(n) * 0.01).astype(np.float32)
    v0 = (rng.random(n) * 1e-3).astype(np.float32)
    lr, inv, b1, b2, eps, wd, step = 1e-3, 1 / 1024.0, 0.9, 0.999, 1e-8, 1e-4, 5
    got_w, got_m, got_v, got8 = oracle.adam_fp16(w16, m0, v0, g8, lr, inv, step, beta1=b1, beta2=b2, eps=eps,
                                                 weight_decay=wd, mode=oracle.RNE, want_w8=True)
    # the textbook formulas in float64
    w = w16.view(np.float16).astype(np.float64)
    g = (g8.astype(np.uint16) << 8).view(np.float16).astype(np.float64) * inv + wd * w
    f = lambda x: float(np.float32(x))                    # the parameters are FP32 numbers
    g = (g8.astype(np.uint16) << 8).view(np.float16).astype(np.float64) * f(inv) + f(wd) * w
    omb1, omb2 = float(np.float32(1) - np.float32(b1)), float(np.float32(1) - np.float32(b2))
    m = f(b1) * m0 + omb1 * g
    v = f(b2) * v0 + omb2 * g * g
    ref = w - f(lr) * (m / (1 - f(b1) ** step)) / (np.sqrt(v / (1 - f(b2) ** step)) + f(eps))
    # a few FP32 roundings on terms of the size of the operands (the two terms of m may cancel)
    assert np.all(np.abs(got_m - m) <= 3e-7 * (np.abs(f(b1) * m0) + np.abs(omb1 * g)))
    assert np.all(np.abs(got_v - v) <= 3e-7 * v)
    assert _half_grid_error(got_w, ref).max() <= 0.5 + 1e-3           # the nearest half, FP32 noise aside
    assert np.array_equal(got8, oracle.quantize_e5m2(got_w.view(np.float16).reshape(1, -1))[0].reshape(-1))
    # the library routine: torch's CPU ADAM in float32 on the same numbers (different operation
    # order, so equal only to FP32 accuracy; its weights are compared on the half grid)
    import torch
    p = torch.nn.Parameter(torch.from_numpy(w16.view(np.float16).astype(np.float32)))
    opt = torch.optim.Adam([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    opt.zero_grad()
    p.grad = torch.from_numpy(((g8.astype(np.uint16) << 8).view(np.float16).astype(np.float32) * np.float32(inv)))
    opt.state[p]["step"] = torch.tensor(float(step - 1))
    opt.state[p]["exp_avg"] = torch.from_numpy(m0.copy())
    opt.state[p]["exp_avg_sq"] = torch.from_numpy(v0.copy())
    opt.step()
    assert np.all(np.abs(got_m - opt.state[p]["exp_avg"].numpy()) <= 1e-6 * (np.abs(f(b1) * m0) + np.abs(omb1 * g)))
    # torch forms 1 - beta2 in double (0.001); the FP32 difference 1 - fl32(0.999) is 4.7e-5 larger
    assert np.all(np.abs(got_v - opt.state[p]["exp_avg_sq"].numpy()) <= 1e-6 * v + 6e-5 * omb2 * g * g)
    assert _half_grid_error(got_w, p.detach().numpy().astype(np.float64)).max() <= 0.5 + 1e-2
