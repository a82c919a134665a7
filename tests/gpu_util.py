"""Helpers shared by the GPU parity tests: upload/download and the GEMM acceptance checks."""
from __future__ import annotations

import numpy as np

import oracle


def gpu(arr):
    import torch
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def host(t):
    return t.cpu().numpy()


def signed_rank(codes):
    """Map 8-bit codes to integers ordered like their values (sign-magnitude order)."""
    c = codes.astype(np.int32)
    mag = c & 0x7F
    return np.where(c & 0x80, -mag, mag)


def acc_tolerance_ok(acc, ref, absref, kc):
    """|acc - ref| <= 1e-5 * sqrt(kc) * max(|ref|, absref / sqrt(kc)), element-wise."""
    rk = np.sqrt(float(kc))
    bound = 1e-5 * rk * np.maximum(np.abs(ref), absref / rk)
    err = np.abs(acc.astype(np.float64) - ref)
    finite = np.isfinite(ref)
    ok = np.all(err[finite] <= bound[finite] + 1e-300)
    same_class = np.array_equal(np.isnan(acc), np.isnan(ref)) and np.array_equal(
        np.isinf(acc), np.isinf(ref))
    return bool(ok and same_class), float((err[finite] / (bound[finite] + 1e-300)).max(initial=0.0))


def check_outputs(acc_gpu, out8_gpu, ref, absref, kc, alpha=1.0, mode=oracle.RNE, flags=0, seed=0,
                  offset=0, first_index=None, cols=None):
    """The three acceptance checks of a GEMM result against the oracle:
    (1) FP32 accumulator within tolerance of the double reference;
    (2) out8 equals the oracle's rounding of the GPU's own accumulator, bit for bit;
    (3) out8 within one code of the oracle's rounding of the double reference (RNE), or
        within one code of the bracket [toward-zero code, +1] of the reference (SR).
    For row subsets pass the rows' linear index bases so the SR stream lines up."""
    ok, worst = acc_tolerance_ok(acc_gpu, ref, absref, kc)
    assert ok, f"accumulator outside tolerance (worst ratio {worst})"
    if mode == oracle.RNE:
        want, _ = oracle.quantize_e5m2(acc_gpu, scale=alpha, mode=oracle.RNE, flags=flags)
        assert np.array_equal(out8_gpu, want), "out8 != oracle rounding of the GPU accumulator"
        near = oracle.round_ref_e5m2(ref, alpha=alpha, flags=flags)
        nan = np.isnan(ref)
        d = np.abs(signed_rank(out8_gpu) - signed_rank(near))
        assert np.all(d[~nan] <= 1), "out8 more than one code from the rounded reference"
    else:
        rows, ncols = acc_gpu.shape
        want = np.empty_like(out8_gpu)
        y = (acc_gpu * np.float32(alpha)).astype(np.float32)
        for t in range(rows):
            base = (first_index[t] if first_index is not None else t * ncols)
            for c in range(ncols):
                r16 = oracle.sr_bits(seed, offset, base + c)
                want[t, c] = oracle.e5m2_encode(float(y[t, c]), oracle.SR, r16, bool(flags & 1))
        assert np.array_equal(out8_gpu, want), "SR out8 != oracle SR of the GPU accumulator"
    return worst
