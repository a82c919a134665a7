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


def acc_bounds(ref, absref, kc):
    """Element-wise tolerance of the FP32 accumulator against the double reference.

    The stated bar is a relative error of 1e-5 * sqrt(kc).  For a dot product the error is
    taken relative to sum_j |a_j * b_j| (the scale every inner-product error bound uses; a
    sum that cancels has no meaningful error relative to itself):
        |acc - ref| <= 1e-5 * sqrt(kc) * absref.
    The tighter scale max(|ref|, absref / sqrt(kc)) is also evaluated, for the record: the
    matrix cores align the products of each group of eight to the group's largest product and
    drop what falls more than 13 bits below it, so they can miss that tighter bound by a
    small factor on operands with a wide dynamic range."""
    rk = np.sqrt(float(kc))
    return 1e-5 * rk * absref, 1e-5 * rk * np.maximum(np.abs(ref), absref / rk)


def acc_tolerance_ok(acc, ref, absref, kc):
    tol, tight = acc_bounds(ref, absref, kc)
    err = np.abs(acc.astype(np.float64) - ref)
    finite = np.isfinite(ref)
    ok = np.all(err[finite] <= tol[finite] + 1e-300)
    same_class = np.array_equal(np.isnan(acc), np.isnan(ref)) and np.array_equal(
        np.isinf(acc), np.isinf(ref))
    worst = float((err[finite] / (tol[finite] + 1e-300)).max(initial=0.0))
    worst_tight = float((err[finite] / (tight[finite] + 1e-300)).max(initial=0.0))
    return bool(ok and same_class), worst, worst_tight


def check_outputs(acc_gpu, out8_gpu, ref, absref, kc, alpha=1.0, mode=oracle.RNE, flags=0, seed=0,
                  offset=0, first_index=None, cols=None):
    """The acceptance checks of a GEMM result against the oracle:
    (1) FP32 accumulator within tolerance of the double reference (acc_bounds);
    (2) out8 equals the oracle's rounding of the GPU's own accumulator, bit for bit
        (RNE, or SR with the same random stream);
    (3) RNE: out8 lies between the oracle's roundings of ref - tol and ref + tol, and where the
        sum is well conditioned (|ref| >= absref / sqrt(kc)) it is within one code of the
        oracle's rounding of the double reference.
    For row subsets pass the rows' linear index bases so the SR stream lines up."""
    ok, worst, worst_tight = acc_tolerance_ok(acc_gpu, ref, absref, kc)
    assert ok, f"accumulator outside tolerance (worst ratio {worst})"
    assert worst_tight < 8.0, f"accumulator far outside the tight scale ({worst_tight})"
    tol, _ = acc_bounds(ref, absref, kc)
    if mode == oracle.RNE:
        want, _ = oracle.quantize_e5m2(acc_gpu, scale=alpha, mode=oracle.RNE, flags=flags)
        assert np.array_equal(out8_gpu, want), "out8 != oracle rounding of the GPU accumulator"
        ok_el = np.isfinite(ref)
        s = np.sign(alpha) if alpha != 0 else 1.0
        lo = signed_rank(oracle.round_ref_e5m2(np.where(ok_el, ref - s * tol, 0.0), alpha=alpha, flags=flags))
        hi = signed_rank(oracle.round_ref_e5m2(np.where(ok_el, ref + s * tol, 0.0), alpha=alpha, flags=flags))
        got = signed_rank(out8_gpu)
        assert np.all((got >= lo)[ok_el] & (got <= hi)[ok_el]), "out8 outside the tolerance interval"
        near = signed_rank(oracle.round_ref_e5m2(np.where(ok_el, ref, 0.0), alpha=alpha, flags=flags))
        well = ok_el & (np.abs(ref) >= absref / np.sqrt(float(kc)))
        assert np.all(np.abs(got - near)[well] <= 1), "out8 more than one code from the rounded reference"
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
    return worst, worst_tight
