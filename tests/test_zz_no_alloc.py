"""GPU test of mp8_gemm_fp8_static, the entry point for callers that cannot allocate: the scratch
of the two-pass GEMM paths lives in a static device array of the library.  Its results must be
those of mp8_gemm_fp8 with a caller's workspace, bit for bit (and both are held against the
oracle here), on two calls in a row that share the array -- the second with a smaller input --
and a shape beyond the array's size must be refused."""
import numpy as np
import pytest

import oracle
from gpu_util import gpu, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mp8():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1905_12334_amd as m
    m.lib()
    return m


def _exact_sum_codes(rng, shape):
    """Codes of {1, 1.25, 1.5, 1.75} * 2^{0..3}, both signs: short sums of their products are
    exact in FP32 in any order, so the accumulator must equal the oracle's reference exactly."""
    return ((rng.integers(0, 2, shape) << 7) | (rng.integers(15, 19, shape) << 2)
            | rng.integers(0, 4, shape)).astype(np.uint8)


def _both_ways(mp8, op, dims, a8, b8, rows, cols, **kw):
    """The same GEMM through mp8_gemm_fp8 (caller's workspace) and mp8_gemm_fp8_static."""
    import torch
    M, N, K = dims
    a, b = gpu(a8), gpu(b8)
    ws = torch.empty(max(mp8.gemm_fp8_workspace_bytes(op, M, N, K), 16), dtype=torch.uint8, device="cuda")
    res = []
    for static in (False, True):
        acc = torch.full((rows * cols + 16,), 7.0, dtype=torch.float32, device="cuda")
        out = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
        out_t = torch.full((rows * cols + 64,), 0xAA, dtype=torch.uint8, device="cuda")
        st = mp8.new_stats()
        args = dict(out8=out[: rows * cols], out8_t=out_t[: rows * cols], acc=acc[: rows * cols], acc_mode=1,
                    stats=st, **kw)
        if static:
            mp8.gemm_fp8_static(op, M, N, K, a, b, **args)
        else:
            mp8.gemm_fp8(op, M, N, K, a, b, workspace=ws, **args)
        torch.cuda.synchronize()
        assert bool((out[rows * cols:] == 0xAA).all()) and bool((out_t[rows * cols:] == 0xAA).all())
        assert bool((acc[rows * cols:] == 7.0).all())
        res.append((host(acc[: rows * cols]).reshape(rows, cols), host(out[: rows * cols]).reshape(rows, cols),
                    host(out_t[: rows * cols]).reshape(cols, rows), mp8.read_stats(st)))
    return res


def test_static_scratch_gemm_equals_the_workspace_gemm_on_two_calls_in_a_row(mp8):
    rng = np.random.default_rng(7)
    assert mp8.static_scratch_bytes() == 32 << 20
    # first call: a weight gradient whose contraction is split into several slices (FP32 tiles of
    # every slice pass through the scratch), stochastic rounding; second call: a smaller GEMM with
    # a ragged column count (unfused epilogue through the scratch), RNE
    cases = [
        (mp8.WGRAD, (8192, 64, 64), 64, 64, 8192, dict(round=oracle.SR, seed=77, offset=3, alpha=2.0 ** -6)),
        (mp8.FWD, (96, 50, 256), 96, 50, 256, dict(alpha=2.0 ** -4)),
    ]
    for op, dims, rows, cols, kc, kw in cases:
        a8, b8 = _exact_sum_codes(rng, (rows, kc)), _exact_sum_codes(rng, (cols, kc))
        if kc > 1024:
            a8[:, rng.random(kc) < 0.9] = 0          # keeps every partial sum exact in FP32
        if op == mp8.WGRAD:
            assert mp8.gemm_fp8_plan(op, *dims, 0)[1] > 1, "this case is meant to split the contraction"
            assert mp8.gemm_fp8_workspace_bytes(op, *dims) > 0
        (acc_w, out_w, out_t_w, st_w), (acc_s, out_s, out_t_s, st_s) = _both_ways(mp8, op, dims, a8, b8, rows, cols, **kw)
        assert np.array_equal(acc_s.view(np.uint32), acc_w.view(np.uint32)), "FP32 result differs"
        assert np.array_equal(out_s, out_w) and np.array_equal(out_t_s, out_t_w), "8-bit result differs"
        assert st_s == st_w
        # and both are the oracle's: exact sums, its rounding of them
        ref, _ = oracle.gemm_ref(a8, b8, want_abs=False)
        assert np.array_equal(acc_s.astype(np.float64), ref)
        want = oracle.quantize_e5m2(acc_s, scale=kw.get("alpha", 1.0), mode=kw.get("round", oracle.RNE),
                                    seed=kw.get("seed", 0), offset=kw.get("offset", 0))[0]
        assert np.array_equal(out_s, want) and np.array_equal(out_t_s, want.T)


def test_static_scratch_gemm_refuses_what_does_not_fit(mp8):
    import torch
    # a split weight gradient whose FP32 slices need more than the 32 MiB the library holds
    M, N, K = 256, 4096, 4096
    need = mp8.gemm_fp8_workspace_bytes(mp8.WGRAD, M, N, K)
    assert need > mp8.static_scratch_bytes()
    a = torch.zeros((K, M), dtype=torch.uint8, device="cuda")
    b = torch.zeros((N, M), dtype=torch.uint8, device="cuda")
    out = torch.full((K * N,), 0xAA, dtype=torch.uint8, device="cuda")
    with pytest.raises(mp8.Mp8Error, match="workspace"):
        mp8.gemm_fp8_static(mp8.WGRAD, M, N, K, a, b, out8=out)
    torch.cuda.synchronize()
    assert bool((out == 0xAA).all()), "a refused call must not write"
