"""CPU-side checks of the product library: it loads, exports every symbol the header
declares, and its host-only logic (Philox block, loss scaler, planning, argument
validation) behaves.  No kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_1905_12334_amd as mp8

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mp8.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mp8_[a-z0-9_]+)\s*\(", header))
    assert declared == set(mp8.EXPORTS)
    L = mp8.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_host_philox_known_answers_and_oracle_agreement(golden_dir):
    with open(f"{golden_dir}/philox4x32_10_kat.txt") as f:
        rows = [[int(t, 16) for t in l.split()] for l in f if l.strip() and not l.startswith("#")]
    for w in rows:
        assert mp8.philox4x32_10(w[0:4], w[4:6]) == w[6:10]
    rng = np.random.default_rng(1)
    for _ in range(2000):
        ctr = rng.integers(0, 2 ** 32, 4, dtype=np.uint64)
        key = rng.integers(0, 2 ** 32, 2, dtype=np.uint64)
        assert mp8.philox4x32_10(ctr, key) == [int(x) for x in oracle.philox4x32_10(ctr, key)]


def test_scaler_matches_oracle_on_random_traces():
    rng = np.random.default_rng(2)
    for trial in range(20):
        floor = float(2 ** rng.integers(0, 12))
        scale = floor * float(2 ** rng.integers(0, 8))
        gi = int(rng.integers(1, 6))
        a = mp8.scaler_new(scale, floor, gi)
        b = oracle.scaler_new(scale, floor, gi)
        for step in range(200):
            nf = int(rng.integers(0, 3) == 0) * int(rng.integers(1, 9))
            assert mp8.scaler_update(a, nf) == oracle.scaler_update(b, nf)
            if step % 50 == 49:
                nfloor = float(2 ** rng.integers(0, 16))
                mp8.scaler_set_floor(a, nfloor)
                oracle.scaler_set_floor(b, nfloor)
            assert (a.scale, a.floor, a.good_steps) == (b.scale, b.floor, b.good_steps)
            assert a.scale >= a.floor


def test_status_strings_and_validation_without_gpu():
    L = mp8.lib()
    assert L.mp8_status_string(0) == b"ok"
    assert all(len(L.mp8_status_string(i)) > 0 for i in range(7))
    one = C.c_void_p(16)
    # bad enum / negative sizes / null pointers are rejected before anything is enqueued
    assert L.mp8_quantize_e5m2(one, 0, one, None, -1, 4, 1.0, 0, 0, 0, 0, None, None) == 1
    assert L.mp8_quantize_e5m2(one, 0, one, None, 4, 4, 1.0, 7, 0, 0, 0, None, None) == 1
    assert L.mp8_quantize_e5m2(None, 0, one, None, 4, 4, 1.0, 0, 0, 0, 0, None, None) == 1
    assert L.mp8_quantize_e5m2(C.c_void_p(8), 0, one, None, 4, 4, 1.0, 0, 0, 0, 0, None, None) == 3
    assert L.mp8_quantize_e5m2(None, 0, None, None, 0, 4, 1.0, 0, 0, 0, 0, None, None) == 0
    assert L.mp8_sgd_update_fp16_sr(None, None, 0, 0.1, 1.0, 1, 0, 0, None, None, None, None) == 0
    assert L.mp8_sgd_update_fp16_sr(None, one, 5, 0.1, 1.0, 1, 0, 0, None, None, None, None) == 1
    assert L.mp8_sgd_update_fp16_sr(one, one, 5, 0.1, 1.0, 9, 0, 0, None, None, None, None) == 1
    g = lambda *a: L.mp8_gemm_fp8(*a)
    assert g(5, 8, 8, 128, one, 128, one, 128, 1.0, None, 0, one, None, 0, 0, 0, 0, None, None, 0, None) == 1
    assert g(0, -1, 8, 128, one, 128, one, 128, 1.0, None, 0, one, None, 0, 0, 0, 0, None, None, 0, None) == 1
    assert g(0, 8, 8, 128, one, 64, one, 128, 1.0, None, 0, one, None, 0, 0, 0, 0, None, None, 0, None) == 1
    assert g(0, 8, 8, 128, one, 128, one, 128, 1.0, None, 1, one, None, 0, 0, 0, 0, None, None, 0, None) == 1
    assert g(0, 0, 8, 128, None, 128, None, 128, 1.0, None, 0, None, None, 0, 0, 0, 0, None, None, 0, None) == 0
    # a split contraction without workspace is refused
    t = L.mp8_gemm_fp8_tuned
    assert t(2, 16384, 4096, 1024, one, 16384, one, 16384, 1.0, None, 0, one, None, 0, 0, 0, 0, None,
             None, 0, None, 1, 4) == 4


def test_workspace_query_is_consistent():
    # the query is an upper bound for any options: one FP32 tile set per contraction slice
    assert mp8.gemm_fp8_workspace_bytes(mp8.FWD, 4096, 4096, 4096) == 4096 * 4096 * 4
    for (op, M, N, K) in [(mp8.WGRAD, 25088, 128, 1152), (mp8.WGRAD, 16384, 4096, 1024),
                          (mp8.FWD, 128, 4096, 2048), (mp8.BWD_DATA, 128, 4096, 2048)]:
        rows, cols, kc = {0: (M, N, K), 1: (M, K, N), 2: (K, N, M)}[op]
        auto = mp8.gemm_fp8_workspace_bytes(op, M, N, K)
        assert auto % (rows * cols * 4) == 0
        for s in (2, 3, 8):
            assert mp8.gemm_fp8_workspace_bytes(op, M, N, K, 1, s) == s * rows * cols * 4
    assert len(mp8.gemm_tile_configs()) == mp8.lib().mp8_gemm_num_tile_configs() >= 4
    assert mp8.gemm_fp8_workspace_bytes(mp8.FWD, 100, 100, 100) == 0   # generic kernel
