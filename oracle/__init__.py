"""ctypes front end of the CPU oracle (``mp8_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``.  It knows nothing about the HIP library and
the HIP library knows nothing about it.  All arrays are host numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mp8_oracle.c")
_LIB = os.path.join(_HERE, "libmp8_oracle.so")

RNE, SR = 0, 1
FLAG_SATURATE = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no contraction); returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Stats(C.Structure):
    _fields_ = [("amax_bits", C.c_uint32), ("nonfinite", C.c_uint32),
                ("zeroed", C.c_uint32), ("rsvd", C.c_uint32)]

    def as_tuple(self):
        return (self.amax_bits, self.nonfinite, self.zeroed)


class Scaler(C.Structure):
    _fields_ = [("scale", C.c_double), ("floor", C.c_double),
                ("growth_interval", C.c_int64), ("good_steps", C.c_int64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_e5m2_decode.restype = C.c_double
        L.orc_e5m2_decode.argtypes = [C.c_uint8]
        L.orc_fp16_decode.restype = C.c_double
        L.orc_fp16_decode.argtypes = [C.c_uint16]
        L.orc_e5m2_encode.restype = C.c_uint8
        L.orc_e5m2_encode.argtypes = [C.c_double, C.c_int, C.c_uint32, C.c_int]
        L.orc_fp16_encode.restype = C.c_uint16
        L.orc_fp16_encode.argtypes = [C.c_double, C.c_int, C.c_uint32]
        L.orc_philox4x32_10.restype = None
        L.orc_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_sr_bits.restype = C.c_uint32
        L.orc_sr_bits.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
        L.orc_quantize_e5m2.restype = None
        L.orc_quantize_e5m2.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int64,
                                        C.c_int64, C.c_float, C.c_int, C.c_int, C.c_uint64,
                                        C.c_uint64, C.c_void_p]
        L.orc_fp16_encode_array.restype = None
        L.orc_fp16_encode_array.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_uint64,
                                            C.c_void_p]
        L.orc_gemm_ref.restype = None
        L.orc_gemm_ref.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int64,
                                   C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                   C.c_void_p]
        for fn in (L.orc_conv3x3_fwd_ref, L.orc_conv3x3_bwd_data_ref, L.orc_conv3x3_wgrad_ref):
            fn.restype = None
            fn.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int64] * 5 + [C.c_void_p, C.c_void_p]
        L.orc_gemm_exact.restype = C.c_int64
        L.orc_gemm_exact.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int64,
                                     C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.orc_round_ref_e5m2.restype = None
        L.orc_round_ref_e5m2.argtypes = [C.c_void_p, C.c_int64, C.c_double, C.c_int, C.c_void_p]
        L.orc_sgd_update_fp16.restype = None
        L.orc_sgd_update_fp16.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_float,
                                          C.c_int, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p,
                                          C.c_void_p]
        L.orc_sgd_momentum_fp16.restype = None
        L.orc_sgd_momentum_fp16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float,
                                            C.c_float, C.c_float, C.c_float, C.c_int, C.c_uint64,
                                            C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_adam_fp16.restype = None
        L.orc_adam_fp16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float,
                                    C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_int64,
                                    C.c_int, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_scaler_update.restype = C.c_int
        L.orc_scaler_update.argtypes = [C.POINTER(Scaler), C.c_uint32]
        L.orc_scaler_set_floor.restype = None
        L.orc_scaler_set_floor.argtypes = [C.POINTER(Scaler), C.c_double]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _carr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# --- scalar helpers -------------------------------------------------------------------

def e5m2_decode(code: int) -> float:
    return lib().orc_e5m2_decode(int(code) & 0xFF)


def fp16_decode(code: int) -> float:
    return lib().orc_fp16_decode(int(code) & 0xFFFF)


def e5m2_encode(y: float, mode: int = RNE, r16: int = 0, saturate: bool = False) -> int:
    return lib().orc_e5m2_encode(float(y), mode, r16, int(saturate))


def fp16_encode(y: float, mode: int = RNE, r16: int = 0) -> int:
    return lib().orc_fp16_encode(float(y), mode, r16)


def e5m2_decode_table() -> np.ndarray:
    return np.array([e5m2_decode(c) for c in range(256)], dtype=np.float64)


def philox4x32_10(ctr, key) -> np.ndarray:
    c = _carr(ctr, np.uint32)
    k = _carr(key, np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sr_bits(seed: int, offset: int, i: int) -> int:
    return lib().orc_sr_bits(seed, offset, i)


# --- tensor operations -----------------------------------------------------------------

def quantize_e5m2(src, scale=1.0, mode=RNE, flags=0, seed=0, offset=0, want_t=False,
                  stats: Stats | None = None):
    """Q(fl32(src*scale)) for a 2-D FP32 (or float16) array -> (codes, codes_t or None)."""
    src = np.ascontiguousarray(src)
    assert src.ndim == 2 and src.dtype in (np.float32, np.float16)
    rows, cols = src.shape
    dst = np.empty((rows, cols), dtype=np.uint8)
    dst_t = np.empty((cols, rows), dtype=np.uint8) if want_t else None
    lib().orc_quantize_e5m2(_p(src), int(src.dtype == np.float16), _p(dst), _p(dst_t), rows, cols,
                            float(scale), mode, flags, seed, offset,
                            C.byref(stats) if stats is not None else None)
    return dst, dst_t


def fp16_encode_array(src, mode=RNE, seed=0, offset=0):
    src = _carr(src, np.float32).reshape(-1)
    out = np.empty(src.size, dtype=np.uint16)
    lib().orc_fp16_encode_array(_p(src), src.size, mode, seed, offset, _p(out))
    return out


def gemm_ref(a, b, row_idx=None, want_abs=True):
    """ref[r,c] = sum_j a[r,j]*b[c,j] in double; a:[rows,kc] b:[cols,kc] uint8 E5M2 codes.

    Strided 2-D views with a contiguous last axis are accepted (leading dim = stride)."""
    assert a.dtype == np.uint8 and b.dtype == np.uint8 and a.ndim == 2 and b.ndim == 2
    assert a.strides[1] == 1 and b.strides[1] == 1 and a.shape[1] == b.shape[1]
    rows, kc = a.shape
    cols = b.shape[0]
    idx = None
    nrows = rows
    if row_idx is not None:
        idx = _carr(row_idx, np.int64)
        nrows = idx.size
    ref = np.empty((nrows, cols), dtype=np.float64)
    absref = np.empty((nrows, cols), dtype=np.float64) if want_abs else None
    lib().orc_gemm_ref(_p(a), a.strides[0], _p(b), b.strides[0], rows, cols, kc, _p(idx),
                       nrows if idx is not None else 0, _p(ref), _p(absref))
    return ref, absref


def conv3x3_ref(op, a, b, want_abs=True):
    """Double-precision 3x3 convolution (stride 1, zero padding 1, channels last) on E5M2 codes.

    op 'fwd':      a = x [B,H,W,Ci], b = w [3,3,Ci,Co]   -> y  [B,H,W,Co]
    op 'bwd_data': a = e [B,H,W,Co], b = w [3,3,Ci,Co]   -> dx [B,H,W,Ci]
    op 'wgrad':    a = x [B,H,W,Ci], b = e [B,H,W,Co]    -> dw [3,3,Ci,Co]
    Returns (ref, absref or None)."""
    a = _carr(a, np.uint8)
    b = _carr(b, np.uint8)
    if op == "fwd":
        B, H, W, Ci = a.shape
        Co = b.shape[3]
        shape, fn = (B, H, W, Co), lib().orc_conv3x3_fwd_ref
        assert b.shape == (3, 3, Ci, Co)
    elif op == "bwd_data":
        B, H, W, Co = a.shape
        Ci = b.shape[2]
        shape, fn = (B, H, W, Ci), lib().orc_conv3x3_bwd_data_ref
        assert b.shape == (3, 3, Ci, Co)
    else:
        B, H, W, Ci = a.shape
        Co = b.shape[3]
        shape, fn = (3, 3, Ci, Co), lib().orc_conv3x3_wgrad_ref
        assert b.shape == (B, H, W, Co)
    ref = np.empty(shape, dtype=np.float64)
    absref = np.empty(shape, dtype=np.float64) if want_abs else None
    fn(_p(a), _p(b), B, H, W, Ci, Co, _p(ref), _p(absref))
    return ref, absref


def gemm_exact(a, b):
    """Exact integer dot products (python ints, units of 2**-32) for tiny finite inputs."""
    a = _carr(a, np.uint8)
    b = _carr(b, np.uint8)
    rows, kc = a.shape
    cols = b.shape[0]
    hi = np.empty((rows, cols), dtype=np.int64)
    lo = np.empty((rows, cols), dtype=np.uint64)
    bad = lib().orc_gemm_exact(_p(a), kc, _p(b), kc, rows, cols, kc, _p(hi), _p(lo))
    out = [[(int(hi[r, c]) << 64) + int(lo[r, c]) for c in range(cols)] for r in range(rows)]
    return out, bad


def round_ref_e5m2(ref, alpha=1.0, flags=0):
    ref = _carr(ref, np.float64)
    out = np.empty(ref.shape, dtype=np.uint8)
    lib().orc_round_ref_e5m2(_p(ref), ref.size, float(alpha), flags, _p(out))
    return out


def sgd_update_fp16(w16, g8, lr, inv_loss_scale, mode=SR, seed=0, offset=0, skip=None,
                    want_w8=False, stats: Stats | None = None):
    """Returns (new_w16, w8 or None); inputs are not modified."""
    w = np.array(w16, dtype=np.uint16, copy=True).reshape(-1)
    g = _carr(g8, np.uint8).reshape(-1)
    assert w.size == g.size
    w8 = np.zeros(w.size, dtype=np.uint8) if want_w8 else None
    sk = None
    if skip is not None:
        sk = np.array([skip], dtype=np.uint32)
    lib().orc_sgd_update_fp16(_p(w), _p(g), w.size, float(lr), float(inv_loss_scale), mode, seed,
                              offset, _p(sk), _p(w8),
                              C.byref(stats) if stats is not None else None)
    return w, w8


def sgd_momentum_fp16(w16, vel, g8, lr, inv_loss_scale, momentum, weight_decay=0.0, mode=SR, seed=0,
                      offset=0, skip=None, want_w8=False, stats: Stats | None = None):
    """Momentum SGD with L2 regularisation on half master weights and an FP32 velocity.
    Returns (new_w16, new_vel, w8 or None); inputs are not modified."""
    w = np.array(w16, dtype=np.uint16, copy=True).reshape(-1)
    v = np.array(vel, dtype=np.float32, copy=True).reshape(-1)
    g = _carr(g8, np.uint8).reshape(-1)
    assert w.size == g.size == v.size
    w8 = np.zeros(w.size, dtype=np.uint8) if want_w8 else None
    sk = None if skip is None else np.array([skip], dtype=np.uint32)
    lib().orc_sgd_momentum_fp16(_p(w), _p(v), _p(g), w.size, float(lr), float(inv_loss_scale),
                                float(momentum), float(weight_decay), mode, seed, offset, _p(sk),
                                _p(w8), C.byref(stats) if stats is not None else None)
    return w, v, w8


def adam_fp16(w16, m, v, g8, lr, inv_loss_scale, step, beta1=0.9, beta2=0.999, eps=1e-8,
              weight_decay=0.0, mode=SR, seed=0, offset=0, skip=None, want_w8=False,
              stats: Stats | None = None):
    """ADAM with L2 regularisation on half master weights and FP32 moments (step counts from 1).
    Returns (new_w16, new_m, new_v, w8 or None); inputs are not modified."""
    w = np.array(w16, dtype=np.uint16, copy=True).reshape(-1)
    m_ = np.array(m, dtype=np.float32, copy=True).reshape(-1)
    v_ = np.array(v, dtype=np.float32, copy=True).reshape(-1)
    g = _carr(g8, np.uint8).reshape(-1)
    assert w.size == g.size == m_.size == v_.size and step >= 1
    w8 = np.zeros(w.size, dtype=np.uint8) if want_w8 else None
    sk = None if skip is None else np.array([skip], dtype=np.uint32)
    lib().orc_adam_fp16(_p(w), _p(m_), _p(v_), _p(g), w.size, float(lr), float(inv_loss_scale),
                        float(beta1), float(beta2), float(eps), float(weight_decay), int(step), mode,
                        seed, offset, _p(sk), _p(w8), C.byref(stats) if stats is not None else None)
    return w, m_, v_, w8


def scaler_new(scale, floor, growth_interval) -> Scaler:
    return Scaler(float(scale), float(floor), int(growth_interval), 0)


def scaler_update(s: Scaler, nonfinite: int) -> int:
    return lib().orc_scaler_update(C.byref(s), int(nonfinite))


def scaler_set_floor(s: Scaler, floor: float) -> None:
    lib().orc_scaler_set_floor(C.byref(s), float(floor))
