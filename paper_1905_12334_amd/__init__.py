"""Python binding of libmp8.so -- the MI355X-native 8-bit floating point training primitive
(arXiv 1905.12334): ``quantize_e5m2``, ``gemm_fp8`` and ``sgd_update_fp16_sr``.

Argument marshalling only: every function takes torch tensors that already live on the GPU,
passes their ``data_ptr()`` and the current HIP stream through the C ABI declared in
``include/mp8.h`` and returns without synchronising.  There is no CPU fallback: if the HIP
library has not been built, loading it raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# MP8_LIB_PATH: another build of the same library (tuning experiments); default: the in-tree build
LIB_PATH = os.environ.get("MP8_LIB_PATH") or os.path.join(_HERE, "libmp8.so")

RNE, SR = 0, 1
FWD, BWD_DATA, WGRAD = 0, 1, 2
FLAG_SATURATE = 1
FLAG_A_CONTRACTION_MAJOR = 2
FLAG_B_CONTRACTION_MAJOR = 4
FLAG_CONTRACTION_MAJOR = 6

EXPORTS = [
    "mp8_quantize_e5m2", "mp8_gemm_fp8", "mp8_gemm_fp8_workspace_bytes", "mp8_gemm_fp8_tuned",
    "mp8_gemm_fp8_workspace_bytes_tuned", "mp8_gemm_num_tile_configs",
    "mp8_gemm_tile_config_name", "mp8_sgd_update_fp16_sr", "mp8_sr_bits", "mp8_philox4x32_10",
    "mp8_scaler_init", "mp8_scaler_update", "mp8_scaler_set_floor", "mp8_status_string",
    "mp8_conv3x3_fp8", "mp8_conv3x3_fp8_workspace_bytes", "mp8_sgd_momentum_fp16_sr",
    "mp8_gemm_fp8_plan", "mp8_gemm_tile_config_lds_bytes", "mp8_adam_fp16_sr",
    "mp8_quantize_e5m2_batch", "mp8_wgrad_update_fp16_sr", "mp8_conv3x3_wgrad_update_fp16_sr",
    "mp8_quantize_gemm_fwd_fp8", "mp8_wgrad_momentum_fp16_sr", "mp8_conv3x3_wgrad_momentum_fp16_sr",
    "mp8_wgrad_adam_fp16_sr", "mp8_gemm_fp8_static", "mp8_static_scratch_bytes",
    "mp8_stream_probe",
]


class Mp8Error(RuntimeError):
    pass


class Scaler(C.Structure):
    """mp8_scaler: host-side dynamic loss scaler with a minimum threshold."""
    _fields_ = [("scale", C.c_double), ("floor", C.c_double),
                ("growth_interval", C.c_int64), ("good_steps", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    """Load libmp8.so (built in-tree by ``build.py``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise Mp8Error(f"{LIB_PATH} not found: build it with `python -m paper_1905_12334_amd.build` "
                       "(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(LIB_PATH)
    i64, u64, vp, f32, ci = C.c_int64, C.c_uint64, C.c_void_p, C.c_float, C.c_int
    L.mp8_quantize_e5m2.restype = ci
    L.mp8_quantize_e5m2.argtypes = [vp, ci, vp, vp, i64, i64, f32, ci, ci, u64, u64, vp, vp]
    gemm_args = [ci, i64, i64, i64, vp, i64, vp, i64, f32, vp, ci, vp, vp, ci, ci, u64, u64, vp,
                 vp, C.c_size_t, vp]
    L.mp8_gemm_fp8.restype = ci
    L.mp8_gemm_fp8.argtypes = gemm_args
    L.mp8_gemm_fp8_tuned.restype = ci
    L.mp8_gemm_fp8_tuned.argtypes = gemm_args + [ci, ci]
    L.mp8_gemm_fp8_static.restype = ci
    L.mp8_gemm_fp8_static.argtypes = gemm_args[:-3] + [vp]
    L.mp8_static_scratch_bytes.restype = C.c_size_t
    L.mp8_static_scratch_bytes.argtypes = []
    L.mp8_gemm_fp8_workspace_bytes.restype = C.c_size_t
    L.mp8_gemm_fp8_workspace_bytes.argtypes = [ci, i64, i64, i64]
    L.mp8_gemm_fp8_workspace_bytes_tuned.restype = C.c_size_t
    L.mp8_gemm_fp8_workspace_bytes_tuned.argtypes = [ci, i64, i64, i64, ci, ci]
    L.mp8_gemm_fp8_plan.restype = ci
    L.mp8_gemm_fp8_plan.argtypes = [ci, i64, i64, i64, ci, ci, ci, C.POINTER(ci), C.POINTER(ci)]
    L.mp8_gemm_num_tile_configs.restype = ci
    L.mp8_gemm_num_tile_configs.argtypes = []
    L.mp8_gemm_tile_config_name.restype = ci
    L.mp8_gemm_tile_config_name.argtypes = [ci, C.c_char_p, C.c_size_t]
    L.mp8_gemm_tile_config_lds_bytes.restype = ci
    L.mp8_gemm_tile_config_lds_bytes.argtypes = [ci, ci]
    L.mp8_sgd_update_fp16_sr.restype = ci
    L.mp8_sgd_update_fp16_sr.argtypes = [vp, vp, i64, f32, f32, ci, u64, u64, vp, vp, vp, vp]
    L.mp8_sgd_momentum_fp16_sr.restype = ci
    L.mp8_sgd_momentum_fp16_sr.argtypes = [vp, vp, vp, i64, f32, f32, f32, f32, ci, u64, u64, vp, vp, vp, vp]
    L.mp8_wgrad_update_fp16_sr.restype = ci
    L.mp8_wgrad_update_fp16_sr.argtypes = [i64, i64, i64, vp, i64, vp, i64, f32, vp, ci, ci, u64, u64, vp,
                                           vp, f32, f32, ci, u64, u64, vp, vp, vp, C.c_size_t, vp]
    L.mp8_conv3x3_wgrad_update_fp16_sr.restype = ci
    L.mp8_conv3x3_wgrad_update_fp16_sr.argtypes = [i64, i64, i64, i64, i64, i64, vp, vp, f32, vp, ci, ci, u64,
                                                   u64, vp, vp, f32, f32, ci, u64, u64, vp, vp, vp,
                                                   C.c_size_t, vp]
    L.mp8_wgrad_momentum_fp16_sr.restype = ci
    L.mp8_wgrad_momentum_fp16_sr.argtypes = [i64, i64, i64, vp, i64, vp, i64, f32, vp, ci, ci, u64, u64, vp,
                                             vp, vp, f32, f32, f32, f32, ci, u64, u64, vp, vp, vp, C.c_size_t,
                                             vp]
    L.mp8_wgrad_adam_fp16_sr.restype = ci
    L.mp8_wgrad_adam_fp16_sr.argtypes = [i64, i64, i64, vp, i64, vp, i64, f32, vp, ci, ci, u64, u64, vp,
                                         vp, vp, vp, f32, f32, f32, f32, f32, f32, i64, ci, u64, u64, vp, vp, vp,
                                         C.c_size_t, vp]
    L.mp8_conv3x3_wgrad_momentum_fp16_sr.restype = ci
    L.mp8_conv3x3_wgrad_momentum_fp16_sr.argtypes = [i64, i64, i64, i64, i64, i64, vp, vp, f32, vp, ci, ci, u64,
                                                     u64, vp, vp, vp, f32, f32, f32, f32, ci, u64, u64, vp, vp,
                                                     vp, C.c_size_t, vp]
    L.mp8_quantize_gemm_fwd_fp8.restype = ci
    L.mp8_quantize_gemm_fwd_fp8.argtypes = [i64, i64, i64, vp, f32, ci, ci, u64, u64, vp, vp, vp, i64, f32,
                                            vp, ci, vp, vp, ci, ci, u64, u64, vp, vp, C.c_size_t, vp]
    L.mp8_quantize_e5m2_batch.restype = ci
    L.mp8_quantize_e5m2_batch.argtypes = [vp, ci, vp]
    L.mp8_adam_fp16_sr.restype = ci
    L.mp8_adam_fp16_sr.argtypes = [vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, f32, i64, ci, u64, u64,
                                   vp, vp, vp, vp]
    L.mp8_stream_probe.restype = ci
    L.mp8_stream_probe.argtypes = [vp, vp, i64, ci, vp]
    L.mp8_sr_bits.restype = ci
    L.mp8_sr_bits.argtypes = [vp, i64, u64, u64, vp]
    L.mp8_philox4x32_10.restype = None
    L.mp8_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                    C.POINTER(C.c_uint32)]
    L.mp8_scaler_init.restype = None
    L.mp8_scaler_init.argtypes = [C.POINTER(Scaler), C.c_double, C.c_double, i64]
    L.mp8_scaler_update.restype = ci
    L.mp8_scaler_update.argtypes = [C.POINTER(Scaler), C.c_uint32]
    L.mp8_scaler_set_floor.restype = None
    L.mp8_scaler_set_floor.argtypes = [C.POINTER(Scaler), C.c_double]
    L.mp8_conv3x3_fp8.restype = ci
    L.mp8_conv3x3_fp8.argtypes = [ci, i64, i64, i64, i64, i64, i64, vp, vp, f32, vp, ci, vp, ci, ci,
                                  u64, u64, vp, vp, C.c_size_t, vp]
    L.mp8_conv3x3_fp8_workspace_bytes.restype = C.c_size_t
    L.mp8_conv3x3_fp8_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, i64, i64]
    L.mp8_status_string.restype = C.c_char_p
    L.mp8_status_string.argtypes = [ci]
    _lib = L
    return L


def _check(status: int, what: str) -> None:
    if status != 0:
        raise Mp8Error(f"{what}: {lib().mp8_status_string(status).decode()} (status {status})")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, name, dtype=None):
    if t is None:
        return
    if not t.is_cuda:
        raise Mp8Error(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise Mp8Error(f"{name} must be contiguous")
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise Mp8Error(f"{name} has dtype {t.dtype}, expected {dtype}")


def stream_probe(src, dst, reads_per_write):
    """mp8_stream_probe: read all of src, write 1/reads_per_write as many bytes to dst (diagnostic)."""
    _dev(src, "src")
    _dev(dst, "dst")
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes // reads_per_write:
        raise Mp8Error("dst is too small")
    _check(lib().mp8_stream_probe(_ptr(src), _ptr(dst), nbytes, reads_per_write, _stream()), "mp8_stream_probe")


def new_stats(device="cuda"):
    """A zeroed mp8_stats on the device: uint32 [amax_bits, nonfinite, zeroed, rsvd] as int32."""
    import torch
    return torch.zeros(4, dtype=torch.int32, device=device)


def read_stats(stats):
    """(amax_bits, nonfinite, zeroed) as python ints (synchronises)."""
    v = [int(x) & 0xFFFFFFFF for x in stats.cpu().tolist()]
    return v[0], v[1], v[2]


def quantize_e5m2(src, dst, dst_t=None, scale=1.0, round=RNE, flags=0, seed=0, offset=0,
                  stats=None):
    """mp8_quantize_e5m2: dst = Q(fl32(src*scale)); src [rows, cols] float32/float16."""
    import torch
    _dev(src, "src", (torch.float32, torch.float16))
    _dev(dst, "dst", torch.uint8)
    _dev(dst_t, "dst_t", torch.uint8)
    if src.dim() != 2:
        raise Mp8Error("src must be 2-D")
    rows, cols = src.shape
    if dst.numel() != rows * cols or (dst_t is not None and dst_t.numel() != rows * cols):
        raise Mp8Error("dst / dst_t size does not match src")
    st = lib().mp8_quantize_e5m2(_ptr(src), int(src.dtype == torch.float16), _ptr(dst), _ptr(dst_t),
                                 rows, cols, float(scale), round, flags, seed, offset,
                                 _ptr(stats), _stream())
    _check(st, "mp8_quantize_e5m2")
    return dst


QUANTIZE_BATCH_MAX = 8


class _QuantizeItem(C.Structure):
    _fields_ = [("src", C.c_void_p), ("src_is_f16", C.c_int), ("dst", C.c_void_p), ("n", C.c_int64),
                ("scale", C.c_float), ("round", C.c_int), ("flags", C.c_int), ("seed", C.c_uint64),
                ("offset", C.c_uint64), ("stats", C.c_void_p)]


def quantize_e5m2_batch(items):
    """mp8_quantize_e5m2_batch: several flat Q nodes in one launch.  `items` is a sequence of
    dicts with keys src, dst and optionally scale, round, flags, seed, offset, stats (as the
    arguments of quantize_e5m2; tensors of any shape are taken flat, no transposed copy)."""
    import torch
    arr = (_QuantizeItem * max(len(items), 1))()
    for i, it in enumerate(items):
        src, dst = it["src"], it["dst"]
        _dev(src, "src", (torch.float32, torch.float16))
        _dev(dst, "dst", torch.uint8)
        if dst.numel() != src.numel():
            raise Mp8Error("dst size does not match src")
        stats = it.get("stats")
        arr[i] = _QuantizeItem(src.data_ptr(), int(src.dtype == torch.float16), dst.data_ptr(), src.numel(),
                               float(it.get("scale", 1.0)), it.get("round", RNE), it.get("flags", 0),
                               it.get("seed", 0), it.get("offset", 0),
                               None if stats is None else stats.data_ptr())
    _check(lib().mp8_quantize_e5m2_batch(arr, len(items), _stream()), "mp8_quantize_e5m2_batch")


def _op_dims(op, M, N, K):
    return {FWD: (M, N, K), BWD_DATA: (M, K, N), WGRAD: (K, N, M)}[op]


def gemm_fp8_workspace_bytes(op, M, N, K, tile_config=0, split_k=0) -> int:
    return int(lib().mp8_gemm_fp8_workspace_bytes_tuned(op, M, N, K, tile_config, split_k))


def gemm_fp8(op, M, N, K, a, b, out8=None, out8_t=None, acc=None, acc_mode=0, alpha=1.0,
             round=RNE, flags=0, seed=0, offset=0, stats=None, workspace=None, lda=None,
             ldb=None, tile_config=0, split_k=0, static_scratch=False):
    """mp8_gemm_fp8(_tuned): out[r,c] = sum_j a[r,j]*b[c,j] with the operand orientation of
    include/mp8.h.  All tensors are caller-allocated GPU tensors; workspace is a uint8/any
    tensor of at least gemm_fp8_workspace_bytes(...) bytes when that is non-zero."""
    import torch
    _dev(a, "a", torch.uint8)
    _dev(b, "b", torch.uint8)
    _dev(out8, "out8", torch.uint8)
    _dev(out8_t, "out8_t", torch.uint8)
    _dev(acc, "acc", torch.float32)
    rows, cols, kc = _op_dims(op, M, N, K)
    a_km, b_km = bool(flags & FLAG_A_CONTRACTION_MAJOR), bool(flags & FLAG_B_CONTRACTION_MAJOR)
    if lda is None:
        lda = rows if a_km else kc
    if ldb is None:
        ldb = cols if b_km else kc
    need_a = ((kc - 1) * lda + rows if a_km else (rows - 1) * lda + kc) if rows > 0 and kc > 0 else 0
    need_b = ((kc - 1) * ldb + cols if b_km else (cols - 1) * ldb + kc) if cols > 0 and kc > 0 else 0
    if a.numel() < need_a:
        raise Mp8Error("a is smaller than its shape and leading dimension require")
    if b.numel() < need_b:
        raise Mp8Error("b is smaller than its shape and leading dimension require")
    for t, name in ((out8, "out8"), (out8_t, "out8_t"), (acc, "acc")):
        if t is not None and t.numel() < rows * cols:
            raise Mp8Error(f"{name} is smaller than rows*cols")
    if static_scratch:
        if workspace is not None or tile_config or split_k:
            raise Mp8Error("static_scratch takes no workspace, tile_config or split_k")
        st = lib().mp8_gemm_fp8_static(op, M, N, K, _ptr(a), lda, _ptr(b), ldb, float(alpha), _ptr(acc),
                                       acc_mode, _ptr(out8), _ptr(out8_t), round, flags, seed, offset,
                                       _ptr(stats), _stream())
        _check(st, "mp8_gemm_fp8_static")
        return out8
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_gemm_fp8_tuned(op, M, N, K, _ptr(a), lda, _ptr(b), ldb, float(alpha), _ptr(acc),
                                  acc_mode, _ptr(out8), _ptr(out8_t), round, flags, seed, offset,
                                  _ptr(stats), _ptr(workspace), ws_bytes, _stream(), tile_config,
                                  split_k)
    _check(st, "mp8_gemm_fp8")
    return out8


def gemm_fp8_static(op, M, N, K, a, b, **kw):
    """mp8_gemm_fp8_static: gemm_fp8 with the library's own static scratch (allocates nothing)."""
    return gemm_fp8(op, M, N, K, a, b, static_scratch=True, **kw)


def static_scratch_bytes() -> int:
    return int(lib().mp8_static_scratch_bytes())


def quantize_gemm_fwd_fp8(M, N, K, x, x8_out, w8, out8=None, out8_t=None, acc=None, acc_mode=0,
                          x_scale=1.0, x_round=RNE, x_flags=0, x_seed=0, x_offset=0, x_stats=None,
                          alpha=1.0, round=RNE, flags=0, seed=0, offset=0, stats=None, workspace=None,
                          ldw=None):
    """mp8_quantize_gemm_fwd_fp8: x8_out = Q(x * x_scale) [M, K] and out = x8_out . w8 [K, N] in one
    call (one kernel when N <= 128)."""
    import torch
    _dev(x, "x", torch.float32)
    _dev(x8_out, "x8_out", torch.uint8)
    _dev(w8, "w8", torch.uint8)
    _dev(out8, "out8", torch.uint8)
    _dev(out8_t, "out8_t", torch.uint8)
    _dev(acc, "acc", torch.float32)
    ldw = N if ldw is None else ldw
    if x.numel() != M * K or x8_out.numel() != M * K:
        raise Mp8Error("x and x8_out must have M*K elements")
    if K > 0 and N > 0 and w8.numel() < (K - 1) * ldw + N:
        raise Mp8Error("w8 is smaller than its shape and leading dimension require")
    for t, name in ((out8, "out8"), (out8_t, "out8_t"), (acc, "acc")):
        if t is not None and t.numel() < M * N:
            raise Mp8Error(f"{name} is smaller than M*N")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_quantize_gemm_fwd_fp8(M, N, K, _ptr(x), float(x_scale), x_round, x_flags, x_seed,
                                         x_offset, _ptr(x_stats), _ptr(x8_out), _ptr(w8), ldw,
                                         float(alpha), _ptr(acc), acc_mode, _ptr(out8), _ptr(out8_t),
                                         round, flags, seed, offset, _ptr(stats), _ptr(workspace),
                                         ws_bytes, _stream())
    _check(st, "mp8_quantize_gemm_fwd_fp8")
    return out8


def conv_prows(B, H, W) -> int:
    """Rows of a padded channels-last tensor: B*(H+2)*(W+2) rounded up to a multiple of 128."""
    return -(-(B * (H + 2) * (W + 2)) // 128) * 128


def conv_buffer(prows, channels, W, dtype=None, device="cuda"):
    """A zeroed [prows, channels] tensor for mp8_conv3x3_fp8 with the W+3 guard rows it wants
    readable before and after (the returned view starts behind the leading guard)."""
    import torch
    guard = (W + 3) * channels
    store = torch.zeros(prows * channels + 2 * guard, dtype=dtype or torch.uint8, device=device)
    return store[guard:guard + prows * channels].view(prows, channels)


def _has_guard(t, guard_elems):
    after = t.untyped_storage().nbytes() // t.element_size() - (t.storage_offset() + t.numel())
    return t.storage_offset() >= guard_elems and after >= guard_elems


def conv3x3_fp8_workspace_bytes(op, B, H, W, Cin, Cout, prows=None) -> int:
    prows = conv_prows(B, H, W) if prows is None else prows
    return int(lib().mp8_conv3x3_fp8_workspace_bytes(op, B, H, W, Cin, Cout, prows))


def conv3x3_fp8(op, B, H, W, Cin, Cout, a, b, out8=None, acc=None, acc_mode=0, alpha=1.0, round=RNE,
                flags=0, seed=0, offset=0, stats=None, workspace=None, prows=None):
    """mp8_conv3x3_fp8 on padded channels-last tensors (see include/mp8.h): a / b are
    [prows, C] views with guard rows around them (conv_buffer), weights are [3, 3, Cin, Cout]."""
    import torch
    prows = conv_prows(B, H, W) if prows is None else prows
    _dev(a, "a", torch.uint8)
    _dev(b, "b", torch.uint8)
    _dev(out8, "out8", torch.uint8)
    _dev(acc, "acc", torch.float32)
    ca = Cout if op == BWD_DATA else Cin
    shapes = {FWD: (prows * Cin, 9 * Cin * Cout, prows * Cout),
              BWD_DATA: (prows * Cout, 9 * Cin * Cout, prows * Cin),
              WGRAD: (prows * Cin, prows * Cout, 9 * Cin * Cout)}[op]
    if a.numel() != shapes[0] or b.numel() != shapes[1]:
        raise Mp8Error("a / b do not have the sizes the operation implies")
    for t, name in ((out8, "out8"), (acc, "acc")):
        if t is not None and t.numel() < shapes[2]:
            raise Mp8Error(f"{name} is smaller than the output")
    if not _has_guard(a, (W + 3) * ca):
        raise Mp8Error("the padded tensor `a` needs W+3 readable guard rows before and after "
                       "(allocate it with conv_buffer)")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_conv3x3_fp8(op, B, H, W, Cin, Cout, prows, _ptr(a), _ptr(b), float(alpha), _ptr(acc),
                               acc_mode, _ptr(out8), round, flags, seed, offset, _ptr(stats),
                               _ptr(workspace), ws_bytes, _stream())
    _check(st, "mp8_conv3x3_fp8")
    return out8


def conv3x3_wgrad_update_fp16_sr(B, H, W, Cin, Cout, x8, e8, w16, lr, inv_loss_scale, g8_out=None, alpha=1.0,
                                 g_round=RNE, flags=0, g_seed=0, g_offset=0, stats=None, w_round=SR, w_seed=0,
                                 w_offset=0, skip_if_nonzero=None, w8_out=None, workspace=None, prows=None):
    """mp8_conv3x3_wgrad_update_fp16_sr: weight gradient of the 3x3 convolution, its rounding to
    8 bits and the update of the FP16 master weights w16 [3, 3, Cin, Cout] in one call."""
    import torch
    prows = conv_prows(B, H, W) if prows is None else prows
    _dev(x8, "x8", torch.uint8)
    _dev(e8, "e8", torch.uint8)
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(g8_out, "g8_out", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    if x8.numel() != prows * Cin or e8.numel() != prows * Cout:
        raise Mp8Error("x8 / e8 do not have the sizes the operation implies")
    for t, name in ((w16, "w16"), (g8_out, "g8_out"), (w8_out, "w8_out")):
        if t is not None and t.numel() != 9 * Cin * Cout:
            raise Mp8Error(f"{name} must have 9*Cin*Cout elements")
    if not _has_guard(x8, (W + 3) * Cin):
        raise Mp8Error("the padded tensor x8 needs W+3 readable guard rows before and after "
                       "(allocate it with conv_buffer)")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_conv3x3_wgrad_update_fp16_sr(B, H, W, Cin, Cout, prows, _ptr(x8), _ptr(e8), float(alpha),
                                                _ptr(g8_out), g_round, flags, g_seed, g_offset, _ptr(stats),
                                                _ptr(w16), float(lr), float(inv_loss_scale), w_round, w_seed,
                                                w_offset, _ptr(skip_if_nonzero), _ptr(w8_out), _ptr(workspace),
                                                ws_bytes, _stream())
    _check(st, "mp8_conv3x3_wgrad_update_fp16_sr")
    return w16


def wgrad_momentum_fp16_sr(M, N, K, a, b, w16, velocity, lr, inv_loss_scale, momentum, weight_decay=0.0,
                           g8_out=None, alpha=1.0, g_round=RNE, flags=0, g_seed=0, g_offset=0, stats=None,
                           w_round=SR, w_seed=0, w_offset=0, skip_if_nonzero=None, w8_out=None,
                           workspace=None, lda=None, ldb=None):
    """mp8_wgrad_momentum_fp16_sr: wgrad_update_fp16_sr with the momentum optimizer (velocity [K, N]
    FP32 in place) in the finishing pass."""
    import torch
    _dev(a, "a", torch.uint8)
    _dev(b, "b", torch.uint8)
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(velocity, "velocity", torch.float32)
    _dev(g8_out, "g8_out", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    rows, cols, kc = _op_dims(WGRAD, M, N, K)
    a_km, b_km = bool(flags & FLAG_A_CONTRACTION_MAJOR), bool(flags & FLAG_B_CONTRACTION_MAJOR)
    lda = (rows if a_km else kc) if lda is None else lda
    ldb = (cols if b_km else kc) if ldb is None else ldb
    need_a = ((kc - 1) * lda + rows if a_km else (rows - 1) * lda + kc) if rows > 0 and kc > 0 else 0
    need_b = ((kc - 1) * ldb + cols if b_km else (cols - 1) * ldb + kc) if cols > 0 and kc > 0 else 0
    if a.numel() < need_a or b.numel() < need_b:
        raise Mp8Error("a / b is smaller than its shape and leading dimension require")
    for t, name in ((w16, "w16"), (velocity, "velocity"), (g8_out, "g8_out"), (w8_out, "w8_out")):
        if t is not None and t.numel() != rows * cols:
            raise Mp8Error(f"{name} must have K*N elements")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_wgrad_momentum_fp16_sr(M, N, K, _ptr(a), lda, _ptr(b), ldb, float(alpha), _ptr(g8_out),
                                          g_round, flags, g_seed, g_offset, _ptr(stats), _ptr(w16),
                                          _ptr(velocity), float(lr), float(inv_loss_scale), float(momentum),
                                          float(weight_decay), w_round, w_seed, w_offset,
                                          _ptr(skip_if_nonzero), _ptr(w8_out), _ptr(workspace), ws_bytes,
                                          _stream())
    _check(st, "mp8_wgrad_momentum_fp16_sr")
    return w16


def wgrad_adam_fp16_sr(M, N, K, a, b, w16, m, v, lr, inv_loss_scale, step, beta1=0.9, beta2=0.999, eps=1e-8,
                       weight_decay=0.0, g8_out=None, alpha=1.0, g_round=RNE, flags=0, g_seed=0, g_offset=0,
                       stats=None, w_round=SR, w_seed=0, w_offset=0, skip_if_nonzero=None, w8_out=None,
                       workspace=None, lda=None, ldb=None):
    """mp8_wgrad_adam_fp16_sr: wgrad_update_fp16_sr with ADAM (m, v [K, N] FP32 in place, step from 1)
    in the finishing pass."""
    import torch
    _dev(a, "a", torch.uint8)
    _dev(b, "b", torch.uint8)
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(m, "m", torch.float32)
    _dev(v, "v", torch.float32)
    _dev(g8_out, "g8_out", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    rows, cols, kc = _op_dims(WGRAD, M, N, K)
    a_km, b_km = bool(flags & FLAG_A_CONTRACTION_MAJOR), bool(flags & FLAG_B_CONTRACTION_MAJOR)
    lda = (rows if a_km else kc) if lda is None else lda
    ldb = (cols if b_km else kc) if ldb is None else ldb
    need_a = ((kc - 1) * lda + rows if a_km else (rows - 1) * lda + kc) if rows > 0 and kc > 0 else 0
    need_b = ((kc - 1) * ldb + cols if b_km else (cols - 1) * ldb + kc) if cols > 0 and kc > 0 else 0
    if a.numel() < need_a or b.numel() < need_b:
        raise Mp8Error("a / b is smaller than its shape and leading dimension require")
    for t, name in ((w16, "w16"), (m, "m"), (v, "v"), (g8_out, "g8_out"), (w8_out, "w8_out")):
        if t is not None and t.numel() != rows * cols:
            raise Mp8Error(f"{name} must have K*N elements")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_wgrad_adam_fp16_sr(M, N, K, _ptr(a), lda, _ptr(b), ldb, float(alpha), _ptr(g8_out), g_round,
                                      flags, g_seed, g_offset, _ptr(stats), _ptr(w16), _ptr(m), _ptr(v),
                                      float(lr), float(inv_loss_scale), float(beta1), float(beta2), float(eps),
                                      float(weight_decay), int(step), w_round, w_seed, w_offset,
                                      _ptr(skip_if_nonzero), _ptr(w8_out), _ptr(workspace), ws_bytes, _stream())
    _check(st, "mp8_wgrad_adam_fp16_sr")
    return w16


def conv3x3_wgrad_momentum_fp16_sr(B, H, W, Cin, Cout, x8, e8, w16, velocity, lr, inv_loss_scale, momentum,
                                   weight_decay=0.0, g8_out=None, alpha=1.0, g_round=RNE, flags=0, g_seed=0,
                                   g_offset=0, stats=None, w_round=SR, w_seed=0, w_offset=0,
                                   skip_if_nonzero=None, w8_out=None, workspace=None, prows=None):
    """mp8_conv3x3_wgrad_momentum_fp16_sr: conv3x3_wgrad_update_fp16_sr with the momentum optimizer
    (velocity [3, 3, Cin, Cout] FP32 in place) in the finishing pass."""
    import torch
    prows = conv_prows(B, H, W) if prows is None else prows
    _dev(x8, "x8", torch.uint8)
    _dev(e8, "e8", torch.uint8)
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(velocity, "velocity", torch.float32)
    _dev(g8_out, "g8_out", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    if x8.numel() != prows * Cin or e8.numel() != prows * Cout:
        raise Mp8Error("x8 / e8 do not have the sizes the operation implies")
    for t, name in ((w16, "w16"), (velocity, "velocity"), (g8_out, "g8_out"), (w8_out, "w8_out")):
        if t is not None and t.numel() != 9 * Cin * Cout:
            raise Mp8Error(f"{name} must have 9*Cin*Cout elements")
    if not _has_guard(x8, (W + 3) * Cin):
        raise Mp8Error("the padded tensor x8 needs W+3 readable guard rows before and after "
                       "(allocate it with conv_buffer)")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_conv3x3_wgrad_momentum_fp16_sr(
        B, H, W, Cin, Cout, prows, _ptr(x8), _ptr(e8), float(alpha), _ptr(g8_out), g_round, flags, g_seed,
        g_offset, _ptr(stats), _ptr(w16), _ptr(velocity), float(lr), float(inv_loss_scale), float(momentum),
        float(weight_decay), w_round, w_seed, w_offset, _ptr(skip_if_nonzero), _ptr(w8_out), _ptr(workspace),
        ws_bytes, _stream())
    _check(st, "mp8_conv3x3_wgrad_momentum_fp16_sr")
    return w16


def gemm_fp8_plan(op, M, N, K, flags=0, tile_config=0, split_k=0):
    """(tile configuration name or None for the any-shape kernel, contraction slices)."""
    t, s = C.c_int(0), C.c_int(0)
    _check(lib().mp8_gemm_fp8_plan(op, M, N, K, flags, tile_config, split_k, C.byref(t), C.byref(s)),
           "mp8_gemm_fp8_plan")
    return (gemm_tile_configs()[t.value - 1] if t.value else None), s.value


def gemm_tile_configs():
    n = lib().mp8_gemm_num_tile_configs()
    names = []
    for i in range(1, n + 1):
        buf = C.create_string_buffer(64)
        lib().mp8_gemm_tile_config_name(i, buf, 64)
        names.append(buf.value.decode())
    return names


def gemm_tile_config_lds_bytes(tile_config, epi):
    """Static LDS bytes of a tile configuration's row-major kernel, as the runtime reports them."""
    return lib().mp8_gemm_tile_config_lds_bytes(tile_config, epi)


def sgd_update_fp16_sr(w16, g8, lr, inv_loss_scale, round=SR, seed=0, offset=0,
                       skip_if_nonzero=None, w8_out=None, stats=None):
    """mp8_sgd_update_fp16_sr: in-place SGD step on float16 master weights from 8-bit grads."""
    import torch
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(g8, "g8", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    n = w16.numel()
    if g8.numel() != n or (w8_out is not None and w8_out.numel() != n):
        raise Mp8Error("g8 / w8_out size does not match w16")
    st = lib().mp8_sgd_update_fp16_sr(_ptr(w16), _ptr(g8), n, float(lr), float(inv_loss_scale),
                                      round, seed, offset, _ptr(skip_if_nonzero), _ptr(w8_out),
                                      _ptr(stats), _stream())
    _check(st, "mp8_sgd_update_fp16_sr")
    return w16


def sgd_momentum_fp16_sr(w16, velocity, g8, lr, inv_loss_scale, momentum, weight_decay=0.0, round=SR,
                         seed=0, offset=0, skip_if_nonzero=None, w8_out=None, stats=None):
    """mp8_sgd_momentum_fp16_sr: momentum SGD with L2 regularisation, FP32 velocity in place."""
    import torch
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(velocity, "velocity", torch.float32)
    _dev(g8, "g8", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    n = w16.numel()
    if g8.numel() != n or velocity.numel() != n or (w8_out is not None and w8_out.numel() != n):
        raise Mp8Error("velocity / g8 / w8_out size does not match w16")
    st = lib().mp8_sgd_momentum_fp16_sr(_ptr(w16), _ptr(velocity), _ptr(g8), n, float(lr),
                                        float(inv_loss_scale), float(momentum), float(weight_decay),
                                        round, seed, offset, _ptr(skip_if_nonzero), _ptr(w8_out),
                                        _ptr(stats), _stream())
    _check(st, "mp8_sgd_momentum_fp16_sr")
    return w16


def wgrad_update_fp16_sr(M, N, K, a, b, w16, lr, inv_loss_scale, g8_out=None, alpha=1.0, g_round=RNE,
                         flags=0, g_seed=0, g_offset=0, stats=None, w_round=SR, w_seed=0, w_offset=0,
                         skip_if_nonzero=None, w8_out=None, workspace=None, lda=None, ldb=None):
    """mp8_wgrad_update_fp16_sr: weight-gradient GEMM, its rounding to 8 bits and the update of the
    FP16 master weights w16 [K, N] in one call (operands as gemm_fp8 with op = WGRAD)."""
    import torch
    _dev(a, "a", torch.uint8)
    _dev(b, "b", torch.uint8)
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(g8_out, "g8_out", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    rows, cols, kc = _op_dims(WGRAD, M, N, K)
    a_km, b_km = bool(flags & FLAG_A_CONTRACTION_MAJOR), bool(flags & FLAG_B_CONTRACTION_MAJOR)
    lda = (rows if a_km else kc) if lda is None else lda
    ldb = (cols if b_km else kc) if ldb is None else ldb
    need_a = ((kc - 1) * lda + rows if a_km else (rows - 1) * lda + kc) if rows > 0 and kc > 0 else 0
    need_b = ((kc - 1) * ldb + cols if b_km else (cols - 1) * ldb + kc) if cols > 0 and kc > 0 else 0
    if a.numel() < need_a or b.numel() < need_b:
        raise Mp8Error("a / b is smaller than its shape and leading dimension require")
    for t, name in ((w16, "w16"), (g8_out, "g8_out"), (w8_out, "w8_out")):
        if t is not None and t.numel() != rows * cols:
            raise Mp8Error(f"{name} must have K*N elements")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().mp8_wgrad_update_fp16_sr(M, N, K, _ptr(a), lda, _ptr(b), ldb, float(alpha), _ptr(g8_out),
                                        g_round, flags, g_seed, g_offset, _ptr(stats), _ptr(w16), float(lr),
                                        float(inv_loss_scale), w_round, w_seed, w_offset,
                                        _ptr(skip_if_nonzero), _ptr(w8_out), _ptr(workspace), ws_bytes,
                                        _stream())
    _check(st, "mp8_wgrad_update_fp16_sr")
    return w16


def adam_fp16_sr(w16, m, v, g8, lr, inv_loss_scale, step, beta1=0.9, beta2=0.999, eps=1e-8,
                 weight_decay=0.0, round=SR, seed=0, offset=0, skip_if_nonzero=None, w8_out=None,
                 stats=None):
    """mp8_adam_fp16_sr: ADAM with L2 regularisation, FP32 moments in place (step counts from 1)."""
    import torch
    _dev(w16, "w16", (torch.float16, torch.int16, torch.uint16))
    _dev(m, "m", torch.float32)
    _dev(v, "v", torch.float32)
    _dev(g8, "g8", torch.uint8)
    _dev(w8_out, "w8_out", torch.uint8)
    n = w16.numel()
    if g8.numel() != n or m.numel() != n or v.numel() != n or (w8_out is not None and w8_out.numel() != n):
        raise Mp8Error("m / v / g8 / w8_out size does not match w16")
    st = lib().mp8_adam_fp16_sr(_ptr(w16), _ptr(m), _ptr(v), _ptr(g8), n, float(lr), float(inv_loss_scale),
                                float(beta1), float(beta2), float(eps), float(weight_decay), int(step),
                                round, seed, offset, _ptr(skip_if_nonzero), _ptr(w8_out), _ptr(stats),
                                _stream())
    _check(st, "mp8_adam_fp16_sr")
    return w16


def sr_bits(out, seed=0, offset=0):
    """mp8_sr_bits: out[i] (int16/uint16 GPU tensor) = the 16 random bits of element i."""
    _dev(out, "out")
    if out.element_size() != 2:
        raise Mp8Error("out must have 2-byte elements")
    _check(lib().mp8_sr_bits(_ptr(out), out.numel(), seed, offset, _stream()), "mp8_sr_bits")
    return out


def philox4x32_10(ctr, key):
    """Host: one Philox4x32-10 block; ctr 4 words, key 2 words -> list of 4 ints."""
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().mp8_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def scaler_new(scale, floor, growth_interval=2000) -> Scaler:
    s = Scaler()
    lib().mp8_scaler_init(C.byref(s), float(scale), float(floor), int(growth_interval))
    return s


def scaler_update(s: Scaler, nonfinite: int) -> int:
    return int(lib().mp8_scaler_update(C.byref(s), int(nonfinite)))


def scaler_set_floor(s: Scaler, floor: float) -> None:
    lib().mp8_scaler_set_floor(C.byref(s), float(floor))
