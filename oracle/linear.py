"""NumPy-facing wrappers around the oracle's C routines (test infrastructure only).

Arrays: activations are uint16 bf16 bit patterns [M, K]; quantized values are int8 in
[-8, 7], one per element; packed buffers are uint8 [rows, K/2] in the canonical layout
(even index in the low nibble); accumulators int64 or int32 [M, N]; outputs uint16 bf16
bit patterns [M, N].

Each function names the passage of the paper it follows; the arithmetic itself lives in
fptq_oracle.c.
"""
import ctypes
import os

import numpy as np

from . import build as _build

MODE_NONE, MODE_RMS, MODE_GIVEN = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, f32, p = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
        L.oracle_bf16_to_f32.restype = f32
        L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.oracle_f32_to_bf16.argtypes = [f32]
        L.oracle_row_scale.restype = ctypes.c_int
        L.oracle_row_scale.argtypes = [p, i64, i64, ctypes.c_int, f32, p, p]
        L.oracle_quantize_scalar.restype = ctypes.c_int8
        L.oracle_quantize_scalar.argtypes = [ctypes.c_uint16, f32]
        L.oracle_row_multiplier.restype = f32
        L.oracle_row_multiplier.argtypes = [f32, f32, ctypes.c_int]
        L.oracle_quantize.restype = ctypes.c_int
        L.oracle_quantize.argtypes = [p, i64, i64, p, f32, p]
        L.oracle_pack.restype = ctypes.c_int
        L.oracle_pack.argtypes = [p, i64, i64, p]
        L.oracle_unpack.restype = ctypes.c_int
        L.oracle_unpack.argtypes = [p, i64, i64, p]
        L.oracle_gemm_i64.restype = i64
        L.oracle_gemm_i64.argtypes = [p, p, i64, i64, i64, p]
        L.oracle_gemm_i32.restype = ctypes.c_int
        L.oracle_gemm_i32.argtypes = [p, p, i64, i64, i64, p]
        L.oracle_gemm_i64_samples.restype = ctypes.c_int
        L.oracle_gemm_i64_samples.argtypes = [p, p, i64, p, p, i64, p]
        L.oracle_epilogue.restype = ctypes.c_int
        L.oracle_epilogue.argtypes = [p, i64, i64, f32, p, p, p]
        L.oracle_w4a4_linear.restype = ctypes.c_int
        L.oracle_w4a4_linear.argtypes = [p, p, i64, i64, i64, ctypes.c_int, f32, p, f32, p, p, p, p, p, p]
        L.oracle_hadamard_rows.restype = ctypes.c_int
        L.oracle_hadamard_rows.argtypes = [p, i64, i64, i64, p]
        L.oracle_hadamard_multiplier.restype = f32
        L.oracle_hadamard_multiplier.argtypes = [f32, f32, ctypes.c_int, i64]
        L.oracle_quantize_f32.restype = ctypes.c_int
        L.oracle_quantize_f32.argtypes = [p, i64, i64, p, f32, i64, p]
        L.oracle_quantize_dynamic.restype = ctypes.c_int
        L.oracle_quantize_dynamic.argtypes = [p, i64, i64, p, p]
        L.oracle_quantize_scalar_zp.restype = ctypes.c_int8
        L.oracle_quantize_scalar_zp.argtypes = [ctypes.c_uint16, f32, ctypes.c_int]
        L.oracle_quantize_zp.restype = ctypes.c_int
        L.oracle_quantize_zp.argtypes = [p, i64, i64, p, f32, ctypes.c_int, p]
        L.oracle_weight_row_sums.restype = ctypes.c_int
        L.oracle_weight_row_sums.argtypes = [p, i64, i64, p]
        L.oracle_epilogue_zp.restype = ctypes.c_int
        L.oracle_epilogue_zp.argtypes = [p, i64, i64, f32, p, p, ctypes.c_int, p, p]
        L.oracle_residual_norm_quantize.restype = ctypes.c_int
        L.oracle_residual_norm_quantize.argtypes = [p, p, i64, i64, p, f32, f32, p, p, p]
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def bf16_to_f32(bits):
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def row_scale(x_bits, mode=MODE_RMS, eps=0.0, row_scale_in=None):
    """Sec. 3.1.3 Step 1: S = 1 / RMS(x) per token, fp64 sum, fp32 result."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    out = np.empty(M, dtype=np.float32)
    rin = None if row_scale_in is None else _c(row_scale_in, np.float32)
    rc = lib().oracle_row_scale(_ptr(x_bits), M, K, mode, float(eps), _ptr(rin), _ptr(out))
    if rc:
        raise ValueError("bad scale mode")
    return out


def quantize(x_bits, s_a, row_scale=None):
    """App. B static quantization: q = clamp(rne(x * S / s_a), -8, 7) as int8 [M, K]."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    q = np.empty((M, K), dtype=np.int8)
    r = None if row_scale is None else _c(row_scale, np.float32)
    lib().oracle_quantize(_ptr(x_bits), M, K, _ptr(r), float(np.float32(s_a)), _ptr(q))
    return q


def hadamard_rows(x_bits, block):
    """App. D block-wise Walsh-Hadamard transform of every row (unnormalised, fp32 butterflies)."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    out = np.empty((M, K), dtype=np.float32)
    if lib().oracle_hadamard_rows(_ptr(x_bits), M, K, int(block), _ptr(out)):
        raise ValueError("block must be a power of two dividing K")
    return out


def quantize_hadamard(x_bits, s_a, block, row_scale=None):
    """Online Hadamard (Sec. 3.1.4, App. D) followed by the static quantizer (App. B): int8 [M, K]."""
    h = hadamard_rows(x_bits, block)
    M, K = h.shape
    q = np.empty((M, K), dtype=np.int8)
    r = None if row_scale is None else _c(row_scale, np.float32)
    lib().oracle_quantize_f32(_ptr(h), M, K, _ptr(r), float(np.float32(s_a)), int(block), _ptr(q))
    return q


def quantize_dynamic(x_bits):
    """App. B dynamic quantization: per-token s_t = max|x_t| / 7 at run time; returns (int8 [M, K], fp32 [M])."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    q = np.empty((M, K), dtype=np.int8)
    s = np.empty(M, dtype=np.float32)
    lib().oracle_quantize_dynamic(_ptr(x_bits), M, K, _ptr(s), _ptr(q))
    return q, s


def quantize_zp(x_bits, s_a, zero_point, row_scale=None):
    """Asymmetric static grid (App. D): v = clamp(rne(x * S / s_a) + z, -8, 7), representing s_a (v - z)."""
    x_bits = _c(x_bits, np.uint16)
    M, K = x_bits.shape
    q = np.empty((M, K), dtype=np.int8)
    r = None if row_scale is None else _c(row_scale, np.float32)
    if lib().oracle_quantize_zp(_ptr(x_bits), M, K, _ptr(r), float(np.float32(s_a)), int(zero_point), _ptr(q)):
        raise ValueError("zero point outside [-8, 7]")
    return q


def weight_row_sums(w_int):
    w_int = _c(w_int, np.int8)
    N, K = w_int.shape
    out = np.empty(N, dtype=np.int32)
    lib().oracle_weight_row_sums(_ptr(w_int), N, K, _ptr(out))
    return out


def epilogue_zp(acc, s_a, s_w, zero_point, w_row_sum, row_out_scale=None):
    """y = bf16((acc - z * wsum[o]) * (s_a * s_w[o]) [* d_t])."""
    acc = _c(acc, np.int32)
    M, N = acc.shape
    s_w, ws = _c(s_w, np.float32), _c(w_row_sum, np.int32)
    d = None if row_out_scale is None else _c(row_out_scale, np.float32)
    y = np.empty((M, N), dtype=np.uint16)
    lib().oracle_epilogue_zp(_ptr(acc), M, N, float(np.float32(s_a)), _ptr(s_w), _ptr(d), int(zero_point), _ptr(ws), _ptr(y))
    return y


def residual_norm_quantize(x_res_bits, y_bits, s_a, s_prev=None, eps=0.0):
    """Sec. 3.1.3 Eq. (5)-(7): Z~ = X~ + Y~, S_n = S_{n-1} / RMS(Z~), X~_n = Z~ / RMS(Z~), q = quantize(X~_n / s_a).
    Returns dict(x_next (bf16 bits), s_next (fp32 [M]), q (int8 [M, K]))."""
    x_res_bits, y_bits = _c(x_res_bits, np.uint16), _c(y_bits, np.uint16)
    M, K = x_res_bits.shape
    sp = None if s_prev is None else _c(s_prev, np.float32)
    x_next = np.empty((M, K), np.uint16)
    s_next = np.empty(M, np.float32)
    q = np.empty((M, K), np.int8)
    lib().oracle_residual_norm_quantize(_ptr(x_res_bits), _ptr(y_bits), M, K, _ptr(sp), float(eps), float(np.float32(s_a)),
                                        _ptr(x_next), _ptr(s_next), _ptr(q))
    return {"x_next": x_next, "s_next": s_next, "q": q}


def pack(v):
    """App. J double-packed storage, canonical nibble order."""
    v = _c(v, np.int8)
    rows, K = v.shape
    out = np.empty((rows, K // 2), dtype=np.uint8)
    if lib().oracle_pack(_ptr(v), rows, K, _ptr(out)):
        raise ValueError("K must be even")
    return out


def unpack(packed, K):
    packed = _c(packed, np.uint8)
    rows = packed.shape[0]
    out = np.empty((rows, K), dtype=np.int8)
    if lib().oracle_unpack(_ptr(packed), rows, K, _ptr(out)):
        raise ValueError("K must be even")
    return out


def gemm_i64(q, w):
    """App. J integer matmul acc[t, o] = sum_k q[t, k] w[o, k], 64-bit; asserts the int32 fit."""
    q, w = _c(q, np.int8), _c(w, np.int8)
    M, K = q.shape
    N, K2 = w.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int64)
    bad = lib().oracle_gemm_i64(_ptr(q), _ptr(w), M, N, K, _ptr(acc))
    if bad:
        raise OverflowError(f"{bad} accumulators exceed int32")
    return acc


def gemm_i32(q, w):
    q, w = _c(q, np.int8), _c(w, np.int8)
    M, K = q.shape
    N, _ = w.shape
    acc = np.empty((M, N), dtype=np.int32)
    lib().oracle_gemm_i32(_ptr(q), _ptr(w), M, N, K, _ptr(acc))
    return acc


def gemm_i64_samples(q, w, rows, cols):
    """acc[i] = <q[rows[i]], w[cols[i]]> for sampled entries of a result too large to form."""
    q, w = _c(q, np.int8), _c(w, np.int8)
    rows, cols = _c(rows, np.int64), _c(cols, np.int64)
    K = q.shape[1]
    assert w.shape[1] == K and rows.shape == cols.shape
    out = np.empty(rows.shape[0], dtype=np.int64)
    lib().oracle_gemm_i64_samples(_ptr(q), _ptr(w), K, _ptr(rows), _ptr(cols), rows.shape[0], _ptr(out))
    return out


def epilogue(acc, s_a, s_w, row_out_scale=None):
    """App. B: y = bf16(acc * (s_a * s_w[o]) [* d_t]); returns bf16 bit patterns."""
    acc = _c(acc, np.int32)
    M, N = acc.shape
    s_w = _c(s_w, np.float32)
    d = None if row_out_scale is None else _c(row_out_scale, np.float32)
    y = np.empty((M, N), dtype=np.uint16)
    lib().oracle_epilogue(_ptr(acc), M, N, float(np.float32(s_a)), _ptr(s_w), _ptr(d), _ptr(y))
    return y


def w4a4_linear(x_bits, w_int, s_a, s_w, mode=MODE_RMS, eps=0.0, row_scale_in=None, row_out_scale=None):
    """The whole path, checked build: returns dict(r, q, acc (int32), y (bf16 bits))."""
    r = row_scale(x_bits, mode, eps, row_scale_in)
    q = quantize(x_bits, s_a, None if mode == MODE_NONE else r)
    acc = gemm_i64(q, w_int).astype(np.int32)
    y = epilogue(acc, s_a, s_w, row_out_scale)
    return {"r": r, "q": q, "acc": acc, "y": y}


def w4a4_linear_timed(x_bits, w_int, s_a, s_w, mode=MODE_RMS, eps=0.0, row_scale_in=None):
    """The whole path in one C call with the 32-bit accumulator (the build that is timed)."""
    x_bits, w_int, s_w = _c(x_bits, np.uint16), _c(w_int, np.int8), _c(s_w, np.float32)
    M, K = x_bits.shape
    N = w_int.shape[0]
    r = np.empty(M, np.float32)
    q = np.empty((M, K), np.int8)
    acc = np.empty((M, N), np.int32)
    y = np.empty((M, N), np.uint16)
    rin = None if row_scale_in is None else _c(row_scale_in, np.float32)
    rc = lib().oracle_w4a4_linear(_ptr(x_bits), _ptr(w_int), M, N, K, mode, float(eps), _ptr(rin),
                                  float(np.float32(s_a)), _ptr(s_w), None, _ptr(r), _ptr(q), _ptr(acc), _ptr(y))
    assert rc == 0
    return y


def num_threads():
    return int(lib().oracle_num_threads())
