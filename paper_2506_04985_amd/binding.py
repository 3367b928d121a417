"""ctypes view of the fptq C-ABI library (include/fptq.h).  Argument marshalling only: every
step of the layer runs in the library's HIP kernels.  PyTorch supplies device memory and the
current stream, nothing else.  Without the built library (csrc/libfptq.so) importing works but
every call raises -- there is no CPU fallback.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "csrc", "libfptq.so")

SCALE_NONE, SCALE_RMS, SCALE_GIVEN = 0, 1, 2
ERR_NAMES = {-1: "FPTQ_ERR_NULL", -2: "FPTQ_ERR_SHAPE", -3: "FPTQ_ERR_SIZE", -4: "FPTQ_ERR_MODE",
             -5: "FPTQ_ERR_HIP", -6: "FPTQ_ERR_VALUE", -7: "FPTQ_ERR_ALIGN"}

# every symbol include/fptq.h declares, and the test knob of include/fptq_testing.h
EXPORTS = ["fptq_version", "fptq_last_error", "fptq_init", "fptq_packed_bytes", "fptq_pack_weights", "fptq_quantize_act",
           "fptq_quantize_act_hadamard", "fptq_quantize_act_dynamic", "fptq_quantize_act_asym",
           "fptq_weight_row_sums", "fptq_w4a4_linear_zp", "fptq_residual_norm_quantize",
           "fptq_w4a4_linear", "fptq_w4a4_linear_ref", "fptq_unpack", "fptq_linear_workspace_bytes", "fptq_w4a4_linear_ws",
           "fptq_w4a4_linear_noalloc"]
TESTING_EXPORTS = ["fptq_set_gemm_tile", "fptq_set_gemm_map", "fptq_set_decode_shape", "fptq_linear_launch_plan"]

_lib = None


class FptqError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


def lib():
    """Load csrc/libfptq.so (build it first with paper_2506_04985_amd.build.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2506_04985_amd.build` "
                               "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        i64, f32, p, i32 = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int
        L.fptq_version.restype = i32
        L.fptq_init.restype = i32
        L.fptq_last_error.restype = ctypes.c_char_p
        L.fptq_packed_bytes.restype = i64
        L.fptq_packed_bytes.argtypes = [i64, i64]
        L.fptq_pack_weights.restype = i32
        L.fptq_pack_weights.argtypes = [p, i64, i64, p, i64, p]
        L.fptq_quantize_act.restype = i32
        L.fptq_quantize_act.argtypes = [p, i64, i64, i32, f32, p, f32, p, i64, p, p]
        L.fptq_quantize_act_hadamard.restype = i32
        L.fptq_quantize_act_hadamard.argtypes = [p, i64, i64, i32, i32, f32, p, f32, p, i64, p, p]
        L.fptq_quantize_act_asym.restype = i32
        L.fptq_quantize_act_asym.argtypes = [p, i64, i64, i32, f32, p, f32, i32, p, i64, p, p]
        L.fptq_weight_row_sums.restype = i32
        L.fptq_weight_row_sums.argtypes = [p, i64, i64, p, p]
        L.fptq_w4a4_linear_zp.restype = i32
        L.fptq_w4a4_linear_zp.argtypes = [p, p, i64, i64, i64, f32, p, p, i32, p, p, p, p]
        L.fptq_residual_norm_quantize.restype = i32
        L.fptq_residual_norm_quantize.argtypes = [p, p, i64, i64, p, f32, f32, p, p, p, i64, p]
        L.fptq_quantize_act_dynamic.restype = i32
        L.fptq_quantize_act_dynamic.argtypes = [p, i64, i64, p, i64, p, p]
        for name in ("fptq_w4a4_linear", "fptq_w4a4_linear_ref", "fptq_w4a4_linear_noalloc"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = [p, p, i64, i64, i64, f32, p, p, p, p, p]
        L.fptq_linear_launch_plan.restype = i32
        L.fptq_linear_launch_plan.argtypes = [i64, i64, i64, i32, ctypes.c_char_p, i32, ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.fptq_set_gemm_map.restype = i32
        L.fptq_set_gemm_map.argtypes = [i32]
        L.fptq_set_decode_shape.restype = i32
        L.fptq_set_decode_shape.argtypes = [i32]
        L.fptq_set_gemm_tile.restype = i32
        L.fptq_set_gemm_tile.argtypes = [i32]
        L.fptq_unpack.restype = i32
        L.fptq_unpack.argtypes = [p, i64, i64, p, p]
        L.fptq_linear_workspace_bytes.restype = i64
        L.fptq_linear_workspace_bytes.argtypes = [i64, i64, i64]
        L.fptq_w4a4_linear_ws.restype = i32
        L.fptq_w4a4_linear_ws.argtypes = [p, p, i64, i64, i64, f32, p, p, p, p, p, i64, p]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise FptqError(rc, lib().fptq_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous device tensor of {dtype}")
    return t


def fptq_version():
    return lib().fptq_version()


def fptq_init():
    """Set the current device up (kernel attributes, device properties); the first launching call does it otherwise."""
    _check(lib().fptq_init())


def fptq_packed_bytes(rows, K):
    n = lib().fptq_packed_bytes(rows, K)
    if n < 0:
        _check(int(n))
    return int(n)


def _need(rows, K):
    # same formula as the library's fptq_packed_bytes, kept in Python to spare a foreign call per argument check
    return ((K + 127) // 128) * rows * 64


def fptq_pack_weights(w_int, out=None):
    """int8 [N, K] device tensor with values in [-8, 7] -> packed uint8 blob."""
    _dev(w_int, torch.int8, "w_int")
    N, K = w_int.shape
    nbytes = fptq_packed_bytes(N, K)
    out = torch.empty(nbytes, dtype=torch.uint8, device=w_int.device) if out is None else out
    _check(lib().fptq_pack_weights(_ptr(w_int), N, K, _ptr(out), out.numel(), _stream()))
    return out


def fptq_quantize_act(x_bf16, s_a, scale_mode=SCALE_RMS, eps=0.0, row_scale_in=None, out=None, row_scale_out=None,
                      want_row_scale=True):
    """bf16 [M, K] -> (packed uint8 blob, fp32 [M] per-token scale or None)."""
    _dev(x_bf16, torch.bfloat16, "x_bf16")
    M, K = x_bf16.shape
    if row_scale_in is not None:
        _dev(row_scale_in, torch.float32, "row_scale_in")
    out = torch.empty(_need(M, K), dtype=torch.uint8, device=x_bf16.device) if out is None else out
    if row_scale_out is None and want_row_scale:
        row_scale_out = torch.empty(M, dtype=torch.float32, device=x_bf16.device)
    _check(lib().fptq_quantize_act(_ptr(x_bf16), M, K, scale_mode, float(eps), _ptr(row_scale_in), float(s_a),
                                   _ptr(out), out.numel(), _ptr(row_scale_out), _stream()))
    return out, row_scale_out


def fptq_quantize_act_hadamard(x_bf16, s_a, hadamard_block=256, scale_mode=SCALE_GIVEN, eps=0.0, row_scale_in=None, out=None,
                               row_scale_out=None, want_row_scale=True):
    """bf16 [M, K] -> block-wise Hadamard, per-token scale, static INT4 quantizer, packed."""
    _dev(x_bf16, torch.bfloat16, "x_bf16")
    M, K = x_bf16.shape
    if row_scale_in is not None:
        _dev(row_scale_in, torch.float32, "row_scale_in")
    out = torch.empty(_need(M, K), dtype=torch.uint8, device=x_bf16.device) if out is None else out
    if row_scale_out is None and want_row_scale:
        row_scale_out = torch.empty(M, dtype=torch.float32, device=x_bf16.device)
    _check(lib().fptq_quantize_act_hadamard(_ptr(x_bf16), M, K, int(hadamard_block), scale_mode, float(eps),
                                            _ptr(row_scale_in), float(s_a), _ptr(out), out.numel(), _ptr(row_scale_out),
                                            _stream()))
    return out, row_scale_out


def fptq_quantize_act_asym(x_bf16, s_a, zero_point, scale_mode=SCALE_NONE, eps=0.0, row_scale_in=None, out=None):
    """bf16 [M, K] -> packed codes of the asymmetric grid v = clamp(rne(x S / s_a) + z, -8, 7)."""
    _dev(x_bf16, torch.bfloat16, "x_bf16")
    M, K = x_bf16.shape
    if row_scale_in is not None:
        _dev(row_scale_in, torch.float32, "row_scale_in")
    out = torch.empty(_need(M, K), dtype=torch.uint8, device=x_bf16.device) if out is None else out
    r = torch.empty(M, dtype=torch.float32, device=x_bf16.device)
    _check(lib().fptq_quantize_act_asym(_ptr(x_bf16), M, K, scale_mode, float(eps), _ptr(row_scale_in), float(s_a),
                                        int(zero_point), _ptr(out), out.numel(), _ptr(r), _stream()))
    return out, r


def fptq_weight_row_sums(w_int):
    _dev(w_int, torch.int8, "w_int")
    N, K = w_int.shape
    out = torch.empty(N, dtype=torch.int32, device=w_int.device)
    _check(lib().fptq_weight_row_sums(_ptr(w_int), N, K, _ptr(out), _stream()))
    return out


def fptq_w4a4_linear_zp(xq, wq, M, N, K, s_a, s_w, zero_point, w_row_sum, row_out_scale=None, out=None, want_acc=False):
    _dev(w_row_sum, torch.int32, "w_row_sum")
    fn = lambda a, b, m, n, k, sa, sw, d, y, acc, st: lib().fptq_w4a4_linear_zp(a, b, m, n, k, sa, sw, d, int(zero_point),
                                                                                 _ptr(w_row_sum), y, acc, st)
    return _linear(fn, xq, wq, M, N, K, s_a, s_w, row_out_scale, out, want_acc, None)


def fptq_residual_norm_quantize(x_res, y_blk, s_a, s_prev=None, eps=0.0, x_next=None, s_next=None, out=None):
    """Residual add + norm + S_n update + quantizer in one pass: returns (X~_n bf16, S_n fp32 [M], packed uint8)."""
    _dev(x_res, torch.bfloat16, "x_res")
    _dev(y_blk, torch.bfloat16, "y_blk")
    M, K = x_res.shape
    if s_prev is not None:
        _dev(s_prev, torch.float32, "s_prev")
    x_next = torch.empty_like(x_res) if x_next is None else x_next
    s_next = torch.empty(M, dtype=torch.float32, device=x_res.device) if s_next is None else s_next
    out = torch.empty(_need(M, K), dtype=torch.uint8, device=x_res.device) if out is None else out
    _check(lib().fptq_residual_norm_quantize(_ptr(x_res), _ptr(y_blk), M, K, _ptr(s_prev), float(eps), float(s_a),
                                             _ptr(x_next), _ptr(s_next), _ptr(out), out.numel(), _stream()))
    return x_next, s_next, out


def fptq_quantize_act_dynamic(x_bf16, out=None, token_scale_out=None):
    """bf16 [M, K] -> (packed uint8 blob, fp32 [M] per-token scales s_t computed at run time)."""
    _dev(x_bf16, torch.bfloat16, "x_bf16")
    M, K = x_bf16.shape
    out = torch.empty(_need(M, K), dtype=torch.uint8, device=x_bf16.device) if out is None else out
    if token_scale_out is None:
        token_scale_out = torch.empty(M, dtype=torch.float32, device=x_bf16.device)
    _check(lib().fptq_quantize_act_dynamic(_ptr(x_bf16), M, K, _ptr(out), out.numel(), _ptr(token_scale_out), _stream()))
    return out, token_scale_out


def _linear(fn, xq, wq, M, N, K, s_a, s_w, row_out_scale, out, want_acc, acc):
    _dev(xq, torch.uint8, "xq")
    _dev(wq, torch.uint8, "wq")
    _dev(s_w, torch.float32, "s_w")
    if xq.numel() < _need(M, K) or wq.numel() < _need(N, K) or s_w.numel() < N:
        raise FptqError(-3, "packed buffer or s_w smaller than the shape needs")
    if row_out_scale is not None:
        _dev(row_out_scale, torch.float32, "row_out_scale")
    out = torch.empty((M, N), dtype=torch.bfloat16, device=xq.device) if out is None else out
    if acc is None and want_acc:
        acc = torch.empty((M, N), dtype=torch.int32, device=xq.device)
    _check(fn(_ptr(xq), _ptr(wq), M, N, K, float(s_a), _ptr(s_w), _ptr(row_out_scale), _ptr(out), _ptr(acc),
              _stream()))
    return (out, acc) if (want_acc or acc is not None) else out


def fptq_w4a4_linear(xq, wq, M, N, K, s_a, s_w, row_out_scale=None, out=None, want_acc=False, acc=None):
    """Packed activations x packed weights -> bf16 [M, N] (and the int32 accumulators if asked)."""
    return _linear(lib().fptq_w4a4_linear, xq, wq, M, N, K, s_a, s_w, row_out_scale, out, want_acc, acc)


def fptq_linear_workspace_bytes(M, N, K):
    """Bytes of workspace fptq_w4a4_linear_ws would use for this shape (0: it would not use one)."""
    n = lib().fptq_linear_workspace_bytes(M, N, K)
    if n < 0:
        _check(int(n))
    return int(n)


def fptq_w4a4_linear_ws(xq, wq, M, N, K, s_a, s_w, workspace, row_out_scale=None, out=None, want_acc=False, acc=None):
    """fptq_w4a4_linear with a zero-initialised uint8 device workspace (or None) for the split over K."""
    if workspace is not None:
        _dev(workspace, torch.uint8, "workspace")
    fn = lambda a, b, m, n, k, sa, sw, d, y, ac, st: lib().fptq_w4a4_linear_ws(
        a, b, m, n, k, sa, sw, d, y, ac, _ptr(workspace), 0 if workspace is None else workspace.numel(), st)
    return _linear(fn, xq, wq, M, N, K, s_a, s_w, row_out_scale, out, want_acc, acc)


def fptq_w4a4_linear_noalloc(xq, wq, M, N, K, s_a, s_w, row_out_scale=None, out=None, want_acc=False, acc=None):
    """fptq_w4a4_linear_ws on the library's built-in scratch area.  The library allocates nothing; pass `out` (and `acc`)
    to keep this wrapper from allocating the result tensors."""
    return _linear(lib().fptq_w4a4_linear_noalloc, xq, wq, M, N, K, s_a, s_w, row_out_scale, out, want_acc, acc)


def fptq_w4a4_linear_ref(xq, wq, M, N, K, s_a, s_w, row_out_scale=None, out=None, want_acc=False, acc=None):
    return _linear(lib().fptq_w4a4_linear_ref, xq, wq, M, N, K, s_a, s_w, row_out_scale, out, want_acc, acc)


def fptq_set_gemm_map(mode):
    _check(lib().fptq_set_gemm_map(int(mode)))


def fptq_set_decode_shape(code):
    _check(lib().fptq_set_decode_shape(int(code)))


def fptq_set_gemm_tile(tile):
    _check(lib().fptq_set_gemm_tile(int(tile)))


def fptq_linear_launch_plan(M, N, K, with_workspace=False):
    """(kernel name fragment, workgroups, threads per workgroup) of the launch a linear call would make; host only."""
    buf = ctypes.create_string_buffer(96)
    wgs, thr = ctypes.c_int64(0), ctypes.c_int(0)
    _check(lib().fptq_linear_launch_plan(M, N, K, int(bool(with_workspace)), buf, len(buf), ctypes.byref(wgs), ctypes.byref(thr)))
    return buf.value.decode(), int(wgs.value), int(thr.value)


def fptq_unpack(packed, rows, K):
    _dev(packed, torch.uint8, "packed")
    if packed.numel() < fptq_packed_bytes(rows, K):
        raise FptqError(-3, "packed buffer smaller than the shape needs")
    out = torch.empty((rows, K), dtype=torch.int8, device=packed.device)
    _check(lib().fptq_unpack(_ptr(packed), rows, K, _ptr(out), _stream()))
    return out
