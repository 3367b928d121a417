"""ctypes view of the measurement aids (include/fptq_probe.h, csrc/libfptq_probe.so): an MFMA-only loop and a
streaming read, so a benchmark can report what the device sustains next to the layer's own kernels.  Not part of
the quantized linear layer; only the benchmark and its test load this."""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "csrc", "libfptq_probe.so")
EXPORTS = ["fptq_probe_last_error", "fptq_probe_mfma_rate", "fptq_probe_read", "fptq_probe_read_burst", "fptq_probe_mfma_rate_ex"]

_lib = None


class ProbeError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"fptq_probe error {code}: {msg}")
        self.code = code


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2506_04985_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.fptq_probe_last_error.restype = ctypes.c_char_p
        L.fptq_probe_mfma_rate.restype = ctypes.c_int64
        L.fptq_probe_mfma_rate.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.fptq_probe_read.restype = ctypes.c_int
        L.fptq_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        L.fptq_probe_mfma_rate_ex.restype = ctypes.c_int64
        L.fptq_probe_mfma_rate_ex.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.fptq_probe_read_burst.restype = ctypes.c_int
        L.fptq_probe_read_burst.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        _lib = L
    return _lib


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _fail(code):
    raise ProbeError(int(code), lib().fptq_probe_last_error().decode())


def mfma_rate(iters, dense, out=None):
    """Launch the MFMA-only loop; returns (integer operations launched, per-thread checksums).  The caller times it."""
    out = torch.empty(65536, dtype=torch.int32, device="cuda") if out is None else out
    ops = lib().fptq_probe_mfma_rate(int(iters), int(dense), ctypes.c_void_p(out.data_ptr()), _stream())
    if ops < 0:
        _fail(ops)
    return int(ops), out


def read(src, xor4=None, nbytes=None):
    """Stream a device buffer (its first nbytes) once; returns the XOR of its 16-byte words as 4 int32 (xor4 is zeroed
    here if not given)."""
    if not src.is_cuda or not src.is_contiguous():
        raise TypeError("src must be a contiguous CUDA tensor")
    xor4 = torch.zeros(4, dtype=torch.int32, device=src.device) if xor4 is None else xor4
    n = src.numel() * src.element_size() if nbytes is None else int(nbytes)
    rc = lib().fptq_probe_read(ctypes.c_void_p(src.data_ptr()), n, ctypes.c_void_p(xor4.data_ptr()), _stream())
    if rc != 0:
        _fail(rc)
    return xor4


def read_burst(src, xor1024, threads=1024, loads=2, nbytes=None):
    """Stream a device buffer once as a single burst of loads (threads per workgroup x loads per thread in flight).
    xor1024: 1024 zeroed int32 on the device (256 slots of 4); XOR the slots together for the buffer's checksum."""
    xor4 = xor1024
    if not src.is_cuda or not src.is_contiguous():
        raise TypeError("src must be a contiguous CUDA tensor")
    n = src.numel() * src.element_size() if nbytes is None else int(nbytes)
    rc = lib().fptq_probe_read_burst(ctypes.c_void_p(src.data_ptr()), n, ctypes.c_void_p(xor4.data_ptr()), int(threads), int(loads), _stream())
    if rc != 0:
        _fail(rc)
    return xor4


def mfma_rate_ex(iters, operands, workgroups_per_cu, out):
    """The MFMA loop with explicit operand mode (0 zero, 1 fixed, 2 fresh, 3 fresh instruction stream on zeros) and one or
    two workgroups per CU; out: 65536 x workgroups_per_cu int32 on the device.  Returns the operations launched."""
    ops = lib().fptq_probe_mfma_rate_ex(int(iters), int(operands), int(workgroups_per_cu), ctypes.c_void_p(out.data_ptr()), _stream())
    if ops < 0:
        _fail(ops)
    return int(ops)
