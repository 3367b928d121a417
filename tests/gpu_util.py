"""Helpers shared by the GPU parity tests: host <-> device marshalling and the comparison rules.

Comparison bar: per-token scales, quantized values and int32 accumulators bit-exact; bf16 outputs
within 1e-2 of the oracle, max-abs normalised (the tests also report how many differ at all).
"""
import numpy as np
import torch

from paper_2506_04985_amd import binding as fptq

Y_TOL = 1e-2


def dev_bf16(x_bits):
    return torch.from_numpy(np.ascontiguousarray(x_bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(y):
    return y.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_f64(b):
    return (np.asarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def y_error(y_bits_gpu, y_bits_ref):
    """max |y_gpu - y_ref| / max |y_ref| on finite values."""
    a, b = bits_to_f64(y_bits_gpu), bits_to_f64(y_bits_ref)
    denom = max(np.abs(b).max(), 1e-30)
    return float(np.abs(a - b).max() / denom)


def layout_from_canonical(canon, rows, K):
    """Library layout spelled out from its documentation: 128-value K tiles outermost, one 64-byte
    segment per (tile, row), K zero-padded.  canon is uint8 [rows, K/2] (K even)."""
    kt = (K + 127) // 128
    padded = np.zeros((rows, kt * 64), np.uint8)
    padded[:, :canon.shape[1]] = canon
    return np.ascontiguousarray(padded.reshape(rows, kt, 64).transpose(1, 0, 2)).reshape(-1)


def run_gpu_linear(inp, M=None, use_ref=False, want_acc=True, undo_scale=False):
    """Quantize + linear on the GPU for one synthetic case; returns host arrays."""
    case = inp.case
    x = dev_bf16(inp.x_bits)
    w_packed = fptq.fptq_pack_weights(dev(inp.w_int))
    s_w = dev(inp.s_w)
    r_in = dev(inp.row_scale_in)
    Mx, K = inp.x_bits.shape
    N = inp.w_int.shape[0]
    xq, r = fptq.fptq_quantize_act(x, float(inp.s_a), case.mode, case.eps, r_in)
    d = (1.0 / r) if undo_scale else None
    fn = fptq.fptq_w4a4_linear_ref if use_ref else fptq.fptq_w4a4_linear
    out = fn(xq, w_packed, Mx, N, K, float(inp.s_a), s_w, d, want_acc=want_acc)
    y, acc = out if want_acc else (out, None)
    q = fptq.fptq_unpack(xq, Mx, K)
    torch.cuda.synchronize()
    return {"r": r.cpu().numpy(), "q": q.cpu().numpy(), "acc": None if acc is None else acc.cpu().numpy(),
            "y": host_bits(y), "d": None if d is None else d.cpu().numpy()}
