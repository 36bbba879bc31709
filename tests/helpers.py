"""Shared test plumbing: parameter conversion between the oracle's dataclasses and the
library's ctypes structs (both carry the same integers), and GPU upload helpers."""
import numpy as np

import paper_2511_15369_amd as ip
from oracle import ref


def lib_dyadic(d: ref.Dyadic) -> ip.Dyadic:
    return ip.Dyadic(d.m, d.s, d.zp, d.qmin, d.qmax)


def lib_softmax(p: ref.SoftmaxParams, algo: int = 0) -> ip.SoftmaxParams:
    return ip.SoftmaxParams(p.variant, p.i0, p.n_shift, p.m_bits, p.out_bits, p.pre_m, p.pre_s,
                            lib_dyadic(p.post), p.out_is_signed, algo)


def lib_gelu(p: ref.GeluParams, algo: int = 0) -> ip.GeluParams:
    return ip.GeluParams(p.variant, p.q_b, p.q_c, p.k, p.zp_in, p.max_abs_q, p.pre_m, p.pre_s,
                         lib_dyadic(p.post), algo)


def softmax_fields(p):
    return (p.variant, p.i0, p.n_shift, p.m_bits, p.out_bits, p.pre_m, p.pre_s, p.post.m, p.post.s,
            p.post.zp, p.post.qmin, p.post.qmax, p.out_is_signed)


def gelu_fields(p):
    return (p.variant, p.q_b, p.q_c, p.k, p.zp_in, p.max_abs_q, p.pre_m, p.pre_s, p.post.m,
            p.post.s, p.post.zp, p.post.qmin, p.post.qmax)


def gpu_softmax(scores: np.ndarray, p: ref.SoftmaxParams, bias=None, period=0, algo=0) -> np.ndarray:
    import torch
    rows, cols = scores.shape
    d_in = torch.from_numpy(np.ascontiguousarray(scores)).cuda()
    d_bias = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias)).cuda()

    def run(which):
        d_out = torch.full((rows, cols), 0x5A, dtype=torch.int8 if p.out_is_signed else torch.uint8,
                           device="cuda")
        ip.softmax_i32(d_in, d_bias, period, d_out, rows, cols, lib_softmax(p, which))
        torch.cuda.synchronize()
        return d_out.cpu().numpy()

    out = run(algo)
    if algo == 0:
        # a call of few rows goes to one wavefront per row; the slab kernels must agree on it too
        assert np.array_equal(run(4), out), "IPTQ_ALGO_SLAB differs from IPTQ_ALGO_AUTO"
    return out


def gpu_gelu_i8(x: np.ndarray, p: ref.GeluParams, algo=0, inplace=False) -> np.ndarray:
    import torch
    d_in = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    d_out = d_in if inplace else torch.full_like(d_in, 0x5A)
    ip.gelu_i8(d_in, d_out, x.size, lib_gelu(p, algo))
    torch.cuda.synchronize()
    return d_out.cpu().numpy()


def gpu_gelu_i32(x: np.ndarray, p: ref.GeluParams, algo=0) -> np.ndarray:
    import torch
    d_in = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    d_out = torch.full(x.shape, 0x5A, dtype=torch.int8, device="cuda")
    ip.gelu_i32(d_in, d_out, x.size, lib_gelu(p, algo))
    torch.cuda.synchronize()
    return d_out.cpu().numpy()


def gpu_requant(x: np.ndarray, d: ref.Dyadic, out_is_signed: int) -> np.ndarray:
    import torch
    d_in = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    d_out = torch.full(x.shape, 0x5A, dtype=torch.int8 if out_is_signed else torch.uint8,
                       device="cuda")
    ip.requant(d_in, d_out, x.size, out_is_signed, lib_dyadic(d))
    torch.cuda.synchronize()
    return d_out.cpu().numpy()


def gpu_softmax_windowed(scores: np.ndarray, p: ref.SoftmaxParams, bias, period, mask, heads, algo=0) -> np.ndarray:
    import torch
    rows, cols = scores.shape
    d_in = torch.from_numpy(np.ascontiguousarray(scores)).cuda()
    d_bias = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias)).cuda()
    d_mask = None if mask is None else torch.from_numpy(np.ascontiguousarray(mask)).cuda()
    n_w = 0 if mask is None else mask.shape[0]
    d_out = torch.full((rows, cols), 0x5A, dtype=torch.int8 if p.out_is_signed else torch.uint8, device="cuda")
    ip.softmax_i32_windowed(d_in, d_bias, period, d_mask, n_w, heads, d_out, rows, cols, lib_softmax(p, algo))
    torch.cuda.synchronize()
    return d_out.cpu().numpy()


def gpu_pack_window_mask(mask: np.ndarray):
    """The library's packing of an int32 window mask; returns (device words as int64, host uint64 view)."""
    import torch
    n_w, cols, _ = mask.shape
    d_mask = torch.from_numpy(np.ascontiguousarray(mask)).cuda()
    d_bits = torch.full((n_w, cols, (cols + 63) // 64), 0x5A5A5A5A, dtype=torch.int64, device="cuda")
    ip.pack_window_mask(d_mask, n_w, cols, d_bits)
    torch.cuda.synchronize()
    return d_bits, d_bits.cpu().numpy().view(np.uint64)


def gpu_softmax_windowed_bits(scores: np.ndarray, p: ref.SoftmaxParams, bias, period, bits: np.ndarray, heads,
                              algo=0) -> np.ndarray:
    """bits: uint64 [n_windows, cols, words] on the host (the oracle's packing)."""
    import torch
    rows, cols = scores.shape
    d_in = torch.from_numpy(np.ascontiguousarray(scores)).cuda()
    d_bias = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias)).cuda()
    d_bits = torch.from_numpy(np.ascontiguousarray(bits).view(np.int64)).cuda()
    d_out = torch.full((rows, cols), 0x5A, dtype=torch.int8 if p.out_is_signed else torch.uint8, device="cuda")
    ip.softmax_i32_windowed_bits(d_in, d_bias, period, d_bits, bits.shape[0], heads, d_out, rows, cols,
                                 lib_softmax(p, algo))
    torch.cuda.synchronize()
    return d_out.cpu().numpy()
