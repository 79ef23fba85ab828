"""numpy front end of the CPU oracle (oracle/dlcx_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  Nothing on the product path imports this module
and this module imports nothing from the GPU package.

Shapes: a matrix is an (m, n) float32 C-contiguous array.  A factor with r
columns of length L is an (r, L) float32 C-contiguous array, i.e. row c of the
numpy array is column c of the mathematical factor.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16 = 0, 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _declare(_lib)
    return _lib


_fp = C.POINTER(C.c_float)
_dp = C.POINTER(C.c_double)
_bp = C.POINTER(C.c_uint8)
_ip = C.POINTER(C.c_int32)


def _declare(L):
    L.orc_delta_ef.argtypes = [_fp, C.c_void_p, C.c_int, _fp, _fp, C.c_int64]
    L.orc_project_p.argtypes = [C.c_int64, C.c_int64, C.c_int, _fp, _fp, _fp]
    L.orc_project_q.argtypes = [C.c_int64, C.c_int64, C.c_int, _fp, _fp, _fp]
    L.orc_project_q_row.argtypes = [C.c_int64, C.c_int64, C.c_int, _fp, _fp, C.c_int64, _fp]
    L.orc_reconstruct.argtypes = [C.c_int64, C.c_int64, C.c_int, _fp, _fp, _fp]
    L.orc_orthonormalize.argtypes = [C.c_int64, C.c_int, _fp]
    L.orc_quantize.argtypes = [_fp, C.c_int64, C.c_int, C.c_int, _bp, _fp]
    L.orc_dequantize.argtypes = [_bp, _fp, C.c_int64, C.c_int, C.c_int, _fp]
    L.orc_dequant_average.argtypes = [C.c_int, C.POINTER(_bp), C.POINTER(_fp), C.c_int64,
                                      C.c_int, C.c_int, _fp]
    L.orc_ef_update.argtypes = [_fp, _fp, C.c_int64]
    L.orc_outer_nesterov.argtypes = [_fp, _fp, _fp, C.c_int64, C.c_double, C.c_double]
    L.orc_gram_eigenvalues.argtypes = [C.c_int64, C.c_int, _fp, _dp]
    L.orc_effective_rank.argtypes = [C.c_int64, C.c_int, _fp, C.c_double]
    L.orc_effective_rank.restype = C.c_int
    L.orc_adagradcmp.argtypes = [_ip, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                 C.c_int32, _ip, _ip]
    for name in ("orc_delta_ef", "orc_project_p", "orc_project_q", "orc_project_q_row",
                 "orc_reconstruct", "orc_orthonormalize", "orc_quantize", "orc_dequantize",
                 "orc_dequant_average", "orc_ef_update", "orc_outer_nesterov",
                 "orc_gram_eigenvalues", "orc_adagradcmp"):
        getattr(L, name).restype = None


def _f(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"], (a.dtype, a.flags)
    return a.ctypes.data_as(_fp)


def _b(a):
    assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_bp)


def payload_bytes(count, qbits, group):
    """(code bytes, number of fp32 scales) of a quantised factor of `count` elements."""
    assert count % group == 0 and qbits in (4, 8)
    return (count // 2 if qbits == 4 else count), count // group


def delta_ef(theta_g, theta_l, e):
    """delta = (theta_g - theta_l) + e.  theta_l float32, or uint16 holding bf16 bits."""
    out = np.empty_like(e)
    if theta_l.dtype == np.uint16:
        dt = BF16
    else:
        assert theta_l.dtype == np.float32
        dt = F32
    assert theta_l.flags["C_CONTIGUOUS"] and theta_g.size == theta_l.size == e.size
    lib().orc_delta_ef(_f(theta_g), theta_l.ctypes.data_as(C.c_void_p), dt, _f(e), _f(out),
                       theta_g.size)
    return out


def project_p(M, q_in):
    m, n = M.shape
    r = q_in.shape[0]
    assert q_in.shape == (r, n)
    p = np.empty((r, m), np.float32)
    lib().orc_project_p(m, n, r, _f(M), _f(q_in), _f(p))
    return p


def project_q(M, p_hat):
    m, n = M.shape
    r = p_hat.shape[0]
    assert p_hat.shape == (r, m)
    q = np.empty((r, n), np.float32)
    lib().orc_project_q(m, n, r, _f(M), _f(p_hat), _f(q))
    return q


def project_q_row(M, p_hat, j0):
    m, n = M.shape
    r = p_hat.shape[0]
    out = np.empty(r, np.float32)
    lib().orc_project_q_row(m, n, r, _f(M), _f(p_hat), int(j0), _f(out))
    return out


def reconstruct(p_hat, q_bar):
    r, m = p_hat.shape
    n = q_bar.shape[1]
    assert q_bar.shape[0] == r
    out = np.empty((m, n), np.float32)
    lib().orc_reconstruct(m, n, r, _f(p_hat), _f(q_bar), _f(out))
    return out


def orthonormalize(p):
    r, m = p.shape
    out = np.ascontiguousarray(p.copy())
    lib().orc_orthonormalize(m, r, _f(out))
    return out


def quantize(x, qbits, group):
    x = np.ascontiguousarray(x)
    count = x.size
    nb, ns = payload_bytes(count, qbits, group)
    codes = np.zeros(nb, np.uint8)
    scales = np.empty(ns, np.float32)
    lib().orc_quantize(_f(x), count, qbits, group, _b(codes), _f(scales))
    return codes, scales


def dequantize(codes, scales, count, qbits, group):
    out = np.empty(count, np.float32)
    lib().orc_dequantize(_b(codes), _f(scales), count, qbits, group, _f(out))
    return out


def unpack_codes(codes, count, qbits):
    """Signed integer value of every code (numpy helper for tests)."""
    if qbits == 8:
        return codes.view(np.int8).astype(np.int32)[:count]
    lo = (codes & 0xF).astype(np.int32)
    hi = (codes >> 4).astype(np.int32)
    v = np.empty(codes.size * 2, np.int32)
    v[0::2] = lo
    v[1::2] = hi
    v = np.where(v >= 8, v - 16, v)
    return v[:count]


def dequant_average(codes_list, scales_list, count, qbits, group):
    K = len(codes_list)
    cp = (_bp * K)(*[_b(c) for c in codes_list])
    sp = (_fp * K)(*[_f(s) for s in scales_list])
    out = np.empty(count, np.float32)
    lib().orc_dequant_average(K, cp, sp, count, qbits, group, _f(out))
    return out


def ef_update(e_inout, delta_hat):
    assert e_inout.size == delta_hat.size
    lib().orc_ef_update(_f(e_inout), _f(delta_hat), e_inout.size)
    return e_inout


def outer_nesterov(theta, v, g, lr, mu):
    assert theta.size == v.size == g.size
    lib().orc_outer_nesterov(_f(theta), _f(v), _f(g), theta.size, float(lr), float(mu))
    return theta, v


def gram_eigenvalues(q_bar):
    r, n = q_bar.shape
    eig = np.empty(r, np.float64)
    lib().orc_gram_eigenvalues(n, r, _f(q_bar), eig.ctypes.data_as(_dp))
    return eig


def effective_rank(q_bar, tau):
    r, n = q_bar.shape
    return int(lib().orc_effective_rank(n, r, _f(q_bar), float(tau)))


def adagradcmp(hist, t, c, r1, rmin, rmax, H1):
    h = np.ascontiguousarray(np.asarray(hist, np.int32))
    assert h.size >= t
    r_out = C.c_int32(0)
    H_out = C.c_int32(0)
    lib().orc_adagradcmp(h.ctypes.data_as(_ip), t, c, r1, rmin, rmax, H1,
                         C.byref(r_out), C.byref(H_out))
    return int(r_out.value), int(H_out.value)
