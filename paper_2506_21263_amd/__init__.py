"""Python binding of libdlcx_hip.so (see include/dlcx.h for the contract).

Argument marshalling only: every function below has the name of the C entry point it calls,
takes torch tensors that live on the GPU (PyTorch is used for device memory and streams and for
nothing else) and passes their addresses through.  There is no fallback: if the HIP library is
missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdlcx_hip.so")

OK, EINVAL, EUNSUPPORTED, ELAUNCH, ETOOBIG = 0, -1, -2, -3, -4
PHASE_P, PHASE_Q = 0, 1
F32, BF16 = 0, 1
MMA_FMA, MMA_F32, MMA_BF16, MMA_F16 = 0, 1, 2, 3
MAX_RANK, MAX_WORKERS = 256, 16


class DlcxError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        detail = lib().dlcx_last_hip_error().decode() if code == ELAUNCH else ""
        super().__init__("%s: %s (%d) %s" % (what, lib().dlcx_strerror(code).decode(), code, detail))


class Desc(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64), ("r", C.c_int32), ("qbits", C.c_int32),
                ("group", C.c_int32), ("mma", C.c_int32)]


def desc(m, n, r, qbits, group, mma=MMA_FMA):
    return Desc(m, n, r, qbits, group, mma)


_lib = None
_vp, _i64, _i32, _int = C.c_void_p, C.c_int64, C.c_int32, C.c_int
_dp = C.POINTER(Desc)

SYMBOLS = {
    "dlcx_delta_ef": (_int, [_vp, _vp, _int, _vp, _i64, _vp]),
    "dlcx_compress": (_int, [_dp, _int, _vp, _vp, _vp, _vp, _vp, _vp]),
    "dlcx_compress_batched": (_int, [_dp, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp]),
    "dlcx_average": (_int, [_dp, _int, _int, _vp, _vp, _vp, _vp, _vp]),
    "dlcx_average_static": (_int, [_dp, _int, _int, _vp, _vp, _vp, _vp]),
    "dlcx_static_scratch_bytes": (C.c_size_t, []),
    "dlcx_static_scratch_need": (C.c_size_t, [_dp, _int]),
    "dlcx_decompress": (_int, [_dp, _vp, _vp, _vp, _int, _vp, _vp, _vp]),
    "dlcx_decompress_apply": (_int, [_dp, _vp, _vp, _int, _vp, _vp, _vp, C.c_float, C.c_float, _vp,
                                     _vp]),
    "dlcx_ef_delta_apply": (_int, [_dp, _vp, _vp, _int, _vp, _int, _vp, _vp, _vp, C.c_float,
                                   C.c_float, _vp, _vp]),
    "dlcx_ef_delta_apply_compress": (_int, [_dp, _i32, _vp, _vp, _int, _vp, _int, _vp, _vp, _vp,
                                            C.c_float, C.c_float, _vp, _vp, _vp, _vp, _vp]),
    "dlcx_outer_nesterov": (_int, [_vp, _vp, _vp, _i64, C.c_float, C.c_float, _vp]),
    "dlcx_quant_round": (_int, [_i64, _int, _int, _int, _vp, _int, _vp, _vp, _vp, C.c_double,
                                C.c_double, _vp, _vp, _int, _vp, _vp, _vp]),
    "dlcx_ef_update": (_int, [_int, _vp, _vp, _i64, _vp]),
    "dlcx_requantize": (_int, [_vp, _i64, _int, _int, _vp]),
    "dlcx_mfma_peak_probe": (_int, [_int, _int, _int, _vp, _vp]),
    "dlcx_traffic_probe": (_int, [_int, _vp, _int, _vp, _vp, _vp, _i64, _vp]),
    "dlcx_comm_seconds": (C.c_double, [C.c_double, _int, C.c_double]),
    "dlcx_plan_overlap": (_int, [_dp, _int, C.c_double, _int, _i32, _i32, _int, C.c_double,
                                 C.c_double, _i32, _vp, _vp, _vp]),
    "dlcx_select_rank": (_int, [_dp, _vp, _int, C.c_double, _vp, _i32, _i32, _i32, _i32, _i32,
                                _i32, _vp, _vp, _vp, _vp, _vp]),
    "dlcx_select_rank_from": (_int, [_vp, _int, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp,
                                     _vp]),
    "dlcx_batched_workspace_bytes": (C.c_size_t, [_dp, _int]),
    "dlcx_orthonormalize_batched": (_int, [_dp, _vp, _int, _vp, _vp]),
    "dlcx_effective_rank_batched": (_int, [_dp, _vp, _int, C.c_double, _vp, _vp, _vp]),
    "dlcx_payload_bytes": (C.c_size_t, [_dp, _int, _vp, _vp]),
    "dlcx_workspace_bytes": (C.c_size_t, [_dp, _int]),
    "dlcx_select_rank_workspace_bytes": (C.c_size_t, [_dp, _int]),
    "dlcx_project": (_int, [_dp, _int, _int, _vp, _vp, _vp, _vp, _vp]),
    "dlcx_quantize": (_int, [_vp, _i64, _int, _int, _vp, _vp, _vp]),
    "dlcx_dequant_average": (_int, [_int, _vp, _vp, _i64, _int, _int, _vp, _vp]),
    "dlcx_orthonormalize": (_int, [_i64, _i32, _vp, _vp, _vp]),
    "dlcx_effective_rank": (_int, [_i64, _i32, _vp, C.c_double, _vp, _vp, _vp]),
    "dlcx_profile_enable": (_int, [_int]),
    "dlcx_profile_kernels": (_int, []),
    "dlcx_profile_name": (C.c_char_p, [_int]),
    "dlcx_profile_read": (_int, [_int, _vp, _vp]),
    "dlcx_strerror": (C.c_char_p, [_int]),
    "dlcx_last_hip_error": (C.c_char_p, []),
}


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: build it with `python paper_2506_21263_amd/build.py` "
                              "(there is no CPU fallback)" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            f = getattr(L, name)
            f.restype = res
            f.argtypes = args
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _ptr_array(ts):
    if ts is None:
        return None
    arr = (C.c_void_p * len(ts))(*[_ptr(t) for t in ts])
    return C.cast(arr, C.c_void_p), arr  # keep `arr` alive with the caller


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(code, what):
    if code != OK:
        raise DlcxError(code, what)


def dlcx_payload_bytes(d, phase):
    cb, sb = C.c_size_t(0), C.c_size_t(0)
    total = lib().dlcx_payload_bytes(C.byref(d), phase, C.addressof(cb), C.addressof(sb))
    return total, cb.value, sb.value


def dlcx_workspace_bytes(d, K):
    return lib().dlcx_workspace_bytes(C.byref(d), K)


def dlcx_delta_ef(theta_g, theta_l, ef_inout, numel=None, stream=None):
    dt = BF16 if theta_l.dtype == torch.bfloat16 else F32
    n = theta_g.numel() if numel is None else numel
    _check(lib().dlcx_delta_ef(_ptr(theta_g), _ptr(theta_l), dt, _ptr(ef_inout), n,
                               _stream(stream)), "dlcx_delta_ef")


def dlcx_compress(d, phase, delta, basis, codes_out, scales_out, workspace, stream=None):
    _check(lib().dlcx_compress(C.byref(d), phase, _ptr(delta), _ptr(basis), _ptr(codes_out),
                               _ptr(scales_out), _ptr(workspace), _stream(stream)),
           "dlcx_compress")


def dlcx_compress_batched(d, phase, deltas, basis, codes_out, scales_out, workspace, stream=None):
    dp, k1 = _ptr_array(deltas)
    cp, k2 = _ptr_array(codes_out)
    sp, k3 = _ptr_array(scales_out)
    _check(lib().dlcx_compress_batched(C.byref(d), phase, len(deltas), dp, _ptr(basis), cp, sp,
                                       _ptr(workspace), _stream(stream)), "dlcx_compress_batched")


def dlcx_average(d, phase, codes, scales, factor_out, workspace, stream=None):
    cp, k1 = _ptr_array(codes)
    sp, k2 = _ptr_array(scales)
    _check(lib().dlcx_average(C.byref(d), phase, len(codes), cp, sp, _ptr(factor_out),
                              _ptr(workspace), _stream(stream)), "dlcx_average")


def dlcx_average_static(d, phase, codes, scales, factor_out, stream=None):
    cp, k1 = _ptr_array(codes)
    sp, k2 = _ptr_array(scales)
    _check(lib().dlcx_average_static(C.byref(d), phase, len(codes), cp, sp, _ptr(factor_out),
                                     _stream(stream)), "dlcx_average_static")


def dlcx_static_scratch_bytes():
    return lib().dlcx_static_scratch_bytes()


def dlcx_static_scratch_need(d, phase):
    return lib().dlcx_static_scratch_need(C.byref(d), phase)


def dlcx_decompress(d, p_hat, q_bar, delta_hat_out, ef_inout=(), workspace=None, stream=None):
    ep, keep = _ptr_array(list(ef_inout)) if len(ef_inout) else (None, None)
    _check(lib().dlcx_decompress(C.byref(d), _ptr(p_hat), _ptr(q_bar), _ptr(delta_hat_out),
                                 len(ef_inout), ep, _ptr(workspace), _stream(stream)),
           "dlcx_decompress")


def dlcx_decompress_apply(d, p_hat, q_bar, ef_inout, theta_g, v, lr, mu, workspace=None,
                          stream=None):
    ep, keep = _ptr_array(list(ef_inout)) if len(ef_inout) else (None, None)
    _check(lib().dlcx_decompress_apply(C.byref(d), _ptr(p_hat), _ptr(q_bar), len(ef_inout), ep,
                                       _ptr(theta_g), _ptr(v), lr, mu, _ptr(workspace),
                                       _stream(stream)), "dlcx_decompress_apply")


def dlcx_ef_delta_apply(d, p_hat, q_bar, theta_l, ef_inout, theta_g, v, lr, mu, workspace=None,
                        stream=None):
    dt = BF16 if theta_l[0].dtype == torch.bfloat16 else F32
    tp, k1 = _ptr_array(list(theta_l))
    ep, k2 = _ptr_array(list(ef_inout))
    _check(lib().dlcx_ef_delta_apply(C.byref(d), _ptr(p_hat), _ptr(q_bar), len(ef_inout), tp, dt,
                                     ep, _ptr(theta_g), _ptr(v), lr, mu, _ptr(workspace),
                                     _stream(stream)), "dlcx_ef_delta_apply")


def dlcx_ef_delta_apply_compress(d, r_prev, p_hat, q_bar, theta_l, ef_inout, theta_g, v, lr, mu,
                                 basis, codes_out, scales_out, workspace, stream=None):
    dt = BF16 if theta_l[0].dtype == torch.bfloat16 else F32
    tp, k1 = _ptr_array(list(theta_l))
    ep, k2 = _ptr_array(list(ef_inout))
    cp, k3 = _ptr_array(list(codes_out))
    sp, k4 = _ptr_array(list(scales_out))
    _check(lib().dlcx_ef_delta_apply_compress(
        C.byref(d), r_prev, _ptr(p_hat), _ptr(q_bar), len(ef_inout), tp, dt, ep, _ptr(theta_g),
        _ptr(v), lr, mu, _ptr(basis), cp, sp, _ptr(workspace), _stream(stream)),
        "dlcx_ef_delta_apply_compress")


def dlcx_outer_nesterov(theta_g, v, delta_hat, lr, mu, numel=None, stream=None):
    n = theta_g.numel() if numel is None else numel
    _check(lib().dlcx_outer_nesterov(_ptr(theta_g), _ptr(v), _ptr(delta_hat), n, lr, mu,
                                     _stream(stream)), "dlcx_outer_nesterov")


def dlcx_quant_round(numel, qbits, group, theta_l, ef_inout, theta_g, v, lr, mu, prev_codes,
                     prev_scales, codes_out, scales_out, requant=False, stream=None):
    """prev_codes / prev_scales None: outer step 1."""
    dt = BF16 if theta_l[0].dtype == torch.bfloat16 else F32
    tp, k1 = _ptr_array(list(theta_l))
    ep, k2 = _ptr_array(list(ef_inout))
    pc, k3 = _ptr_array(list(prev_codes)) if prev_codes is not None else (None, None)
    ps, k4 = _ptr_array(list(prev_scales)) if prev_scales is not None else (None, None)
    cp, k5 = _ptr_array(list(codes_out))
    sp, k6 = _ptr_array(list(scales_out))
    _check(lib().dlcx_quant_round(numel, qbits, group, len(ef_inout), tp, dt, ep, _ptr(theta_g),
                                  _ptr(v), lr, mu, pc, ps, 1 if requant else 0, cp, sp,
                                  _stream(stream)), "dlcx_quant_round")


def dlcx_ef_update(ef_inout, delta_hat, numel=None, stream=None):
    n = delta_hat.numel() if numel is None else numel
    ep, keep = _ptr_array(list(ef_inout))
    _check(lib().dlcx_ef_update(len(ef_inout), ep, _ptr(delta_hat), n, _stream(stream)),
           "dlcx_ef_update")


def dlcx_mfma_peak_probe(workgroups, iters, out, random_operands=False, stream=None):
    _check(lib().dlcx_mfma_peak_probe(workgroups, iters, 1 if random_operands else 0, _ptr(out),
                                      _stream(stream)), "dlcx_mfma_peak_probe")


def dlcx_traffic_probe(theta_l, ef_inout, theta_g, v, numel=None, stream=None):
    dt = BF16 if theta_l[0].dtype == torch.bfloat16 else F32
    n = theta_g.numel() if numel is None else numel
    tp, k1 = _ptr_array(list(theta_l))
    ep, k2 = _ptr_array(list(ef_inout))
    _check(lib().dlcx_traffic_probe(len(ef_inout), tp, dt, ep, _ptr(theta_g), _ptr(v), n,
                                    _stream(stream)), "dlcx_traffic_probe")


def dlcx_requantize(x_inout, count, qbits, group, stream=None):
    _check(lib().dlcx_requantize(_ptr(x_inout), count, qbits, group, _stream(stream)),
           "dlcx_requantize")


def dlcx_comm_seconds(payload_bytes, clusters, bits_per_second):
    return lib().dlcx_comm_seconds(payload_bytes, clusters, bits_per_second)


def dlcx_plan_overlap(descs, extra_bytes, rmin, rmax, clusters, bits_per_second, step_seconds, H,
                      power_iters=1):
    """Returns (rank, H, seconds of the exchange at that rank).  Host only."""
    n = len(descs)
    arr = (Desc * max(n, 1))(*descs)
    r, h, t = _i32(0), _i32(0), C.c_double(0.0)
    _check(lib().dlcx_plan_overlap(arr, n, extra_bytes, power_iters, rmin, rmax, clusters,
                                   bits_per_second, step_seconds, H, C.addressof(r),
                                   C.addressof(h), C.addressof(t)), "dlcx_plan_overlap")
    return r.value, h.value, t.value


def dlcx_select_rank_workspace_bytes(descs):
    arr = (Desc * max(len(descs), 1))(*descs)
    return lib().dlcx_select_rank_workspace_bytes(arr, len(descs))


def dlcx_select_rank(descs, q_bars, tau, rprime_hist, t, c, r1, rmin, rmax, H1, workspace=None,
                     rprime=None, stream=None):
    """rprime_hist: ctypes int32 array of length c (the caller's ring).  Returns (r', r_t, H_t)."""
    n = len(descs)
    arr = (Desc * max(n, 1))(*descs)
    qp, keep = _ptr_array(list(q_bars)) if n else (None, None)
    rp = C.c_int32(0 if rprime is None else rprime)
    r_next, h_next = C.c_int32(0), C.c_int32(0)
    _check(lib().dlcx_select_rank(arr, qp, n, tau, C.addressof(rprime_hist), t, c, r1, rmin, rmax,
                                  H1, C.addressof(rp), C.addressof(r_next), C.addressof(h_next),
                                  _ptr(workspace), _stream(stream) if n else None),
           "dlcx_select_rank")
    return rp.value, r_next.value, h_next.value


def dlcx_select_rank_from(rprime_dev, n, rprime_hist, t, c, r1, rmin, rmax, H1, rprime=None,
                          stream=None):
    """Window rule on r' values already measured into the device int32 tensor rprime_dev."""
    rp = C.c_int32(0 if rprime is None else rprime)
    r_next, h_next = C.c_int32(0), C.c_int32(0)
    _check(lib().dlcx_select_rank_from(_ptr(rprime_dev) if n else None, n,
                                       C.addressof(rprime_hist), t, c, r1, rmin, rmax, H1,
                                       C.addressof(rp), C.addressof(r_next), C.addressof(h_next),
                                       _stream(stream) if n else None), "dlcx_select_rank_from")
    return rp.value, r_next.value, h_next.value


def dlcx_batched_workspace_bytes(descs):
    arr = (Desc * max(len(descs), 1))(*descs)
    return lib().dlcx_batched_workspace_bytes(arr, len(descs))


def dlcx_orthonormalize_batched(descs, p_inout, workspace, stream=None):
    arr = (Desc * max(len(descs), 1))(*descs)
    pp, keep = _ptr_array(list(p_inout))
    _check(lib().dlcx_orthonormalize_batched(arr, pp, len(descs), _ptr(workspace), _stream(stream)),
           "dlcx_orthonormalize_batched")


def dlcx_effective_rank_batched(descs, q_bars, tau, rprime_out_dev, workspace, stream=None):
    arr = (Desc * max(len(descs), 1))(*descs)
    qp, keep = _ptr_array(list(q_bars))
    _check(lib().dlcx_effective_rank_batched(arr, qp, len(descs), tau, _ptr(rprime_out_dev),
                                             _ptr(workspace), _stream(stream)),
           "dlcx_effective_rank_batched")


def dlcx_project(d, phase, deltas, basis, factors_out, workspace, stream=None):
    dp, k1 = _ptr_array(deltas)
    fp, k2 = _ptr_array(factors_out)
    _check(lib().dlcx_project(C.byref(d), phase, len(deltas), dp, _ptr(basis), fp, _ptr(workspace),
                              _stream(stream)), "dlcx_project")


def dlcx_quantize(x, qbits, group, codes_out, scales_out, count=None, stream=None):
    n = x.numel() if count is None else count
    _check(lib().dlcx_quantize(_ptr(x), n, qbits, group, _ptr(codes_out), _ptr(scales_out),
                               _stream(stream)), "dlcx_quantize")


def dlcx_dequant_average(codes, scales, count, qbits, group, mean_out, stream=None):
    cp, k1 = _ptr_array(codes)
    sp, k2 = _ptr_array(scales)
    _check(lib().dlcx_dequant_average(len(codes), cp, sp, count, qbits, group, _ptr(mean_out),
                                      _stream(stream)), "dlcx_dequant_average")


def dlcx_orthonormalize(L, r, p_inout, workspace, stream=None):
    _check(lib().dlcx_orthonormalize(L, r, _ptr(p_inout), _ptr(workspace), _stream(stream)),
           "dlcx_orthonormalize")


def dlcx_effective_rank(L, r, q_bar, tau, rprime_out_dev, workspace, stream=None):
    _check(lib().dlcx_effective_rank(L, r, _ptr(q_bar), tau, _ptr(rprime_out_dev),
                                     _ptr(workspace), _stream(stream)), "dlcx_effective_rank")


def dlcx_profile_enable(on):
    _check(lib().dlcx_profile_enable(1 if on else 0), "dlcx_profile_enable")


def dlcx_profile_read():
    """{kernel name: (total ms, launches)} of the launches recorded since dlcx_profile_enable(1)."""
    out = {}
    for kid in range(lib().dlcx_profile_kernels()):
        ms, cnt = C.c_double(0.0), C.c_int64(0)
        _check(lib().dlcx_profile_read(kid, C.addressof(ms), C.addressof(cnt)), "dlcx_profile_read")
        if cnt.value:
            out[lib().dlcx_profile_name(kid).decode()] = (ms.value, cnt.value)
    return out
