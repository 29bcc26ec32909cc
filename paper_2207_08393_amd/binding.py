"""Thin ctypes binding of libgleam.so: argument marshalling only.

Every function has the name and argument order of its C declaration in include/gleam.h and
forwards device pointers of torch tensors (torch is used for device memory and streams only).
There is no CPU path: if the shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgleam.so")

GLEAM_OK = 0
GLEAM_E_NULL = -1
GLEAM_E_DIMS = -2
GLEAM_E_UNSUPPORTED_SIZE = -3
GLEAM_E_WORKSPACE = -4
GLEAM_E_DESC = -5
GLEAM_E_LAUNCH = -6


class gleam_geom(C.Structure):
    _fields_ = [("ndim_fft", C.c_int32), ("centred", C.c_int32), ("B", C.c_int64), ("C", C.c_int64), ("T", C.c_int64),
                ("D", C.c_int64), ("H", C.c_int64), ("W", C.c_int64)]


class gleam_conv(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("cin", "cout", "kt", "kd", "kh", "kw", "relu_in", "relu_out",
                                         "has_bias", "skip_src")]


class gleam_prox_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(gleam_conv)), ("dtype", C.c_int32),
                ("loss_kind", C.c_int32)]


class gleam_kernel_record(C.Structure):
    _fields_ = [("name", C.c_char * 56), ("flops", C.c_double), ("bytes", C.c_double), ("mfma_flops", C.c_double),
                ("ms", C.c_float)]


class gleam_adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float)]


class GleamError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """Loads libgleam.so (built by paper_2207_08393_amd/csrc/build.sh); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run paper_2207_08393_amd/csrc/build.sh "
                               "(or __graft_entry__.build()); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, sz = C.c_void_p, C.c_size_t
        pg, pp = C.POINTER(gleam_geom), C.POINTER(gleam_prox_desc)
        L.gleam_strerror.restype = C.c_char_p
        L.gleam_strerror.argtypes = [C.c_int]
        L.gleam_fft_size_supported.argtypes = [C.c_int64]
        L.gleam_set_kernel_policy.argtypes = [C.c_uint32]
        L.gleam_get_kernel_policy.argtypes = []
        L.gleam_get_kernel_policy.restype = C.c_uint32
        L.gleam_theta_count.argtypes = [pp, C.POINTER(sz)]
        L.gleam_workspace_bytes.argtypes = [pg, pp, C.POINTER(sz), C.POINTER(sz)]
        L.gleam_sense_normal.argtypes = [pg, vp, vp, vp, vp, vp, sz, vp]
        L.gleam_sense_normal_static.argtypes = [pg, vp, vp, vp, vp, vp]
        L.gleam_module_fwd.argtypes = [pg, pp, vp, vp, vp, vp, C.c_float, vp, vp, vp, vp, vp, sz, vp, sz, vp]
        L.gleam_module_bwd.argtypes = [pg, pp, vp, vp, sz, vp, vp, sz, vp]
        L.gleam_module_bwd_alpha.argtypes = [pg, pp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, sz, vp]
        L.gleam_deep_workspace_bytes.argtypes = [pg, pp, C.c_int, C.POINTER(sz), C.POINTER(sz)]
        L.gleam_deep_module_fwd.argtypes = [pg, pp, C.c_int, vp, vp, vp, vp, C.c_float, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp]
        L.gleam_deep_module_bwd.argtypes = [pg, pp, C.c_int, vp, vp, C.c_float, vp, vp, sz, vp, vp, sz, vp]
        L.gleam_sense_adjoint.argtypes = [pg, vp, vp, vp, vp, vp, sz, vp]
        L.gleam_kspace_to_hybrid.argtypes = [pg, vp, vp, vp]
        L.gleam_mask_constant_along_outer_axis.argtypes = [pg, vp, C.POINTER(C.c_int)]
        L.gleam_modl_workspace_bytes.argtypes = [pg, pp, C.POINTER(sz), C.POINTER(sz)]
        L.gleam_modl_module_fwd.argtypes = [pg, pp, vp, vp, vp, vp, C.c_float, C.c_int, vp, vp, vp, vp, vp, sz, vp, sz, vp]
        L.gleam_modl_module_bwd.argtypes = [pg, pp, vp, vp, C.c_float, C.c_int, vp, vp, sz, vp, vp, sz, vp]
        L.gleam_adam_step.argtypes = [C.POINTER(gleam_adam), C.c_int64, sz, vp, vp, vp, vp, vp]
        L.gleam_greedy_iteration.argtypes = [pg, pp, C.c_int, vp, vp, vp, vp, C.c_float, vp, vp, vp, C.POINTER(gleam_adam),
                                             C.c_int64, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp]
        L.gleam_unrolled_infer.argtypes = [pg, pp, C.c_int, vp, vp, vp, vp, C.c_float, vp, vp, vp, vp, sz, vp]
        L.gleam_profile_begin.argtypes = []
        L.gleam_profile_end.argtypes = [C.POINTER(gleam_kernel_record), C.c_int, C.POINTER(C.c_int)]
        _lib = L
    return _lib


EXPORTS = ("gleam_strerror", "gleam_fft_size_supported", "gleam_set_kernel_policy", "gleam_get_kernel_policy", "gleam_theta_count", "gleam_workspace_bytes",
           "gleam_sense_normal", "gleam_sense_normal_static", "gleam_module_fwd", "gleam_module_bwd", "gleam_module_bwd_alpha", "gleam_deep_workspace_bytes",
           "gleam_deep_module_fwd", "gleam_deep_module_bwd", "gleam_sense_adjoint", "gleam_kspace_to_hybrid",
           "gleam_mask_constant_along_outer_axis", "gleam_modl_workspace_bytes",
           "gleam_modl_module_fwd", "gleam_modl_module_bwd", "gleam_adam_step",
           "gleam_greedy_iteration", "gleam_unrolled_infer", "gleam_profile_begin", "gleam_profile_end")


def strerror(status: int) -> str:
    return lib().gleam_strerror(int(status)).decode()


def make_geom(g) -> gleam_geom:
    """From any object with ndim_fft, B, C, T, D, H, W (and optionally centred) attributes."""
    return gleam_geom(int(g.ndim_fft), int(getattr(g, "centred", 0)), int(g.B), int(g.C), int(g.T), int(g.D), int(g.H), int(g.W))


def make_prox(p) -> gleam_prox_desc:
    """From any object with `layers` (cin, cout, kt, kd, kh, kw, relu_in, relu_out, has_bias, skip_src),
    `dtype` and `loss_kind`.  The returned struct keeps its layer array alive."""
    arr = (gleam_conv * len(p.layers))()
    for i, l in enumerate(p.layers):
        arr[i] = gleam_conv(l.cin, l.cout, l.kt, l.kd, l.kh, l.kw, l.relu_in, l.relu_out, l.has_bias, l.skip_src)
    d = gleam_prox_desc(len(p.layers), C.cast(arr, C.POINTER(gleam_conv)), int(p.dtype), int(p.loss_kind))
    d._keep = arr
    return d


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors passed to libgleam must be contiguous")
    return t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(rc: int, where: str):
    if rc != GLEAM_OK:
        raise GleamError(rc, where)


POLICY_NO_WINOGRAD, POLICY_NO_BF16_2D, POLICY_NO_THIN_MFMA, POLICY_NO_WGRAD_BALANCE, POLICY_NO_FRAME_WALK = 1, 2, 4, 8, 16


def gleam_set_kernel_policy(policy: int):
    _check(lib().gleam_set_kernel_policy(int(policy)), "gleam_set_kernel_policy")


def gleam_get_kernel_policy() -> int:
    return int(lib().gleam_get_kernel_policy())


def gleam_fft_size_supported(n: int) -> bool:
    return bool(lib().gleam_fft_size_supported(int(n)))


def gleam_theta_count(prox: gleam_prox_desc) -> int:
    n = C.c_size_t(0)
    _check(lib().gleam_theta_count(C.byref(prox), C.byref(n)), "gleam_theta_count")
    return n.value


def gleam_workspace_bytes(geom: gleam_geom, prox: Optional[gleam_prox_desc]):
    ws, saved = C.c_size_t(0), C.c_size_t(0)
    _check(lib().gleam_workspace_bytes(C.byref(geom), C.byref(prox) if prox is not None else None,
                                       C.byref(ws), C.byref(saved)), "gleam_workspace_bytes")
    return ws.value, saved.value


def gleam_sense_normal(geom, x, S, M, out, ws, stream=None):
    _check(lib().gleam_sense_normal(C.byref(geom), _ptr(x), _ptr(S), _ptr(M), _ptr(out), _ptr(ws), _nbytes(ws),
                                    _stream(stream)), "gleam_sense_normal")


STATIC_SCRATCH_BYTES = 64 << 20   # GLEAM_STATIC_SCRATCH_BYTES of include/gleam.h


def gleam_sense_normal_static(geom, x, S, M, out, stream=None):
    _check(lib().gleam_sense_normal_static(C.byref(geom), _ptr(x), _ptr(S), _ptr(M), _ptr(out), _stream(stream)),
           "gleam_sense_normal_static")


def gleam_module_fwd(geom, prox, x_in, S, M, y, alpha, theta, x_ref, x_out, loss, saved, ws, stream=None):
    _check(lib().gleam_module_fwd(C.byref(geom), C.byref(prox), _ptr(x_in), _ptr(S), _ptr(M), _ptr(y),
                                  C.c_float(alpha), _ptr(theta), _ptr(x_ref), _ptr(x_out), _ptr(loss),
                                  _ptr(saved), _nbytes(saved), _ptr(ws), _nbytes(ws), _stream(stream)),
           "gleam_module_fwd")


def gleam_module_bwd(geom, prox, theta, saved, grad_theta, ws, stream=None):
    _check(lib().gleam_module_bwd(C.byref(geom), C.byref(prox), _ptr(theta), _ptr(saved), _nbytes(saved),
                                  _ptr(grad_theta), _ptr(ws), _nbytes(ws), _stream(stream)), "gleam_module_bwd")


def gleam_module_bwd_alpha(geom, prox, x_in, S, M, y, theta, saved, grad_theta, grad_alpha, ws, stream=None):
    _check(lib().gleam_module_bwd_alpha(C.byref(geom), C.byref(prox), _ptr(x_in), _ptr(S), _ptr(M), _ptr(y), _ptr(theta),
                                        _ptr(saved), _nbytes(saved), _ptr(grad_theta), _ptr(grad_alpha), _ptr(ws),
                                        _nbytes(ws), _stream(stream)), "gleam_module_bwd_alpha")


def gleam_deep_workspace_bytes(geom, prox, n_iter):
    ws, saved = C.c_size_t(0), C.c_size_t(0)
    _check(lib().gleam_deep_workspace_bytes(C.byref(geom), C.byref(prox), int(n_iter), C.byref(ws), C.byref(saved)),
           "gleam_deep_workspace_bytes")
    return ws.value, saved.value


def gleam_deep_module_fwd(geom, prox, n_iter, x_in, S, M, y, alpha, theta, x_ref, x_out, x_tmp, loss, saved, ws, stream=None):
    _check(lib().gleam_deep_module_fwd(C.byref(geom), C.byref(prox), int(n_iter), _ptr(x_in), _ptr(S), _ptr(M), _ptr(y),
                                       C.c_float(alpha), _ptr(theta), _ptr(x_ref), _ptr(x_out), _ptr(x_tmp), _ptr(loss),
                                       _ptr(saved), _nbytes(saved), _ptr(ws), _nbytes(ws), _stream(stream)),
           "gleam_deep_module_fwd")


def gleam_deep_module_bwd(geom, prox, n_iter, S, M, alpha, theta, saved, grad_theta, ws, stream=None):
    _check(lib().gleam_deep_module_bwd(C.byref(geom), C.byref(prox), int(n_iter), _ptr(S), _ptr(M), C.c_float(alpha),
                                       _ptr(theta), _ptr(saved), _nbytes(saved), _ptr(grad_theta), _ptr(ws), _nbytes(ws),
                                       _stream(stream)), "gleam_deep_module_bwd")


def gleam_sense_adjoint(geom, S, M, y, out, ws, stream=None):
    _check(lib().gleam_sense_adjoint(C.byref(geom), _ptr(S), _ptr(M), _ptr(y), _ptr(out), _ptr(ws), _nbytes(ws),
                                     _stream(stream)), "gleam_sense_adjoint")


def gleam_kspace_to_hybrid(geom, y_in, y_out, stream=None):
    _check(lib().gleam_kspace_to_hybrid(C.byref(geom), _ptr(y_in), _ptr(y_out), _stream(stream)), "gleam_kspace_to_hybrid")


def gleam_mask_constant_along_outer_axis(geom, mask_host) -> bool:
    """mask_host: contiguous uint8 numpy array [B][T][D][H][W] in host memory."""
    import numpy as np
    m = np.ascontiguousarray(mask_host, dtype=np.uint8)
    if m.size != geom.B * geom.T * geom.D * geom.H * geom.W:
        raise ValueError("mask size does not match the geometry")
    out = C.c_int(0)
    _check(lib().gleam_mask_constant_along_outer_axis(C.byref(geom), m.ctypes.data_as(C.c_void_p), C.byref(out)),
           "gleam_mask_constant_along_outer_axis")
    return bool(out.value)


def gleam_modl_workspace_bytes(geom, prox):
    ws, saved = C.c_size_t(0), C.c_size_t(0)
    _check(lib().gleam_modl_workspace_bytes(C.byref(geom), C.byref(prox), C.byref(ws), C.byref(saved)),
           "gleam_modl_workspace_bytes")
    return ws.value, saved.value


def gleam_modl_module_fwd(geom, prox, x_in, S, M, aty, mu, n_cg, theta, x_ref, x_out, loss, saved, ws, stream=None):
    _check(lib().gleam_modl_module_fwd(C.byref(geom), C.byref(prox), _ptr(x_in), _ptr(S), _ptr(M), _ptr(aty), C.c_float(mu),
                                       int(n_cg), _ptr(theta), _ptr(x_ref), _ptr(x_out), _ptr(loss), _ptr(saved),
                                       _nbytes(saved), _ptr(ws), _nbytes(ws), _stream(stream)), "gleam_modl_module_fwd")


def gleam_modl_module_bwd(geom, prox, S, M, mu, n_cg, theta, saved, grad_theta, ws, stream=None):
    _check(lib().gleam_modl_module_bwd(C.byref(geom), C.byref(prox), _ptr(S), _ptr(M), C.c_float(mu), int(n_cg),
                                       _ptr(theta), _ptr(saved), _nbytes(saved), _ptr(grad_theta), _ptr(ws), _nbytes(ws),
                                       _stream(stream)), "gleam_modl_module_bwd")


def make_adam(lr, beta1=0.9, beta2=0.999, eps=1e-8) -> gleam_adam:
    return gleam_adam(float(lr), float(beta1), float(beta2), float(eps))


def gleam_adam_step(hyper, t, theta, grad, m, v, stream=None):
    _check(lib().gleam_adam_step(C.byref(hyper), int(t), theta.numel(), _ptr(theta), _ptr(grad), _ptr(m), _ptr(v),
                                 _stream(stream)), "gleam_adam_step")


def gleam_greedy_iteration(geom, prox, n_modules, x0, S, M, y, alpha, theta, adam_m, adam_v, hyper, t, x_ref, x_out,
                           x_tmp, losses, grad, saved, ws, stream=None):
    _check(lib().gleam_greedy_iteration(C.byref(geom), C.byref(prox), int(n_modules), _ptr(x0), _ptr(S), _ptr(M), _ptr(y),
                                        C.c_float(alpha), _ptr(theta), _ptr(adam_m), _ptr(adam_v), C.byref(hyper), int(t),
                                        _ptr(x_ref), _ptr(x_out), _ptr(x_tmp), _ptr(losses), _ptr(grad), _ptr(saved),
                                        _nbytes(saved), _ptr(ws), _nbytes(ws), _stream(stream)), "gleam_greedy_iteration")


def gleam_unrolled_infer(geom, prox, n_modules, x0, S, M, y, alpha, theta, x_out, x_tmp, ws, stream=None):
    _check(lib().gleam_unrolled_infer(C.byref(geom), C.byref(prox), int(n_modules), _ptr(x0), _ptr(S), _ptr(M), _ptr(y),
                                      C.c_float(alpha), _ptr(theta), _ptr(x_out), _ptr(x_tmp), _ptr(ws), _nbytes(ws),
                                      _stream(stream)), "gleam_unrolled_infer")


def gleam_profile_begin():
    _check(lib().gleam_profile_begin(), "gleam_profile_begin")


def gleam_profile_end(capacity: int = 65536):
    """Returns a list of (name, flops, bytes, ms, mfma_flops), one per kernel launch since gleam_profile_begin."""
    arr = (gleam_kernel_record * capacity)()
    n = C.c_int(0)
    _check(lib().gleam_profile_end(arr, capacity, C.byref(n)), "gleam_profile_end")
    return [(arr[i].name.decode(), arr[i].flops, arr[i].bytes, arr[i].ms, arr[i].mfma_flops)
            for i in range(min(n.value, capacity))]
