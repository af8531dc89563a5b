"""ctypes front end of the CPU oracle (oracle/bd_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.

All arrays are host numpy arrays.  binary16 tensors are passed as np.float16 (or
np.uint16 bit patterns); packed signs are np.uint32 [out, in/32] with the least
significant bit first along `in` and bit 1 meaning +1 (Eq. 2 of the paper).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bd_ref.cpp")
_LIB = os.path.join(_HERE, "libbd_ref.so")


def build(force: bool = False) -> str:
    """Compile bd_ref.cpp with g++ (no HIP, no GPU headers)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c_u16p = ctypes.POINTER(ctypes.c_uint16)
        c_u32p = ctypes.POINTER(ctypes.c_uint32)
        c_f32p = ctypes.POINTER(ctypes.c_float)
        c_f64p = ctypes.POINTER(ctypes.c_double)
        c_i32p = ctypes.POINTER(ctypes.c_int32)
        c_i8p = ctypes.POINTER(ctypes.c_int8)
        i64 = ctypes.c_int64
        L.bd_ref_f16_to_f32.restype = ctypes.c_float
        L.bd_ref_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.bd_ref_f32_to_f16.restype = ctypes.c_uint16
        L.bd_ref_f32_to_f16.argtypes = [ctypes.c_float]
        L.bd_ref_f64_to_f16.restype = ctypes.c_uint16
        L.bd_ref_f64_to_f16.argtypes = [ctypes.c_double]
        L.bd_ref_num_threads.restype = ctypes.c_int
        L.bd_ref_pack_signs.argtypes = [c_u16p, i64, i64, c_u32p]
        L.bd_ref_unpack_signs.argtypes = [c_u32p, i64, i64, c_i8p]
        L.bd_ref_compress.argtypes = [c_u16p, c_u16p, i64, i64, c_u32p, c_f32p, c_f64p]
        L.bd_ref_linear_multitenant.argtypes = [c_u16p, c_u16p, ctypes.POINTER(c_u32p), c_f32p, c_i32p,
                                                c_u16p, c_f32p, i64, i64, i64, ctypes.c_int32]
        L.bd_ref_linear_multitenant_f64.argtypes = [c_u16p, c_u16p, ctypes.POINTER(c_u32p), c_f32p, c_i32p,
                                                    c_f64p, i64, i64, i64, ctypes.c_int32]
        L.bd_ref_compress_iterated.argtypes = [c_u16p, c_u16p, i64, i64, ctypes.c_int32, c_u32p, c_f32p, c_f64p, c_f64p]
        L.bd_ref_linear_multitenant_kbit.argtypes = [c_u16p, c_u16p, ctypes.POINTER(c_u32p), c_f32p, c_i32p,
                                                     c_u16p, c_f32p, i64, i64, i64, ctypes.c_int32, ctypes.c_int32]
        L.bd_ref_linear_multitenant_kbit_f64.argtypes = [c_u16p, c_u16p, ctypes.POINTER(c_u32p), c_f32p, c_i32p,
                                                         c_f64p, i64, i64, i64, ctypes.c_int32, ctypes.c_int32]
        L.bd_ref_quantize_rtn8.argtypes = [c_u16p, i64, i64, c_i8p, c_f32p]
        L.bd_ref_compress_q8.argtypes = [c_i8p, c_f32p, c_u16p, i64, i64, c_u32p, c_f32p, c_f64p]
        L.bd_ref_linear_multitenant_q8.argtypes = [c_u16p, c_i8p, c_f32p, ctypes.POINTER(c_u32p), c_f32p, c_i32p,
                                                   c_u16p, c_f32p, i64, i64, i64, ctypes.c_int32]
        L.bd_ref_linear_multitenant_q8_f64.argtypes = [c_u16p, c_i8p, c_f32p, ctypes.POINTER(c_u32p), c_f32p, c_i32p,
                                                       c_f64p, i64, i64, i64, ctypes.c_int32]
        L.bd_ref_linear_materialised.argtypes = [c_u16p, c_u16p, c_u32p, ctypes.c_float, c_f32p, c_f32p,
                                                 i64, i64, i64]
        L.bd_ref_linear_naive.argtypes = [c_u16p, ctypes.POINTER(c_u16p), c_i32p, c_u16p, c_f32p,
                                          i64, i64, i64, ctypes.c_int32]
        L.bd_ref_materialise_f16.argtypes = [c_u16p, c_u32p, ctypes.c_float, c_u16p, i64, i64]
        _lib = L
    return _lib


def _u16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype == np.uint16:
        return a
    raise TypeError(f"expected float16/uint16, got {a.dtype}")


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def num_threads() -> int:
    return int(lib().bd_ref_num_threads())


def f16_to_f32(bits: int) -> float:
    return float(lib().bd_ref_f16_to_f32(int(bits)))


def f32_to_f16(v: float) -> int:
    return int(lib().bd_ref_f32_to_f16(float(v)))


def f64_to_f16(v: float) -> int:
    """binary64 -> binary16 bits, one rounding to nearest even (what the scale of Eq. 4 goes through)."""
    return int(lib().bd_ref_f64_to_f16(float(v)))


def pack_signs(delta: np.ndarray) -> np.ndarray:
    d = _u16(delta)
    out, inn = d.shape
    packed = np.empty((out, inn // 32 if inn % 32 == 0 else 0), dtype=np.uint32)
    rc = lib().bd_ref_pack_signs(_p(d, ctypes.c_uint16), out, inn, _p(packed, ctypes.c_uint32))
    if rc != 0:
        raise ValueError("in must be a multiple of 32")
    return packed


def unpack_signs(packed: np.ndarray, inn: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    out = packed.shape[0]
    signs = np.empty((out, inn), dtype=np.int8)
    rc = lib().bd_ref_unpack_signs(_p(packed, ctypes.c_uint32), out, inn, _p(signs, ctypes.c_int8))
    if rc != 0:
        raise ValueError("in must be a multiple of 32")
    return signs


def compress(w_base: np.ndarray, w_ft: np.ndarray):
    """Returns (packed uint32 [out,in/32], alpha as float (binary16-representable), mean before rounding)."""
    b, f = _u16(w_base), _u16(w_ft)
    assert b.shape == f.shape
    out, inn = b.shape
    if inn % 32 != 0:
        raise ValueError("in must be a multiple of 32")
    packed = np.empty((out, inn // 32), dtype=np.uint32)
    alpha = ctypes.c_float(0.0)
    mean = ctypes.c_double(0.0)
    rc = lib().bd_ref_compress(_p(b, ctypes.c_uint16), _p(f, ctypes.c_uint16), out, inn,
                               _p(packed, ctypes.c_uint32), ctypes.byref(alpha), ctypes.byref(mean))
    assert rc == 0
    return packed, float(alpha.value), float(mean.value)


def compress_iterated(w_base: np.ndarray, w_ft: np.ndarray, k: int):
    """The compressor iterated k times (Sec. 4.2, fidelity of Delta).  Returns (packed uint32 [k,out,in/32],
    alpha float32 [k] (binary16-representable), means before rounding float64 [k], residual sum of squares
    float64 [k+1] before each iteration and after the last)."""
    b, f = _u16(w_base), _u16(w_ft)
    assert b.shape == f.shape
    out, inn = b.shape
    if inn % 32 != 0 or k < 1:
        raise ValueError("in must be a multiple of 32 and k >= 1")
    packed = np.empty((k, out, inn // 32), dtype=np.uint32)
    alpha = np.empty(k, dtype=np.float32)
    mean = np.empty(k, dtype=np.float64)
    rsq = np.empty(k + 1, dtype=np.float64)
    rc = lib().bd_ref_compress_iterated(_p(b, ctypes.c_uint16), _p(f, ctypes.c_uint16), out, inn, k,
                                        _p(packed, ctypes.c_uint32), _p(alpha, ctypes.c_float),
                                        _p(mean, ctypes.c_double), _p(rsq, ctypes.c_double))
    assert rc == 0
    return packed, alpha, mean, rsq


def _kbit_args(x, w_base, planes_by_tenant, alpha_by_tenant, tenant_of_token):
    xb, wb = _u16(x), _u16(w_base)
    T, inn = xb.shape
    out = wb.shape[0]
    assert wb.shape[1] == inn
    k = len(planes_by_tenant[0])
    flat = []
    for planes in planes_by_tenant:
        assert len(planes) == k
        for p in planes:
            p = np.ascontiguousarray(p, dtype=np.uint32)
            assert p.shape == (out, inn // 32)
            flat.append(p)
    ptrs, keep = _tenant_ptrs(flat, ctypes.c_uint32)
    alpha = np.ascontiguousarray(alpha_by_tenant, dtype=np.float32)
    assert alpha.shape == (len(planes_by_tenant), k)
    tok = np.ascontiguousarray(tenant_of_token, dtype=np.int32)
    assert tok.shape == (T,)
    return xb, wb, T, out, inn, k, ptrs, keep, alpha, tok


def linear_multitenant_kbit(x, w_base, planes_by_tenant, alpha_by_tenant, tenant_of_token):
    """Eq. 6 with k sign planes per tenant: planes_by_tenant[e][j] uint32 [out,in/32], alpha_by_tenant [n_tenants,k].
    Returns (y float16 [T,out], y float32 before rounding)."""
    xb, wb, T, out, inn, k, ptrs, keep, alpha, tok = _kbit_args(x, w_base, planes_by_tenant, alpha_by_tenant, tenant_of_token)
    y16 = np.empty((T, out), dtype=np.uint16)
    y32 = np.empty((T, out), dtype=np.float32)
    rc = lib().bd_ref_linear_multitenant_kbit(_p(xb, ctypes.c_uint16), _p(wb, ctypes.c_uint16), ptrs,
                                              _p(alpha, ctypes.c_float), _p(tok, ctypes.c_int32),
                                              _p(y16, ctypes.c_uint16), _p(y32, ctypes.c_float),
                                              T, out, inn, len(planes_by_tenant), k)
    if rc == -1:
        raise ValueError("in must be a multiple of 32")
    if rc == -2:
        raise IndexError("tenant id out of range")
    del keep
    return y16.view(np.float16), y32


def linear_multitenant_kbit_f64(x, w_base, planes_by_tenant, alpha_by_tenant, tenant_of_token):
    xb, wb, T, out, inn, k, ptrs, keep, alpha, tok = _kbit_args(x, w_base, planes_by_tenant, alpha_by_tenant, tenant_of_token)
    y = np.empty((T, out), dtype=np.float64)
    rc = lib().bd_ref_linear_multitenant_kbit_f64(_p(xb, ctypes.c_uint16), _p(wb, ctypes.c_uint16), ptrs,
                                                  _p(alpha, ctypes.c_float), _p(tok, ctypes.c_int32),
                                                  _p(y, ctypes.c_double), T, out, inn, len(planes_by_tenant), k)
    if rc == -1:
        raise ValueError("in must be a multiple of 32")
    if rc == -2:
        raise IndexError("tenant id out of range")
    del keep
    return y


def quantize_rtn8(w: np.ndarray):
    """8-bit round-to-nearest base (Sec. 4.2, quantized base models): returns (q int8 [out,in], scale float32 [out])."""
    wb = _u16(w)
    out, inn = wb.shape
    q = np.empty((out, inn), dtype=np.int8)
    scale = np.empty(out, dtype=np.float32)
    assert lib().bd_ref_quantize_rtn8(_p(wb, ctypes.c_uint16), out, inn, _p(q, ctypes.c_int8), _p(scale, ctypes.c_float)) == 0
    return q, scale


def compress_q8(q: np.ndarray, scale: np.ndarray, w_ft: np.ndarray):
    """The 1-bit compressor against the quantised base scale[n] * q[n,k]: (packed, alpha, mean before rounding)."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    f = _u16(w_ft)
    out, inn = f.shape
    assert q.shape == (out, inn) and scale.shape == (out,)
    if inn % 32 != 0:
        raise ValueError("in must be a multiple of 32")
    packed = np.empty((out, inn // 32), dtype=np.uint32)
    alpha, mean = ctypes.c_float(0.0), ctypes.c_double(0.0)
    rc = lib().bd_ref_compress_q8(_p(q, ctypes.c_int8), _p(scale, ctypes.c_float), _p(f, ctypes.c_uint16), out, inn,
                                  _p(packed, ctypes.c_uint32), ctypes.byref(alpha), ctypes.byref(mean))
    assert rc == 0
    return packed, float(alpha.value), float(mean.value)


def _q8_args(x, q, scale, packed_by_tenant, alpha_by_tenant, tenant_of_token):
    xb = _u16(x)
    q = np.ascontiguousarray(q, dtype=np.int8)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    T, inn = xb.shape
    out = q.shape[0]
    assert q.shape == (out, inn) and scale.shape == (out,)
    packed = [np.ascontiguousarray(p, dtype=np.uint32) for p in packed_by_tenant]
    for p in packed:
        assert p.shape == (out, inn // 32)
    ptrs, keep = _tenant_ptrs(packed, ctypes.c_uint32)
    alpha = np.ascontiguousarray(alpha_by_tenant, dtype=np.float32)
    tok = np.ascontiguousarray(tenant_of_token, dtype=np.int32)
    assert tok.shape == (T,)
    return xb, q, scale, T, out, inn, ptrs, keep, alpha, tok, len(packed)


def linear_multitenant_q8(x, q, scale, packed_by_tenant, alpha_by_tenant, tenant_of_token):
    """Eq. 6 over the quantised base.  Returns (y float16 [T,out], y float32 before rounding)."""
    xb, q, scale, T, out, inn, ptrs, keep, alpha, tok, nt = _q8_args(x, q, scale, packed_by_tenant, alpha_by_tenant, tenant_of_token)
    y16 = np.empty((T, out), dtype=np.uint16)
    y32 = np.empty((T, out), dtype=np.float32)
    rc = lib().bd_ref_linear_multitenant_q8(_p(xb, ctypes.c_uint16), _p(q, ctypes.c_int8), _p(scale, ctypes.c_float), ptrs,
                                            _p(alpha, ctypes.c_float), _p(tok, ctypes.c_int32), _p(y16, ctypes.c_uint16),
                                            _p(y32, ctypes.c_float), T, out, inn, nt)
    if rc == -1:
        raise ValueError("in must be a multiple of 32")
    if rc == -2:
        raise IndexError("tenant id out of range")
    del keep
    return y16.view(np.float16), y32


def linear_multitenant_q8_f64(x, q, scale, packed_by_tenant, alpha_by_tenant, tenant_of_token):
    xb, q, scale, T, out, inn, ptrs, keep, alpha, tok, nt = _q8_args(x, q, scale, packed_by_tenant, alpha_by_tenant, tenant_of_token)
    y = np.empty((T, out), dtype=np.float64)
    rc = lib().bd_ref_linear_multitenant_q8_f64(_p(xb, ctypes.c_uint16), _p(q, ctypes.c_int8), _p(scale, ctypes.c_float), ptrs,
                                                _p(alpha, ctypes.c_float), _p(tok, ctypes.c_int32), _p(y, ctypes.c_double),
                                                T, out, inn, nt)
    if rc == -1:
        raise ValueError("in must be a multiple of 32")
    if rc == -2:
        raise IndexError("tenant id out of range")
    del keep
    return y


def _tenant_ptrs(arrs: Sequence[np.ndarray], ctype):
    keep = [np.ascontiguousarray(a) for a in arrs]
    PT = ctypes.POINTER(ctype)
    ptrs = (PT * len(keep))(*[_p(a, ctype) for a in keep])
    return ptrs, keep


def linear_multitenant(x, w_base, packed_by_tenant, alpha_by_tenant, tenant_of_token):
    """Eq. 6, fused form, binary32 accumulation.  Returns (y float16 [T,out], y float32 before rounding)."""
    xb, wb = _u16(x), _u16(w_base)
    T, inn = xb.shape
    out = wb.shape[0]
    assert wb.shape[1] == inn
    packed = [np.ascontiguousarray(p, dtype=np.uint32) for p in packed_by_tenant]
    for p in packed:
        assert p.shape == (out, inn // 32)
    ptrs, keep = _tenant_ptrs(packed, ctypes.c_uint32)
    alpha = np.ascontiguousarray(alpha_by_tenant, dtype=np.float32)
    tok = np.ascontiguousarray(tenant_of_token, dtype=np.int32)
    assert tok.shape == (T,)
    y16 = np.empty((T, out), dtype=np.uint16)
    y32 = np.empty((T, out), dtype=np.float32)
    rc = lib().bd_ref_linear_multitenant(_p(xb, ctypes.c_uint16), _p(wb, ctypes.c_uint16), ptrs,
                                         _p(alpha, ctypes.c_float), _p(tok, ctypes.c_int32),
                                         _p(y16, ctypes.c_uint16), _p(y32, ctypes.c_float),
                                         T, out, inn, len(packed))
    if rc == -1:
        raise ValueError("in must be a multiple of 32")
    if rc == -2:
        raise IndexError("tenant id out of range")
    del keep
    return y16.view(np.float16), y32


def linear_multitenant_f64(x, w_base, packed_by_tenant, alpha_by_tenant, tenant_of_token):
    xb, wb = _u16(x), _u16(w_base)
    T, inn = xb.shape
    out = wb.shape[0]
    packed = [np.ascontiguousarray(p, dtype=np.uint32) for p in packed_by_tenant]
    ptrs, keep = _tenant_ptrs(packed, ctypes.c_uint32)
    alpha = np.ascontiguousarray(alpha_by_tenant, dtype=np.float32)
    tok = np.ascontiguousarray(tenant_of_token, dtype=np.int32)
    y = np.empty((T, out), dtype=np.float64)
    rc = lib().bd_ref_linear_multitenant_f64(_p(xb, ctypes.c_uint16), _p(wb, ctypes.c_uint16), ptrs,
                                             _p(alpha, ctypes.c_float), _p(tok, ctypes.c_int32),
                                             _p(y, ctypes.c_double), T, out, inn, len(packed))
    if rc == -1:
        raise ValueError("in must be a multiple of 32")
    if rc == -2:
        raise IndexError("tenant id out of range")
    del keep
    return y


def linear_materialised(x, w_base, packed, alpha: float):
    """y = x . (f32(W_base) + alpha*s), one tenant; returns (y float32 [T,out], sum_k |x*W_eff| float32)."""
    xb, wb = _u16(x), _u16(w_base)
    T, inn = xb.shape
    out = wb.shape[0]
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    y = np.empty((T, out), dtype=np.float32)
    a = np.empty((T, out), dtype=np.float32)
    rc = lib().bd_ref_linear_materialised(_p(xb, ctypes.c_uint16), _p(wb, ctypes.c_uint16),
                                          _p(packed, ctypes.c_uint32), float(alpha),
                                          _p(y, ctypes.c_float), _p(a, ctypes.c_float), T, out, inn)
    assert rc == 0
    return y, a


def linear_naive(x, w_by_tenant, tenant_of_token):
    xb = _u16(x)
    T, inn = xb.shape
    ws = [_u16(w) for w in w_by_tenant]
    out = ws[0].shape[0]
    ptrs, keep = _tenant_ptrs(ws, ctypes.c_uint16)
    tok = np.ascontiguousarray(tenant_of_token, dtype=np.int32)
    y16 = np.empty((T, out), dtype=np.uint16)
    y32 = np.empty((T, out), dtype=np.float32)
    rc = lib().bd_ref_linear_naive(_p(xb, ctypes.c_uint16), ptrs, _p(tok, ctypes.c_int32),
                                   _p(y16, ctypes.c_uint16), _p(y32, ctypes.c_float), T, out, inn, len(ws))
    if rc == -2:
        raise IndexError("tenant id out of range")
    del keep
    return y16.view(np.float16), y32


def materialise_f16(w_base, packed, alpha: float) -> np.ndarray:
    wb = _u16(w_base)
    out, inn = wb.shape
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    w = np.empty((out, inn), dtype=np.uint16)
    rc = lib().bd_ref_materialise_f16(_p(wb, ctypes.c_uint16), _p(packed, ctypes.c_uint32), float(alpha),
                                      _p(w, ctypes.c_uint16), out, inn)
    assert rc == 0
    return w.view(np.float16)
