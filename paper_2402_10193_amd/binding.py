"""Thin ctypes binding of libbitdelta.so: same names as the C ABI, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the library's
kernels.  There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# BITDELTA_LIB may name another build of the same library (e.g. an instrumented one)
LIB_PATH = os.environ.get("BITDELTA_LIB") or os.path.join(_PKG, "libbitdelta.so")

BD_OK = 0
STATUS_NAMES = {0: "BD_OK", 1: "BD_ERR_NULL", 2: "BD_ERR_SHAPE", 3: "BD_ERR_ALIGN", 4: "BD_ERR_TENANT",
                5: "BD_ERR_WORKSPACE", 6: "BD_ERR_DEVICE", 7: "BD_ERR_UNSUPPORTED", 8: "BD_ERR_ALIAS",
                9: "BD_ERR_FORMAT", 10: "BD_ERR_IO", 11: "BD_ERR_TOO_LARGE"}
OP_PACK_SIGNS, OP_COMPRESS, OP_LINEAR_MULTITENANT, OP_LINEAR_GEMM, OP_LINEAR_TILED_GEMM = 0, 1, 2, 3, 4

# every symbol include/bitdelta.h declares
EXPORTS = ["bd_status_string", "bd_version", "bd_workspace_bytes", "bd_pack_signs", "bd_compress", "bd_compress_noalloc", "bd_compress_batch",
           "bd_group_tokens",
           "bd_linear_multitenant", "bd_linear_multitenant_variant", "bd_materialize", "bd_linear_naive",
           "bd_probe_read", "bd_probe_copy", "bd_tiled_base_bytes", "bd_tiled_signs_bytes", "bd_tile_base",
           "bd_tile_signs", "bd_linear_multitenant_tiled", "bd_linear_multitenant_tiled_gemm", "bd_linear_multitenant_tiled_group",
           "bd_compress_iterated",
           "bd_linear_multitenant_tiled_kbit", "bd_linear_multitenant_tiled_group_kbit", "bd_delta_image_bytes",
           "bd_delta_image_build", "bd_delta_image_check", "bd_delta_image_entry", "bd_delta_file_write",
           "bd_delta_file_bytes", "bd_delta_file_read", "bd_delta_upload", "bd_delta_install", "bd_quantize_base_q8",
           "bd_compress_q8", "bd_tiled_base_q8_bytes", "bd_tile_base_q8", "bd_linear_multitenant_tiled_q8",
           "bd_linear_multitenant_tiled_group_q8", "bd_linear_multitenant_kbit", "bd_linear_multitenant_gemm_kbit",
           "bd_linear_multitenant_gemm_q8", "bd_linear_multitenant_q8"]


class BitDeltaError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (python -m paper_2402_10193_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2402_10193_amd.build` "
                                    "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
        L.bd_status_string.restype = ctypes.c_char_p
        L.bd_status_string.argtypes = [ctypes.c_int]
        L.bd_version.restype = ctypes.c_int
        L.bd_version.argtypes = []
        L.bd_workspace_bytes.restype = sz
        L.bd_workspace_bytes.argtypes = [ctypes.c_int, i64, i64, i64, i32]
        L.bd_pack_signs.argtypes = [vp, i64, i64, vp, vp]
        L.bd_compress.argtypes = [vp, vp, i64, i64, vp, vp, vp, sz, vp]
        L.bd_compress_noalloc.argtypes = [vp, vp, i64, i64, vp, vp, vp]
        L.bd_linear_multitenant.argtypes = [vp, vp, vp, vp, ctypes.POINTER(i32), vp, i64, i64, i64, i32, vp, sz, vp]
        L.bd_linear_multitenant_variant.argtypes = [vp, vp, vp, vp, ctypes.POINTER(i32), vp, i64, i64, i64, i32, vp,
                                                    sz, vp, i32]
        pi = ctypes.POINTER(i32)
        L.bd_group_tokens.argtypes = [pi, i32, pi, pi, pi, pi, pi, pi]
        L.bd_group_tokens.restype = ctypes.c_int
        L.bd_materialize.argtypes = [vp, vp, vp, vp, i64, i64, vp]
        L.bd_linear_naive.argtypes = [vp, vp, ctypes.POINTER(i32), vp, i64, i64, i64, i32, vp]
        L.bd_probe_read.argtypes = [vp, sz, vp, vp]
        L.bd_probe_copy.argtypes = [vp, vp, sz, vp]
        L.bd_tiled_base_bytes.restype = sz
        L.bd_tiled_base_bytes.argtypes = [i64, i64]
        L.bd_tiled_signs_bytes.restype = sz
        L.bd_tiled_signs_bytes.argtypes = [i64, i64]
        L.bd_tile_base.argtypes = [vp, i64, i64, vp, vp]
        L.bd_tile_signs.argtypes = [vp, i64, i64, vp, vp]
        pvp, pi64 = ctypes.POINTER(vp), ctypes.POINTER(i64)
        L.bd_linear_multitenant_tiled.argtypes = [vp, vp, pvp, vp, pi, vp, i64, i64, i64, i32, vp]
        L.bd_linear_multitenant_tiled_group.argtypes = [i32, vp, pvp, pvp, pvp, pi, pvp, i64, pi64, i64, i32, vp]
        L.bd_linear_multitenant_tiled_gemm.argtypes = [vp, vp, pvp, vp, pi, vp, i64, i64, i64, i32, i32, vp, sz, vp]
        L.bd_linear_multitenant_tiled_gemm.restype = ctypes.c_int
        psz = ctypes.POINTER(sz)
        L.bd_delta_image_bytes.restype = sz
        L.bd_delta_image_bytes.argtypes = [i32, pi64, pi64, i32]
        L.bd_delta_image_build.argtypes = [vp, sz, i32, pi64, pi64, i32, pvp, pvp]
        L.bd_delta_image_check.argtypes = [vp, sz, i32, pi, pi]
        L.bd_delta_image_entry.argtypes = [vp, sz, i32, pi64, pi64, psz, psz]
        L.bd_delta_file_write.argtypes = [ctypes.c_char_p, vp, sz]
        L.bd_delta_file_bytes.argtypes = [ctypes.c_char_p, psz]
        L.bd_delta_file_read.argtypes = [ctypes.c_char_p, vp, sz]
        L.bd_delta_upload.argtypes = [vp, sz, vp, vp]
        L.bd_delta_install.argtypes = [vp, sz, vp, i32, i32, pvp, pvp, vp]
        L.bd_quantize_base_q8.argtypes = [vp, i64, i64, vp, vp, vp]
        L.bd_compress_q8.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp, sz, vp]
        L.bd_tiled_base_q8_bytes.restype = sz
        L.bd_tiled_base_q8_bytes.argtypes = [i64, i64]
        L.bd_tile_base_q8.argtypes = [vp, vp, i64, i64, vp, vp]
        L.bd_linear_multitenant_tiled_q8.argtypes = [vp, vp, pvp, vp, pi, vp, i64, i64, i64, i32, vp]
        L.bd_linear_multitenant_tiled_group_q8.argtypes = [i32, vp, pvp, pvp, pvp, pi, pvp, i64, pi64, i64, i32, vp]
        L.bd_compress_iterated.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, sz, vp]
        L.bd_linear_multitenant_kbit.argtypes = [vp, vp, vp, vp, pi, vp, i64, i64, i64, i32, i32, vp]
        L.bd_linear_multitenant_gemm_kbit.argtypes = [vp, vp, vp, vp, pi, vp, i64, i64, i64, i32, i32, vp, sz, vp]
        L.bd_linear_multitenant_gemm_q8.argtypes = [vp, vp, vp, vp, vp, pi, vp, i64, i64, i64, i32, vp, sz, vp]
        L.bd_linear_multitenant_q8.argtypes = [vp, vp, vp, vp, vp, pi, vp, i64, i64, i64, i32, vp]
        L.bd_compress_batch.argtypes = [i32, pvp, pvp, pi64, pi64, pvp, vp, vp, sz, vp]
        L.bd_compress_batch.restype = ctypes.c_int
        L.bd_linear_multitenant_tiled_kbit.argtypes = [vp, vp, pvp, vp, pi, vp, i64, i64, i64, i32, i32, vp]
        L.bd_linear_multitenant_tiled_group_kbit.argtypes = [i32, vp, pvp, pvp, pvp, pi, pvp, i64, pi64, i64, i32, i32, vp]
        for name in ("bd_pack_signs", "bd_compress", "bd_linear_multitenant", "bd_linear_multitenant_variant",
                     "bd_materialize", "bd_linear_naive", "bd_probe_read", "bd_probe_copy", "bd_tile_base",
                     "bd_tile_signs", "bd_linear_multitenant_tiled", "bd_linear_multitenant_tiled_group"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().bd_status_string(int(status)).decode()


def version() -> int:
    return int(lib().bd_version())


def workspace_bytes(op: int, T: int, out: int, inn: int, n_tenants: int) -> int:
    return int(lib().bd_workspace_bytes(int(op), T, out, inn, n_tenants))


def _stream(stream) -> int:
    if stream is None:
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, torch.cuda.Stream):
        return int(stream.cuda_stream)
    return int(stream)


def _ptr(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else int(t.data_ptr())


def _check(status: int, what: str) -> None:
    if status != BD_OK:
        raise BitDeltaError(status, what)


def _dev(t: torch.Tensor, dtype, what: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{what} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def new_workspace(nbytes: int, device) -> torch.Tensor:
    """Caller-owned scratch (torch's allocations are at least 256-byte aligned)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def pack_signs(delta: torch.Tensor, packed: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """bd_pack_signs: delta fp16 [out, in] -> packed int32 [out, in/32] (uint32 bit patterns)."""
    _dev(delta, torch.float16, "delta")
    out, inn = delta.shape
    if packed is None:
        packed = torch.empty((out, max(inn // 32, 0)), dtype=torch.int32, device=delta.device)
    _dev(packed, torch.int32, "packed")
    _check(lib().bd_pack_signs(_ptr(delta), out, inn, _ptr(packed), _stream(stream)), "bd_pack_signs")
    return packed


def compress(w_base: torch.Tensor, w_ft: torch.Tensor, packed: Optional[torch.Tensor] = None,
             alpha: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """bd_compress: returns (packed int32 [out, in/32], alpha float32 [1]) on the device."""
    _dev(w_base, torch.float16, "w_base")
    _dev(w_ft, torch.float16, "w_ft")
    if w_base.shape != w_ft.shape:
        raise ValueError("w_base and w_ft differ in shape")
    out, inn = w_base.shape
    dev = w_base.device
    if packed is None:
        packed = torch.empty((out, max(inn // 32, 0)), dtype=torch.int32, device=dev)
    if alpha is None:
        alpha = torch.empty((1,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(workspace_bytes(OP_COMPRESS, 0, out, inn, 1), dev)
    _check(lib().bd_compress(_ptr(w_base), _ptr(w_ft), out, inn, _ptr(packed), _ptr(alpha), _ptr(workspace),
                             workspace.numel(), _stream(stream)), "bd_compress")
    return packed, alpha


COMPRESS_NOALLOC_MAX_ELEMENTS = 1 << 32


def compress_noalloc(w_base: torch.Tensor, w_ft: torch.Tensor, packed: torch.Tensor, alpha: torch.Tensor, stream=None):
    """bd_compress_noalloc: the caller brings both outputs (packed int32 [out, in/32], alpha float32 [1]);
    nothing is allocated here or in the library."""
    _dev(w_base, torch.float16, "w_base")
    _dev(w_ft, torch.float16, "w_ft")
    _dev(packed, torch.int32, "packed")
    _dev(alpha, torch.float32, "alpha")
    if w_base.shape != w_ft.shape:
        raise ValueError("w_base and w_ft differ in shape")
    out, inn = w_base.shape
    if packed.numel() != out * (inn // 32) or alpha.numel() < 1:
        raise ValueError("packed must hold out * in / 32 words and alpha one float")
    _check(lib().bd_compress_noalloc(_ptr(w_base), _ptr(w_ft), out, inn, _ptr(packed), _ptr(alpha), _stream(stream)),
           "bd_compress_noalloc")
    return packed, alpha


COMPRESS_BATCH_MAX = 8


def compress_batch(w_bases: Sequence[torch.Tensor], w_fts: Sequence[torch.Tensor],
                   workspace: Optional[torch.Tensor] = None, stream=None):
    """bd_compress_batch: several matrices of one fine-tune in one call.  Returns (list of packed int32 [out, in/32],
    alpha float32 [n]) on the device."""
    n = len(w_bases)
    if len(w_fts) != n:
        raise ValueError("one fine-tuned matrix per base matrix")
    if n == 0:
        return [], torch.empty((0,), dtype=torch.float32)
    dev = w_bases[0].device
    packed = []
    for b, f in zip(w_bases, w_fts):
        _dev(b, torch.float16, "w_base")
        _dev(f, torch.float16, "w_ft")
        if b.shape != f.shape:
            raise ValueError("w_base and w_ft differ in shape")
        packed.append(torch.empty((b.shape[0], max(b.shape[1] // 32, 0)), dtype=torch.int32, device=dev))
    alpha = torch.empty((n,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(COMPRESS_BATCH_MAX * workspace_bytes(OP_COMPRESS, 0, 1, 32, 1), dev)
    ptrs = lambda ts: (ctypes.c_void_p * n)(*[_ptr(t) or None for t in ts])
    outs = (ctypes.c_int64 * n)(*[int(b.shape[0]) for b in w_bases])
    ins = (ctypes.c_int64 * n)(*[int(b.shape[1]) for b in w_bases])
    _check(lib().bd_compress_batch(n, ptrs(w_bases), ptrs(w_fts), outs, ins, ptrs(packed), _ptr(alpha), _ptr(workspace),
                                   workspace.numel(), _stream(stream)), "bd_compress_batch")
    return packed, alpha


MAX_PLANES = 8


def compress_iterated(w_base: torch.Tensor, w_ft: torch.Tensor, k: int, packed: Optional[torch.Tensor] = None,
                      alpha: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """bd_compress_iterated: returns (packed int32 [k, out, in/32], alpha float32 [k]) on the device."""
    _dev(w_base, torch.float16, "w_base")
    _dev(w_ft, torch.float16, "w_ft")
    if w_base.shape != w_ft.shape:
        raise ValueError("w_base and w_ft differ in shape")
    out, inn = w_base.shape
    dev = w_base.device
    if packed is None:
        packed = torch.empty((max(k, 0), out, max(inn // 32, 0)), dtype=torch.int32, device=dev)
    if alpha is None:
        alpha = torch.empty((max(k, 1),), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(workspace_bytes(OP_COMPRESS, 0, out, inn, 1), dev)
    _check(lib().bd_compress_iterated(_ptr(w_base), _ptr(w_ft), out, inn, k, _ptr(packed), _ptr(alpha), _ptr(workspace),
                                      workspace.numel(), _stream(stream)), "bd_compress_iterated")
    return packed, alpha


class TenantTable:
    """Device-side arrays the linear takes: pointers to each tenant's packed delta and the scales."""

    def __init__(self, packed_by_tenant: Sequence[torch.Tensor], alpha_by_tenant):
        self.packed = list(packed_by_tenant)
        for p in self.packed:
            _dev(p, torch.int32, "packed delta")
        dev = self.packed[0].device
        self.ptrs = torch.tensor([p.data_ptr() for p in self.packed], dtype=torch.int64, device=dev)
        if isinstance(alpha_by_tenant, torch.Tensor):
            self.alpha = alpha_by_tenant.to(device=dev, dtype=torch.float32).reshape(-1).contiguous()
        else:
            self.alpha = torch.cat([a.reshape(1).to(torch.float32) for a in alpha_by_tenant]).to(dev).contiguous()
        if self.alpha.numel() != len(self.packed):
            raise ValueError("one alpha per tenant")

    @property
    def n_tenants(self) -> int:
        return len(self.packed)


def _tok_array(tenant_of_token: Sequence[int]):
    n = len(tenant_of_token)
    return (ctypes.c_int32 * max(n, 1))(*[int(t) for t in tenant_of_token])


def linear_multitenant(x: torch.Tensor, w_base: torch.Tensor, tenants: TenantTable, tenant_of_token: Sequence[int],
                       y: Optional[torch.Tensor] = None, stream=None, variant: int = 0,
                       tok_array=None, workspace="auto") -> torch.Tensor:
    """bd_linear_multitenant (variant 0) or bd_linear_multitenant_variant: y fp16 [T, out].
    workspace: "auto" allocates what bd_workspace_bytes asks for (more than 32 tokens: the prefill GEMM),
    None passes no workspace (the call then runs as decode launches), or a caller-owned uint8 tensor."""
    _dev(x, torch.float16, "x")
    _dev(w_base, torch.float16, "w_base")
    T, inn = x.shape
    out = w_base.shape[0]
    if w_base.shape[1] != inn:
        raise ValueError("x and w_base disagree on `in`")
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    L = lib()
    if isinstance(workspace, str):
        need = workspace_bytes(OP_LINEAR_MULTITENANT, T, out, inn, tenants.n_tenants)
        workspace = new_workspace(need, x.device) if need > 0 else None
    ws_ptr, ws_bytes = (_ptr(workspace), workspace.numel()) if workspace is not None else (0, 0)
    if variant == 0:
        st = L.bd_linear_multitenant(_ptr(x), _ptr(w_base), _ptr(tenants.ptrs), _ptr(tenants.alpha), tok, _ptr(y),
                                     T, out, inn, tenants.n_tenants, ws_ptr, ws_bytes, _stream(stream))
    else:
        st = L.bd_linear_multitenant_variant(_ptr(x), _ptr(w_base), _ptr(tenants.ptrs), _ptr(tenants.alpha), tok,
                                             _ptr(y), T, out, inn, tenants.n_tenants, ws_ptr, ws_bytes, _stream(stream),
                                             int(variant))
    _check(st, "bd_linear_multitenant")
    return y


def group_tokens(tenant_of_token: Sequence[int]):
    """bd_group_tokens: returns (token_of_col, jobs) with jobs = [(tenant, tile, col_begin, col_end), ...]."""
    T = len(tenant_of_token)
    n = max(T, 1)
    tok = _tok_array(tenant_of_token)
    arrs = [(ctypes.c_int32 * n)() for _ in range(5)]
    nj = ctypes.c_int32(0)
    _check(lib().bd_group_tokens(tok, T, arrs[0], arrs[1], arrs[2], arrs[3], arrs[4], ctypes.byref(nj)),
           "bd_group_tokens")
    jobs = [(arrs[1][j], arrs[2][j], arrs[3][j], arrs[4][j]) for j in range(nj.value)]
    return list(arrs[0][:T]), jobs


def materialize(w_base: torch.Tensor, packed: torch.Tensor, alpha: torch.Tensor,
                w_out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    _dev(w_base, torch.float16, "w_base")
    _dev(packed, torch.int32, "packed")
    _dev(alpha, torch.float32, "alpha")
    out, inn = w_base.shape
    if w_out is None:
        w_out = torch.empty_like(w_base)
    _check(lib().bd_materialize(_ptr(w_base), _ptr(packed), _ptr(alpha), _ptr(w_out), out, inn, _stream(stream)),
           "bd_materialize")
    return w_out


class WeightTable:
    """Device array of pointers to full fp16 matrices, one per tenant (the naive system)."""

    def __init__(self, w_by_tenant: Sequence[torch.Tensor]):
        self.w = list(w_by_tenant)
        for w in self.w:
            _dev(w, torch.float16, "tenant weight")
        self.ptrs = torch.tensor([w.data_ptr() for w in self.w], dtype=torch.int64, device=self.w[0].device)


def linear_naive(x: torch.Tensor, weights: WeightTable, tenant_of_token: Sequence[int],
                 y: Optional[torch.Tensor] = None, stream=None, tok_array=None) -> torch.Tensor:
    _dev(x, torch.float16, "x")
    T, inn = x.shape
    out = weights.w[0].shape[0]
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_naive(_ptr(x), _ptr(weights.ptrs), tok, _ptr(y), T, out, inn, len(weights.w),
                                 _stream(stream)), "bd_linear_naive")
    return y


def probe_read(buf: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    nbytes = buf.numel() * buf.element_size()
    _check(lib().bd_probe_read(_ptr(buf), nbytes, _ptr(sink), _stream(stream)), "bd_probe_read")


def probe_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().bd_probe_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "bd_probe_copy")


# ---- tiled serving layout ------------------------------------------------------------------

def tiled_base_bytes(out: int, inn: int) -> int:
    return int(lib().bd_tiled_base_bytes(out, inn))


def tiled_signs_bytes(out: int, inn: int) -> int:
    return int(lib().bd_tiled_signs_bytes(out, inn))


def tile_base(w: torch.Tensor, w_tiled: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """bd_tile_base: fp16 [out, in] -> flat fp16 tensor in the serving layout."""
    _dev(w, torch.float16, "w")
    out, inn = w.shape
    if w_tiled is None:
        w_tiled = torch.empty((max(tiled_base_bytes(out, inn) // 2, 8),), dtype=torch.float16, device=w.device)
    _check(lib().bd_tile_base(_ptr(w), out, inn, _ptr(w_tiled), _stream(stream)), "bd_tile_base")
    return w_tiled


def tile_signs(packed: torch.Tensor, out: int, inn: int, signs_tiled: Optional[torch.Tensor] = None,
               stream=None) -> torch.Tensor:
    """bd_tile_signs: int32 [out, in/32] -> flat int32 tensor in the serving layout."""
    _dev(packed, torch.int32, "packed")
    if signs_tiled is None:
        signs_tiled = torch.empty((max(tiled_signs_bytes(out, inn) // 4, 4),), dtype=torch.int32, device=packed.device)
    _check(lib().bd_tile_signs(_ptr(packed), out, inn, _ptr(signs_tiled), _stream(stream)), "bd_tile_signs")
    return signs_tiled


class TiledTenantTable:
    """What the tiled linear takes for one matrix: a HOST array of device pointers to each tenant's
    tiled delta (None = tenant absent) and the device array of scales."""

    def __init__(self, tiled_by_tenant: Sequence[Optional[torch.Tensor]], alpha_by_tenant):
        self.tiled = list(tiled_by_tenant)
        dev = next(t for t in self.tiled if t is not None).device
        for t in self.tiled:
            if t is not None:
                _dev(t, torch.int32, "tiled delta")
        self.host_ptrs = (ctypes.c_void_p * max(len(self.tiled), 1))(*[_ptr(t) or None for t in self.tiled])
        if isinstance(alpha_by_tenant, torch.Tensor):
            self.alpha = alpha_by_tenant.to(device=dev, dtype=torch.float32).reshape(-1).contiguous()
        else:
            self.alpha = torch.cat([a.reshape(1).to(torch.float32) for a in alpha_by_tenant]).to(dev).contiguous()
        if self.alpha.numel() != len(self.tiled):
            raise ValueError("one alpha per tenant")

    @property
    def n_tenants(self) -> int:
        return len(self.tiled)


def linear_multitenant_tiled(x: torch.Tensor, w_tiled: torch.Tensor, out: int, tenants: TiledTenantTable,
                             tenant_of_token: Sequence[int], y: Optional[torch.Tensor] = None, stream=None,
                             tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_tiled: y fp16 [T, out]."""
    _dev(x, torch.float16, "x")
    _dev(w_tiled, torch.float16, "w_tiled")
    T, inn = x.shape
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_tiled(_ptr(x), _ptr(w_tiled), tenants.host_ptrs, _ptr(tenants.alpha), tok,
                                             _ptr(y), T, out, inn, tenants.n_tenants, _stream(stream)),
           "bd_linear_multitenant_tiled")
    return y


def linear_multitenant_tiled_gemm(x: torch.Tensor, w_tiled: torch.Tensor, out: int, tenants: TiledTenantTable,
                                  tenant_of_token: Sequence[int], one_product: bool = False, y: Optional[torch.Tensor] = None,
                                  workspace: Optional[torch.Tensor] = None, stream=None, tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_tiled_gemm: all tokens in one matrix-core GEMM launch on the serving layout; y fp16 [T, out].
    workspace: a caller-owned uint8 tensor of bd_workspace_bytes(OP_LINEAR_TILED_GEMM, ...) bytes, or None to allocate one."""
    _dev(x, torch.float16, "x")
    _dev(w_tiled, torch.float16, "w_tiled")
    T, inn = x.shape
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    if workspace is None:
        workspace = new_workspace(workspace_bytes(OP_LINEAR_TILED_GEMM, T, out, inn, tenants.n_tenants), x.device)
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_tiled_gemm(_ptr(x), _ptr(w_tiled), tenants.host_ptrs, _ptr(tenants.alpha), tok, _ptr(y), T,
                                                  out, inn, tenants.n_tenants, 1 if one_product else 0, _ptr(workspace),
                                                  workspace.numel(), _stream(stream)), "bd_linear_multitenant_tiled_gemm")
    return y


class PlaneTable:
    """Device-side arrays of bd_linear_multitenant_kbit: pointers to every tenant's k row-major planes (entry
    tenant * k + plane) and the scales [n_tenants * k].  planes_by_tenant: list of int32 tensors [k, out, in/32]."""

    def __init__(self, planes_by_tenant: Sequence[torch.Tensor], alpha_by_tenant: torch.Tensor):
        self.planes = list(planes_by_tenant)
        self.k = int(self.planes[0].shape[0])
        for p in self.planes:
            _dev(p, torch.int32, "planes")
            if p.shape[0] != self.k:
                raise ValueError("every tenant needs the same number of planes")
        dev = self.planes[0].device
        self.ptrs = torch.tensor([p[j].data_ptr() for p in self.planes for j in range(self.k)], dtype=torch.int64, device=dev)
        self.alpha = alpha_by_tenant.to(device=dev, dtype=torch.float32).reshape(-1).contiguous()
        if self.alpha.numel() != len(self.planes) * self.k:
            raise ValueError("one alpha per tenant and plane")

    @property
    def n_tenants(self) -> int:
        return len(self.planes)


def linear_multitenant_kbit(x: torch.Tensor, w_base: torch.Tensor, tenants: PlaneTable, tenant_of_token: Sequence[int],
                            y: Optional[torch.Tensor] = None, stream=None, tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_kbit: y fp16 [T, out] from the row-major base and k row-major planes per tenant."""
    _dev(x, torch.float16, "x")
    _dev(w_base, torch.float16, "w_base")
    T, inn = x.shape
    out = w_base.shape[0]
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_kbit(_ptr(x), _ptr(w_base), _ptr(tenants.ptrs), _ptr(tenants.alpha), tok, _ptr(y), T, out,
                                            inn, tenants.n_tenants, tenants.k, _stream(stream)), "bd_linear_multitenant_kbit")
    return y


def linear_multitenant_gemm_kbit(x: torch.Tensor, w_base: torch.Tensor, tenants: PlaneTable, tenant_of_token: Sequence[int],
                                 y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                                 tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_gemm_kbit: the GEMM form (any T >= 1) with k row-major planes per tenant."""
    _dev(x, torch.float16, "x")
    _dev(w_base, torch.float16, "w_base")
    T, inn = x.shape
    out = w_base.shape[0]
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = new_workspace(workspace_bytes(OP_LINEAR_GEMM, T, out, inn, tenants.n_tenants), x.device)
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_gemm_kbit(_ptr(x), _ptr(w_base), _ptr(tenants.ptrs), _ptr(tenants.alpha), tok, _ptr(y), T,
                                                 out, inn, tenants.n_tenants, tenants.k, _ptr(workspace), workspace.numel(),
                                                 _stream(stream)), "bd_linear_multitenant_gemm_kbit")
    return y


def linear_multitenant_q8(x: torch.Tensor, q: torch.Tensor, scale: torch.Tensor, tenants: "TenantTable",
                          tenant_of_token: Sequence[int], y: Optional[torch.Tensor] = None, stream=None,
                          tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_q8: decode launches on the row-major 8-bit base (q int8 [out, in], scale [out])."""
    _dev(x, torch.float16, "x")
    _dev(q, torch.int8, "q")
    _dev(scale, torch.float32, "scale")
    T, inn = x.shape
    out = q.shape[0]
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_q8(_ptr(x), _ptr(q), _ptr(scale), _ptr(tenants.ptrs), _ptr(tenants.alpha), tok, _ptr(y), T,
                                          out, inn, tenants.n_tenants, _stream(stream)), "bd_linear_multitenant_q8")
    return y


def linear_multitenant_gemm_q8(x: torch.Tensor, q: torch.Tensor, scale: torch.Tensor, tenants: "TenantTable",
                               tenant_of_token: Sequence[int], y: Optional[torch.Tensor] = None,
                               workspace: Optional[torch.Tensor] = None, stream=None, tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_gemm_q8: the GEMM form (any T >= 1) on the row-major 8-bit base (q int8 [out, in], scale [out])."""
    _dev(x, torch.float16, "x")
    _dev(q, torch.int8, "q")
    _dev(scale, torch.float32, "scale")
    T, inn = x.shape
    out = q.shape[0]
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = new_workspace(workspace_bytes(OP_LINEAR_GEMM, T, out, inn, tenants.n_tenants), x.device)
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_gemm_q8(_ptr(x), _ptr(q), _ptr(scale), _ptr(tenants.ptrs), _ptr(tenants.alpha), tok, _ptr(y),
                                               T, out, inn, tenants.n_tenants, _ptr(workspace), workspace.numel(),
                                               _stream(stream)), "bd_linear_multitenant_gemm_q8")
    return y


class TiledPlaneTable:
    """What the k-plane tiled linear takes for one matrix: a HOST array [n_tenants * k] of device pointers to
    every tenant's tiled planes (None = tenant absent) and the device array [n_tenants * k] of scales."""

    def __init__(self, planes_by_tenant: Sequence[Optional[Sequence[torch.Tensor]]], alpha_by_tenant: torch.Tensor):
        present = [p for p in planes_by_tenant if p is not None]
        self.k = len(present[0])
        if any(len(p) != self.k for p in present):
            raise ValueError("every tenant needs the same number of planes")
        self.planes = [list(p) if p is not None else None for p in planes_by_tenant]
        flat = []
        for p in self.planes:
            for j in range(self.k):
                t = p[j] if p is not None else None
                if t is not None:
                    _dev(t, torch.int32, "tiled plane")
                flat.append(t)
        dev = present[0][0].device
        self.host_ptrs = (ctypes.c_void_p * max(len(flat), 1))(*[_ptr(t) or None for t in flat])
        self.alpha = alpha_by_tenant.to(device=dev, dtype=torch.float32).reshape(-1).contiguous()
        if self.alpha.numel() != len(self.planes) * self.k:
            raise ValueError("one alpha per tenant and plane")

    @property
    def n_tenants(self) -> int:
        return len(self.planes)


def linear_multitenant_tiled_kbit(x: torch.Tensor, w_tiled: torch.Tensor, out: int, tenants: TiledPlaneTable,
                                  tenant_of_token: Sequence[int], y: Optional[torch.Tensor] = None, stream=None,
                                  tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_tiled_kbit: y fp16 [T, out]."""
    _dev(x, torch.float16, "x")
    _dev(w_tiled, torch.float16, "w_tiled")
    T, inn = x.shape
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_tiled_kbit(_ptr(x), _ptr(w_tiled), tenants.host_ptrs, _ptr(tenants.alpha), tok,
                                                  _ptr(y), T, out, inn, tenants.n_tenants, tenants.k, _stream(stream)),
           "bd_linear_multitenant_tiled_kbit")
    return y


class TiledPlaneGroup:
    """Marshalled arguments of bd_linear_multitenant_tiled_group_kbit for a fixed set of matrices."""

    def __init__(self, w_tiled: Sequence[torch.Tensor], outs: Sequence[int], tables: Sequence[TiledPlaneTable]):
        self.n = len(w_tiled)
        self.keep = (list(w_tiled), list(tables))
        self.outs = [int(o) for o in outs]
        nt, k = tables[0].n_tenants, tables[0].k
        if any(t.n_tenants != nt or t.k != k for t in tables):
            raise ValueError("every matrix needs the same tenants and planes")
        self.n_tenants, self.k = nt, k
        self.w = (ctypes.c_void_p * self.n)(*[_ptr(w) for w in w_tiled])
        self.signs = (ctypes.c_void_p * (self.n * max(nt * k, 1)))(*[p for tab in tables for p in tab.host_ptrs])
        self.alpha = (ctypes.c_void_p * self.n)(*[_ptr(tab.alpha) for tab in tables])
        self.out_arr = (ctypes.c_int64 * self.n)(*self.outs)


def linear_multitenant_tiled_group_kbit(x: torch.Tensor, group: TiledPlaneGroup, tenant_of_token: Sequence[int],
                                        ys: Optional[Sequence[torch.Tensor]] = None, stream=None, tok_array=None):
    """bd_linear_multitenant_tiled_group_kbit: list of y_m fp16 [T, out_m]."""
    _dev(x, torch.float16, "x")
    T, inn = x.shape
    if ys is None:
        ys = [torch.empty((T, o), dtype=torch.float16, device=x.device) for o in group.outs]
    yarr = (ctypes.c_void_p * group.n)(*[_ptr(_dev(y, torch.float16, "y")) for y in ys])
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_tiled_group_kbit(group.n, _ptr(x), group.w, group.signs, group.alpha, tok, yarr, T,
                                                        group.out_arr, inn, group.n_tenants, group.k, _stream(stream)),
           "bd_linear_multitenant_tiled_group_kbit")
    return list(ys)


class TiledGroup:
    """Marshalled arguments of bd_linear_multitenant_tiled_group for a fixed set of matrices."""

    def __init__(self, w_tiled: Sequence[torch.Tensor], outs: Sequence[int], tables: Sequence[TiledTenantTable]):
        self.n = len(w_tiled)
        self.keep = (list(w_tiled), list(tables))
        self.outs = [int(o) for o in outs]
        nt = tables[0].n_tenants
        if any(t.n_tenants != nt for t in tables):
            raise ValueError("every matrix needs the same tenants")
        self.n_tenants = nt
        self.w = (ctypes.c_void_p * self.n)(*[_ptr(w) for w in w_tiled])
        self.signs = (ctypes.c_void_p * (self.n * max(nt, 1)))(
            *[_ptr(t) or None for tab in tables for t in tab.tiled])
        self.alpha = (ctypes.c_void_p * self.n)(*[_ptr(tab.alpha) for tab in tables])
        self.out_arr = (ctypes.c_int64 * self.n)(*self.outs)


def linear_multitenant_tiled_group(x: torch.Tensor, group: TiledGroup, tenant_of_token: Sequence[int],
                                   ys: Optional[Sequence[torch.Tensor]] = None, stream=None, tok_array=None):
    """bd_linear_multitenant_tiled_group: list of y_m fp16 [T, out_m]."""
    _dev(x, torch.float16, "x")
    T, inn = x.shape
    if ys is None:
        ys = [torch.empty((T, o), dtype=torch.float16, device=x.device) for o in group.outs]
    yarr = (ctypes.c_void_p * group.n)(*[_ptr(_dev(y, torch.float16, "y")) for y in ys])
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_tiled_group(group.n, _ptr(x), group.w, group.signs, group.alpha, tok, yarr, T,
                                                   group.out_arr, inn, group.n_tenants, _stream(stream)),
           "bd_linear_multitenant_tiled_group")
    return list(ys)


# ---- delta images and hot swap (host-side calls take CPU tensors) --------------------------------------

def _host_u8(n: int, pinned: bool) -> torch.Tensor:
    return torch.empty(n, dtype=torch.uint8, pin_memory=bool(pinned and torch.cuda.is_available()))


def delta_image_bytes(outs: Sequence[int], ins: Sequence[int], k: int) -> int:
    n = len(outs)
    return int(lib().bd_delta_image_bytes(n, (ctypes.c_int64 * n)(*outs), (ctypes.c_int64 * n)(*ins), k))


def delta_image_build(packed: Sequence[torch.Tensor], alpha: Sequence[torch.Tensor], outs: Sequence[int],
                      ins: Sequence[int], k: int, pinned: bool = True) -> torch.Tensor:
    """bd_delta_image_build from CPU tensors: packed[m] int32 [k, out_m, in_m/32], alpha[m] float32 [k].
    Returns the image as a uint8 CPU tensor (pinned if asked and a GPU is present)."""
    n = len(outs)
    nbytes = delta_image_bytes(outs, ins, k)
    if nbytes == 0:
        raise BitDeltaError(2, "bd_delta_image_bytes")
    pk = [p.contiguous() for p in packed]
    al = [a.to(torch.float32).contiguous() for a in alpha]
    for m in range(n):
        if pk[m].device.type != "cpu" or pk[m].dtype != torch.int32 or pk[m].numel() != k * outs[m] * (ins[m] // 32):
            raise ValueError("packed[m]: int32 CPU tensor [k, out, in/32]")
        if al[m].device.type != "cpu" or al[m].numel() != k:
            raise ValueError("alpha[m]: float32 CPU tensor [k]")
    image = _host_u8(nbytes, pinned)
    _check(lib().bd_delta_image_build(_ptr(image), nbytes, n, (ctypes.c_int64 * n)(*outs), (ctypes.c_int64 * n)(*ins), k,
                                      (ctypes.c_void_p * n)(*[_ptr(p) or None for p in pk]),
                                      (ctypes.c_void_p * n)(*[_ptr(a) for a in al])), "bd_delta_image_build")
    return image


def delta_image_check(image: torch.Tensor, verify_checksum: bool = True):
    """Returns (n_mats, k) of a valid image, raises BitDeltaError otherwise."""
    n, k = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().bd_delta_image_check(_ptr(image), image.numel(), int(verify_checksum), ctypes.byref(n), ctypes.byref(k)),
           "bd_delta_image_check")
    return n.value, k.value


def delta_image_entry(image: torch.Tensor, m: int):
    """(out, in, packed_offset, alpha_offset) of matrix m."""
    o, i = ctypes.c_int64(0), ctypes.c_int64(0)
    po, ao = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().bd_delta_image_entry(_ptr(image), image.numel(), m, ctypes.byref(o), ctypes.byref(i), ctypes.byref(po),
                                      ctypes.byref(ao)), "bd_delta_image_entry")
    return o.value, i.value, po.value, ao.value


def delta_file_write(path: str, image: torch.Tensor) -> None:
    _check(lib().bd_delta_file_write(os.fsencode(path), _ptr(image), image.numel()), "bd_delta_file_write")


def delta_file_read(path: str, pinned: bool = True) -> torch.Tensor:
    n = ctypes.c_size_t(0)
    _check(lib().bd_delta_file_bytes(os.fsencode(path), ctypes.byref(n)), "bd_delta_file_bytes")
    image = _host_u8(n.value, pinned)
    _check(lib().bd_delta_file_read(os.fsencode(path), _ptr(image), n.value), "bd_delta_file_read")
    return image


def delta_upload(image: torch.Tensor, arena: Optional[torch.Tensor] = None, device="cuda", stream=None) -> torch.Tensor:
    """bd_delta_upload: one asynchronous copy of the image into a device arena (allocated here if not given)."""
    if arena is None:
        arena = torch.empty(image.numel(), dtype=torch.uint8, device=device)
    _check(lib().bd_delta_upload(_ptr(image), image.numel(), _ptr(arena), _stream(stream)), "bd_delta_upload")
    return arena


def delta_install(image: torch.Tensor, arena: torch.Tensor, tenant: int, n_tenants: int,
                  tiled_dst: Sequence[Sequence[torch.Tensor]], alpha_by_tenant: Sequence[torch.Tensor], stream=None) -> None:
    """bd_delta_install: tiled_dst[m][j] int32 device buffers in the serving layout, alpha_by_tenant[m] float32 device
    arrays [n_tenants * k]."""
    flat = [t for planes in tiled_dst for t in planes]
    _check(lib().bd_delta_install(_ptr(image), image.numel(), _ptr(arena), tenant, n_tenants,
                                  (ctypes.c_void_p * max(len(flat), 1))(*[_ptr(t) for t in flat]),
                                  (ctypes.c_void_p * max(len(alpha_by_tenant), 1))(*[_ptr(a) for a in alpha_by_tenant]),
                                  _stream(stream)), "bd_delta_install")


# ---- 8-bit round-to-nearest base -----------------------------------------------------------------------

def quantize_base_q8(w: torch.Tensor, stream=None):
    """bd_quantize_base_q8: returns (q int8 [out, in], scale float32 [out]) on the device."""
    _dev(w, torch.float16, "w")
    out, inn = w.shape
    q = torch.empty((out, inn), dtype=torch.int8, device=w.device)
    scale = torch.empty((out,), dtype=torch.float32, device=w.device)
    _check(lib().bd_quantize_base_q8(_ptr(w), out, inn, _ptr(q), _ptr(scale), _stream(stream)), "bd_quantize_base_q8")
    return q, scale


def compress_q8(q: torch.Tensor, scale: torch.Tensor, w_ft: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                stream=None):
    """bd_compress_q8: returns (packed int32 [out, in/32], alpha float32 [1]) on the device."""
    _dev(q, torch.int8, "q")
    _dev(scale, torch.float32, "scale")
    _dev(w_ft, torch.float16, "w_ft")
    out, inn = w_ft.shape
    if q.shape != w_ft.shape or scale.numel() != out:
        raise ValueError("q, scale and w_ft disagree in shape")
    dev = w_ft.device
    packed = torch.empty((out, max(inn // 32, 0)), dtype=torch.int32, device=dev)
    alpha = torch.empty((1,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(workspace_bytes(OP_COMPRESS, 0, out, inn, 1), dev)
    _check(lib().bd_compress_q8(_ptr(q), _ptr(scale), _ptr(w_ft), out, inn, _ptr(packed), _ptr(alpha), _ptr(workspace),
                                workspace.numel(), _stream(stream)), "bd_compress_q8")
    return packed, alpha


def tiled_base_q8_bytes(out: int, inn: int) -> int:
    return int(lib().bd_tiled_base_q8_bytes(out, inn))


def tile_base_q8(q: torch.Tensor, scale: torch.Tensor, stream=None) -> torch.Tensor:
    """bd_tile_base_q8: the 8-bit base in the serving layout (uint8 tensor: tiles, then the padded scales)."""
    _dev(q, torch.int8, "q")
    _dev(scale, torch.float32, "scale")
    out, inn = q.shape
    n = tiled_base_q8_bytes(out, inn)
    if n == 0 and out * inn > 0:
        raise BitDeltaError(2, "bd_tiled_base_q8_bytes")
    wq = torch.empty(n, dtype=torch.uint8, device=q.device)
    _check(lib().bd_tile_base_q8(_ptr(q), _ptr(scale), out, inn, _ptr(wq), _stream(stream)), "bd_tile_base_q8")
    return wq


def linear_multitenant_tiled_q8(x: torch.Tensor, wq_tiled: torch.Tensor, out: int, tenants: TiledTenantTable,
                                tenant_of_token: Sequence[int], y: Optional[torch.Tensor] = None, stream=None,
                                tok_array=None) -> torch.Tensor:
    """bd_linear_multitenant_tiled_q8: y fp16 [T, out]."""
    _dev(x, torch.float16, "x")
    _dev(wq_tiled, torch.uint8, "wq_tiled")
    T, inn = x.shape
    if y is None:
        y = torch.empty((T, out), dtype=torch.float16, device=x.device)
    _dev(y, torch.float16, "y")
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_tiled_q8(_ptr(x), _ptr(wq_tiled), tenants.host_ptrs, _ptr(tenants.alpha), tok,
                                                _ptr(y), T, out, inn, tenants.n_tenants, _stream(stream)),
           "bd_linear_multitenant_tiled_q8")
    return y


def linear_multitenant_tiled_group_q8(x: torch.Tensor, group: TiledGroup, tenant_of_token: Sequence[int],
                                      ys: Optional[Sequence[torch.Tensor]] = None, stream=None, tok_array=None):
    """bd_linear_multitenant_tiled_group_q8: `group` built from 8-bit tiled bases (TiledGroup takes any tensors)."""
    _dev(x, torch.float16, "x")
    T, inn = x.shape
    if ys is None:
        ys = [torch.empty((T, o), dtype=torch.float16, device=x.device) for o in group.outs]
    yarr = (ctypes.c_void_p * group.n)(*[_ptr(_dev(y, torch.float16, "y")) for y in ys])
    tok = tok_array if tok_array is not None else _tok_array(tenant_of_token)
    _check(lib().bd_linear_multitenant_tiled_group_q8(group.n, _ptr(x), group.w, group.signs, group.alpha, tok, yarr, T,
                                                      group.out_arr, inn, group.n_tenants, _stream(stream)),
           "bd_linear_multitenant_tiled_group_q8")
    return list(ys)
