"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
arguments on the host before anything is enqueued (no GPU needed, no compute call is made)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bd():
    from paper_2402_10193_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2402_10193_amd import build
        build.build_library()
    binding.lib()
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "bitdelta.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(bd):
    names = _declared_functions()
    assert set(names) == set(bd.EXPORTS)
    L = bd.lib()
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_strings(bd):
    assert bd.version() >= 100
    seen = set()
    for code in range(9):
        s = bd.status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert bd.status_string(99) == "unknown status"


def test_workspace_bytes(bd):
    assert bd.workspace_bytes(bd.OP_COMPRESS, 0, 4096, 4096, 1) >= 2048 * 8
    assert bd.workspace_bytes(bd.OP_LINEAR_MULTITENANT, 16, 4096, 4096, 16) == 0
    assert bd.workspace_bytes(bd.OP_LINEAR_MULTITENANT, 32, 4096, 4096, 16) == 0
    # prefill: (ceil(T / rows) + min(tenants, T)) tiles x (rows + 1) ints for token tiles of rows = 128 and of 256 rows
    # (the one-product form), the larger of the two, rounded up to 256 bytes
    assert bd.workspace_bytes(bd.OP_LINEAR_MULTITENANT, 4096, 11008, 4096, 8) == (max(40 * 129, 24 * 257) * 4 + 255) // 256 * 256
    assert bd.workspace_bytes(bd.OP_LINEAR_MULTITENANT, 33, 64, 64, 100) == (max(34 * 129, 34 * 257) * 4 + 255) // 256 * 256
    assert bd.workspace_bytes(bd.OP_PACK_SIGNS, 0, 4096, 4096, 1) == 0
    assert bd.workspace_bytes(bd.OP_COMPRESS, 0, 4096, 4100, 1) == 0   # rejected shape


def _tok(*ids):
    return (ctypes.c_int32 * max(len(ids), 1))(*ids)


A = 0x10000  # a fake, 16-byte aligned, never dereferenced device address


def test_linear_argument_errors_are_caught_on_the_host(bd):
    L = bd.lib()
    f = L.bd_linear_multitenant
    ok_args = dict(x=A, w=2 * A, pk=3 * A, al=4 * A, tok=_tok(0), y=5 * A, T=1, out=16, inn=128, nt=1)

    def call(**kw):
        a = dict(ok_args, **kw)
        return f(a["x"], a["w"], a["pk"], a["al"], a["tok"], a["y"], a["T"], a["out"], a["inn"], a["nt"], 0, 0, 0)

    assert call(inn=48) == 2 and call(T=-1) == 2 and call(out=-1) == 2 and call(T=70000) == 2
    assert call(x=0) == 1 and call(w=0) == 1 and call(pk=0) == 1 and call(al=0) == 1 and call(y=0) == 1
    assert call(x=A + 2) == 3 and call(w=2 * A + 8) == 3 and call(y=5 * A + 4) == 3
    assert call(tok=_tok(1)) == 4 and call(tok=_tok(-1)) == 4 and call(tok=_tok(0, 0, 5), T=3, nt=5) == 4
    assert call(y=A) == 8 and call(y=2 * A + 64) == 8            # y overlapping x / w
    # no-ops succeed without touching any pointer
    assert call(T=0, x=0, y=0) == 0 and call(out=0, w=0, y=0) == 0
    # unknown kernel variant, and a matrix-core variant on a shape it cannot run
    fv = L.bd_linear_multitenant_variant
    assert fv(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 0, 0, 0, 99) == 7
    assert fv(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 96, 1, 0, 0, 0, 3) == 7
    # the GEMM variants: one decode launch worth of tokens, no workspace, a reduction length the large tiles cannot run
    many = _tok(*([0] * 64))
    for v in (4, 5, 6, 7, 8):
        assert fv(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 0, 0, 0, v) == 7
        assert fv(A, 2 * A, 3 * A, 4 * A, many, 5 * A, 64, 16, 128, 1, 0, 0, 0, v) == 5
    for v in (5, 6, 7, 8):
        assert fv(A, 2 * A, 3 * A, 4 * A, many, 5 * A, 64, 16, 96, 1, 6 * A, 1 << 20, 0, v) == 7
    assert fv(A, 2 * A, 3 * A, 4 * A, many, 5 * A, 64, 16, 128, 1, 6 * A, 1 << 20, 0, 9) == 7


def test_tiled_gemm_argument_errors(bd):
    """bd_linear_multitenant_tiled_gemm: every error is found on the host before anything is launched."""
    L = bd.lib()
    f = L.bd_linear_multitenant_tiled_gemm
    ptrs = (ctypes.c_void_p * 2)(3 * A, 6 * A)
    tok = _tok(*([0] * 40))
    W = 0x100000   # a fake, 256-byte aligned workspace address
    need = bd.workspace_bytes(bd.OP_LINEAR_TILED_GEMM, 40, 64, 128, 2)
    # the token tables of either tile height (1 + 2 tiles x 129 ints, or x 257) and the table of 2 pointers
    assert need == (3 * 257 * 4 + 255) // 256 * 256 + 256
    assert bd.workspace_bytes(bd.OP_LINEAR_TILED_GEMM, 0, 64, 128, 2) == 0

    def call(x=A, w=2 * A, p=ptrs, al=4 * A, t=tok, y=5 * A, T=40, out=64, inn=128, nt=2, ws=W, nb=need):
        return f(x, w, p, al, t, y, T, out, inn, nt, 0, ws, nb, 0)

    assert call(inn=100) == 2 and call(T=-1) == 2 and call(T=70000) == 2
    assert call(x=0) == 1 and call(w=0) == 1 and call(al=0) == 1 and call(y=0) == 1 and call(p=None) == 1
    assert call(p=(ctypes.c_void_p * 2)(None, 6 * A)) == 1            # tenant 0 has tokens but no delta
    assert call(x=A + 2) == 3 and call(p=(ctypes.c_void_p * 2)(3 * A + 4, 6 * A)) == 3
    assert call(t=_tok(*([0] * 39 + [2]))) == 4 and call(t=_tok(*([0] * 39 + [-1]))) == 4
    assert call(y=A + 64) == 8 and call(y=2 * A + 1024) == 8
    assert call(inn=96) == 7                                          # no whole step of 64
    assert call(ws=0, nb=0) == 5 and call(nb=need - 1) == 5 and call(ws=W + 16) == 5
    assert call(T=0, x=0, y=0) == 0 and call(out=0, w=0, y=0) == 0


def test_compress_and_pack_argument_errors(bd):
    L = bd.lib()
    need = bd.workspace_bytes(bd.OP_COMPRESS, 0, 16, 128, 1)
    c = L.bd_compress
    assert c(A, 2 * A, 16, 100, 3 * A, 4 * A, 5 * A, need, 0) == 2
    assert c(0, 2 * A, 16, 128, 3 * A, 4 * A, 5 * A, need, 0) == 1
    assert c(A, 2 * A, 16, 128, 3 * A, 0, 5 * A, need, 0) == 1
    assert c(A + 4, 2 * A, 16, 128, 3 * A, 4 * A, 5 * A, need, 0) == 3
    assert c(A, 2 * A, 16, 128, 3 * A, 4 * A, 0, need, 0) == 5
    assert c(A, 2 * A, 16, 128, 3 * A, 4 * A, 5 * A, need - 1, 0) == 5
    assert c(A, 2 * A, 16, 128, 3 * A, 4 * A, 5 * A + 16, need, 0) == 5
    assert c(A, 2 * A, 16, 128, A + 1024, 4 * A, 5 * A, need, 0) == 8
    p = L.bd_pack_signs
    assert p(A, 16, 40, 2 * A, 0) == 2 and p(0, 16, 64, 2 * A, 0) == 1 and p(A, 16, 64, 2 * A + 4, 0) == 3
    assert p(0, 0, 64, 0, 0) == 0
    assert L.bd_probe_read(A, 24, 2 * A, 0) == 2 and L.bd_probe_copy(A, A + 16, 64, 0) == 8
    assert L.bd_linear_naive(A, 2 * A, _tok(3), 3 * A, 1, 16, 64, 2, 0) == 4
    assert L.bd_materialize(A, 2 * A, 0, 3 * A, 16, 64, 0) == 1


def test_linear_kbit_row_major_argument_errors(bd):
    f = bd.lib().bd_linear_multitenant_kbit
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 0, 0) == 2      # k out of range
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 9, 0) == 2
    assert f(A, 2 * A, 0, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 2, 0) == 1
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(1), 5 * A, 1, 16, 128, 1, 2, 0) == 4
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 96, 1, 2, 0) == 7       # in % 128: no kernel for it
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 0, 16, 128, 1, 2, 0) == 0      # no tokens: nothing to do


def test_gemm_variants_argument_errors(bd):
    """bd_linear_multitenant_gemm_kbit / _gemm_q8: every error is found on the host before anything is launched."""
    L = bd.lib()
    f, g = L.bd_linear_multitenant_gemm_kbit, L.bd_linear_multitenant_gemm_q8
    W = 0x100000   # a fake, 256-byte aligned workspace address
    # the token tables: (ceil(T / 128) + min(tenants, T)) tiles x 129 ints, for any T >= 1
    assert bd.workspace_bytes(bd.OP_LINEAR_GEMM, 1, 64, 64, 3) == (2 * 129 * 4 + 255) // 256 * 256
    assert bd.workspace_bytes(bd.OP_LINEAR_GEMM, 4096, 11008, 4096, 8) == (40 * 129 * 4 + 255) // 256 * 256
    assert bd.workspace_bytes(bd.OP_LINEAR_GEMM, 0, 64, 64, 3) == 0
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 0, W, 4096, 0) == 2     # k out of range
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 9, W, 4096, 0) == 2
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 100, 1, 2, W, 4096, 0) == 2     # in % 32
    assert f(A, 2 * A, 0, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 2, W, 4096, 0) == 1
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(1), 5 * A, 1, 16, 128, 1, 2, W, 4096, 0) == 4
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 2, 0, 0, 0) == 5         # no workspace
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 2, W, 16, 0) == 5        # too small
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 2, W + 64, 4096, 0) == 5  # misaligned
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 0, 1, 2, W, 4096, 0) == 7        # empty reduction: not here
    assert f(A, 2 * A, 3 * A, 4 * A, _tok(0), 5 * A, 0, 16, 128, 1, 2, 0, 0, 0) == 0         # no tokens: nothing to do
    assert g(A, 2 * A, 0, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, W, 4096, 0) == 1      # scales missing
    assert g(A, 2 * A, 6 * A + 2, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, W, 4096, 0) == 3
    assert g(A, 2 * A, 6 * A, 3 * A, 4 * A, _tok(2), 5 * A, 1, 16, 128, 2, W, 4096, 0) == 4
    assert g(A, 2 * A, 6 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 0, 0, 0) == 5
    assert g(A, A, 6 * A, 3 * A, 4 * A, _tok(0), A, 1, 16, 128, 1, W, 4096, 0) == 8          # y on top of x
    d = L.bd_linear_multitenant_q8                                                          # the decode form
    assert d(A, 2 * A, 0, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 128, 1, 0) == 1
    assert d(A, 2 * A, 6 * A, 3 * A, 4 * A, _tok(1), 5 * A, 1, 16, 128, 1, 0) == 4
    assert d(A, 2 * A, 6 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 96, 1, 0) == 7           # in % 128: no kernel for it
    assert d(A, 2 * A, 6 * A, 3 * A, 4 * A, _tok(0), 5 * A, 1, 16, 100, 1, 0) == 2
    assert d(A, 2 * A, 6 * A, 3 * A, 4 * A, _tok(0), 5 * A, 0, 16, 128, 1, 0) == 0


def test_compress_noalloc_argument_errors(bd):
    """Errors of the entry point that brings its own scratch are host-side and come before any launch or look-up."""
    c = bd.lib().bd_compress_noalloc
    assert c(A, 2 * A, 16, 100, 3 * A, 4 * A, 0) == 2
    assert c(A, 2 * A, -1, 128, 3 * A, 4 * A, 0) == 2
    assert c(0, 2 * A, 16, 128, 3 * A, 4 * A, 0) == 1
    assert c(A, 2 * A, 16, 128, 3 * A, 0, 0) == 1
    assert c(A + 4, 2 * A, 16, 128, 3 * A, 4 * A, 0) == 3
    assert c(A, 2 * A, 16, 128, A + 1024, 4 * A, 0) == 8
    # beyond 2^32 elements: its own status, also where out * in would overflow 64 bits
    assert c(A, 2 * A, 1 << 17, (1 << 15) + 32, 3 * A, 4 * A, 0) == 11
    assert c(A, 2 * A, 1 << 40, 1 << 40, 3 * A, 4 * A, 0) == 11
    assert bd.status_string(11) != "unknown status"


def test_compress_batch_argument_errors(bd):
    import ctypes
    L = bd.lib()
    need = bd.COMPRESS_BATCH_MAX * bd.workspace_bytes(bd.OP_COMPRESS, 0, 16, 128, 1)
    c = L.bd_compress_batch

    def ptrs(*v):
        return (ctypes.c_void_p * len(v))(*[x or None for x in v])

    def i64s(*v):
        return (ctypes.c_int64 * len(v))(*v)

    MB = 1 << 20   # far enough apart that the 16 x 128 matrices never overlap
    bases, fts, pk = ptrs(A, A + MB), ptrs(A + 2 * MB, A + 3 * MB), ptrs(A + 4 * MB, A + 5 * MB)
    outs, ins = i64s(16, 16), i64s(128, 128)
    assert c(0, None, None, None, None, None, 0, 0, 0, 0) == 0                       # nothing to do
    assert c(-1, bases, fts, outs, ins, pk, 6 * A, 7 * A, need, 0) == 2
    assert c(2, bases, fts, outs, i64s(128, 100), pk, 6 * A, 7 * A, need, 0) == 2      # in % 32
    assert c(2, None, fts, outs, ins, pk, 6 * A, 7 * A, need, 0) == 1
    assert c(2, bases, fts, outs, ins, pk, 0, 7 * A, need, 0) == 1                     # alpha
    assert c(2, ptrs(A, 0), fts, outs, ins, pk, 6 * A, 7 * A, need, 0) == 1            # one matrix missing
    assert c(2, ptrs(A, A + MB + 4), fts, outs, ins, pk, 6 * A, 7 * A, need, 0) == 3
    assert c(2, bases, fts, outs, ins, pk, 6 * A, 0, need, 0) == 5
    assert c(2, bases, fts, outs, ins, pk, 6 * A, 7 * A, need - 1, 0) == 5
    assert c(2, bases, fts, outs, ins, ptrs(A + 4 * MB, A + 1024), 6 * A, 7 * A, need, 0) == 8   # signs of 1 over base 0
    assert c(2, bases, fts, outs, ins, ptrs(A + 4 * MB, A + 4 * MB + 128), 6 * A, 7 * A, need, 0) == 8   # signs over signs
    # an empty matrix needs no pointers
    assert c(1, ptrs(0), ptrs(0), i64s(0), i64s(128), ptrs(0), 6 * A, 0, 0, 0) == 5    # but the call still wants its workspace


def test_tiled_sizes_and_argument_errors(bd):
    L = bd.lib()
    # sizes: tiles of 16 rows x 256 k, 8 KiB of base and 512 B of signs each; zero for rejected shapes
    assert bd.tiled_base_bytes(4096, 4096) == 4096 * 4096 * 2 and bd.tiled_signs_bytes(4096, 4096) == 4096 * 4096 // 8
    assert bd.tiled_base_bytes(50, 640) == 4 * 3 * 8192 and bd.tiled_signs_bytes(50, 640) == 4 * 3 * 512
    assert bd.tiled_base_bytes(16, 40) == 0 and bd.tiled_signs_bytes(-1, 64) == 0
    assert bd.tiled_base_bytes(1 << 20, 1 << 20) == 0          # a tiled tensor of 4 GiB or more is rejected
    tb, ts = L.bd_tile_base, L.bd_tile_signs
    assert tb(A, 16, 40, 2 * A, 0) == 2 and tb(0, 16, 64, 2 * A, 0) == 1 and tb(A, 16, 64, 2 * A + 8, 0) == 3
    assert tb(A, 16, 256, A + 4096, 0) == 8 and tb(0, 0, 64, 0, 0) == 0
    assert ts(A, 16, 40, 2 * A, 0) == 2 and ts(A, 16, 64, 0, 0) == 1 and ts(A + 4, 16, 64, 2 * A, 0) == 3
    vp = ctypes.c_void_p
    f = L.bd_linear_multitenant_tiled
    ok = dict(x=A, w=2 * A, pk=(vp * 1)(3 * A), al=4 * A, tok=_tok(0), y=5 * A, T=1, out=16, inn=128, nt=1)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["x"], a["w"], a["pk"], a["al"], a["tok"], a["y"], a["T"], a["out"], a["inn"], a["nt"], 0)

    assert call(inn=48) == 2 and call(T=-1) == 2 and call(T=70000) == 2
    assert call(x=0) == 1 and call(w=0) == 1 and call(al=0) == 1 and call(y=0) == 1
    assert call(pk=(vp * 1)(None)) == 1                          # the token's tenant has no delta
    assert call(x=A + 2) == 3 and call(w=2 * A + 8) == 3 and call(pk=(vp * 1)(3 * A + 4)) == 3
    assert call(tok=_tok(1)) == 4 and call(tok=_tok(-1)) == 4
    assert call(y=A) == 8 and call(y=2 * A + 64) == 8
    assert call(T=0, x=0, y=0) == 0 and call(out=0, w=0, y=0) == 0
    g = L.bd_linear_multitenant_tiled_group
    i64 = ctypes.c_int64
    args = [A, (vp * 1)(2 * A), (vp * 1)(3 * A), (vp * 1)(4 * A), _tok(0), (vp * 1)(5 * A), 1, (i64 * 1)(16), 128, 1, 0]
    assert g(0, *args) == 2 and g(4, *args) == 2                 # 1..3 matrices per launch


def test_kbit_argument_errors(bd):
    L = bd.lib()
    vp = ctypes.c_void_p
    need = bd.workspace_bytes(bd.OP_COMPRESS, 0, 16, 128, 1)
    c = L.bd_compress_iterated
    assert c(A, 2 * A, 16, 128, 0, 3 * A, 4 * A, 5 * A, need, 0) == 2            # k outside 1..BD_MAX_PLANES
    assert c(A, 2 * A, 16, 128, 9, 3 * A, 4 * A, 5 * A, need, 0) == 2
    assert c(A, 2 * A, 16, 100, 2, 3 * A, 4 * A, 5 * A, need, 0) == 2
    assert c(0, 2 * A, 16, 128, 2, 3 * A, 4 * A, 5 * A, need, 0) == 1
    assert c(A, 2 * A, 16, 128, 2, 3 * A, 0, 5 * A, need, 0) == 1
    assert c(A, 2 * A, 16, 128, 2, 3 * A + 8, 4 * A, 5 * A, need, 0) == 3
    assert c(A, 2 * A, 16, 128, 2, 3 * A, 4 * A, 5 * A, need - 1, 0) == 5
    assert c(A, 2 * A, 16, 128, 2, A + 4096 - 256, 4 * A, 5 * A, need, 0) == 0x8     # the second plane would overwrite w_base
    f = L.bd_linear_multitenant_tiled_kbit
    ok = dict(x=A, w=2 * A, pk=(vp * 2)(3 * A, 3 * A + 4096), al=4 * A, tok=_tok(0), y=5 * A, T=1, out=16, inn=128, nt=1, k=2)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["x"], a["w"], a["pk"], a["al"], a["tok"], a["y"], a["T"], a["out"], a["inn"], a["nt"], a["k"], 0)

    assert call(k=0) == 2 and call(k=9) == 2 and call(inn=48) == 2
    assert call(pk=(vp * 2)(3 * A, None)) == 1                   # every plane of an active tenant is needed
    assert call(pk=(vp * 2)(3 * A, 3 * A + 4)) == 3
    assert call(tok=_tok(1)) == 4 and call(x=0) == 1 and call(y=A) == 8
    assert call(T=0, x=0, y=0) == 0
    g = L.bd_linear_multitenant_tiled_group_kbit
    i64 = ctypes.c_int64
    args = [A, (vp * 1)(2 * A), (vp * 2)(3 * A, 3 * A + 4096), (vp * 1)(4 * A), _tok(0), (vp * 1)(5 * A), 1, (i64 * 1)(16), 128, 1]
    assert g(0, *args, 2, 0) == 2 and g(1, *args, 0, 0) == 2


def test_q8_argument_errors(bd):
    L = bd.lib()
    vp = ctypes.c_void_p
    assert bd.tiled_base_q8_bytes(4096, 4096) == 4096 * 4096 + 4096 * 4
    assert bd.tiled_base_q8_bytes(50, 640) == 4 * 3 * 4096 + 64 * 4 and bd.tiled_base_q8_bytes(16, 40) == 0
    qz = L.bd_quantize_base_q8
    assert qz(A, -1, 64, 2 * A, 3 * A, 0) == 2 and qz(0, 4, 64, 2 * A, 3 * A, 0) == 1 and qz(A, 4, 64, 2 * A, 0, 0) == 1
    assert qz(A, 4, 64, A + 64, 3 * A, 0) == 8 and qz(0, 0, 64, 0, 0, 0) == 0
    need = bd.workspace_bytes(bd.OP_COMPRESS, 0, 16, 128, 1)
    c = L.bd_compress_q8
    assert c(A, 2 * A, 3 * A, 16, 100, 4 * A, 5 * A, 6 * A, need, 0) == 2
    assert c(0, 2 * A, 3 * A, 16, 128, 4 * A, 5 * A, 6 * A, need, 0) == 1
    assert c(A + 4, 2 * A, 3 * A, 16, 128, 4 * A, 5 * A, 6 * A, need, 0) == 3
    assert c(A, 2 * A, 3 * A, 16, 128, 4 * A, 5 * A, 6 * A, need - 1, 0) == 5
    assert c(A, 2 * A, 3 * A, 16, 128, A + 256, 5 * A, 6 * A, need, 0) == 8
    t = L.bd_tile_base_q8
    assert t(A, 2 * A, 16, 40, 3 * A, 0) == 2 and t(A, 0, 16, 64, 3 * A, 0) == 1 and t(A, 2 * A, 16, 64, 3 * A + 4, 0) == 3
    assert t(A, 2 * A, 16, 256, A + 1024, 0) == 8
    f = L.bd_linear_multitenant_tiled_q8
    ok = dict(x=A, w=2 * A, pk=(vp * 1)(3 * A), al=4 * A, tok=_tok(0), y=5 * A, T=1, out=16, inn=128, nt=1)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["x"], a["w"], a["pk"], a["al"], a["tok"], a["y"], a["T"], a["out"], a["inn"], a["nt"], 0)

    assert call(inn=48) == 2 and call(w=0) == 1 and call(w=2 * A + 8) == 3 and call(tok=_tok(1)) == 4
    assert call(y=2 * A + 4096) == 8          # y inside the scales that follow the tiles
    assert call(T=0, x=0, y=0) == 0


def test_group_tokens_sorts_stably_and_cuts_jobs_at_the_tile_boundary(bd):
    import random
    rng = random.Random(5)
    for T in [1, 2, 5, 16, 17, 31, 32]:
        for n_tenants in [1, 3, 40]:
            tok = [rng.randrange(n_tenants) for _ in range(T)]
            cols, jobs = bd.group_tokens(tok)
            assert sorted(cols) == list(range(T))                      # a permutation
            keys = [(tok[t], t) for t in cols]
            assert keys == sorted(keys)                                # sorted by tenant, stable
            covered = []
            for tenant, tile, cb, ce in jobs:
                assert 0 <= cb < ce <= 16 and tile in (0, 1)
                for c in range(cb, ce):
                    assert tok[cols[tile * 16 + c]] == tenant
                    covered.append(tile * 16 + c)
            assert covered == list(range(T))                           # every column in exactly one job, in order
            per_tile = {}
            for tenant, tile, _, _ in jobs:
                assert (tenant, tile) not in per_tile                  # a delta is streamed once per tile
                per_tile[(tenant, tile)] = True
            assert len(jobs) <= len(set(tok)) + 1                      # at most one tenant straddles the boundary
    assert bd.lib().bd_group_tokens(_tok(0), 0, _tok(0), _tok(0), _tok(0), _tok(0), _tok(0), _tok(0)) == 2
    assert bd.lib().bd_group_tokens(_tok(0), 33, _tok(0), _tok(0), _tok(0), _tok(0), _tok(0), _tok(0)) == 2


def test_loading_fails_loudly_without_the_library(bd, tmp_path, monkeypatch):
    monkeypatch.setattr(bd, "_lib", None)
    monkeypatch.setattr(bd, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        bd.lib()
