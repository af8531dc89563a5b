"""GPU parity of the tiled serving path: the re-layout kernels bit for bit against an index
permutation written out in numpy here, and bd_linear_multitenant_tiled(_group) element by element
against the CPU oracle (which only knows the row-major tensors) within 2e-3."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from paper_2402_10193_amd import synth           # noqa: E402
from gpu_util import Problem, TiledProblem, check_close, packed_to_np, to_np   # noqa: E402

DEV = "cuda"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    bd.lib()


def _p(msg):
    print(msg, flush=True)


def tiled_base_np(w: np.ndarray) -> np.ndarray:
    """Wt[rb][kt][v][l][e] = W[16 rb + l%16][256 kt + 32 v + 8 (l/16) + e], zero padded."""
    out, inn = w.shape
    RB, KT = (out + 15) // 16, (inn + 255) // 256
    pad = np.zeros((RB * 16, KT * 256), dtype=w.dtype)
    pad[:out, :inn] = w
    t = pad.reshape(RB, 16, KT, 8, 4, 8)            # rb, r, kt, v, g, e
    return np.ascontiguousarray(t.transpose(0, 2, 3, 4, 1, 5)).reshape(-1)   # rb, kt, v, g, r, e  (l = 16 g + r)


def tiled_signs_np(bits: np.ndarray) -> np.ndarray:
    """St[rb][kt][l][v] byte, bit e = bits[16 rb + l%16][256 kt + 32 v + 8 (l/16) + e], zero padded."""
    out, inn = bits.shape
    RB, KT = (out + 15) // 16, (inn + 255) // 256
    pad = np.zeros((RB * 16, KT * 256), dtype=np.uint8)
    pad[:out, :inn] = bits
    t = pad.reshape(RB, 16, KT, 8, 4, 8)            # rb, r, kt, v, g, e
    byte = (t << np.arange(8, dtype=np.uint8)).sum(axis=-1).astype(np.uint8)   # rb, r, kt, v, g
    return np.ascontiguousarray(byte.transpose(0, 2, 4, 1, 3)).reshape(-1)      # rb, kt, g, r, v


@pytest.mark.parametrize("out,inn", [(16, 256), (1, 32), (50, 640), (33, 1056), (272, 2176), (4096, 4096), (100, 11008)])
def test_tile_layouts_bit_exact(ref, out, inn):
    _p(f"tile {out}x{inn}")
    w = synth.base_weight(out, inn, device=DEV, tag=("tile", out, inn))
    wt = bd.tile_base(w)
    assert wt.numel() * 2 == bd.tiled_base_bytes(out, inn)
    assert np.array_equal(to_np(wt).view(np.uint16), tiled_base_np(to_np(w).view(np.uint16)))
    packed = torch.randint(-2**31, 2**31 - 1, (out, inn // 32), dtype=torch.int32, device=DEV)
    st = bd.tile_signs(packed, out, inn)
    assert st.numel() * 4 == bd.tiled_signs_bytes(out, inn)
    bits = ((ref.unpack_signs(packed_to_np(packed), inn) + 1) // 2).astype(np.uint8)    # +-1 -> 1/0
    assert np.array_equal(to_np(st).view(np.uint8), tiled_signs_np(bits))


CASES = [
    # out, in, n_tenants, tenant_of_token
    (4096, 4096, 4, [0, 1, 2, 3]),                                   # the single-linear config
    (50, 640, 3, [2, 0, 1]),                                         # ragged rows, K = 2.5 tiles
    (16, 256, 1, [0]),                                               # one tile, one wavefront
    (16, 32, 2, [1, 0]),                                             # K far below one tile
    (33, 1024, 5, [4, 4, 1, 0, 4, 1, 3]),                            # repeats, unsorted, an idle tenant
    (272, 2176, 16, list(range(16))),                                # 16 tenants, K = 8.5 tiles
    (4112, 512, 9, [8, 7, 6, 5, 4, 3, 2, 1, 0, 8, 8]),               # more row blocks than compute units: 4-wave groups
    (100, 4096, 20, [19, 3, 3, 7, 0, 1, 2, 4, 5, 6, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18]),   # 21 tokens: two launches
    (64, 1536, 32, list(range(32))),                                 # 32 tenants
    (40, 96, 2, [1, 0, 1]),                                          # K % 128 != 0
    (64, 11008, 16, list(range(15, -1, -1))),                        # the down-projection's K: 43 tiles
    (80, 2048, 6, [5] * 6 + [1] * 5 + [2] * 5 + [0] * 4 + [1] * 3),  # 23 tokens of 4 tenants: two column tiles, few jobs each
    (48, 1024, 9, [(7 * i) % 9 for i in range(70)]),                 # 70 interleaved tokens: three launches, each tenant's tokens gathered from all over the batch
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_tiled_linear_matches_oracle(ref, case):
    out, inn, nt, tok = CASES[case]
    _p(f"tiled linear case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = TiledProblem(ref, out, inn, nt, tag=("tlin", case))
    x = prob.x(len(tok))
    y = bd.linear_multitenant_tiled(x, prob.w_tiled, out, prob.ttable, tok)
    torch.cuda.synchronize()
    y16, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y32, f"tiled case {case}")
    y64 = ref.linear_multitenant_f64(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y64, f"tiled case {case} vs f64")
    ulp = np.abs(to_np(y).view(np.int16).astype(np.int32) - y16.view(np.int16).astype(np.int32))
    same_sign = np.sign(to_np(y).astype(np.float32)) == np.sign(y16.astype(np.float32))
    assert np.mean((ulp <= 1) | ~same_sign) > 0.99
    # bitwise reproducible
    assert torch.equal(bd.linear_multitenant_tiled(x, prob.w_tiled, out, prob.ttable, tok), y)


def test_tiled_special_inputs(ref):
    """alpha = 0, all-ones / all-zero sign words, one-hot x: exact consequences of Eq. 6."""
    out, inn = 32, 1024
    prob = TiledProblem(ref, out, inn, 1, tag="tspecial")
    x = prob.x(3)
    ones = bd.tile_signs(torch.full((out, inn // 32), -1, dtype=torch.int32, device=DEV), out, inn)
    zeros = bd.tile_signs(torch.zeros((out, inn // 32), dtype=torch.int32, device=DEV), out, inn)
    a = torch.tensor([0.0015], dtype=torch.float32, device=DEV)
    xb = to_np(x).astype(np.float64)
    base = xb @ prob.w_base_np.astype(np.float64).T
    y = bd.linear_multitenant_tiled(x, prob.w_tiled, out, bd.TiledTenantTable([prob.ttable.tiled[0]], torch.zeros(1)), [0, 0, 0])
    check_close(y, base, "alpha=0")
    y = bd.linear_multitenant_tiled(x, prob.w_tiled, out, bd.TiledTenantTable([ones], a), [0, 0, 0])
    check_close(y, base + float(a.item()) * xb.sum(1, keepdims=True), "all +1")
    y = bd.linear_multitenant_tiled(x, prob.w_tiled, out, bd.TiledTenantTable([zeros], a), [0, 0, 0])
    check_close(y, base - float(a.item()) * xb.sum(1, keepdims=True), "all -1")
    for k in (0, 17, 255, 256, 511, 1023):
        xe = torch.zeros((1, inn), dtype=torch.float16, device=DEV)
        xe[0, k] = 1.0
        y = bd.linear_multitenant_tiled(xe, prob.w_tiled, out, prob.ttable, [0])
        s = ref.unpack_signs(prob.packed_np[0], inn)[:, k].astype(np.float32)
        want = (prob.w_base_np[:, k].astype(np.float32) + np.float32(prob.alpha_np[0]) * s).astype(np.float16)
        assert np.array_equal(to_np(y)[0].view(np.uint16), want.view(np.uint16)), k


def test_tiled_matches_row_major_entry_point_and_errors(ref):
    prob = TiledProblem(ref, 48, 1024, 4, tag="tmisc")
    tok = [3, 1, 1, 0, 3, 2, 0]
    x = prob.x(len(tok))
    y_rm = bd.linear_multitenant(x, prob.w_base, prob.table, tok)
    y_t = bd.linear_multitenant_tiled(x, prob.w_tiled, 48, prob.ttable, tok)
    check_close(y_t, to_np(y_rm).astype(np.float32), "tiled vs row-major entry point")
    # an idle tenant's pointer may be NULL
    tt = bd.TiledTenantTable([prob.ttable.tiled[0], None, prob.ttable.tiled[2], None], prob.table.alpha)
    y2 = bd.linear_multitenant_tiled(x[:2].contiguous(), prob.w_tiled, 48, tt, [2, 0])
    y2_ref = bd.linear_multitenant_tiled(x[:2].contiguous(), prob.w_tiled, 48, prob.ttable, [2, 0])
    assert torch.equal(y2, y2_ref)
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled(x[:1].contiguous(), prob.w_tiled, 48, tt, [1])   # tenant 1 has a token but no delta
    assert e.value.status == 1
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled(x[:1].contiguous(), prob.w_tiled, 48, prob.ttable, [4])
    assert e.value.status == 4
    assert bd.linear_multitenant_tiled(x[:0], prob.w_tiled, 48, prob.ttable, []).shape == (0, 48)
    # an empty reduction (in = 0) is a sum of nothing: y = 0, and nothing else is read
    y0 = torch.full((3, 48), 7.0, dtype=torch.float16, device=DEV)
    x0 = torch.empty((3, 0), dtype=torch.float16, device=DEV)
    empty = bd.TiledTenantTable([torch.empty(0, dtype=torch.int32, device=DEV)] * 4, prob.table.alpha)
    bd.linear_multitenant_tiled(x0, torch.empty(0, dtype=torch.float16, device=DEV), 48, empty, [1, 0, 3], y=y0)
    assert float(y0.abs().max().item()) == 0.0


def test_tiled_group_equals_separate_calls(ref):
    """q, k, v style: three matrices over the same x in one launch give the bits of three launches."""
    inn, nt = 1024, 6
    outs = [80, 48, 272]
    probs = [TiledProblem(ref, o, inn, nt, tag=("grp", i)) for i, o in enumerate(outs)]
    tok = [5, 0, 3, 3, 1, 2, 4, 0]
    x = probs[0].x(len(tok))
    group = bd.TiledGroup([p.w_tiled for p in probs], outs, [p.ttable for p in probs])
    ys = bd.linear_multitenant_tiled_group(x, group, tok)
    for i, p in enumerate(probs):
        y1 = bd.linear_multitenant_tiled(x, p.w_tiled, outs[i], p.ttable, tok)
        assert torch.equal(ys[i], y1), i
        _, y32 = ref.linear_multitenant(to_np(x), p.w_base_np, p.packed_np, p.alpha_np, tok)
        check_close(ys[i], y32, f"group matrix {i}")
