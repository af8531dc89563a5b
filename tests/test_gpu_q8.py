"""GPU parity of the 8-bit base (Sec. 4.2 of the paper, quantized base models): quantiser, compressor and re-layout
bit for bit against the oracle / an index permutation written out here, the linear within 2e-3."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from paper_2402_10193_amd import synth           # noqa: E402
from gpu_util import check_close, packed_to_device, packed_to_np, to_np   # noqa: E402

DEV = "cuda"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    bd.lib()


def _p(msg):
    print(msg, flush=True)


def tiled_q8_np(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Wq[rb][kt][i][l][h][e] = 128 + q[16 rb + l%16][256 kt + 32 (2 i + h) + 8 (l/16) + e], then 16 scales per row block."""
    out, inn = q.shape
    RB, KT = (out + 15) // 16, (inn + 255) // 256
    pad = np.zeros((RB * 16, KT * 256), dtype=np.int16)
    pad[:out, :inn] = q
    u = (pad + 128).astype(np.uint8)
    t = u.reshape(RB, 16, KT, 4, 2, 4, 8)                       # rb, r, kt, i, h, g, e
    tiles = np.ascontiguousarray(t.transpose(0, 2, 3, 5, 1, 4, 6)).reshape(-1)   # rb, kt, i, g, r, h, e   (l = 16 g + r)
    sc = np.zeros(RB * 16, dtype=np.float32)
    sc[:out] = scale
    return np.concatenate([tiles, sc.view(np.uint8)])


@pytest.mark.parametrize("out,inn", [(16, 256), (3, 96), (50, 640), (272, 2176), (4096, 4096), (100, 11008)])
def test_quantiser_compressor_and_layout_bit_exact(ref, out, inn):
    _p(f"q8 {out}x{inn}")
    w = synth.base_weight(out, inn, device=DEV, tag=("q8", out, inn))
    if out > 2:
        w[1].zero_()                                             # an all-zero row: scale 1, q 0
        w[2, :8] = torch.tensor([1.5, 2.5, -0.5, -1.5, 127, -127, 63.5, 0.25], dtype=torch.float16, device=DEV) / 64
        w[2, 8:] = 0                                             # scale exactly 1/64: ties go to even
    q, scale = bd.quantize_base_q8(w)
    q_ref, s_ref = ref.quantize_rtn8(to_np(w))
    assert np.array_equal(to_np(scale), s_ref)
    assert np.array_equal(to_np(q), q_ref)
    ft = synth.finetuned_weight(w, sigma=0.002, tag=("q8", out, inn, "ft"))
    packed, alpha = bd.compress_q8(q, scale, ft)
    p_ref, a_ref, _ = ref.compress_q8(q_ref, s_ref, to_np(ft))
    assert np.array_equal(packed_to_np(packed), p_ref)
    assert float(alpha.item()) == a_ref
    wq = bd.tile_base_q8(q, scale)
    assert wq.numel() == bd.tiled_base_q8_bytes(out, inn)
    assert np.array_equal(to_np(wq), tiled_q8_np(q_ref, s_ref))


class Q8Problem:
    def __init__(self, ref, out, inn, n_tenants, tag):
        self.out, self.inn = out, inn
        w = synth.base_weight(out, inn, device=DEV, tag=(tag, "base"))
        self.q_np, self.s_np = ref.quantize_rtn8(to_np(w))
        q = torch.from_numpy(self.q_np).to(DEV)
        s = torch.from_numpy(self.s_np).to(DEV)
        self.wq = bd.tile_base_q8(q, s)
        self.packed_np, self.alpha_np = [], []
        for t in range(n_tenants):
            ft = synth.finetuned_weight(w, sigma=0.002, tag=(tag, "ft", t))
            p, a, _ = ref.compress_q8(self.q_np, self.s_np, to_np(ft))
            self.packed_np.append(p)
            self.alpha_np.append(a)
        self.table = bd.TiledTenantTable([bd.tile_signs(packed_to_device(p, DEV), out, inn) for p in self.packed_np],
                                         torch.tensor(self.alpha_np, dtype=torch.float32, device=DEV))

    def x(self, T):
        return synth.activations(T, self.inn, device=DEV, tag=("q8x", T))


Q8_CASES = [
    (4096, 4096, 4, [0, 1, 2, 3]),
    (50, 640, 3, [2, 0, 1]),
    (16, 32, 2, [1, 0]),
    (33, 1024, 5, [4, 4, 1, 0, 4, 1, 3]),
    (272, 2176, 16, list(range(16))),
    (4112, 512, 9, [8, 7, 6, 5, 4, 3, 2, 1, 0, 8, 8]),
    (100, 4096, 20, [19, 3, 3, 7, 0, 1, 2, 4, 5, 6, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18]),
    (64, 1536, 32, list(range(32))),
    (64, 11008, 16, list(range(15, -1, -1))),
]


@pytest.mark.parametrize("case", range(len(Q8_CASES)))
def test_q8_linear_matches_oracle(ref, case):
    out, inn, nt, tok = Q8_CASES[case]
    _p(f"q8 linear case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = Q8Problem(ref, out, inn, nt, ("q8lin", case))
    x = prob.x(len(tok))
    y = bd.linear_multitenant_tiled_q8(x, prob.wq, out, prob.table, tok)
    torch.cuda.synchronize()
    y16, y32 = ref.linear_multitenant_q8(to_np(x), prob.q_np, prob.s_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y32, f"q8 case {case}")
    y64 = ref.linear_multitenant_q8_f64(to_np(x), prob.q_np, prob.s_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y64, f"q8 case {case} vs f64")
    ulp = np.abs(to_np(y).view(np.int16).astype(np.int32) - y16.view(np.int16).astype(np.int32))
    same_sign = np.sign(to_np(y).astype(np.float32)) == np.sign(y16.astype(np.float32))
    assert np.mean((ulp <= 1) | ~same_sign) > 0.99
    assert torch.equal(bd.linear_multitenant_tiled_q8(x, prob.wq, out, prob.table, tok), y)


@pytest.mark.parametrize("case", range(len(Q8_CASES)))
def test_q8_linear_on_row_major_tensors_matches_oracle(ref, case):
    """bd_linear_multitenant_q8: the same linear read from the row-major int8 base and its `out` scales."""
    out, inn, nt, tok = Q8_CASES[case]
    _p(f"q8 row-major case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = Q8Problem(ref, out, inn, nt, ("q8lin", case))
    x = prob.x(len(tok))
    q = torch.from_numpy(prob.q_np).to(DEV)
    s = torch.from_numpy(prob.s_np).to(DEV)
    table = bd.TenantTable([packed_to_device(p, DEV) for p in prob.packed_np],
                           torch.tensor(prob.alpha_np, dtype=torch.float32, device=DEV))
    if inn % 128 != 0:
        with pytest.raises(bd.BitDeltaError) as e:
            bd.linear_multitenant_q8(x, q, s, table, tok)
        assert e.value.status == 7
        return
    y = bd.linear_multitenant_q8(x, q, s, table, tok)
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant_q8(to_np(x), prob.q_np, prob.s_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y32, f"q8 row-major case {case}")
    assert torch.equal(y, bd.linear_multitenant_q8(x, q, s, table, tok))   # reproducible
    y_tiled = bd.linear_multitenant_tiled_q8(x, prob.wq, out, prob.table, tok)
    check_close(y, to_np(y_tiled).astype(np.float32), f"q8 row-major against tiled, case {case}")


def test_q8_row_major_more_tokens_than_one_launch(ref):
    """75 tokens of 5 tenants: three decode launches of the row-major 8-bit kernel, tokens grouped by tenant across them."""
    out, inn, nt = 80, 1152, 5
    rng = np.random.default_rng(5)
    tok = [int(t) for t in rng.integers(0, nt, size=75)]
    prob = Q8Problem(ref, out, inn, nt, ("q8many",))
    x = prob.x(len(tok))
    q = torch.from_numpy(prob.q_np).to(DEV)
    s = torch.from_numpy(prob.s_np).to(DEV)
    table = bd.TenantTable([packed_to_device(p, DEV) for p in prob.packed_np],
                           torch.tensor(prob.alpha_np, dtype=torch.float32, device=DEV))
    y = bd.linear_multitenant_q8(x, q, s, table, tok)
    _, y32 = ref.linear_multitenant_q8(to_np(x), prob.q_np, prob.s_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y32, "q8 row-major, 75 tokens")
    check_close(bd.linear_multitenant_gemm_q8(x, q, s, table, tok), y32, "q8 gemm, 75 tokens")


def test_q8_row_major_output_right_behind_the_int8_base(ref):
    """y may start right where the out * in BYTES of q end (the alias check must not take q for an fp16 tensor)."""
    out, inn, nt, tok = 50, 640, 3, [2, 0, 1]
    prob = Q8Problem(ref, out, inn, nt, ("q8adj",))
    x = prob.x(len(tok))
    buf = torch.empty(out * inn + len(tok) * out * 2, dtype=torch.uint8, device=DEV)
    q = buf[:out * inn].view(torch.int8).view(out, inn)
    q.copy_(torch.from_numpy(prob.q_np).to(DEV))
    y = buf[out * inn:].view(torch.float16).view(len(tok), out)
    s = torch.from_numpy(prob.s_np).to(DEV)
    table = bd.TenantTable([packed_to_device(p, DEV) for p in prob.packed_np],
                           torch.tensor(prob.alpha_np, dtype=torch.float32, device=DEV))
    _, y32 = ref.linear_multitenant_q8(to_np(x), prob.q_np, prob.s_np, prob.packed_np, prob.alpha_np, tok)
    bd.linear_multitenant_q8(x, q, s, table, tok, y=y)
    check_close(y, y32, "y behind q, decode")
    y.zero_()
    bd.linear_multitenant_gemm_q8(x, q, s, table, tok, y=y)
    check_close(y, y32, "y behind q, gemm")
    with pytest.raises(bd.BitDeltaError) as e:   # and one byte earlier it does overlap
        bd.linear_multitenant_q8(x, q, s, table, tok, y=buf[out * inn - 16:out * inn - 16 + len(tok) * out * 2].view(torch.float16).view(len(tok), out))
    assert e.value.status == 8


def test_q8_group_and_errors(ref):
    inn, nt = 1024, 3
    probs = [Q8Problem(ref, o, inn, nt, ("q8grp", i)) for i, o in enumerate((48, 80, 32))]
    tok = [2, 0, 1, 1]
    x = probs[0].x(len(tok))
    g = bd.TiledGroup([p.wq for p in probs], [p.out for p in probs], [p.table for p in probs])
    ys = bd.linear_multitenant_tiled_group_q8(x, g, tok)
    for p, y in zip(probs, ys):
        assert torch.equal(y, bd.linear_multitenant_tiled_q8(x, p.wq, p.out, p.table, tok))
    p = probs[0]
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled_q8(x[:1].contiguous(), p.wq, p.out, p.table, [3])
    assert e.value.status == 4
    assert bd.linear_multitenant_tiled_q8(x[:0], p.wq, p.out, p.table, []).shape == (0, p.out)
    assert bd.tiled_base_q8_bytes(50, 640) == 4 * 3 * 4096 + 4 * 16 * 4 and bd.tiled_base_q8_bytes(16, 40) == 0


@pytest.mark.timeout(600)
def test_q8_llama2_7b_gate_b16_full_output(ref):
    out, inn, B = 11008, 4096, 16
    _p("7B gate q8 B=16")
    w = synth.base_weight(out, inn, device=DEV, tag=("q87b", "base"))
    q, scale = bd.quantize_base_q8(w)
    q_np, s_np = ref.quantize_rtn8(to_np(w))
    assert np.array_equal(to_np(q), q_np) and np.array_equal(to_np(scale), s_np)
    ws = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, out, inn, 1), DEV)
    tiled, alphas, packed_np, alphas_ref = [], [], [], []
    for t in range(B):
        ft = synth.finetuned_weight(w, sigma=0.002, tag=("q87b", t))
        p, a = bd.compress_q8(q, scale, ft, workspace=ws)
        p_ref, a_ref, _ = ref.compress_q8(q_np, s_np, to_np(ft))
        del ft
        assert np.array_equal(packed_to_np(p), p_ref) and float(a.item()) == a_ref
        tiled.append(bd.tile_signs(p, out, inn))
        alphas.append(a)
        packed_np.append(p_ref)
        alphas_ref.append(a_ref)
    table = bd.TiledTenantTable(tiled, alphas)
    x = synth.activations(B, inn, device=DEV, tag=("q87b", "x"))
    tok = synth.one_token_per_tenant(B)
    y = bd.linear_multitenant_tiled_q8(x, bd.tile_base_q8(q, scale), out, table, tok)
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant_q8(to_np(x), q_np, s_np, packed_np, alphas_ref, tok)
    err = check_close(y, y32, "7B gate q8")
    _p(f"   max rel err {err:.2e}")
