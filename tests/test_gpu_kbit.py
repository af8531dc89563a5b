"""GPU parity of the k-plane extension (iterated compression, Sec. 4.2 of the paper): bd_compress_iterated bit
for bit against the oracle (planes and scales), bd_linear_multitenant_tiled_kbit(_group) element by element
within 2e-3.  The linear is fed the ORACLE's planes and scales, so compressor noise cannot hide in its budget."""
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


@pytest.mark.parametrize("out,inn,k,sigma", [(64, 256, 1, 0.002), (50, 640, 2, 0.002), (33, 1024, 3, 0.002),
                                             (272, 2176, 5, 0.002), (1024, 4096, 8, 0.002), (4096, 4096, 4, 0.001),
                                             (4, 32, 8, 0.25)])
def test_compress_iterated_bit_exact(ref, out, inn, k, sigma):
    _p(f"compress_iterated {out}x{inn} k={k}")
    base = synth.base_weight(out, inn, device=DEV, tag=("kc", out, inn))
    ft = synth.finetuned_weight(base, sigma=sigma, tag=("kc", out, inn, "ft"))
    packed, alpha = bd.compress_iterated(base, ft, k)
    torch.cuda.synchronize()
    p_ref, a_ref, mean_ref, rsq = ref.compress_iterated(to_np(base), to_np(ft), k)
    assert np.array_equal(to_np(alpha), a_ref), (to_np(alpha), a_ref, mean_ref)
    got = packed_to_np(packed)
    for j in range(k):
        assert np.array_equal(got[j], p_ref[j]), f"plane {j}"
    assert np.all(np.diff(rsq) <= 0)
    # plane 0 is the plain compressor
    p1, a1 = bd.compress(base, ft)
    assert torch.equal(p1, packed[0]) and float(a1.item()) == float(alpha[0].item())


def test_compress_iterated_specials_and_errors(ref):
    base = synth.base_weight(8, 64, device=DEV, tag="kspecial")
    # W_fine == W_base: every residual is zero -> all bits 0, all scales 0
    packed, alpha = bd.compress_iterated(base, base.clone(), 3)
    assert int(packed.abs().sum().item()) == 0 and float(alpha.abs().sum().item()) == 0.0
    ws = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, 8, 64, 1), DEV)
    for k, status in [(0, 2), (9, 2)]:
        with pytest.raises(bd.BitDeltaError) as e:
            bd.compress_iterated(base, base.clone(), k, workspace=ws)
        assert e.value.status == status
    odd = synth.base_weight(3, 96, device=DEV, tag="kodd")       # planes that do not start on 16-byte boundaries
    odd_ft = synth.finetuned_weight(odd, sigma=0.002, tag=("kodd", "ft"))
    packed, alpha = bd.compress_iterated(odd, odd_ft, 3)
    p_ref, a_ref, _, _ = ref.compress_iterated(to_np(odd), to_np(odd_ft), 3)
    assert np.array_equal(packed_to_np(packed), p_ref) and np.array_equal(to_np(alpha), a_ref)


class PlaneProblem:
    """n_tenants fine-tunes of one matrix, each compressed to k planes by the ORACLE; tiled on the device."""

    def __init__(self, ref, out, inn, n_tenants, k, sigma=0.002, tag="kp"):
        self.out, self.inn, self.k = out, inn, k
        self.w_base = synth.base_weight(out, inn, device=DEV, tag=(tag, "base"))
        self.w_base_np = to_np(self.w_base)
        self.planes_np, self.alpha_np = [], []
        for t in range(n_tenants):
            ft = synth.finetuned_weight(self.w_base, sigma=sigma, tag=(tag, "ft", t))
            p, a, _, _ = ref.compress_iterated(self.w_base_np, to_np(ft), k)
            self.planes_np.append([p[j] for j in range(k)])
            self.alpha_np.append(a)
        self.alpha_np = np.array(self.alpha_np, dtype=np.float32)
        self.w_tiled = bd.tile_base(self.w_base)
        self.tiled = [[bd.tile_signs(packed_to_device(p, DEV), out, inn) for p in planes] for planes in self.planes_np]
        self.table = bd.TiledPlaneTable(self.tiled, torch.from_numpy(self.alpha_np).to(DEV))

    def x(self, T):
        return synth.activations(T, self.inn, device=DEV, tag=("kx", T))


KBIT_CASES = [
    # out, in, n_tenants, k, tenant_of_token
    (64, 1024, 3, 2, [2, 0, 1]),                                   # 6 columns, one tile
    (50, 640, 4, 3, [3, 3, 0, 1, 2]),                              # 5 tokens x 3 planes = 15 columns, ragged rows
    (48, 2176, 8, 2, list(range(8))),                              # 16 columns: a full tile of 16 jobs
    (272, 1536, 9, 2, [8, 1, 1, 5, 0, 2, 3, 4, 6, 7, 7, 1]),       # 12 tokens: two column tiles
    (100, 4096, 5, 4, [4, 0, 1, 2, 3, 3, 0]),                      # 4 planes: 4 tokens per tile, 7 tokens = 8 + 8 + ... two tiles
    (80, 512, 3, 8, [1, 2, 0, 1, 1]),                              # 8 planes: 2 tokens per tile, 5 tokens = two launches
    (40, 96, 2, 5, [1, 0, 1]),                                     # 5 planes: 3 tokens per tile, K far below one tile
    (4112, 512, 6, 2, [5, 4, 3, 2, 1, 0, 5, 5]),                   # more row blocks than compute units
    (64, 11008, 4, 2, [0, 1, 2, 3, 3, 2, 1, 0, 0, 1, 2, 3, 0, 1, 2, 3, 1, 1, 2]),   # 19 tokens: two launches; K = 43 tiles
    (32, 256, 2, 1, [1, 0, 1]),                                    # one plane: the 1-bit path
]


@pytest.mark.parametrize("case", range(len(KBIT_CASES)))
def test_kbit_linear_matches_oracle(ref, case):
    out, inn, nt, k, tok = KBIT_CASES[case]
    _p(f"kbit linear case={case} out={out} in={inn} tenants={nt} k={k} T={len(tok)}")
    prob = PlaneProblem(ref, out, inn, nt, k, tag=("klin", case))
    x = prob.x(len(tok))
    y = bd.linear_multitenant_tiled_kbit(x, prob.w_tiled, out, prob.table, tok)
    torch.cuda.synchronize()
    y16, y32 = ref.linear_multitenant_kbit(to_np(x), prob.w_base_np, prob.planes_np, prob.alpha_np, tok)
    check_close(y, y32, f"kbit case {case}")
    y64 = ref.linear_multitenant_kbit_f64(to_np(x), prob.w_base_np, prob.planes_np, prob.alpha_np, tok)
    check_close(y, y64, f"kbit case {case} vs f64")
    ulp = np.abs(to_np(y).view(np.int16).astype(np.int32) - y16.view(np.int16).astype(np.int32))
    same_sign = np.sign(to_np(y).astype(np.float32)) == np.sign(y16.astype(np.float32))
    assert np.mean((ulp <= 1) | ~same_sign) > 0.99
    assert torch.equal(bd.linear_multitenant_tiled_kbit(x, prob.w_tiled, out, prob.table, tok), y)   # reproducible
    if k == 1:
        tt = bd.TiledTenantTable([p[0] for p in prob.tiled], prob.table.alpha)
        assert torch.equal(bd.linear_multitenant_tiled(x, prob.w_tiled, out, tt, tok), y)


@pytest.mark.parametrize("case", range(len(KBIT_CASES)))
def test_kbit_linear_on_row_major_tensors_matches_oracle_and_tiled_call(ref, case):
    """bd_linear_multitenant_kbit: the same k-plane linear read from the row-major base and planes.  Same arithmetic as the
    tiled call up to the order of additions (the k tiles are dealt to the wavefronts differently): the same bits from call to
    call, at most a rounding step from the tiled call's; shapes the row-major kernel cannot run are refused."""
    out, inn, nt, k, tok = KBIT_CASES[case]
    _p(f"kbit row-major case={case} out={out} in={inn} tenants={nt} k={k} T={len(tok)}")
    prob = PlaneProblem(ref, out, inn, nt, k, tag=("klin", case))
    x = prob.x(len(tok))
    planes = [torch.stack([packed_to_device(p, DEV) for p in pl]).contiguous() for pl in prob.planes_np]
    table = bd.PlaneTable(planes, torch.from_numpy(prob.alpha_np).to(DEV))
    if inn % 128 != 0:
        with pytest.raises(bd.BitDeltaError) as e:
            bd.linear_multitenant_kbit(x, prob.w_base, table, tok)
        assert e.value.status == 7
        return
    y = bd.linear_multitenant_kbit(x, prob.w_base, table, tok)
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant_kbit(to_np(x), prob.w_base_np, prob.planes_np, prob.alpha_np, tok)
    check_close(y, y32, f"kbit row-major case {case}")
    assert torch.equal(y, bd.linear_multitenant_kbit(x, prob.w_base, table, tok))   # reproducible
    y_tiled = bd.linear_multitenant_tiled_kbit(x, prob.w_tiled, out, prob.table, tok)
    check_close(y, to_np(y_tiled).astype(np.float32), f"kbit row-major against tiled, case {case}")
    assert np.mean(to_np(y) == to_np(y_tiled)) > 0.9   # most sums round to the same binary16 either way


def test_kbit_more_planes_come_closer_to_the_fine_tuned_weight(ref):
    """The point of the extension: y with k planes approaches x W_fine^T as k grows."""
    out, inn, T = 64, 2048, 4
    base = synth.base_weight(out, inn, device=DEV, tag="kconv")
    ft = synth.finetuned_weight(base, sigma=0.002, tag=("kconv", "ft"))
    x = synth.activations(T, inn, device=DEV, tag="kconv")
    want = to_np(x).astype(np.float64) @ to_np(ft).astype(np.float64).T
    base_only = to_np(x).astype(np.float64) @ to_np(base).astype(np.float64).T
    wt = bd.tile_base(base)
    errs = [float(np.sqrt(np.mean((base_only - want) ** 2)))]
    for k in (1, 2, 4, 8):
        packed, alpha = bd.compress_iterated(base, ft, k)
        table = bd.TiledPlaneTable([[bd.tile_signs(packed[j].contiguous(), out, inn) for j in range(k)]], alpha)
        y = bd.linear_multitenant_tiled_kbit(x, wt, out, table, [0] * T)
        errs.append(float(np.sqrt(np.mean((to_np(y).astype(np.float64) - want) ** 2))))
    _p(f"rms error vs x.W_fine^T for 0,1,2,4,8 planes: {errs}")
    assert errs[1] < 0.7 * errs[0] and errs[2] < 0.8 * errs[1] and errs[3] < 0.8 * errs[2]


def test_kbit_group_and_errors(ref):
    k, nt, inn = 2, 3, 1024
    probs = [PlaneProblem(ref, o, inn, nt, k, tag=("kgrp", i)) for i, o in enumerate((48, 80))]
    tok = [2, 0, 1, 1]
    x = probs[0].x(len(tok))
    g = bd.TiledPlaneGroup([p.w_tiled for p in probs], [p.out for p in probs], [p.table for p in probs])
    ys = bd.linear_multitenant_tiled_group_kbit(x, g, tok)
    for p, y in zip(probs, ys):
        assert torch.equal(y, bd.linear_multitenant_tiled_kbit(x, p.w_tiled, p.out, p.table, tok))
        _, y32 = ref.linear_multitenant_kbit(to_np(x), p.w_base_np, p.planes_np, p.alpha_np, tok)
        check_close(y, y32, "kbit group")
    p = probs[0]
    # an idle tenant may have no planes; an active one must have all of them
    t2 = bd.TiledPlaneTable([p.tiled[0], None, p.tiled[2]], p.table.alpha)
    assert torch.equal(bd.linear_multitenant_tiled_kbit(x[:2].contiguous(), p.w_tiled, p.out, t2, [2, 0]),
                       bd.linear_multitenant_tiled_kbit(x[:2].contiguous(), p.w_tiled, p.out, p.table, [2, 0]))
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled_kbit(x[:1].contiguous(), p.w_tiled, p.out, t2, [1])
    assert e.value.status == 1
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled_kbit(x[:1].contiguous(), p.w_tiled, p.out, p.table, [3])
    assert e.value.status == 4
    assert bd.linear_multitenant_tiled_kbit(x[:0], p.w_tiled, p.out, p.table, []).shape == (0, p.out)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("k,tok", [(2, list(range(8))), (4, [0, 1, 2, 3, 3, 2, 1, 0])])
def test_kbit_llama2_7b_gate_full_output(ref, k, tok):
    """Full size: the gate projection (11008 x 4096) with k planes per tenant, GPU-compressed planes checked bit for
    bit against the oracle's and the linear compared over the whole output."""
    out, inn = 11008, 4096
    nt = max(tok) + 1
    _p(f"7B gate k={k} T={len(tok)} tenants={nt}")
    base = synth.base_weight(out, inn, device=DEV, tag=("k7b", k))
    base_np = to_np(base)
    ws = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, out, inn, 1), DEV)
    tiled, alphas, planes_np = [], [], []
    for t in range(nt):
        ft = synth.finetuned_weight(base, sigma=0.002, tag=("k7b", k, t))
        packed, alpha = bd.compress_iterated(base, ft, k, workspace=ws)
        p_ref, a_ref, _, _ = ref.compress_iterated(base_np, to_np(ft), k)
        del ft
        assert np.array_equal(to_np(alpha), a_ref)
        assert np.array_equal(packed_to_np(packed), p_ref)
        tiled.append([bd.tile_signs(packed[j].contiguous(), out, inn) for j in range(k)])
        alphas.append(alpha)
        planes_np.append([p_ref[j] for j in range(k)])
    table = bd.TiledPlaneTable(tiled, torch.stack(alphas))
    x = synth.activations(len(tok), inn, device=DEV, tag=("k7b", k))
    y = bd.linear_multitenant_tiled_kbit(x, bd.tile_base(base), out, table, tok)
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant_kbit(to_np(x), base_np, planes_np, to_np(torch.stack(alphas)), tok)
    err = check_close(y, y32, f"7B gate k={k}")
    _p(f"   max rel err {err:.2e}")
