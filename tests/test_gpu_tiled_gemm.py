"""GPU parity of bd_linear_multitenant_tiled_gemm: the prefill GEMM reading the serving layout (one copy of the base and
of every delta for decode and prefill).  Both forms against the CPU oracle, and bit for bit against the same kernels on
the row-major tensors (same arithmetic in the same order; only the addresses differ)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from gpu_util import TiledProblem, check_close, to_np   # noqa: E402

DEV = "cuda"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    bd.lib()


def _p(msg):
    print(msg, flush=True)


CASES = [
    # out, in, n_tenants, tokens per tenant (shuffled)
    (300, 512, 5, [70, 1, 0, 129, 40]),          # out not a multiple of 16 (padded row block), an idle tenant
    (1024, 2048, 8, [160] * 8),                  # 8 k tiles of the serving layout
    (520, 192, 3, [40, 3, 90]),                  # in below one k tile of 256: three steps inside a partly filled tile
    (256, 64, 2, [33, 1]),                       # one step
    (300, 320, 4, [257, 512, 130, 128]),         # five steps across two k tiles; token tiles of 256: whole, short, single row
    (64, 1088, 2, [20, 13]),                     # 17 steps: 4 whole k tiles and a quarter; T = 33
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_tiled_gemm_matches_oracle_and_the_row_major_kernels(ref, case):
    out, inn, nt, counts = CASES[case]
    tok = [t for t, c in enumerate(counts) for _ in range(c)]
    perm = torch.randperm(len(tok), generator=torch.Generator().manual_seed(100 + case)).tolist()
    tok = [tok[i] for i in perm]
    _p(f"tiled gemm case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = TiledProblem(ref, out, inn, nt, tag=("tg", case))
    # tenants without a token may be absent from the table
    ttable = bd.TiledTenantTable([t if counts[i] > 0 else None for i, t in enumerate(prob.ttable.tiled)], prob.ttable.alpha)
    x = prob.x(len(tok))
    _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    y = bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, out, ttable, tok)
    torch.cuda.synchronize()
    check_close(y, y32, f"tiled gemm case {case}")
    assert torch.equal(y, bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=5)), "two products: tiled != row-major"
    assert torch.equal(bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, out, ttable, tok), y)
    # one product on W + alpha S rounded to fp16: the oracle's materialised weights; bit for bit variant 8 on row-major tensors
    w_ft = [ref.materialise_f16(prob.w_base_np, prob.packed_np[t], prob.alpha_np[t]) for t in range(nt)]
    _, n32 = ref.linear_naive(to_np(x), w_ft, tok)
    y1 = bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, out, ttable, tok, one_product=True)
    torch.cuda.synchronize()
    check_close(y1, n32, f"tiled gemm case {case}, one product")
    check_close(y1, y32, f"tiled gemm case {case}, one product against the two products", elementwise=False)
    assert torch.equal(y1, bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=8)), "one product: tiled != row-major"


def test_tiled_gemm_tokens_grouped_by_tenant_and_a_single_token(ref):
    out, inn, nt = 272, 256, 3
    prob = TiledProblem(ref, out, inn, nt, tag=("tg", "grouped"))
    for name, tok in (("grouped", [0] * 140 + [1] * 5 + [2] * 260), ("one token", [1])):
        _p(f"tiled gemm {name}, T={len(tok)}")
        x = prob.x(len(tok))
        _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
        for one in (False, True):
            y = bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, out, prob.ttable, tok, one_product=one)
            check_close(y, y32, f"tiled gemm {name}, one_product={one}", elementwise=not one)


def test_tiled_gemm_errors(ref):
    prob = TiledProblem(ref, 64, 96, 2, tag=("tg", "err"))        # 96: whole sign words, but no whole step of 64
    tok = [0] * 40
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled_gemm(prob.x(40), prob.w_tiled, 64, prob.ttable, tok)
    assert e.value.status == 7
    prob = TiledProblem(ref, 64, 128, 2, tag=("tg", "err2"))
    x = prob.x(40)
    need = bd.workspace_bytes(bd.OP_LINEAR_TILED_GEMM, 40, 64, 128, 2)
    assert need > 0 and need % 256 == 0
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, 64, prob.ttable, tok, workspace=bd.new_workspace(need, DEV)[:need - 256])
    assert e.value.status == 5
    absent = bd.TiledTenantTable([None, prob.ttable.tiled[1]], prob.ttable.alpha)
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, 64, absent, tok)           # tenant 0 has tokens but no delta
    assert e.value.status == 1
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, 64, prob.ttable, [0] * 39 + [2])
    assert e.value.status == 4
    y = bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, 64, absent, [1] * 40)       # the absent tenant is idle: fine
    _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, [1] * 40)
    check_close(y, y32, "tiled gemm with an absent idle tenant")
