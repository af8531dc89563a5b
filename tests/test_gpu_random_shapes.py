"""Seeded sweep over shapes nobody picked by hand: every entry point of the linear (Eq. 6 of the paper) against the
oracle on small random problems -- ragged out, K from one 32-element word up to a few tiles, idle and repeated
tenants, token counts on both sides of the decode / prefill boundary."""
import random

import pytest
import torch

from paper_2402_10193_amd import binding as bd
from gpu_util import Problem, TiledProblem, check_close, to_np

pytestmark = pytest.mark.gpu


def _p(msg):
    print(msg, flush=True)


def _draw(case):
    """out, in, n_tenants, tenant_of_token for case number `case` (pure function of the number)."""
    r = random.Random(9100 + case)
    out = r.choice([1, 7, 16, 31, 48, 100, 129, 255, 256, 300, 513, 700])
    inn = 32 * r.choice([1, 2, 3, 4, 5, 8, 9, 16, 17, 24, 40])
    n_tenants = r.randint(1, 12)
    if case % 3 == 0:
        T = r.randint(1, 32)        # decode launches
    elif case % 3 == 1:
        T = r.randint(33, 140)      # just beyond: the GEMM with mostly empty tiles
    else:
        T = r.randint(141, 420)     # several tiles per tenant
    live = r.sample(range(n_tenants), r.randint(1, n_tenants))   # the other tenants stay idle
    tok = [r.choice(live) for _ in range(T)]
    return out, inn, n_tenants, tok


@pytest.mark.parametrize("case", range(18))
def test_random_shapes_row_major_entry_point(ref, case):
    out, inn, nt, tok = _draw(case)
    _p(f"random shape case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = Problem(ref, out, inn, nt, tag=("rnd", case))
    x = prob.x(len(tok))
    _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    y = bd.linear_multitenant(x, prob.w_base, prob.table, tok)                      # library's choice, workspace given
    check_close(y, y32, f"random case {case}")
    y_nows = bd.linear_multitenant(x, prob.w_base, prob.table, tok, workspace=None)  # decode launches only
    check_close(y_nows, y32, f"random case {case}, no workspace")
    y1 = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=1)           # vector-ALU kernel
    check_close(y1, y32, f"random case {case}, variant 1")
    if len(tok) > 32:
        variants = [4] + ([5, 6, 7, 8] if inn % 64 == 0 else [])
        for v in variants:
            yv = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=v)
            # (8: one product on W + alpha S rounded to fp16; the bar on the largest error holds against the two products)
            check_close(yv, y32, f"random case {case}, variant {v}", elementwise=v != 8)
    torch.cuda.synchronize()


@pytest.mark.parametrize("case", range(0, 18, 3))
def test_random_shapes_tiled_entry_point(ref, case):
    out, inn, nt, tok = _draw(case)
    _p(f"random shape, tiled layout, case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = TiledProblem(ref, out, inn, nt, tag=("rnd", case))
    x = prob.x(len(tok))
    _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    y = bd.linear_multitenant_tiled(x, prob.w_tiled, out, prob.ttable, tok)
    check_close(y, y32, f"random case {case}, tiled")
    assert torch.equal(bd.linear_multitenant_tiled(x, prob.w_tiled, out, prob.ttable, tok), y)   # bitwise reproducible
    torch.cuda.synchronize()
