"""GPU parity of the GEMM form (prefill regime, Sec. 4.3 of the paper) of the two extensions of Sec. 4.2: k sign planes per
tenant (bd_linear_multitenant_gemm_kbit) and the 8-bit base (bd_linear_multitenant_gemm_q8), element by element against the
oracle's k-plane / 8-bit-base linear, within the linear's tolerance."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from paper_2402_10193_amd import synth           # noqa: E402
from gpu_util import check_close, packed_to_device, to_np   # noqa: E402
from test_gpu_kbit import PlaneProblem           # noqa: E402
from test_gpu_q8 import Q8Problem                # noqa: E402

DEV = "cuda"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    bd.lib()


def _p(msg):
    print(msg, flush=True)


def mixed_tokens(n_tenants, counts, seed):
    """counts[i] tokens of tenant i (0 = idle), shuffled."""
    tok = [t for t in range(n_tenants) for _ in range(counts[t])]
    rng = np.random.default_rng(seed)
    rng.shuffle(tok)
    return [int(t) for t in tok]


GEMM_KBIT_CASES = [
    # out, in, n_tenants, k, tokens per tenant
    (64, 1024, 3, 2, [5, 0, 2]),                 # far below one tile, an idle tenant
    (50, 640, 4, 3, [130, 1, 0, 40]),            # ragged rows and k, a tenant with two tiles
    (272, 96, 2, 5, [129, 127]),                 # in = 96: a ragged last k step
    (300, 2176, 5, 8, [33, 64, 1, 128, 7]),      # eight planes
    (128, 512, 2, 1, [200, 100]),                # one plane: the 1-bit formula
    (4112, 512, 3, 2, [128, 128, 3]),            # more output tiles than one round
]


@pytest.mark.parametrize("case", range(len(GEMM_KBIT_CASES)))
def test_gemm_kbit_matches_oracle(ref, case):
    out, inn, nt, k, counts = GEMM_KBIT_CASES[case]
    tok = mixed_tokens(nt, counts, 100 + case)
    _p(f"gemm kbit case={case} out={out} in={inn} tenants={nt} k={k} T={len(tok)}")
    prob = PlaneProblem(ref, out, inn, nt, k, tag=("gk", case))
    x = prob.x(len(tok))
    planes = [torch.stack([packed_to_device(p, DEV) for p in pl]).contiguous() for pl in prob.planes_np]
    table = bd.PlaneTable(planes, torch.from_numpy(prob.alpha_np).to(DEV))
    y = bd.linear_multitenant_gemm_kbit(x, prob.w_base, table, tok)
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant_kbit(to_np(x), prob.w_base_np, prob.planes_np, prob.alpha_np, tok)
    check_close(y, y32, f"gemm kbit case {case}")
    assert torch.equal(y, bd.linear_multitenant_gemm_kbit(x, prob.w_base, table, tok))   # reproducible
    if inn % 128 == 0:   # the decode launches of the same call family agree within the same tolerance
        check_close(bd.linear_multitenant_kbit(x, prob.w_base, table, tok), y32, f"decode kbit case {case}")


GEMM_Q8_CASES = [
    (64, 1024, 3, [5, 0, 2]),
    (50, 640, 4, [130, 1, 0, 40]),
    (272, 96, 2, [129, 127]),
    (300, 2176, 5, [33, 64, 1, 128, 7]),
    (4112, 512, 3, [128, 128, 3]),
]


def q8_device(prob):
    q = torch.from_numpy(prob.q_np).to(DEV)
    s = torch.from_numpy(prob.s_np).to(DEV)
    table = bd.TenantTable([packed_to_device(p, DEV) for p in prob.packed_np],
                           torch.tensor(prob.alpha_np, dtype=torch.float32, device=DEV))
    return q, s, table


@pytest.mark.parametrize("case", range(len(GEMM_Q8_CASES)))
def test_gemm_q8_matches_oracle(ref, case):
    out, inn, nt, counts = GEMM_Q8_CASES[case]
    tok = mixed_tokens(nt, counts, 200 + case)
    _p(f"gemm q8 case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = Q8Problem(ref, out, inn, nt, ("gq", case))
    q, s, table = q8_device(prob)
    x = prob.x(len(tok))
    y = bd.linear_multitenant_gemm_q8(x, q, s, table, tok)
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant_q8(to_np(x), prob.q_np, prob.s_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y32, f"gemm q8 case {case}")
    y64 = ref.linear_multitenant_q8_f64(to_np(x), prob.q_np, prob.s_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y64, f"gemm q8 case {case} vs f64")
    assert torch.equal(y, bd.linear_multitenant_gemm_q8(x, q, s, table, tok))
    # same tenants through the decode kernel on the tiled 8-bit base: within the tolerance of each other as well
    if len(tok) <= 32:
        check_close(bd.linear_multitenant_tiled_q8(x, prob.wq, out, prob.table, tok), y32, "tiled q8")


def test_gemm_variants_errors(ref):
    prob = PlaneProblem(ref, 64, 256, 2, 2, tag=("gke", 0))
    planes = [torch.stack([packed_to_device(p, DEV) for p in pl]).contiguous() for pl in prob.planes_np]
    table = bd.PlaneTable(planes, torch.from_numpy(prob.alpha_np).to(DEV))
    x = prob.x(3)
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    need = bd.workspace_bytes(bd.OP_LINEAR_GEMM, 3, 64, 256, 2)
    assert need > 0 and need % 256 == 0
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_gemm_kbit(x, prob.w_base, table, [0, 1, 1], workspace=small[:16])
    assert e.value.status == 5   # workspace too small
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant_gemm_kbit(x, prob.w_base, table, [0, 2, 1])
    assert e.value.status == 4   # tenant out of range
    assert bd.linear_multitenant_gemm_kbit(x[:0], prob.w_base, table, []).shape == (0, 64)


@pytest.mark.timeout(900)
def test_gemm_kbit_and_q8_llama2_7b_gate(ref):
    """The 7B gate projection (11008 x 4096), 4 tenants x 40 tokens: two planes per tenant, then the 8-bit base."""
    out, inn, nt, per = 11008, 4096, 4, 40
    tok = mixed_tokens(nt, [per] * nt, 7)
    _p(f"7B gate, gemm kbit k=2 and q8, T={len(tok)}")
    prob = PlaneProblem(ref, out, inn, nt, 2, tag=("gk7b",))
    x = prob.x(len(tok))
    planes = [torch.stack([packed_to_device(p, DEV) for p in pl]).contiguous() for pl in prob.planes_np]
    table = bd.PlaneTable(planes, torch.from_numpy(prob.alpha_np).to(DEV))
    y = bd.linear_multitenant_gemm_kbit(x, prob.w_base, table, tok)
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant_kbit(to_np(x), prob.w_base_np, prob.planes_np, prob.alpha_np, tok)
    check_close(y, y32, "7B gate gemm kbit")
    del prob, planes, table
    qp = Q8Problem(ref, out, inn, nt, ("gq7b",))
    q, s, qtable = q8_device(qp)
    xq = qp.x(len(tok))
    yq = bd.linear_multitenant_gemm_q8(xq, q, s, qtable, tok)
    torch.cuda.synchronize()
    _, yq32 = ref.linear_multitenant_q8(to_np(xq), qp.q_np, qp.s_np, qp.packed_np, qp.alpha_np, tok)
    check_close(yq, yq32, "7B gate gemm q8")
