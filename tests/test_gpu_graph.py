"""The library's calls under HIP graph capture: a graph of decode launches, one of the prefill GEMMs (whose token tables
travel in kernel arguments, so nothing is copied from the host at replay) and one of the compressor that brings its own
scratch, each replayed several times with new inputs, eager work of the program and synchronisations between the
replays, and every replay compared with the eager call on the same inputs (bit for bit: fixed summation orders)."""
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from paper_2402_10193_amd import synth           # noqa: E402
from gpu_util import TiledProblem, check_close, to_np   # noqa: E402

DEV = "cuda"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    bd.lib()


def _p(msg):
    print(msg, flush=True)


def _capture(run):
    """Once eagerly (kernel attributes are set on first use, outside any capture), once on a side stream, then captured."""
    run()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    return graph


def test_decode_launches_replayed_from_a_graph(ref):
    """A grouped launch (two matrices on one x), then a linear on its own with streamed x, 16 and 32 tokens."""
    out_a, out_b, inn, nt = 272, 96, 1024, 6
    pa = TiledProblem(ref, out_a, inn, nt, tag=("graph", "a"))
    pb = TiledProblem(ref, out_b, inn, nt, tag=("graph", "b"))
    pc = TiledProblem(ref, 64, 2304, nt, tag=("graph", "c"))             # in = 2304: x streamed per task
    group = bd.TiledGroup([pa.w_tiled, pb.w_tiled], [out_a, out_b], [pa.ttable, pb.ttable])
    for T in (16, 32):
        _p(f"decode graph, T={T}")
        tok = [(5 * i + 1) % nt for i in range(T)]
        tok_arr = bd._tok_array(tok)
        x, xc = torch.empty((T, inn), dtype=torch.float16, device=DEV), torch.empty((T, 2304), dtype=torch.float16, device=DEV)
        ys = [torch.empty((T, o), dtype=torch.float16, device=DEV) for o in (out_a, out_b)]
        yc = torch.empty((T, 64), dtype=torch.float16, device=DEV)

        def run():
            bd.linear_multitenant_tiled_group(x, group, tok, ys=ys, tok_array=tok_arr)
            bd.linear_multitenant_tiled(xc, pc.w_tiled, 64, pc.ttable, tok, y=yc, tok_array=tok_arr)
        x.copy_(synth.activations(T, inn, device=DEV, tag=("graph", "x", T, -1)))
        xc.copy_(synth.activations(T, 2304, device=DEV, tag=("graph", "xc", T, -1)))
        graph = _capture(run)
        for rep in range(4):
            x.copy_(synth.activations(T, inn, device=DEV, tag=("graph", "x", T, rep)))
            xc.copy_(synth.activations(T, 2304, device=DEV, tag=("graph", "xc", T, rep)))
            for y in ys + [yc]:
                y.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            got = [y.clone() for y in ys + [yc]]
            # the program's own eager work between the replays: the same launches outside the graph
            want = bd.linear_multitenant_tiled_group(x, group, tok) + [bd.linear_multitenant_tiled(xc, pc.w_tiled, 64, pc.ttable, tok)]
            torch.cuda.synchronize()
            for g, w in zip(got, want):
                assert torch.equal(g, w), f"replay {rep}"
            if rep == 0:
                _, y32 = ref.linear_multitenant(to_np(x), pa.w_base_np, pa.packed_np, pa.alpha_np, tok)
                check_close(got[0], y32, "graph replay against the oracle")


def test_prefill_gemms_replayed_from_a_graph(ref):
    """The GEMM on the row-major tensors (two products, one product) and on the serving layout in one graph."""
    out, inn, nt = 300, 512, 4
    counts = [70, 1, 129, 300]
    tok = [t for t, c in enumerate(counts) for _ in range(c)]
    perm = torch.randperm(len(tok), generator=torch.Generator().manual_seed(7)).tolist()
    tok = [tok[i] for i in perm]
    T = len(tok)
    tok_arr = bd._tok_array(tok)
    prob = TiledProblem(ref, out, inn, nt, tag=("graph", "pf"))
    x = torch.empty((T, inn), dtype=torch.float16, device=DEV)
    y2, y1, yt = (torch.empty((T, out), dtype=torch.float16, device=DEV) for _ in range(3))
    ws = [bd.new_workspace(bd.workspace_bytes(bd.OP_LINEAR_MULTITENANT, T, out, inn, nt), DEV) for _ in range(2)]
    ws_t = bd.new_workspace(bd.workspace_bytes(bd.OP_LINEAR_TILED_GEMM, T, out, inn, nt), DEV)

    def run():
        bd.linear_multitenant(x, prob.w_base, prob.table, tok, y=y2, tok_array=tok_arr, workspace=ws[0], variant=5)
        bd.linear_multitenant(x, prob.w_base, prob.table, tok, y=y1, tok_array=tok_arr, workspace=ws[1], variant=8)
        bd.linear_multitenant_tiled_gemm(x, prob.w_tiled, out, prob.ttable, tok, y=yt, workspace=ws_t, tok_array=tok_arr)
    x.copy_(prob.x(T, tag="warm"))
    graph = _capture(run)
    for rep in range(3):
        _p(f"prefill graph, replay {rep}")
        x.copy_(prob.x(T, tag=("rep", rep)))
        for w in ws + [ws_t]:
            w.zero_()                              # the tables are written again by the graph's own first kernels
        for y in (y2, y1, yt):
            y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [y2.clone(), y1.clone(), yt.clone()]
        want2 = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=5)
        want1 = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=8)
        torch.cuda.synchronize()
        assert torch.equal(got[0], want2) and torch.equal(got[2], want2), f"replay {rep}, two products"
        assert torch.equal(got[1], want1), f"replay {rep}, one product"
        if rep == 0:
            _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
            check_close(got[0], y32, "prefill graph replay against the oracle")


def test_compressor_without_allocation_replayed_from_a_graph(ref):
    out, inn = 272, 1024
    base = synth.base_weight(out, inn, device=DEV, tag=("graph", "cb"))
    ft = torch.empty_like(base)
    packed = torch.empty((out, inn // 32), dtype=torch.int32, device=DEV)
    alpha = torch.empty(1, dtype=torch.float32, device=DEV)

    def run():
        bd.compress_noalloc(base, ft, packed=packed, alpha=alpha)
    ft.copy_(synth.finetuned_weight(base, tag=("graph", "ft", -1)))
    graph = _capture(run)
    for rep in range(3):
        _p(f"compress graph, replay {rep}")
        ft.copy_(synth.finetuned_weight(base, tag=("graph", "ft", rep)))
        packed.zero_()
        alpha.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        p_ref, a_ref, _ = ref.compress(to_np(base), to_np(ft))
        assert (to_np(packed).view("uint32") == p_ref).all(), f"replay {rep}"
        assert float(alpha.item()) == a_ref, f"replay {rep}"
