"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element, on the same
seeded inputs.  Integer work (sign bits, packing) must be bit-exact; the linear must match within
max |y - y_ref| / max |y_ref| <= 2e-3 (fp16 output, fp32 accumulation) and an element-wise bound."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from paper_2402_10193_amd import synth           # noqa: E402
from gpu_util import Problem, check_close, packed_to_np, to_np, packed_to_device   # noqa: E402

DEV = "cuda"
VARIANTS = [0, 1, 2]   # library's choice, vector-ALU kernel, matrix-core kernel on the row-major tensors


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    bd.lib()


def _p(msg):
    print(msg, flush=True)


# ----------------------------------------------------------------------------- packing / compression
@pytest.mark.parametrize("out,inn", [(1, 32), (7, 96), (64, 4096), (50, 640), (4096, 4096), (333, 11008)])
def test_pack_signs_bit_exact(ref, out, inn):
    _p(f"pack_signs {out}x{inn}")
    d = synth.finetune_delta(out, inn, device=DEV, tag=("pk", out, inn))
    flat = d.view(-1)
    flat[::17] = 0.0
    flat[5::29] = -0.0
    if flat.numel() > 40:
        flat[3], flat[9], flat[11], flat[21] = float("inf"), float("-inf"), float("nan"), 6e-8
    got = packed_to_np(bd.pack_signs(d))
    want = ref.pack_signs(to_np(d))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("out,inn,sigma", [(1, 32, 0.002), (16, 128, 0.002), (50, 640, 0.002), (4096, 4096, 0.002),
                                           (1000, 11008, 0.002), (1024, 8192, 0.001)])
def test_compress_bits_exact_alpha_within_one_fp16_ulp(ref, out, inn, sigma):
    _p(f"compress {out}x{inn}")
    base = synth.base_weight(out, inn, device=DEV, tag=("c", out, inn))
    ft = synth.finetuned_weight(base, sigma=sigma, tag=("c", out, inn))
    ft.view(-1)[::13] = base.view(-1)[::13]          # zero deltas must pack as 0
    packed, alpha = bd.compress(base, ft)
    p_ref, a_ref, mean = ref.compress(to_np(base), to_np(ft))
    assert np.array_equal(packed_to_np(packed), p_ref)
    a = float(alpha.item())
    assert a == float(np.float16(a))                 # representable in fp16
    assert abs(a - a_ref) <= 2.0 ** -10 * a_ref      # one fp16 ulp at most
    assert a == a_ref, (a, a_ref)                    # the binary64 sums agree to ~1e-16, so in practice: equal


def test_compress_scale_rounded_once_at_a_binary16_middle(ref):
    """The mean |Delta| of this pair lies 2^-29 above the middle between two binary16 numbers: rounded once it goes up,
    by way of binary32 it would land on the middle and go down.  Kernel and oracle must both go up."""
    from test_oracle_pins import midpoint_scale_matrices
    base_np, ft_np = midpoint_scale_matrices()
    base, ft = torch.from_numpy(base_np).to(DEV), torch.from_numpy(ft_np).to(DEV)
    _, alpha = bd.compress(base, ft)
    _, a_ref, _ = ref.compress(base_np, ft_np)
    assert float(alpha.item()) == a_ref == 1.0 + 2.0**-10
    _, ab = bd.compress_batch([base, base], [ft, ft])
    assert ab.tolist() == [a_ref, a_ref]


def test_compress_propagates_inf_and_handles_empty(ref):
    base = synth.base_weight(8, 64, device=DEV)
    ft = base.clone()
    ft[0, 0] = float("inf")
    _, alpha = bd.compress(base, ft)
    assert torch.isinf(alpha).all()
    p, alpha = bd.compress(base[:0], ft[:0])
    assert float(alpha.item()) == 0.0 and p.numel() == 0
    assert bd.pack_signs(base[:0]).numel() == 0


# ----------------------------------------------------------------------------- the linear
CASES = [
    # out, in, n_tenants, tenant_of_token
    (4096, 4096, 4, [0, 1, 2, 3]),                                   # the single-linear config
    (50, 640, 3, [2, 0, 1]),                                         # ragged rows, K not a multiple of 512
    (16, 128, 1, [0]),                                               # one tile, one step, one lane group live
    (33, 1024, 5, [4, 4, 1, 0, 4, 1, 3]),                            # repeats, unsorted, an idle tenant
    (272, 2176, 16, list(range(16))),                                # 16 tenants, K = 4.25 steps
    (100, 4096, 20, [19, 3, 3, 7, 0, 1, 2, 4, 5, 6, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18]),   # 21 tokens: two tiles
    (64, 1536, 32, list(range(32))),                                 # 32 tenants, two full tiles
    (48, 512, 6, [5, 0, 5, 1, 5, 2, 5, 3, 5, 4] * 4),                # 40 tokens: more than one launch
    (40, 96, 2, [1, 0, 1]),                                          # K not a multiple of 128: vector-ALU kernel only
]


def test_compress_batch_equals_separate_calls_and_the_oracle(ref):
    """Several matrices per call: the same bits and the same scales as one bd_compress per matrix, and as the oracle."""
    shapes = [(48, 1024), (272, 2176), (0, 64), (1, 32), (300, 512), (64, 4096), (1024, 1024), (17, 96), (33, 64), (5, 0), (640, 256)]
    _p(f"compress_batch {len(shapes)} matrices")
    bases = [synth.base_weight(o, i, device=DEV, tag=("cb", n)) for n, (o, i) in enumerate(shapes)]
    fts = [synth.finetuned_weight(b, sigma=0.002, tag=("cb", n, "ft")) for n, b in enumerate(bases)]
    packed, alpha = bd.compress_batch(bases, fts)            # 11 matrices: two launches of the batch kernel
    torch.cuda.synchronize()
    assert alpha.shape == (len(shapes),)
    for n, (o, i) in enumerate(shapes):
        p1, a1 = bd.compress(bases[n], fts[n])
        assert torch.equal(packed[n], p1), f"matrix {n}"
        assert float(alpha[n].item()) == float(a1.item()), f"matrix {n}"
        if o > 0 and i > 0:
            p_ref, a_ref, _ = ref.compress(to_np(bases[n]), to_np(fts[n]))
            assert np.array_equal(packed_to_np(packed[n]), p_ref), f"matrix {n} against the oracle"
            assert float(alpha[n].item()) == a_ref
        else:
            assert float(alpha[n].item()) == 0.0


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("case", range(len(CASES)))
def test_linear_matches_oracle(ref, case, variant):
    out, inn, nt, tok = CASES[case]
    _p(f"linear case={case} out={out} in={inn} tenants={nt} T={len(tok)} variant={variant}")
    if variant >= 2 and inn % 128 != 0:
        prob = Problem(ref, out, inn, nt, tag=("lin", case))
        with pytest.raises(bd.BitDeltaError) as e:
            bd.linear_multitenant(prob.x(len(tok)), prob.w_base, prob.table, tok, variant=variant)
        assert e.value.status == 7
        return
    prob = Problem(ref, out, inn, nt, tag=("lin", case))
    x = prob.x(len(tok))
    y = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=variant)
    torch.cuda.synchronize()
    y16, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y32, f"case {case} variant {variant}")
    y64 = ref.linear_multitenant_f64(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y64, f"case {case} variant {variant} vs f64")
    # the fp16 results differ from the oracle's fp16 by at most a few ulp, almost always 0 or 1
    ulp = np.abs(to_np(y).view(np.int16).astype(np.int32) - y16.view(np.int16).astype(np.int32))
    same_sign = np.sign(to_np(y).astype(np.float32)) == np.sign(y16.astype(np.float32))
    assert np.mean((ulp <= 1) | ~same_sign) > 0.99


PREFILL_CASES = [
    # out, in, n_tenants, tokens per tenant (tokens are then shuffled)
    (300, 512, 5, [70, 1, 0, 129, 40]),          # ragged rows, an idle tenant, a tenant with more than one tile
    (130, 96, 3, [11, 11, 11]),                  # 33 tokens: just beyond one decode launch; two N tiles, 3 k steps
    (128, 1024, 2, [128, 256]),                  # exact tiles
    (1024, 2048, 8, [160] * 8),                  # 1280 tokens
    (64, 32, 4, [9, 9, 9, 9]),                   # a single k step
    (520, 192, 3, [40, 3, 90]),                  # three 64-wide steps (odd), three 256-wide N tiles with a ragged one
    (256, 64, 2, [33, 1]),                       # one 64-wide step
    (300, 320, 4, [257, 512, 130, 128]),         # five steps (odd); tiles of 256 rows: whole ones, short ones, a single row
]


@pytest.mark.parametrize("case", range(len(PREFILL_CASES)))
def test_prefill_gemm_matches_oracle(ref, case):
    """More than 32 tokens with a workspace: the library picks one matrix-core GEMM launch or decode launches, whichever
    its cost model says is quicker; without a workspace: decode launches; variants 4..8 force a GEMM.  Same oracle."""
    out, inn, nt, counts = PREFILL_CASES[case]
    tok = [t for t, c in enumerate(counts) for _ in range(c)]
    perm = torch.randperm(len(tok), generator=torch.Generator().manual_seed(case)).tolist()
    tok = [tok[i] for i in perm]
    _p(f"prefill case={case} out={out} in={inn} tenants={nt} T={len(tok)}")
    prob = Problem(ref, out, inn, nt, tag=("pf", case))
    x = prob.x(len(tok))
    y = bd.linear_multitenant(x, prob.w_base, prob.table, tok)                       # workspace allocated: library's choice
    y_dec = bd.linear_multitenant(x, prob.w_base, prob.table, tok, workspace=None)   # no workspace: decode launches
    torch.cuda.synchronize()
    _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
    check_close(y, y32, f"prefill case {case}")
    check_close(y_dec, y32, f"prefill case {case}, decode launches")
    assert torch.equal(bd.linear_multitenant(x, prob.w_base, prob.table, tok), y)    # bitwise reproducible
    # the GEMM kernels by name: 4 = 128 x 128 tiles; 128 x 256 tiles (in % 64 == 0 only): 5 = one wavefront per SIMD,
    # the tiles of a sparsely filled last round (here: all of them) as halves of 64 token rows, 6 = two wavefronts
    # per SIMD, 7 = as 5 with every tile whole
    y4 = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=4)
    check_close(y4, y32, f"prefill case {case}, 128 x 128 tiles")
    if inn % 64 == 0:
        by_variant = {}
        for v in (5, 6, 7):
            y5 = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=v)
            check_close(y5, y32, f"prefill case {case}, 128 x 256 tiles, variant {v}")
            assert torch.equal(bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=v), y5)
            by_variant[v] = y5
        # half tiles add up every element in the same order as whole tiles
        assert torch.equal(by_variant[5], by_variant[7])
        # variant 8: one product on W + alpha S rounded to fp16 -- the naive per-tenant model's arithmetic (the oracle's
        # materialised fp16 weights through its plain linear); within the same bound of the two-product form as well
        w_ft = [ref.materialise_f16(prob.w_base_np, prob.packed_np[t], prob.alpha_np[t]) for t in range(nt)]
        _, n32 = ref.linear_naive(to_np(x), w_ft, tok)
        y8 = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=8)
        check_close(y8, n32, f"prefill case {case}, one product, against the materialised weights")
        # (the weights' own fp16 rounding separates it from the two products: the bar on the largest error holds, the
        # element-wise one is asked against the materialised weights only)
        check_close(y8, y32, f"prefill case {case}, one product, against the two products", elementwise=False)
        assert torch.equal(bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=8), y8)
    else:
        with pytest.raises(bd.BitDeltaError) as e:
            bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=5)
        assert e.value.status == 7


def test_prefill_token_tables_written_from_runs(ref):
    """Tokens that arrive grouped by tenant: the library writes the GEMM's token tables from a few runs (values counting
    up, padding and tenant ids repeated) instead of value by value; a batch with one stray token in the middle mixes both."""
    out, inn, nt, counts = 300, 512, 5, [70, 1, 0, 129, 300]
    grouped = [t for t, c in enumerate(counts) for _ in range(c)]
    stray = list(grouped)
    stray[100], stray[400] = stray[400], stray[100]
    prob = Problem(ref, out, inn, nt, tag=("pf", "runs"))
    for name, tok in (("grouped", grouped), ("one stray pair", stray)):
        _p(f"prefill tables from runs: {name}, T={len(tok)}")
        x = prob.x(len(tok))
        _, y32 = ref.linear_multitenant(to_np(x), prob.w_base_np, prob.packed_np, prob.alpha_np, tok)
        for v in (4, 5, 8):
            y = bd.linear_multitenant(x, prob.w_base, prob.table, tok, variant=v)
            check_close(y, y32, f"tables from runs, {name}, variant {v}", elementwise=v != 8)


def test_one_product_gemm_special_inputs(ref):
    """Variant 8 on scales and weights at the edges: alpha = 0 (W itself: bit for bit the two-product form), a negative
    and a large scale, a scale that is not a binary16 number (the kernel rounds it first), one-hot x (the materialised
    weight itself, exactly), and non-finite weights (they stay where the oracle puts them)."""
    out, inn, T = 272, 192, 140
    prob = Problem(ref, out, inn, 1, tag=("pf", "special"))
    x = prob.x(T)
    tok = [0] * T
    packed = prob.table.packed[0]

    def table(alpha):
        return bd.TenantTable([packed], torch.tensor([alpha], dtype=torch.float32, device=DEV))
    _p("one product: alpha = 0")
    y0 = bd.linear_multitenant(x, prob.w_base, table(0.0), tok, variant=8)
    assert torch.equal(y0, bd.linear_multitenant(x, prob.w_base, table(0.0), tok, variant=5))
    for alpha in (-0.003, 0.5, 0.0017):                       # 0.0017 is no binary16 number
        _p(f"one product: alpha = {alpha}")
        a16 = float(np.float16(alpha))
        w_ft = ref.materialise_f16(prob.w_base_np, prob.packed_np[0], a16)
        _, n32 = ref.linear_naive(to_np(x), [w_ft], tok)
        check_close(bd.linear_multitenant(x, prob.w_base, table(alpha), tok, variant=8), n32, f"alpha {alpha}")
    _p("one product: one-hot x")
    xe = torch.zeros((inn, inn), dtype=torch.float16, device=DEV)
    xe[torch.arange(inn), torch.arange(inn)] = 1.0
    w_ft = ref.materialise_f16(prob.w_base_np, prob.packed_np[0], prob.alpha_np[0])
    y = bd.linear_multitenant(xe, prob.w_base, prob.table, [0] * inn, variant=8)
    assert np.array_equal(to_np(y).view(np.uint16), np.ascontiguousarray(w_ft.T).view(np.uint16))
    _p("one product: non-finite weights")
    w = prob.w_base.clone()
    w[3, 5], w[100, 77], w[271, 191], w[8, 0] = float("inf"), float("-inf"), float("nan"), 6e-8   # and a subnormal
    w_ft = ref.materialise_f16(to_np(w), prob.packed_np[0], prob.alpha_np[0])
    _, n32 = ref.linear_naive(to_np(x), [w_ft], tok)
    y = to_np(bd.linear_multitenant(x, w, prob.table, tok, variant=8)).astype(np.float32)
    assert np.array_equal(np.isnan(y), np.isnan(n32)) and np.array_equal(np.isinf(y), np.isinf(n32))
    fin = np.isfinite(n32)
    assert np.array_equal(np.sign(y[~fin & ~np.isnan(n32)]), np.sign(n32[~fin & ~np.isnan(n32)]))
    rows = [r for r in range(out) if r not in (3, 100, 271)]
    check_close(torch.from_numpy(y[:, rows]), n32[:, rows], "rows without non-finite weights")


@pytest.mark.parametrize("variant", VARIANTS)
def test_linear_special_inputs(ref, variant):
    """alpha = 0, all-ones / all-zero sign words, one-hot x: exact consequences of Eq. 6."""
    out, inn = 32, 1024
    _p(f"linear specials variant={variant}")
    prob = Problem(ref, out, inn, 1, tag="special")
    x = prob.x(3)
    ones = torch.full((out, inn // 32), -1, dtype=torch.int32, device=DEV)
    zeros = torch.zeros((out, inn // 32), dtype=torch.int32, device=DEV)
    a = torch.tensor([0.0015], dtype=torch.float32, device=DEV)
    xb = to_np(x).astype(np.float64)
    wb = prob.w_base_np.astype(np.float64)
    base = xb @ wb.T
    y = bd.linear_multitenant(x, prob.w_base, bd.TenantTable([prob.table.packed[0]], torch.zeros(1)), [0, 0, 0], variant=variant)
    check_close(y, base, "alpha=0")
    y = bd.linear_multitenant(x, prob.w_base, bd.TenantTable([ones], a), [0, 0, 0], variant=variant)
    check_close(y, base + float(a.item()) * xb.sum(1, keepdims=True), "all +1")
    y = bd.linear_multitenant(x, prob.w_base, bd.TenantTable([zeros], a), [0, 0, 0], variant=variant)
    check_close(y, base - float(a.item()) * xb.sum(1, keepdims=True), "all -1")
    for k in (0, 17, 511, 1023):
        xe = torch.zeros((1, inn), dtype=torch.float16, device=DEV)
        xe[0, k] = 1.0
        y = bd.linear_multitenant(xe, prob.w_base, prob.table, [0], variant=variant)
        s = ref.unpack_signs(prob.packed_np[0], inn)[:, k].astype(np.float32)
        want = (prob.w_base_np[:, k].astype(np.float32) + np.float32(prob.alpha_np[0]) * s).astype(np.float16)
        assert np.array_equal(to_np(y)[0].view(np.uint16), want.view(np.uint16)), k


def test_linear_noops_determinism_and_token_order(ref):
    prob = Problem(ref, 48, 1024, 4, tag="misc")
    tok = [3, 1, 1, 0, 3, 2, 0]
    x = prob.x(len(tok))
    y0 = bd.linear_multitenant(x, prob.w_base, prob.table, tok)
    for _ in range(3):
        assert torch.equal(bd.linear_multitenant(x, prob.w_base, prob.table, tok), y0)      # bitwise deterministic
    order = [4, 2, 0, 5, 1, 3, 6]
    yo = bd.linear_multitenant(x[order].contiguous(), prob.w_base, prob.table, [tok[i] for i in order])
    check_close(yo, to_np(y0).astype(np.float32)[order], "permuted tokens")
    # each token alone
    for t in range(len(tok)):
        yt = bd.linear_multitenant(x[t:t + 1].contiguous(), prob.w_base, prob.table, [tok[t]])
        check_close(yt, to_np(y0).astype(np.float32)[t:t + 1], "single token")
    # T = 0 and out = 0 launch nothing and succeed
    assert bd.linear_multitenant(x[:0], prob.w_base, prob.table, []).shape == (0, 48)
    assert bd.linear_multitenant(x, prob.w_base[:0], bd.TenantTable([p[:0] for p in prob.table.packed], prob.table.alpha),
                                 tok).shape == (len(tok), 0)
    with pytest.raises(bd.BitDeltaError) as e:
        bd.linear_multitenant(x[:1], prob.w_base, prob.table, [4])
    assert e.value.status == 4


def test_gpu_compress_feeds_gpu_linear_end_to_end(ref):
    """Compression and linear both on the GPU (the product path end to end) against the oracle's pair."""
    out, inn, nt = 256, 2048, 4
    base = synth.base_weight(out, inn, device=DEV, tag="e2e")
    fts = [synth.finetuned_weight(base, tag=("e2e", t)) for t in range(nt)]
    comp = [bd.compress(base, ft) for ft in fts]
    table = bd.TenantTable([c[0] for c in comp], [c[1] for c in comp])
    tok = [0, 1, 2, 3]
    x = synth.activations(4, inn, device=DEV, tag="e2e")
    y = bd.linear_multitenant(x, base, table, tok)
    refc = [ref.compress(to_np(base), to_np(ft)) for ft in fts]
    _, y32 = ref.linear_multitenant(to_np(x), to_np(base), [c[0] for c in refc], [c[1] for c in refc], tok)
    check_close(y, y32, "end to end")
    # and BitDelta's output is close to the true fine-tuned product (what the approximation is for)
    y_true = torch.stack([fts[t].float() @ x[i].float() for i, t in enumerate(tok)])
    rel = (y.float() - y_true).norm() / y_true.norm()
    assert rel < 0.1


# ----------------------------------------------------------------------------- naive baseline helpers
def test_materialize_and_naive_match_oracle(ref):
    prob = Problem(ref, 40, 512, 3, tag="naive")
    ws = [bd.materialize(prob.w_base, prob.table.packed[t], prob.table.alpha[t:t + 1]) for t in range(3)]
    for t in range(3):
        want = ref.materialise_f16(prob.w_base_np, prob.packed_np[t], prob.alpha_np[t])
        assert np.array_equal(to_np(ws[t]).view(np.uint16), want.view(np.uint16))
    tok = [2, 0, 1, 2]
    x = prob.x(4)
    y = bd.linear_naive(x, bd.WeightTable(ws), tok)
    _, y32 = ref.linear_naive(to_np(x), [to_np(w) for w in ws], tok)
    check_close(y, y32, "naive")


def test_probes_run():
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    dst = torch.empty_like(src)
    bd.probe_copy(dst, src)
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    bd.probe_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
