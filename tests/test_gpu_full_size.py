"""GPU parity at the benchmark's full sizes (Llama-2-7B and 70B layer shapes), in the launch configuration
bench.py times: the row-major entry point, the tiled entry point and the grouped (q,k,v / gate,up) tiled
launches.  The 7B layer and the 70B matrices (32 tenants) are compared in full; the prefill GEMM (4096 tokens)
on sampled output rows for every token and on every output row for sampled tokens (rows of a linear and tokens
of a batch are independent, so a slice of either is a complete problem for the oracle)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from paper_2402_10193_amd import synth           # noqa: E402
from gpu_util import check_close, packed_to_np, to_np   # noqa: E402

DEV = "cuda"


def _gpu_layer(out, inn, B, sigma, tag):
    base = synth.base_weight(out, inn, device=DEV, tag=(tag, "base"))
    ws = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, out, inn, 1), DEV)
    packed, alphas, fts = [], [], []
    for t in range(B):
        ft = synth.finetuned_weight(base, sigma=sigma, tag=(tag, t))
        p, a = bd.compress(base, ft, workspace=ws)
        packed.append(p)
        alphas.append(a)
        fts.append(ft)
    return base, fts, bd.TenantTable(packed, alphas)


def _oracle_deltas(ref, base, fts, table):
    """The oracle's own compression of the same (base, fine-tuned) pairs -- what the oracle's linear is fed -- and
    the check that the library's compressor, whose output the library's linear is fed, agrees with it bit for bit."""
    base_np = to_np(base)
    packed, alphas = [], []
    for t, ft in enumerate(fts):
        p, a, _ = ref.compress(base_np, to_np(ft))
        assert np.array_equal(packed_to_np(table.packed[t]), p)
        assert float(table.alpha[t].item()) == a
        packed.append(p)
        alphas.append(a)
    return packed, alphas


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,out,inn", [("q", 4096, 4096), ("gate", 11008, 4096), ("down", 4096, 11008)])
def test_llama2_7b_layer_b16_full_output(ref, name, out, inn):
    B = 16
    print(f"7B {name} {out}x{inn} B={B}", flush=True)
    base, fts, table = _gpu_layer(out, inn, B, 0.002, ("7b", name))
    x = synth.activations(B, inn, device=DEV, tag=("7b", name))
    tok = synth.one_token_per_tenant(B)
    y = bd.linear_multitenant(x, base, table, tok)
    ttable = bd.TiledTenantTable([bd.tile_signs(p, out, inn) for p in table.packed], table.alpha)
    y_tiled = bd.linear_multitenant_tiled(x, bd.tile_base(base), out, ttable, tok)
    torch.cuda.synchronize()
    base_np = to_np(base)
    refc = []
    for t in range(B):
        p, a, _ = ref.compress(base_np, to_np(fts[t]))
        assert np.array_equal(packed_to_np(table.packed[t]), p)          # full-size compression parity, bit-exact
        assert float(table.alpha[t].item()) == a
        refc.append((p, a))
    del fts
    _, y32 = ref.linear_multitenant(to_np(x), base_np, [c[0] for c in refc], [c[1] for c in refc], tok)
    err = check_close(y, y32, f"7B {name}")
    err_t = check_close(y_tiled, y32, f"7B {name} tiled")
    print(f"   max rel err {err:.2e} (row-major)  {err_t:.2e} (tiled)", flush=True)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("names,outs,inn", [(("q", "k", "v"), (4096, 4096, 4096), 4096),
                                            (("gate", "up"), (11008, 11008), 4096)])
def test_llama2_7b_grouped_launch_b16_full_output(ref, names, outs, inn):
    """The launches bench.py times: several matrices over the same x in one call."""
    B = 16
    print(f"7B grouped {names} B={B}", flush=True)
    x = synth.activations(B, inn, device=DEV, tag=("7bg", names[0]))
    tok = synth.one_token_per_tenant(B)
    wts, tables, keep = [], [], []
    for name, out in zip(names, outs):
        base, fts, table = _gpu_layer(out, inn, B, 0.002, ("7bg", name))
        oracle_packed, oracle_alphas = _oracle_deltas(ref, base, fts, table)
        del fts
        wts.append(bd.tile_base(base))
        tables.append(bd.TiledTenantTable([bd.tile_signs(p, out, inn) for p in table.packed], table.alpha))
        keep.append((base, oracle_packed, oracle_alphas))
    ys = bd.linear_multitenant_tiled_group(x, bd.TiledGroup(wts, list(outs), tables), tok)
    torch.cuda.synchronize()
    for i, (base, packed, alphas) in enumerate(keep):
        _, y32 = ref.linear_multitenant(to_np(x), to_np(base), packed, alphas, tok)
        err = check_close(ys[i], y32, f"7B grouped {names[i]}")
        print(f"   {names[i]}: max rel err {err:.2e}", flush=True)


MIXED_BATCHES = [
    # resident tenants, tenant of each token (continuous batching: several tokens of some tenants, most tenants idle)
    (24, [3, 3, 3, 3, 3, 3, 0, 0, 0, 0, 7, 7, 7, 9, 12, 20]),                                  # 16 tokens, 6 of 24 tenants
    (40, [5] * 9 + [31] * 7 + [2, 2, 2, 39, 39, 17, 8, 11, 23, 30, 1]),                        # 27 tokens: two column tiles
]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("case", range(len(MIXED_BATCHES)))
def test_llama2_7b_mixed_batch_gate_up_full_output(ref, case):
    """A mixed decode batch on the grouped gate,up launch at full size: only the active tenants' deltas exist
    (idle tenants have no pointer), each is streamed once for all of its tokens."""
    n_res, tok = MIXED_BATCHES[case]
    out, inn = 11008, 4096
    active = sorted(set(tok))
    print(f"7B mixed batch case={case} T={len(tok)} active={len(active)} of {n_res}", flush=True)
    x = synth.activations(len(tok), inn, device=DEV, tag=("7bmix", case))
    ws = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, out, inn, 1), DEV)
    wts, tables, keep = [], [], []
    for name in ("gate", "up"):
        base = synth.base_weight(out, inn, device=DEV, tag=("7bmix", case, name))
        tiled = [None] * n_res
        alpha = torch.zeros(n_res, dtype=torch.float32, device=DEV)
        dummy = np.zeros((out, inn // 32), dtype=np.uint32)              # never selected: idle tenants have no token
        oracle_packed, oracle_alphas = [dummy] * n_res, [0.0] * n_res
        base_np = to_np(base)
        for t in active:
            ft = synth.finetuned_weight(base, sigma=0.002, tag=("7bmix", case, name, t))
            p, a = bd.compress(base, ft, workspace=ws)
            oracle_packed[t], oracle_alphas[t], _ = ref.compress(base_np, to_np(ft))   # the oracle's own deltas
            del ft
            assert np.array_equal(packed_to_np(p), oracle_packed[t]) and float(a.item()) == oracle_alphas[t]
            alpha[t] = a
            tiled[t] = bd.tile_signs(p, out, inn)
        wts.append(bd.tile_base(base))
        tables.append(bd.TiledTenantTable(tiled, alpha))
        keep.append((base_np, oracle_packed, oracle_alphas))
    ys = bd.linear_multitenant_tiled_group(x, bd.TiledGroup(wts, [out, out], tables), tok)
    torch.cuda.synchronize()
    for i, (base_np, packed_np, alphas) in enumerate(keep):
        _, y32 = ref.linear_multitenant(to_np(x), base_np, packed_np, alphas, tok)
        err = check_close(ys[i], y32, f"7B mixed batch {i}")
        print(f"   matrix {i}: max rel err {err:.2e}", flush=True)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,out,inn", [("kv", 1024, 8192), ("qo", 8192, 8192), ("gate", 28672, 8192), ("down", 8192, 28672)])
def test_llama2_70b_b32_full_output(ref, name, out, inn):
    B = 32
    print(f"70B {name} {out}x{inn} B={B}", flush=True)
    base, fts, table = _gpu_layer(out, inn, B, 0.001, ("70b", name))
    x = synth.activations(B, inn, device=DEV, tag=("70b", name))
    tok = synth.one_token_per_tenant(B)
    y = bd.linear_multitenant(x, base, table, tok)
    ttable = bd.TiledTenantTable([bd.tile_signs(p, out, inn) for p in table.packed], table.alpha)
    y_tiled = bd.linear_multitenant_tiled(x, bd.tile_base(base), out, ttable, tok)   # 32 tokens: one launch, two column tiles
    torch.cuda.synchronize()
    base_np = to_np(base)
    refc, alphas = [], []
    for t in range(B):
        p, a, _ = ref.compress(base_np, to_np(fts[t]))                     # oracle compression of the full matrix
        assert np.array_equal(packed_to_np(table.packed[t]), p)
        assert float(table.alpha[t].item()) == a
        refc.append(p)
        alphas.append(a)
        fts[t] = None
    print("   oracle linear ...", flush=True)
    _, y32 = ref.linear_multitenant(to_np(x), base_np, refc, alphas, tok)
    err = check_close(y, y32, f"70B {name}")
    err_t = check_close(y_tiled, y32, f"70B {name} tiled")
    print(f"   max rel err {err:.2e} (row-major)  {err_t:.2e} (tiled)", flush=True)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,out,inn", [("up", 11008, 4096), ("down", 4096, 11008)])
def test_prefill_8_tenants_x_512_tokens_sampled_rows(ref, name, out, inn):
    """The prefill configuration: 8 tenants x 512 tokens through one GEMM launch, checked on sampled output rows."""
    B, per, n_rows = 8, 512, 96
    print(f"prefill {name} {out}x{inn} T={B * per}", flush=True)
    base, fts, table = _gpu_layer(out, inn, B, 0.002, ("pf", name))
    oracle_packed, alphas = _oracle_deltas(ref, base, fts, table)
    del fts
    tok = [t for t in range(B) for _ in range(per)]
    x = synth.activations(B * per, inn, device=DEV, tag=("pf", name))
    y = bd.linear_multitenant(x, base, table, tok)
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(11)
    rows = torch.sort(torch.randperm(out, generator=g)[:n_rows]).values
    rows[0], rows[-1] = 0, out - 1
    packed = [np.ascontiguousarray(p[rows.numpy()]) for p in oracle_packed]
    base_np = np.ascontiguousarray(to_np(base)[rows.numpy()])
    _, y32 = ref.linear_multitenant(to_np(x), base_np, packed, alphas, tok)
    err = check_close(y[:, rows.to(DEV)], y32, f"prefill {name}")
    print(f"   max rel err {err:.2e}", flush=True)
    # the one-product form (W + alpha S rounded to fp16, 256 x 256 tiles) against the oracle's materialised weights
    y8 = bd.linear_multitenant(x, base, table, tok, variant=8)
    torch.cuda.synchronize()
    w_ft = [ref.materialise_f16(base_np, packed[t], alphas[t]) for t in range(B)]
    _, n32 = ref.linear_naive(to_np(x), w_ft, tok)
    err8 = check_close(y8[:, rows.to(DEV)], n32, f"prefill {name}, one product")
    err86 = check_close(y8[:, rows.to(DEV)], y32, f"prefill {name}, one product against the two products", elementwise=False)
    print(f"   one product: max rel err {err8:.2e} (materialised weights)  {err86:.2e} (two products)", flush=True)
    # the same two launches reading the serving layout: same arithmetic in the same order, so the same bits
    ttable = bd.TiledTenantTable([bd.tile_signs(p, out, inn) for p in table.packed], table.alpha)
    w_tiled = bd.tile_base(base)
    assert torch.equal(bd.linear_multitenant_tiled_gemm(x, w_tiled, out, ttable, tok), y)
    assert torch.equal(bd.linear_multitenant_tiled_gemm(x, w_tiled, out, ttable, tok, one_product=True), y8)


@pytest.mark.timeout(900)
def test_prefill_8_tenants_x_512_tokens_every_output_row_of_sampled_tokens(ref):
    """The same launch (all 4096 tokens go through the GEMM) checked the other way round: every output row, i.e. every
    tile of every workgroup, for 8 sampled tokens of each tenant."""
    B, per, out, inn = 8, 512, 11008, 4096
    print(f"prefill up {out}x{inn} T={B * per}, all rows of sampled tokens", flush=True)
    base, fts, table = _gpu_layer(out, inn, B, 0.002, ("pf", "up"))
    oracle_packed, alphas = _oracle_deltas(ref, base, fts, table)
    del fts
    tok = [t for t in range(B) for _ in range(per)]
    x = synth.activations(B * per, inn, device=DEV, tag=("pf", "up"))
    y = bd.linear_multitenant(x, base, table, tok)
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(13)
    picks = []
    for t in range(B):
        p = torch.sort(torch.randperm(per, generator=g)[:8]).values + t * per
        p[0], p[-1] = t * per, (t + 1) * per - 1          # first and last token of the tenant's tiles
        picks.append(p)
    picks = torch.cat(picks)
    _, y32 = ref.linear_multitenant(to_np(x[picks.to(DEV)]), to_np(base), oracle_packed, alphas, [tok[i] for i in picks.tolist()])
    err = check_close(y[picks.to(DEV)], y32, "prefill up, sampled tokens")
    print(f"   max rel err {err:.2e}", flush=True)
