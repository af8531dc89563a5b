"""GPU test of the delta hot swap: a tenant's delta travels GPU -> host image -> file -> pinned host memory ->
device arena -> serving layout while decode launches keep running on another stream, and the linear with the
swapped-in delta must equal, bit for bit, the linear with the delta that never left the GPU; the uploaded arena
must equal the image byte for byte."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2402_10193_amd import binding as bd   # noqa: E402
from paper_2402_10193_amd import synth           # noqa: E402
from gpu_util import check_close, packed_to_np, to_np   # noqa: E402

DEV = "cuda"


@pytest.mark.parametrize("k", [1, 2])
def test_hot_swap_round_trip(ref, tmp_path, k):
    print(f"hot swap k={k}", flush=True)
    shapes = [(256, 1024), (100, 2048), (64, 512)]           # one tenant's "model": three matrices
    n_tenants, new_tenant = 3, 1
    bases = [synth.base_weight(o, i, device=DEV, tag=("hs", k, m)) for m, (o, i) in enumerate(shapes)]
    wts = [bd.tile_base(b) for b in bases]
    # resident tenants 0..2; tenant 1 will be replaced by a new fine-tune
    packed = [[None] * n_tenants for _ in shapes]
    alphas = [torch.zeros(n_tenants * k, dtype=torch.float32, device=DEV) for _ in shapes]
    tiled = [[None] * n_tenants for _ in shapes]
    # the oracle compresses the same pairs itself: its linear is never fed anything the library produced
    ref_planes = [[None] * n_tenants for _ in shapes]
    ref_alphas = [np.zeros((n_tenants, k), dtype=np.float32) for _ in shapes]

    def oracle_delta(m, ft, p, a):
        p_ref, a_ref, _, _ = ref.compress_iterated(to_np(bases[m]), to_np(ft), k)
        assert np.array_equal(packed_to_np(p), p_ref) and np.array_equal(to_np(a), np.asarray(a_ref, dtype=np.float32))
        return [p_ref[j] for j in range(k)], np.asarray(a_ref, dtype=np.float32)

    for m, (o, i) in enumerate(shapes):
        for t in range(n_tenants):
            ft = synth.finetuned_weight(bases[m], sigma=0.002, tag=("hs", k, m, t))
            p, a = bd.compress_iterated(bases[m], ft, k)
            ref_planes[m][t], ref_alphas[m][t] = oracle_delta(m, ft, p, a)
            packed[m][t] = p
            alphas[m][t * k:(t + 1) * k] = a
            tiled[m][t] = [bd.tile_signs(p[j].contiguous(), o, i) for j in range(k)]
    # the incoming delta, compressed on the GPU, brought to the host and written to a file
    new_packed, new_alpha = [], []
    for m, (o, i) in enumerate(shapes):
        ft = synth.finetuned_weight(bases[m], sigma=0.002, tag=("hs", k, m, "new"))
        p, a = bd.compress_iterated(bases[m], ft, k)
        ref_planes[m][new_tenant], ref_alphas[m][new_tenant] = oracle_delta(m, ft, p, a)   # tenant 1 after the swap
        new_packed.append(p)
        new_alpha.append(a)
    torch.cuda.synchronize()
    outs, ins = [s[0] for s in shapes], [s[1] for s in shapes]
    image = bd.delta_image_build([p.cpu() for p in new_packed], [a.cpu() for a in new_alpha], outs, ins, k)
    path = str(tmp_path / "new_tenant.bdlt")
    bd.delta_file_write(path, image)
    staged = bd.delta_file_read(path)                         # pinned host memory
    assert staged.is_pinned() and torch.equal(staged, image)
    assert bd.delta_image_check(staged) == (len(shapes), k)

    # decode keeps running on the main stream while the swap runs on a side stream
    tok = [0, 1, 2, 1]
    x = {i: synth.activations(len(tok), i, device=DEV, tag=("hs", i)) for i in set(ins)}
    tables = [bd.TiledPlaneTable(tiled[m], alphas[m].clone()) for m in range(len(shapes))]
    y_before = [bd.linear_multitenant_tiled_kbit(x[ins[m]], wts[m], outs[m], tables[m], tok) for m in range(len(shapes))]
    side = torch.cuda.Stream()
    new_tiled = [[torch.empty(bd.tiled_signs_bytes(o, i) // 4, dtype=torch.int32, device=DEV) for _ in range(k)]
                 for (o, i) in shapes]
    new_alphas = [a.clone() for a in alphas]
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        arena = bd.delta_upload(staged, stream=side)
        bd.delta_install(staged, arena, new_tenant, n_tenants, new_tiled, new_alphas, stream=side)
        done = torch.cuda.Event()
        done.record(side)
    for _ in range(5):                                        # launches that overlap the swap use the old tables
        y_mid = [bd.linear_multitenant_tiled_kbit(x[ins[m]], wts[m], outs[m], tables[m], tok) for m in range(len(shapes))]
    torch.cuda.current_stream().wait_event(done)
    for m in range(len(shapes)):
        assert torch.equal(y_mid[m], y_before[m])             # the running tenants were not disturbed
    assert np.array_equal(to_np(arena), staged.numpy())        # the arena is the image

    # the swapped-in tenant against the delta that never left the GPU, and against the oracle
    for m, (o, i) in enumerate(shapes):
        swapped = bd.TiledPlaneTable([tiled[m][0], new_tiled[m], tiled[m][2]], new_alphas[m])
        direct_alpha = alphas[m].clone()
        direct_alpha[new_tenant * k:(new_tenant + 1) * k] = new_alpha[m]
        direct = bd.TiledPlaneTable([tiled[m][0], [bd.tile_signs(new_packed[m][j].contiguous(), o, i) for j in range(k)],
                                     tiled[m][2]], direct_alpha)
        y_s = bd.linear_multitenant_tiled_kbit(x[i], wts[m], o, swapped, tok)
        y_d = bd.linear_multitenant_tiled_kbit(x[i], wts[m], o, direct, tok)
        assert torch.equal(y_s, y_d)
        assert not torch.equal(y_s, y_before[m])
        _, y32 = ref.linear_multitenant_kbit(to_np(x[i]), to_np(bases[m]), ref_planes[m], ref_alphas[m], tok)
        check_close(y_s, y32, f"hot swap matrix {m}")
