"""bd_compress_noalloc (the compressor for callers that cannot allocate: its partial sums live in an array inside
the library) against bd_compress with a caller's workspace: same sign words and the same scale, bit for bit, on two
calls in a row of which the second is smaller (so slots of the shared array that the first call wrote stay unread)."""
import numpy as np
import pytest
import torch

from paper_2402_10193_amd import binding as bd
from paper_2402_10193_amd import synth

pytestmark = pytest.mark.gpu


def _pair(out, inn, tag):
    base = synth.base_weight(out, inn, device="cuda", tag=("noalloc", tag))
    return base, synth.finetuned_weight(base, tag=("noalloc", tag, "ft"))


def test_noalloc_matches_workspace_call_twice_second_smaller(ref):
    # 1000 x 11008: 2048 blocks (every slot of the array); 96 x 160: 8 blocks, ragged against the block size
    for out, inn in ((1000, 11008), (96, 160)):
        base, ft = _pair(out, inn, (out, inn))
        packed = torch.full((out, inn // 32), -1, dtype=torch.int32, device="cuda")
        alpha = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        print(f"bd_compress_noalloc {out} x {inn}", flush=True)
        bd.compress_noalloc(base, ft, packed, alpha)
        want_p, want_a = bd.compress(base, ft)
        torch.cuda.synchronize()
        assert torch.equal(packed, want_p)
        assert alpha.item() == want_a.item()
        # and both equal the oracle
        rp, ra, _ = ref.compress(base.cpu().numpy(), ft.cpu().numpy())
        assert np.array_equal(packed.cpu().numpy().view(np.uint32), rp)
        assert alpha.item() == ra


def test_noalloc_empty_and_too_large():
    alpha = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    empty = torch.empty((0, 64), dtype=torch.float16, device="cuda")
    bd.compress_noalloc(empty, empty, torch.empty((0, 2), dtype=torch.int32, device="cuda"), alpha)
    torch.cuda.synchronize()
    assert alpha.item() == 0.0
    # the size limit is checked on the host from the sizes alone
    a = 1 << 20
    assert bd.lib().bd_compress_noalloc(a, 2 * a, 1 << 20, 1 << 13, 3 * a, 4 * a, 0) == 11
