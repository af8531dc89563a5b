"""Helpers of the GPU parity tests: seeded problems on the device, the same tensors on the host for the oracle."""
import numpy as np
import torch

from paper_2402_10193_amd import binding as bd
from paper_2402_10193_amd import synth

REL_TOL = 2e-3   # max |y - y_ref| / max |y_ref|, fp16 output with fp32 accumulation


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def packed_to_device(p: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(p.view(np.int32).copy()).to(device)


def packed_to_np(t: torch.Tensor) -> np.ndarray:
    return to_np(t).view(np.uint32)


class Problem:
    """One linear with n_tenants fine-tunes: device tensors plus the oracle's compression of them."""

    def __init__(self, ref, out, inn, n_tenants, sigma=0.002, seed=synth.DEFAULT_SEED, tag="p", device="cuda"):
        self.out, self.inn, self.n_tenants = out, inn, n_tenants
        self.w_base = synth.base_weight(out, inn, seed=seed, tag=(tag, "base"), device=device)
        self.w_base_np = to_np(self.w_base)
        self.packed_np, self.alpha_np, self.w_ft = [], [], []
        for t in range(n_tenants):
            w_ft = synth.finetuned_weight(self.w_base, sigma=sigma, seed=seed, tag=(tag, "ft", t))
            p, a, _ = ref.compress(self.w_base_np, to_np(w_ft))
            self.packed_np.append(p)
            self.alpha_np.append(a)
            self.w_ft.append(w_ft)
        self.table = bd.TenantTable([packed_to_device(p, device) for p in self.packed_np],
                                    torch.tensor(self.alpha_np, dtype=torch.float32, device=device))

    def x(self, T, seed=synth.DEFAULT_SEED, tag="x"):
        return synth.activations(T, self.inn, seed=seed, tag=(tag, T), device=self.w_base.device)


class TiledProblem(Problem):
    """The same problem with base and deltas also in the tiled serving layout."""

    def __init__(self, ref, out, inn, n_tenants, **kw):
        super().__init__(ref, out, inn, n_tenants, **kw)
        self.w_tiled = bd.tile_base(self.w_base)
        self.ttable = bd.TiledTenantTable([bd.tile_signs(p, out, inn) for p in self.table.packed], self.table.alpha)


def check_close(y_gpu: torch.Tensor, y_ref32: np.ndarray, what="", elementwise=True):
    """max |y - y_ref| / max |y_ref| <= REL_TOL, and (elementwise) every element within REL_TOL |y_ref| + 1e-3 rms(y_ref)."""
    y = to_np(y_gpu).astype(np.float64)
    r = y_ref32.astype(np.float64)
    assert y.shape == r.shape, (y.shape, r.shape)
    if r.size == 0:
        return 0.0
    assert np.all(np.isfinite(y)), what
    scale = np.max(np.abs(r))
    err = np.max(np.abs(y - r)) / scale
    assert err <= REL_TOL, f"{what}: max rel err {err:.3e} > {REL_TOL}"
    if not elementwise:
        return err
    rms = np.sqrt(np.mean(r * r))
    bad = np.abs(y - r) > REL_TOL * np.abs(r) + 1e-3 * rms
    assert not bad.any(), f"{what}: {bad.sum()} elements outside the element-wise bound"
    return err
