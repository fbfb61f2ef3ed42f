"""Dense inputs of the benchmark workloads, built so that the layer step is stationary:
every step refreshes the same fraction of halo rows.

Two versions of each drifting input alternate from step to step. Forward: halo rows in a
seeded subset S (a fraction rho of all halo rows) differ strongly between the versions,
the others differ by far less than the threshold, so exactly the rows of S fail the cache
test on every step after the first. Backward: the upstream gradient differs on a seeded
subset of local rows, which changes the halo gradient rows next to them.

Large matrices come from torch's seeded device generator (fast); the row subsets come from
the counter-based hash so that they are the same on every device.
"""
from dataclasses import dataclass

import torch

from . import rng


@dataclass
class LayerInputs:
    x_local: torch.Tensor       # n_loc x f_in
    fresh: tuple                # two versions of n_halo x f_in
    dH: tuple                   # two versions of n_loc x f_out
    W: torch.Tensor             # f_in x f_out
    sent_set: torch.Tensor      # bool [n_halo], the rows that change between versions


def _randn(shape, gen, device, dtype):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(dtype)


def make_layer_inputs(seed, layer, n_loc, n_halo, f_in, f_out, rho=0.37, phi=0.01, device="cpu",
                      dtype=torch.float32, halo_width=None) -> LayerInputs:
    """halo_width: width of the rows that cross the partition boundary (f_in when the layer
    aggregates first, f_out when it transforms first)."""
    hw = f_in if halo_width is None else halo_width
    gen = torch.Generator(device=device)
    gen.manual_seed(seed * 1000 + layer)
    x_local = _randn((n_loc, f_in), gen, device, dtype)
    fa = _randn((n_halo, hw), gen, device, torch.float32)
    u = rng.uniform01(seed, 300 + layer, torch.arange(n_halo, dtype=torch.int64, device=device))
    in_s = u < rho
    # strong change on S (factor 1 + 0.5 g), faint change elsewhere (1 + 0.002 g)
    amp = torch.where(in_s, torch.tensor(0.5, device=device), torch.tensor(0.002, device=device)).view(-1, 1)
    fb = fa * (1.0 + amp * torch.randn((n_halo, hw), generator=gen, device=device))
    del amp
    lim = (6.0 / (f_in + f_out)) ** 0.5
    W = (torch.rand((f_in, f_out), generator=gen, device=device) * 2 - 1) * lim
    da = _randn((n_loc, f_out), gen, device, torch.float32)
    v = rng.uniform01(seed, 400 + layer, torch.arange(n_loc, dtype=torch.int64, device=device))
    db = torch.where((v < phi).view(-1, 1), da * 1.5, da)
    return LayerInputs(x_local, (fa.to(dtype), fb.to(dtype)), (da, db), W, in_s)
