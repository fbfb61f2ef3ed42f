"""Seeded dense inputs: vertex features, layer weights, upstream gradients and the
drifting stream that stands in for the halo rows other partitions would send.
"""
import math

import torch

from . import rng


def normal_matrix(seed: int, stream: int, rows: int, cols: int, device="cpu",
                  dtype=torch.float32) -> torch.Tensor:
    """rows x cols standard normal, row-major, value (r, c) = draw r*cols + c."""
    return rng.normal(seed, stream, rows * cols, device=device, dtype=dtype).view(rows, cols)


def glorot(seed: int, stream: int, f_in: int, f_out: int, device="cpu") -> torch.Tensor:
    """Glorot-uniform f_in x f_out fp32 weight."""
    lim = math.sqrt(6.0 / (f_in + f_out))
    return rng.uniform(seed, stream, f_in * f_out, -lim, lim, device=device).view(f_in, f_out)


def to_bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """fp32 -> bf16 storage (torch's round-to-nearest-even cast), as a bfloat16 tensor."""
    return x.to(torch.bfloat16)


class HaloStream:
    """Drifting halo rows: epoch 0 is N(0,1); each later epoch multiplies every
    element by (1 + eta_t * u_r * g) with g ~ N(0,1) per element, a per-row rate
    u_r log-uniform in [0.1, 10], and eta_t = eta0 * kappa**t. Updates shrink
    from epoch to epoch the way layer outputs do as parameters settle, so the
    fraction of rows that fail a fixed-threshold cache test falls over time.
    """

    def __init__(self, seed: int, rows: int, cols: int, device="cpu",
                 eta0: float = 0.2, kappa: float = 0.6, stream: int = 40):
        self.seed, self.rows, self.cols, self.device = seed, rows, cols, device
        self.eta0, self.kappa, self.stream = eta0, kappa, stream
        self.t = 0
        self.cur = normal_matrix(seed, stream, rows, cols, device=device)
        lu = rng.uniform(seed, stream + 1, rows, math.log(0.1), math.log(10.0), device=device,
                         dtype=torch.float64)
        self.rate = torch.exp(lu).to(torch.float32).view(rows, 1)

    def value(self) -> torch.Tensor:
        return self.cur

    def advance(self) -> torch.Tensor:
        self.t += 1
        g = normal_matrix(self.seed, self.stream + 1 + self.t, self.rows, self.cols, device=self.device)
        eta = self.eta0 * self.kappa ** self.t
        self.cur = self.cur * (1.0 + (eta * self.rate) * g)
        return self.cur
