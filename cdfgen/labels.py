"""Seeded node-classification task on a synthetic graph: class labels that agree with the
graph's neighbourhoods, features that carry a noisy copy of the label, and a train split.
Input recipe only - nothing of the trained method lives here.
"""
import torch

from . import rng


def planted_labels(g, classes: int, seed: int, rounds: int = 2) -> torch.Tensor:
    """int64 [n] labels. Start: a hashed class per vertex. Then `rounds` synchronous votes:
    every vertex takes the class most frequent among itself and its neighbours (lowest class
    on ties). The result is homophilous, which is what message passing can exploit; two rounds keep
    the largest class below a fifth of the vertices on the power-law graphs used here (a third round
    lets one class take over half of them)."""
    dev = g.lo.device
    n = g.n
    lab = (rng.uniform01(seed, 60, torch.arange(n, dtype=torch.int64, device=dev)) * classes).long().clamp_(0, classes - 1)
    for _ in range(rounds):
        votes = torch.zeros(n * classes, dtype=torch.int32, device=dev)
        one = torch.ones(1, dtype=torch.int32, device=dev)
        votes.index_add_(0, g.lo * classes + lab[g.hi], one.expand(g.lo.numel()))
        votes.index_add_(0, g.hi * classes + lab[g.lo], one.expand(g.lo.numel()))
        votes.index_add_(0, torch.arange(n, device=dev) * classes + lab, one.expand(n))
        lab = torch.argmax(votes.view(n, classes), dim=1)   # first maximum = lowest class
    return lab


def planted_features(labels: torch.Tensor, dim: int, seed: int, signal: float = 0.15) -> torch.Tensor:
    """fp32 [n, dim]: signal * centroid[label] + N(0, 1) noise; centroids are N(0, 1) rows."""
    dev = labels.device
    classes = int(labels.max().item()) + 1 if labels.numel() else 1
    cent = rng.normal(seed, 61, classes * dim, device=dev).view(classes, dim)
    noise = rng.normal(seed, 62, labels.numel() * dim, device=dev).view(labels.numel(), dim)
    return (signal * cent[labels] + noise).contiguous()


def train_mask(n: int, seed: int, fraction: float = 0.6, device="cpu") -> torch.Tensor:
    """bool [n]: hashed Bernoulli(fraction) train membership."""
    return rng.uniform01(seed, 63, torch.arange(n, dtype=torch.int64, device=device)) < fraction
