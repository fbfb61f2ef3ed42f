"""The five benchmark workloads as seeded recipes, and a builder that turns a
recipe into one partition's CSR blocks. `shrink` scales a recipe down (fewer
vertices and samples) for tests that must finish on the host in seconds.
"""
from dataclasses import dataclass, replace
from typing import List, Tuple

from . import graphs


@dataclass
class Workload:
    name: str
    seed: int
    kind: str                 # "rmat" | "chung_lu"
    n_vertices: int
    scale: int                # R-MAT recursion depth (2**scale >= n_vertices)
    n_samples: int            # undirected edge samples before deduplication
    parts: int
    part: int                 # which partition is the workload
    partitioner: str          # "range" | "bfs"
    dims: List[int]           # feature widths f0 -> f1 -> ... -> classes
    dtype: str = "f32"        # "f32" | "bf16" storage of features / gradients
    bits: int = 8
    qscheme: str = "minmax"
    norm: str = "linf"
    eps: float = 0.05
    exponent: float = 2.1     # Chung-Lu only

    def layers(self) -> List[Tuple[int, int]]:
        return list(zip(self.dims[:-1], self.dims[1:]))


# seed = 0xCDF0 + index
TINY = Workload("tiny", 0xCDF0, "rmat", 2048, 11, 2048 * 8 // 2, 4, 0, "range", [128, 16, 8])
MID = Workload("mid", 0xCDF1, "rmat", 100_000, 17, 100_000 * 50 // 2, 8, 0, "range", [602, 256, 41])
LARGE = Workload("large", 0xCDF2, "chung_lu", 2_400_000, 22, 62_000_000, 8, 0, "bfs", [100, 256, 256, 47])
WIDE = Workload("wide", 0xCDF3, "rmat", 1 << 20, 20, (1 << 20) * 30 // 2, 4, 3, "range",
                [1024, 512, 64], dtype="bf16", bits=4)
SHARE = Workload("share", 0xCDF4, "rmat", 1 << 24, 24, (1 << 24) * 20 // 2, 8, 0, "range",
                 [128, 256, 256, 64])

ALL = {w.name: w for w in (TINY, MID, LARGE, WIDE, SHARE)}


def shrink(w: Workload, n_vertices: int) -> Workload:
    """Same recipe on fewer vertices, keeping samples per vertex."""
    per = w.n_samples / w.n_vertices
    scale = max(1, (n_vertices - 1).bit_length())
    return replace(w, name=f"{w.name}@{n_vertices}", n_vertices=n_vertices, scale=scale,
                   n_samples=int(per * n_vertices))


def build_graph(w: Workload, device="cpu") -> graphs.Graph:
    if w.kind == "rmat":
        r, c = graphs.rmat_pairs_bounded(w.scale, w.n_vertices, w.n_samples, w.seed, device=device)
    elif w.kind == "chung_lu":
        r, c = graphs.chung_lu_pairs(w.n_vertices, w.n_samples, w.exponent, w.seed, device=device)
    else:
        raise ValueError(w.kind)
    return graphs.make_graph(w.n_vertices, r, c)


def owner_masks(w: Workload, g: graphs.Graph):
    """List of boolean ownership masks, one per partition."""
    dev = g.lo.device
    if w.partitioner == "range":
        return [graphs.range_mask(g.n, w.parts, p, device=dev) for p in range(w.parts)]
    owner = graphs.bfs_grown_owner(g, w.parts, w.seed)
    return [owner == p for p in range(w.parts)]


def build_partition(w: Workload, device="cpu", part=None, graph=None) -> graphs.Partition:
    g = graph if graph is not None else build_graph(w, device=device)
    p = w.part if part is None else part
    if w.partitioner == "range":
        mask = graphs.range_mask(g.n, w.parts, p, device=g.lo.device)
    else:
        mask = graphs.bfs_grown_owner(g, w.parts, w.seed) == p
    return graphs.extract_partition(g, mask)
