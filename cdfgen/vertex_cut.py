"""Vertex-cut partitions as inputs: every undirected edge belongs to one device, vertices
are replicated on every device that holds one of their edges, and one replica is the master
(Sec. 3.2's framing). Builds the per-device blocks of D^-1/2 (A+I) D^-1/2 whose sum over the
devices is the whole normalised adjacency. Input preparation only.
"""
from dataclasses import dataclass
from typing import List

import torch

from . import rng


@dataclass
class VcPart:
    """One device's subgraph. Local ids: masters first (ascending global id), then mirrors
    (ascending). A is n x n, n = n_master + n_mirror, CSR with ascending columns in a row, and
    symmetric (both directions of an edge live on the edge's device; the self entry of a
    vertex lives with its master)."""
    n_master: int
    n_mirror: int
    vertices: torch.Tensor          # int64 [n] global ids
    rowptr: torch.Tensor            # int64 [n+1]
    colidx: torch.Tensor            # int32 [nnz]
    vals: torch.Tensor              # float32 [nnz]
    mirror_master_dev: torch.Tensor  # int64 [n_mirror] device of the mirror's master
    mirror_master_row: torch.Tensor  # int64 [n_mirror] local row of the master there

    @property
    def n(self) -> int:
        return self.n_master + self.n_mirror

    @property
    def nnz(self) -> int:
        return int(self.colidx.numel())


def hashed_edge_cut(g, p: int, seed: int) -> torch.Tensor:
    """int32 [n_edges]: every edge on a hashed device (a random vertex-cut)."""
    e = torch.arange(g.lo.numel(), dtype=torch.int64, device=g.lo.device)
    return (rng.uniform01(seed, 90, e) * p).to(torch.int32).clamp_(0, p - 1)


def choose_masters(g, part: torch.Tensor, p: int) -> torch.Tensor:
    """int64 [n]: the replica holding most of the vertex's edges, lowest device on ties; a vertex
    without edges lives on device v mod p."""
    n = g.n
    inc = torch.zeros(n * p, dtype=torch.int64)
    one = torch.ones(1, dtype=torch.int64)
    d = part.to(torch.int64)
    inc.index_add_(0, g.lo * p + d, one.expand(d.numel()))
    inc.index_add_(0, g.hi * p + d, one.expand(d.numel()))
    inc = inc.view(n, p)
    m = torch.argmax(inc, dim=1)                      # first maximum = lowest device
    lone = inc.sum(1) == 0
    m[lone] = torch.arange(n)[lone] % p
    return m


def extract_vertex_cut(g, part: torch.Tensor, master: torch.Tensor, p: int) -> List[VcPart]:
    n = g.n
    d = part.to(torch.int64)
    out = []
    local_row = torch.full((p, n), -1, dtype=torch.int64)   # small graphs: dense lookup is fine
    verts = []
    for i in range(p):
        on = d == i
        here = torch.zeros(n, dtype=torch.bool)
        here[g.lo[on]] = True
        here[g.hi[on]] = True
        is_m = master == i
        here |= is_m
        ms = torch.nonzero(here & is_m).flatten()
        mr = torch.nonzero(here & ~is_m).flatten()
        v = torch.cat([ms, mr])
        local_row[i, v] = torch.arange(v.numel())
        verts.append((ms, mr, v))
    deg = g.deg.to(torch.float64)
    for i in range(p):
        ms, mr, v = verts[i]
        on = d == i
        r = torch.cat([g.lo[on], g.hi[on], ms])
        c = torch.cat([g.hi[on], g.lo[on], ms])
        w = (1.0 / torch.sqrt(deg[r] * deg[c])).to(torch.float32)
        lr, lc = local_row[i, r], local_row[i, c]
        nloc = int(v.numel())
        order = torch.argsort(lr * max(nloc, 1) + lc)
        lr, lc, w = lr[order], lc[order], w[order]
        cnt = torch.bincount(lr, minlength=nloc)
        rowptr = torch.zeros(nloc + 1, dtype=torch.int64)
        torch.cumsum(cnt, 0, out=rowptr[1:])
        mdev = master[mr]
        mrow = local_row[mdev, mr]
        out.append(VcPart(int(ms.numel()), int(mr.numel()), v, rowptr, lc.to(torch.int32), w, mdev, mrow))
    return out
