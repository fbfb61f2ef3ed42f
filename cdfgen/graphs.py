"""Seeded synthetic graphs: R-MAT and Chung-Lu edge samples, made simple,
undirected and self-looped, with symmetric-normalised weights.

All routines work on torch tensors of a caller-chosen device so that the large
benchmark graphs can be produced on the accelerator and the small test graphs
on the host; integer results are identical on both.
"""
from dataclasses import dataclass

import torch

from . import rng


def rmat_pairs(scale: int, n_samples: int, seed: int, a=0.57, b=0.19, c=0.19,
               device="cpu", chunk: int = 1 << 25):
    """n_samples (row, col) pairs from the recursive-matrix model on 2**scale ids.

    One 16-bit draw per recursion level picks the quadrant with probabilities
    (a, b, c, 1-a-b-c); four levels share one 64-bit hash.
    """
    ta = int(round(a * 65536))
    tb = int(round((a + b) * 65536))
    tc = int(round((a + b + c) * 65536))
    rows = torch.empty(n_samples, dtype=torch.int64, device=device)
    cols = torch.empty(n_samples, dtype=torch.int64, device=device)
    for s in range(0, n_samples, chunk):
        e = min(n_samples, s + chunk)
        cnt = torch.arange(s, e, dtype=torch.int64, device=device)
        r = torch.zeros(e - s, dtype=torch.int64, device=device)
        q = torch.zeros(e - s, dtype=torch.int64, device=device)
        h = None
        for lvl in range(scale):
            if lvl % 4 == 0:
                h = rng.bits64(seed, 100 + lvl // 4, cnt)
            u = (h >> (16 * (lvl % 4))) & 0xFFFF
            right = ((u >= ta) & (u < tb)) | (u >= tc)     # quadrants b, d
            down = u >= tb                                  # quadrants c, d
            r = (r << 1) | down.to(torch.int64)
            q = (q << 1) | right.to(torch.int64)
        rows[s:e] = r
        cols[s:e] = q
    return rows, cols


def rmat_pairs_bounded(scale: int, n_vertices: int, n_samples: int, seed: int,
                       device="cpu", **kw):
    """R-MAT samples with both ids < n_vertices: draws are taken in counter order
    and those with an id out of range are skipped until n_samples are kept."""
    if n_vertices == (1 << scale):
        return rmat_pairs(scale, n_samples, seed, device=device, **kw)
    over = int(n_samples * 1.6) + 1024
    while True:
        r, c = rmat_pairs(scale, over, seed, device=device, **kw)
        keep = (r < n_vertices) & (c < n_vertices)
        if int(keep.sum()) >= n_samples:
            r, c = r[keep], c[keep]
            return r[:n_samples].contiguous(), c[:n_samples].contiguous()
        over *= 2


def chung_lu_pairs(n_vertices: int, n_samples: int, exponent: float, seed: int,
                   device="cpu", permute=True, chunk: int = 1 << 25):
    """Endpoint pairs drawn independently with probability proportional to a
    power-law expected degree w_i ~ (i + i0)**(-1/(exponent-1)).

    With permute=True vertex ids are shuffled by a seeded permutation so that
    id order carries no degree information.
    """
    i0 = 10.0
    w = (torch.arange(n_vertices, dtype=torch.float64, device=device) + i0) ** (-1.0 / (exponent - 1.0))
    cdf = torch.cumsum(w, 0)
    cdf = cdf / cdf[-1].clone()
    perm = None
    if permute:
        key = rng.bits64(seed, 7, torch.arange(n_vertices, dtype=torch.int64, device=device))
        perm = torch.argsort(key, stable=True)
    out = []
    for side in range(2):
        ids = torch.empty(n_samples, dtype=torch.int64, device=device)
        for s in range(0, n_samples, chunk):
            e = min(n_samples, s + chunk)
            u = rng.uniform01(seed, 8 + side, torch.arange(s, e, dtype=torch.int64, device=device))
            v = torch.searchsorted(cdf, u).clamp_(max=n_vertices - 1)
            ids[s:e] = perm[v] if perm is not None else v
        out.append(ids)
    return out[0], out[1]


@dataclass
class Graph:
    """Simple undirected graph: unique pairs (lo < hi) plus degrees of A + I."""
    n: int
    lo: torch.Tensor       # int64 [m]
    hi: torch.Tensor       # int64 [m]
    deg: torch.Tensor      # int64 [n], degree in A + I (neighbours + 1)

    @property
    def nnz(self) -> int:  # stored entries of A + I
        return 2 * self.lo.numel() + self.n


def make_graph(n: int, rows: torch.Tensor, cols: torch.Tensor) -> Graph:
    """Drop self pairs, merge duplicates and directions."""
    keep = rows != cols
    r, c = rows[keep], cols[keep]
    lo = torch.minimum(r, c)
    hi = torch.maximum(r, c)
    key = torch.unique(lo * n + hi)
    lo = torch.div(key, n, rounding_mode="floor")
    hi = key - lo * n
    deg = torch.bincount(lo, minlength=n) + torch.bincount(hi, minlength=n) + 1
    return Graph(n, lo, hi, deg)


@dataclass
class Partition:
    """One device's share: owned rows plus halo columns, locally renumbered.

    Local ids 0..n_loc-1 are the owned vertices in ascending global id; ids
    n_loc..n_loc+n_halo-1 are the remote neighbours in ascending global id.
    A is n_loc x (n_loc+n_halo) in CSR with ascending column ids in a row; At is
    its transpose, also CSR. vals = 1/sqrt(deg_u deg_v) with global degrees.
    """
    n_loc: int
    n_halo: int
    owned: torch.Tensor     # int64 [n_loc] global ids
    halo: torch.Tensor      # int64 [n_halo] global ids
    rowptr: torch.Tensor    # int64 [n_loc+1]
    colidx: torch.Tensor    # int32 [nnz]
    vals: torch.Tensor      # float32 [nnz]
    t_rowptr: torch.Tensor  # int64 [n_loc+n_halo+1]
    t_colidx: torch.Tensor  # int32 [nnz]
    t_vals: torch.Tensor    # float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.colidx.numel())

    def to(self, device):
        kw = {k: (v.to(device) if torch.is_tensor(v) else v) for k, v in self.__dict__.items()}
        return Partition(**kw)


def _csr_from_sorted_rows(rows: torch.Tensor, n_rows: int) -> torch.Tensor:
    cnt = torch.bincount(rows, minlength=n_rows)
    ptr = torch.zeros(n_rows + 1, dtype=torch.int64, device=rows.device)
    torch.cumsum(cnt, 0, out=ptr[1:])
    return ptr


def extract_partition(g: Graph, owned_mask: torch.Tensor) -> Partition:
    """Rows of D^-1/2 (A+I) D^-1/2 owned by one partition, with halo columns."""
    dev = g.lo.device
    owned = torch.nonzero(owned_mask).flatten()
    n_loc = int(owned.numel())
    m_lo = owned_mask[g.lo]
    m_hi = owned_mask[g.hi]
    # directed entries whose row is owned: (lo->hi), (hi->lo), (v->v)
    r = torch.cat([g.lo[m_lo], g.hi[m_hi], owned])
    c = torch.cat([g.hi[m_lo], g.lo[m_hi], owned])
    del m_lo, m_hi
    col_owned = owned_mask[c]
    halo = torch.unique(c[~col_owned])
    n_halo = int(halo.numel())
    # global -> local id
    loc = torch.full((g.n,), -1, dtype=torch.int64, device=dev)
    loc[owned] = torch.arange(n_loc, dtype=torch.int64, device=dev)
    loc[halo] = n_loc + torch.arange(n_halo, dtype=torch.int64, device=dev)
    w = 1.0 / torch.sqrt(g.deg[r].to(torch.float64) * g.deg[c].to(torch.float64))
    lr, lc = loc[r], loc[c]
    del r, c, loc
    n_cols = n_loc + n_halo
    order = torch.argsort(lr * n_cols + lc)
    lr, lc, w = lr[order], lc[order], w[order].to(torch.float32)
    rowptr = _csr_from_sorted_rows(lr, n_loc)
    # transpose
    order = torch.argsort(lc * n_loc + lr)
    t_rowptr = _csr_from_sorted_rows(lc[order], n_cols)
    return Partition(n_loc, n_halo, owned, halo, rowptr, lc.to(torch.int32), w,
                     t_rowptr, lr[order].to(torch.int32), w[order])


def range_mask(n: int, parts: int, p: int, device="cpu") -> torch.Tensor:
    """Contiguous-range partition p of parts: ids [p*ceil(n/parts), (p+1)*ceil(n/parts))."""
    size = -(-n // parts)
    m = torch.zeros(n, dtype=torch.bool, device=device)
    m[p * size:min(n, (p + 1) * size)] = True
    return m


def bfs_grown_owner(g: Graph, parts: int, seed: int, max_rounds: int = 64) -> torch.Tensor:
    """Balanced region growing: `parts` seeded sources expand breadth-first, one
    level per round and all at once, each capped at ceil(n/parts) vertices. A
    vertex reached by several regions in one round joins the lowest-numbered
    one; within a region lower ids win when the cap cuts a level. Vertices never
    reached fill the remaining room in id order.
    """
    dev = g.lo.device
    n = g.n
    cap = -(-n // parts)
    owner = torch.full((n,), -1, dtype=torch.int64, device=dev)
    key = rng.bits64(seed, 21, torch.arange(n, dtype=torch.int64, device=dev))
    # sources: the `parts` vertices with the smallest hash among those of degree >= 3
    key = torch.where(g.deg >= 3, key, torch.full_like(key, (1 << 63) - 1))
    src = torch.argsort(key, stable=True)[:parts]
    owner[src] = torch.arange(parts, dtype=torch.int64, device=dev)
    size = torch.ones(parts, dtype=torch.int64, device=dev)
    frontier = torch.zeros(n, dtype=torch.bool, device=dev)
    frontier[src] = True
    BIG = parts
    for _ in range(max_rounds):
        cand = torch.full((n,), BIG, dtype=torch.int64, device=dev)
        for a, b in ((g.lo, g.hi), (g.hi, g.lo)):
            m = frontier[a] & (owner[b] < 0)
            cand.scatter_reduce_(0, b[m], owner[a[m]], reduce="amin")
        newv = torch.nonzero(cand < BIG).flatten()       # ascending ids
        if newv.numel() == 0:
            break
        frontier.zero_()
        p_of = cand[newv]
        order = torch.argsort(p_of, stable=True)         # by region, ids ascending inside
        newv, p_of = newv[order], p_of[order]
        cnt = torch.bincount(p_of, minlength=parts)
        start = torch.cumsum(cnt, 0) - cnt
        rank = torch.arange(newv.numel(), device=dev) - start[p_of]
        ok = rank < (cap - size)[p_of]
        newv, p_of = newv[ok], p_of[ok]
        owner[newv] = p_of
        frontier[newv] = True
        size += torch.bincount(p_of, minlength=parts)
    rest = torch.nonzero(owner < 0).flatten()
    if rest.numel():
        room = (cap - size).clamp(min=0)
        fill = torch.repeat_interleave(torch.arange(parts, device=dev), room)[:rest.numel()]
        owner[rest] = fill
    return owner
