"""Training in the paper's own vertex-cut framing on one GPU: every device's subgraph (master
and mirror replicas, Sec. 3.2) is stepped in turn on one stream, and the replicas are reconciled
by Alg. 2 in full - mirrors test and send differences (gather), masters add them and their own
change to the cached total and mark the vertex active, totals of active vertices return to the
mirrors (scatter). Marshalling only: buffers, argument order, call order; all arithmetic is libcdf's.

Layout: device i holds n_i = n_master_i + n_mirror_i consecutive rows (masters first) of every
tall matrix; `base[i]` is its first row. The cached total of a vertex lives in its master's row of
`tot`; a mirror's row of `tot` is that mirror's copy.
"""
from dataclasses import dataclass
from typing import List

import torch

from cdfgen import configs, features, labels as labelgen, vertex_cut as vcut

from . import binding as B
from .layer import DeviceCsr

_QS = {"minmax": B.Q_MINMAX, "symmetric": B.Q_SYMMETRIC, "none": B.Q_NONE}
_NORM = {"linf": B.NORM_LINF, "l2": B.NORM_L2}


@dataclass
class VcEpochStats:
    epoch: int
    eps: float
    loss: float
    train_acc: float
    mean_acc: float
    gather: int            # mirror rows that sent a difference (all exchanges of the epoch)
    scatter: int           # mirror rows that received a total
    master_updates: int
    mirror_rows: int       # mirror rows tested
    message_bytes: int

    @property
    def hit_rate(self) -> float:
        """Share of mirror rows that needed no message in either phase."""
        return 1.0 - (self.gather + self.scatter) / (2 * self.mirror_rows) if self.mirror_rows else 1.0


class _Exchange:
    """Cache state of one exchanged quantity: partial rows of this epoch, what every replica last
    contributed, and the totals (tall matrices of one width)."""

    def __init__(self, rows, dim, device):
        z = lambda: torch.zeros(rows, dim, dtype=torch.float32, device=device)
        self.part, self.zc, self.tot, self.dim = z(), z(), z(), dim


class VcTrainer:
    def __init__(self, w: configs.Workload, device="cuda:0", eps0=None, lr=0.01, adaptive=True, eps_params=None,
                 qscheme=None, qscheme_scatter=None, bits=None, norm=None, edge_part=None, graph=None,
                 train_fraction=0.6, signal=0.15, keep_inputs=False, p=None):
        """edge_part: int32 [n_edges] device of every undirected edge of the workload graph (default:
        the hierarchical EBV partitioner with its default weights on one host)."""
        assert w.dtype == "f32"
        self.w, self.device, self.lr, self.adaptive = w, device, lr, adaptive
        self.eps = float(w.eps if eps0 is None else eps0)
        self.eps_params, self.mean_acc, self.t = eps_params, 0.0, 0
        self.bits = w.bits if bits is None else bits
        self.qs = _QS[w.qscheme if qscheme is None else qscheme]
        self.qs_scatter = self.qs if qscheme_scatter is None else _QS[qscheme_scatter]
        self.norm = _NORM[w.norm if norm is None else norm]
        g = graph if graph is not None else configs.build_graph(w, device="cpu")
        p = w.parts if p is None else p
        if edge_part is None:
            edge_part = B.cdf_ebv_partition(g.n, g.lo.contiguous(), g.hi.contiguous(), p, p, 1.0, 1.0, 0.0, True)
        master = vcut.choose_masters(g, edge_part, p)
        parts = vcut.extract_vertex_cut(g, edge_part, master, p)
        self.parts, self.p, self.n = parts, p, g.n
        dims = w.layers()
        self.dims, self.L, self.classes = dims, len(dims), dims[-1][1]
        L = self.L

        y = labelgen.planted_labels(g, self.classes, w.seed)
        x0 = labelgen.planted_features(y, dims[0][0], w.seed, signal)
        tm = labelgen.train_mask(g.n, w.seed, train_fraction)
        self.n_train = int(tm.sum().item())
        self.inputs = dict(graph=g, x0=x0, labels=y, train=tm, edge_part=edge_part) if keep_inputs else None

        base = [0]
        for P in parts:
            base.append(base[-1] + P.n)
        self.base, self.rows_total = base, base[-1]
        assert self.rows_total < 2 ** 31
        dev = device
        z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=dev)
        self.A = [DeviceCsr(P.n, P.n, P.rowptr, P.colidx, P.vals, dev) for P in parts]
        # tall row of each mirror's master
        self.mmap = [(torch.tensor(base)[P.mirror_master_dev] + P.mirror_master_row).to(torch.int32).to(dev)
                     for P in parts]
        verts = torch.cat([P.vertices for P in parts])
        is_master = torch.cat([torch.arange(P.n) < P.n_master for P in parts])
        self.vertices, self.is_master = verts, is_master
        lab = torch.where(tm, y, torch.full_like(y, -1))[verts]
        self.labels_all = lab.to(torch.int32).to(dev)                                   # every replica
        self.labels_master = torch.where(is_master, lab, torch.full_like(lab, -1)).to(torch.int32).to(dev)

        R = self.rows_total
        self.X = [z(R, f) for f, _ in dims]
        self.X[0].copy_(x0[verts].to(dev))
        self.M = [z(R, f) for f, _ in dims]
        self.zx = [_Exchange(R, gout, dev) for _, gout in dims]                 # forward: partial Z of layer l
        self.dx = [None] + [_Exchange(R, f, dev) for f, _ in dims[1:]]          # backward: partial gradient of X[l]
        self.dM = [None] + [z(R, f) for f, _ in dims[1:]]
        self.dlogits = z(R, self.classes)
        self.W = [features.glorot(w.seed, 70 + l, f, gout).to(dev) for l, (f, gout) in enumerate(dims)]
        self.adam_m = [torch.zeros_like(W) for W in self.W]
        self.adam_v = [torch.zeros_like(W) for W in self.W]
        self.dW = [[z(f, gout) for f, gout in dims] for _ in parts]
        self.loss_sum, self.counts = z(1), z(2, dt=torch.int32)
        self.scratch_loss, self.scratch_counts = z(1), z(2, dt=torch.int32)
        self.scratch_dlogits = z(R, self.classes)
        self.active = z(max(R, 1), dt=torch.uint8)
        self.n_ex = L + (L - 1)
        self.n_sent = z(self.n_ex * p * 3, dt=torch.int32)       # [exchange][device][gather, master, scatter]
        # message scratch, shared by all exchanges (they run one after another)
        dmax = max(max(d) for d in dims)
        cap = max(max(P.n_master, P.n_mirror) for P in parts)
        cap = max(cap, 1)
        self.mask = z(cap, dt=torch.uint8)
        self.idx = z(cap, dt=torch.int32)
        self.idx_owner = z(cap, dt=torch.int32)
        self.codes = z(cap * dmax * 4, dt=torch.uint8)
        self.meta = z(cap, 2)
        self.fresh = z(cap * dmax)
        nbytes = max(B.cdf_workspace_bytes(max(P.n, 1), dmax, max(P.nnz, 1)) for P in parts)
        nbytes = max(nbytes, B.cdf_workspace_bytes(R, dmax, 0))
        self.ws = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        self.history: List[VcEpochStats] = []

    # ---- Alg. 2 ------------------------------------------------------------------------------
    def _ns(self, ex, i, k):
        o = (ex * self.p + i) * 3 + k
        return self.n_sent[o:o + 1]

    def exchange(self, ex: int, st: _Exchange) -> None:
        """Reconcile st.part into st.tot (what every replica works with afterwards)."""
        eps, D = self.eps, st.dim
        self.active.zero_()
        for i, P in enumerate(self.parts):                  # mirrors: test, difference to the master, commit
            if not P.n_mirror:
                continue
            lo, hi = self.base[i] + P.n_master, self.base[i] + P.n
            ns = self._ns(ex, i, 0)
            idx, idxo = self.idx[:P.n_mirror], self.idx_owner[:P.n_mirror]
            B.cdf_cache_filter_quantize(st.part[lo:hi], st.zc[lo:hi], eps, self.norm, self.bits, self.qs, B.COMMIT_CUR,
                                        True, self.mask, idx, ns, self.codes, self.meta, self.ws)
            B.cdf_map_index(idx, ns, self.mmap[i], idxo)   # the master's row; the master adds and becomes active
            B.cdf_dequantize(self.codes, self.meta, idxo, ns, P.n_mirror, self.bits, self.qs, st.tot, True)
            B.cdf_mark_rows(idxo, ns, None, 0, self.active)
        for i, P in enumerate(self.parts):                  # masters: own change, exact (it never leaves the device)
            if not P.n_master:
                continue
            lo, hi = self.base[i], self.base[i] + P.n_master
            ns = self._ns(ex, i, 1)
            idx = self.idx[:P.n_master]
            B.cdf_cache_filter(st.part[lo:hi], st.zc[lo:hi], eps, self.norm, self.mask, idx, ns, self.ws)
            B.cdf_quantize(st.part[lo:hi], st.zc[lo:hi], idx, ns, P.n_master, self.bits, B.Q_NONE, B.COMMIT_CUR, True,
                           self.codes, self.meta)
            B.cdf_dequantize(self.codes, self.meta, idx, ns, P.n_master, self.bits, B.Q_NONE, st.tot[lo:hi], True)
            B.cdf_mark_rows(idx, ns, None, lo, self.active)
        for i, P in enumerate(self.parts):                  # scatter: totals of active vertices to their mirrors
            if not P.n_mirror:
                continue
            lo, hi = self.base[i] + P.n_master, self.base[i] + P.n
            ns = self._ns(ex, i, 2)
            idx = self.idx[:P.n_mirror]
            fresh = self.fresh[:P.n_mirror * D].view(P.n_mirror, D)
            B.cdf_active_rows(self.active, self.mmap[i], self.mask, idx, ns, self.ws)
            B.cdf_gather_rows(st.tot, self.mmap[i], fresh)
            B.cdf_quantize(fresh, None, idx, ns, P.n_mirror, self.bits, self.qs_scatter, B.COMMIT_NONE, False,
                           self.codes, self.meta)
            B.cdf_dequantize(self.codes, self.meta, idx, ns, P.n_mirror, self.bits, self.qs_scatter, st.tot[lo:hi], False)

    # ---- one epoch (Alg. 1) ----------------------------------------------------------------------
    def epoch(self) -> VcEpochStats:
        eps, L, base = self.eps, self.L, self.base
        ex = 0
        for l in range(L):
            st = self.zx[l]
            for i, P in enumerate(self.parts):
                lo, hi = base[i], base[i] + P.n
                B.cdf_spmm_fwd(self.A[i].struct, self.X[l][lo:hi], self.M[l][lo:hi], self.ws)
                B.cdf_dense_fwd(self.M[l][lo:hi], self.W[l], False, st.part[lo:hi], None)
            self.exchange(ex, st)
            ex += 1
            if l + 1 < L:
                B.cdf_relu_fwd(st.tot, self.X[l + 1])
        logits = self.zx[-1].tot
        scale = 1.0 / max(self.n_train, 1)
        B.cdf_softmax_xent(logits, self.labels_all, scale, self.dlogits, self.scratch_loss, self.scratch_counts, self.ws)
        B.cdf_softmax_xent(logits, self.labels_master, scale, self.scratch_dlogits, self.loss_sum, self.counts, self.ws)
        dH = self.dlogits
        for l in reversed(range(L)):
            for i, P in enumerate(self.parts):
                lo, hi = base[i], base[i] + P.n
                dM = self.dM[l][lo:hi] if l else None
                B.cdf_dense_bwd(self.M[l][lo:hi], self.W[l], self.zx[l].tot[lo:hi], dH[lo:hi], l + 1 < L, self.dW[i][l],
                                dM, self.ws)
                if l:
                    B.cdf_spmm_fwd(self.A[i].struct, dM, self.dx[l].part[lo:hi], self.ws)   # A_i is symmetric
            for i in range(1, self.p):
                B.cdf_accumulate(self.dW[0][l], self.dW[i][l])
            if l:
                self.exchange(ex, self.dx[l])
                ex += 1
                dH = self.dx[l].tot
        self.t += 1
        for l in range(L):
            B.cdf_adam_step(self.W[l], self.dW[0][l], self.adam_m[l], self.adam_v[l], self.lr, self.t)
        sent = self.n_sent.cpu().view(self.n_ex, self.p, 3)
        counts = self.counts.tolist()
        loss = float(self.loss_sum.item()) / max(counts[1], 1)
        acc = counts[0] / max(counts[1], 1)
        new_eps, self.mean_acc = B.cdf_eps_update(self.eps, acc, self.mean_acc, self.eps_params)
        if self.adaptive:
            self.eps = new_eps
        widths = [gout for _, gout in self.dims] + [f for f, _ in reversed(self.dims[1:])]
        nbytes = 0
        for e, D in enumerate(widths):
            nbytes += int(sent[e, :, 0].sum()) * (B.cdf_code_row_bytes(D, self.bits, self.qs) + 12)
            nbytes += int(sent[e, :, 2].sum()) * (B.cdf_code_row_bytes(D, self.bits, self.qs_scatter) + 12)
        st = VcEpochStats(len(self.history), eps, loss, acc, self.mean_acc, int(sent[:, :, 0].sum()),
                          int(sent[:, :, 2].sum()), int(sent[:, :, 1].sum()),
                          sum(P.n_mirror for P in self.parts) * self.n_ex, nbytes)
        self.history.append(st)
        return st

    def logits_by_vertex(self) -> torch.Tensor:
        out = torch.zeros(self.n, self.classes)
        t = self.zx[-1].tot.cpu()
        out[self.vertices[self.is_master]] = t[self.is_master]
        return out
