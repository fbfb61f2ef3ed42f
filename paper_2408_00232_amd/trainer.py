"""Full-batch GCN training of ALL partitions of a workload on one device (Alg. 1 with the
adaptive cache of Alg. 2, the quantised messages of Sec. 5 and the threshold controller of
Sec. 4.1). The partitions take turns on the one stream; rows that would cross the network
are moved by cdf_gather_rows (features, owner -> reader) and by cdf_map_index +
cdf_dequantize (gradients, reader -> owner). This module allocates device memory, fills
argument blocks and orders the calls; every number is computed inside libcdf.

Layout. Partition j owns rows_j = n_loc_j + n_halo_j consecutive rows, local rows first,
of one tall matrix per layer input (`X[l]`, and `dX[l]` for its gradient); `base[j]` is its
first row. Output H of layer l on partition j is written straight into the local rows of
X[l+1], and the gradient arriving at those rows is read from dX[l+1] in place. Owner-side
totals of the gradient messages live in `S[l]`, one row per vertex in owner order
(`off[j]` = first row of partition j): difference messages only ever add to them.
"""
import ctypes
from dataclasses import dataclass
from typing import List

import torch

from cdfgen import configs, features, graphs, labels as labelgen

from . import binding as B
from .layer import DeviceCsr

_QS = {"minmax": B.Q_MINMAX, "symmetric": B.Q_SYMMETRIC, "none": B.Q_NONE}
_NORM = {"linf": B.NORM_LINF, "l2": B.NORM_L2}


@dataclass
class EpochStats:
    epoch: int
    eps: float            # threshold the epoch ran with
    loss: float           # mean cross-entropy over the train rows
    train_acc: float
    mean_acc: float       # moving average after this epoch
    sent_fwd: int         # halo rows that failed the cache test, forward, all layers and partitions
    sent_bwd: int
    rows_fwd: int         # halo rows tested, forward
    rows_bwd: int
    message_bytes: int    # codes + per-row range + row index of everything sent

    @property
    def hit_rate(self) -> float:
        tot = self.rows_fwd + self.rows_bwd
        return 1.0 - (self.sent_fwd + self.sent_bwd) / tot if tot else 1.0


class _PartLayer:
    """Device buffers of one (partition, layer) pair that are not slices of the tall matrices."""

    def __init__(self, n_loc, n_halo, f_in, f_out, bits, qs, need_dx, device):
        z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=device)
        nh = max(n_halo, 1)
        rb = B.cdf_code_row_bytes(f_in, bits, qs)
        self.row_bytes = rb
        self.halo_fresh = z(nh, f_in)
        self.cache_sent = z(nh, f_in)
        self.M = z(max(n_loc, 1), f_in)
        self.mask = z(nh, dt=torch.uint8)
        self.idx = z(nh, dt=torch.int32)
        self.codes = z(max(n_halo * rb, 16), dt=torch.uint8)
        self.meta = z(nh, 2)
        self.dW = z(f_in, f_out)
        if need_dx:
            self.dM = z(max(n_loc, 1), f_in)
            self.gcache_sent = z(nh, f_in)
            self.gmask = z(nh, dt=torch.uint8)
            self.gidx = z(nh, dt=torch.int32)
            self.gidx_owner = z(nh, dt=torch.int32)
            self.gcodes = z(max(n_halo * rb, 16), dt=torch.uint8)
            self.gmeta = z(nh, 2)


class Trainer:
    def __init__(self, w: configs.Workload, device="cuda:0", eps0=None, lr=0.01, adaptive=True,
                 eps_params=None, qscheme=None, bits=None, norm=None, commit=B.COMMIT_CUR,
                 train_fraction=0.6, signal=0.15, graph=None, keep_inputs=False, gen_device="cpu", streams=1):
        """eps0: starting threshold (default: the workload's). adaptive=False keeps it fixed.
        Messages are differences (Alg. 2) in both directions. gen_device: where the seeded inputs
        (graph, partitions, labels, features) are generated; the large workloads take minutes on
        the host and seconds on the GPU (same graph and labels; normal draws agree to rounding)."""
        assert w.dtype == "f32", "the trainer steps fp32 workloads"
        self.w, self.device, self.lr, self.adaptive = w, device, lr, adaptive
        self.eps = float(w.eps if eps0 is None else eps0)
        self.eps_params = eps_params
        self.mean_acc = 0.0
        self.t = 0
        bits = w.bits if bits is None else bits
        qs = _QS[w.qscheme if qscheme is None else qscheme]
        norm = _NORM[w.norm if norm is None else norm]
        self.bits, self.qs = bits, qs
        g = graph if graph is not None else configs.build_graph(w, device=gen_device)
        gd = g.lo.device
        masks = configs.owner_masks(w, g)
        parts = [graphs.extract_partition(g, m) for m in masks]
        self.parts = parts
        p = len(parts)
        dims = w.layers()
        L = len(dims)
        classes = dims[-1][1]
        self.p, self.L, self.classes, self.n = p, L, classes, g.n

        # --- the task (inputs) ---
        y = labelgen.planted_labels(g, classes, w.seed)
        x0 = labelgen.planted_features(y, dims[0][0], w.seed, signal)
        tm = labelgen.train_mask(g.n, w.seed, train_fraction, device=gd)
        self.n_train = int(tm.sum().item())
        self.inputs = dict(graph=g, x0=x0.cpu(), labels=y.cpu(), train=tm.cpu()) if keep_inputs else None

        # --- row numbering ---
        rows = [P.n_loc + P.n_halo for P in parts]
        base = [0]
        off = [0]
        for P, r in zip(parts, rows):
            base.append(base[-1] + r)
            off.append(off[-1] + P.n_loc)
        self.base, self.off, self.rows_total = base, off, base[-1]
        assert self.rows_total < 2 ** 31 and off[-1] == g.n
        tall_of = torch.empty(g.n, dtype=torch.int64, device=gd)   # vertex -> its owner's row in the tall matrices
        slot_of = torch.empty(g.n, dtype=torch.int64, device=gd)   # vertex -> row in owner order
        for j, P in enumerate(parts):
            ar = torch.arange(P.n_loc, dtype=torch.int64, device=gd)
            tall_of[P.owned] = base[j] + ar
            slot_of[P.owned] = off[j] + ar
        dev = device
        self.tall_map = [tall_of[P.halo].to(torch.int32).to(dev) for P in parts]
        self.slot_map = [slot_of[P.halo].to(torch.int32).to(dev) for P in parts]
        self.vertex_of_slot = torch.cat([P.owned for P in parts]).cpu()

        # --- device state ---
        z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=dev)
        self.A = [DeviceCsr(P.n_loc, P.n_loc + P.n_halo, P.rowptr, P.colidx, P.vals, dev) for P in parts]
        self.At = [DeviceCsr(P.n_loc + P.n_halo, P.n_loc, P.t_rowptr, P.t_colidx, P.t_vals, dev) for P in parts]
        self.X = [z(self.rows_total, f) for f, _ in dims]
        self.dX = [None] + [z(self.rows_total, f) for f, _ in dims[1:]]
        self.S = [None] + [z(g.n, f) for f, _ in dims[1:]]
        self.logits = z(g.n, classes)
        self.dlogits = z(g.n, classes)
        for j, P in enumerate(parts):
            self.X[0][base[j]:base[j] + P.n_loc] = x0[P.owned].to(dev)
        vos = self.vertex_of_slot.to(gd)
        lab = torch.where(tm, y, torch.full_like(y, -1))[vos]
        self.labels = lab.to(torch.int32).to(dev)
        self.labels_all = y[vos].to(torch.int32).to(dev)
        self.W = [features.glorot(w.seed, 70 + l, f, gout).to(dev) for l, (f, gout) in enumerate(dims)]
        self.adam_m = [torch.zeros_like(W) for W in self.W]
        self.adam_v = [torch.zeros_like(W) for W in self.W]
        self.loss_sum = z(1)
        self.counts = z(2, dt=torch.int32)
        self.n_sent = z(2 * L * p, dt=torch.int32)   # [dir][layer][part]
        self.pl: List[List[_PartLayer]] = [
            [_PartLayer(P.n_loc, P.n_halo, f, gout, bits, qs, l > 0, dev) for l, (f, gout) in enumerate(dims)]
            for P in parts]
        nbytes = max(B.cdf_workspace_bytes(max(r, 1), max(max(d) for d in dims), max(P.nnz, 1))
                     for P, r in zip(parts, rows))
        nbytes = max(nbytes, B.cdf_workspace_bytes(g.n, classes, 0))
        self.ws = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        # streams > 1: the partitions' layer steps of one phase (they do not depend on each other) are
        # spread over that many streams of default priority, each with a workspace of its own; small
        # partitions do not fill the chip alone. Results do not depend on the number of streams.
        self.n_streams = max(1, min(int(streams), p))
        self.side = [torch.cuda.Stream(device=dev) for _ in range(self.n_streams)] if self.n_streams > 1 else []
        self.side_ws = [torch.zeros(nbytes, dtype=torch.uint8, device=dev) for _ in self.side]

        # --- argument blocks ---
        es = 4
        nsp = lambda d, l, j: self.n_sent.data_ptr() + 4 * ((d * L + l) * p + j)
        self.fwd_args, self.bwd_args = [], []
        for j, P in enumerate(parts):
            fa, ba = [], []
            for l, (f, gout) in enumerate(dims):
                q = self.pl[j][l]
                last = l == L - 1
                xfull = self.X[l].data_ptr() + es * base[j] * f
                H = (self.logits.data_ptr() + es * off[j] * classes) if last else \
                    (self.X[l + 1].data_ptr() + es * base[j] * gout)
                dH = (self.dlogits.data_ptr() + es * off[j] * classes) if last else \
                    (self.dX[l + 1].data_ptr() + es * base[j] * gout)
                fa.append(B.cdf_layer_fwd_args(
                    ctypes.pointer(self.A[j].struct), P.n_loc, P.n_halo, f, gout, B.F32, 0 if last else 1, xfull,
                    q.halo_fresh.data_ptr(), q.cache_sent.data_ptr(), self.W[l].data_ptr(), self.eps, norm, bits, qs,
                    commit, 1, q.M.data_ptr(), None, H, q.mask.data_ptr(), q.idx.data_ptr(), nsp(0, l, j),
                    q.codes.data_ptr(), q.meta.data_ptr()))
                if l > 0:
                    ba.append(B.cdf_layer_bwd_args(
                        ctypes.pointer(self.At[j].struct), P.n_loc, P.n_halo, f, gout, B.F32, 0 if last else 1, 1, dH,
                        H, q.M.data_ptr(), self.W[l].data_ptr(), q.dW.data_ptr(), q.dM.data_ptr(),
                        self.dX[l].data_ptr() + es * base[j] * f, q.gcache_sent.data_ptr(), self.eps, norm, bits, qs,
                        commit, 1, q.gmask.data_ptr(), q.gidx.data_ptr(), nsp(1, l, j), q.gcodes.data_ptr(),
                        q.gmeta.data_ptr()))
                else:
                    ba.append(B.cdf_layer_bwd_args(
                        None, P.n_loc, P.n_halo, f, gout, B.F32, 0 if last else 1, 0, dH, H, q.M.data_ptr(),
                        self.W[l].data_ptr(), q.dW.data_ptr(), None, None, None, self.eps, norm, bits, qs, commit, 1,
                        None, None, None, None, None))
            self.fwd_args.append(fa)
            self.bwd_args.append(ba)
        self.rows_fwd = sum(P.n_halo for P in parts) * L
        self.rows_bwd = sum(P.n_halo for P in parts) * (L - 1)
        self.history: List[EpochStats] = []

    # -- one epoch -------------------------------------------------------------------------
    def forward(self) -> None:
        for l in range(self.L):
            for j, P in enumerate(self.parts):
                if P.n_halo:
                    B.cdf_gather_rows(self.X[l], self.tall_map[j], self.pl[j][l].halo_fresh)
            self._per_partition(lambda j, ws, l=l: self._fwd_one(j, l, ws))

    def _fwd_one(self, j, l, ws):
        a = self.fwd_args[j][l]
        a.eps = self.eps
        B.cdf_gcn_layer_fwd(a, ws)

    def _bwd_one(self, j, l, ws):
        a = self.bwd_args[j][l]
        a.eps = self.eps
        B.cdf_gcn_layer_bwd(a, ws)

    def _per_partition(self, fn) -> None:
        """fn(j, workspace) for every partition: in turn on the current stream, or fanned out over the
        side streams (fork after everything queued so far, join before anything queued afterwards)."""
        if not self.side:
            for j in range(self.p):
                fn(j, self.ws)
            return
        main = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(main)
        for k, st in enumerate(self.side):
            st.wait_event(fork)
            with torch.cuda.stream(st):
                for j in range(k, self.p, self.n_streams):
                    fn(j, self.side_ws[k])
            done = torch.cuda.Event()
            done.record(st)
            main.wait_event(done)

    def loss(self) -> None:
        B.cdf_softmax_xent(self.logits, self.labels, 1.0 / max(self.n_train, 1), self.dlogits, self.loss_sum,
                           self.counts, self.ws)

    def backward(self) -> None:
        for l in reversed(range(self.L)):
            self._per_partition(lambda j, ws, l=l: self._bwd_one(j, l, ws))
            for j in range(1, self.p):                       # sum of the partitions' parameter gradients
                B.cdf_accumulate(self.pl[0][l].dW, self.pl[j][l].dW)
            if l == 0:
                continue
            for j, P in enumerate(self.parts):               # gradient messages, reader -> owner
                if not P.n_halo:
                    continue
                q = self.pl[j][l]
                ns = self.n_sent[(self.L + l) * self.p + j:(self.L + l) * self.p + j + 1]
                B.cdf_map_index(q.gidx, ns, self.slot_map[j], q.gidx_owner)
                B.cdf_dequantize(q.gcodes, q.gmeta, q.gidx_owner, ns, P.n_halo, self.bits, self.qs, self.S[l], True)
            for j, P in enumerate(self.parts):               # owner: own part + what the readers sent
                if P.n_loc:
                    B.cdf_accumulate(self.dX[l][self.base[j]:self.base[j] + P.n_loc],
                                     self.S[l][self.off[j]:self.off[j] + P.n_loc])

    def update(self) -> None:
        self.t += 1
        for l in range(self.L):
            B.cdf_adam_step(self.W[l], self.pl[0][l].dW, self.adam_m[l], self.adam_v[l], self.lr, self.t)

    def epoch(self) -> EpochStats:
        eps = self.eps
        self.forward()
        self.loss()
        self.backward()
        self.update()
        sent = self.n_sent.cpu().view(2, self.L, self.p)     # one transfer: the controller runs on the host
        counts = self.counts.tolist()
        loss = float(self.loss_sum.item()) / max(counts[1], 1)
        acc = counts[0] / max(counts[1], 1)
        if self.adaptive:
            self.eps, self.mean_acc = B.cdf_eps_update(self.eps, acc, self.mean_acc, self.eps_params)
        else:
            _, self.mean_acc = B.cdf_eps_update(self.eps, acc, self.mean_acc, self.eps_params)
        nbytes = 0
        for j in range(self.p):
            for l in range(self.L):
                per = self.pl[j][l].row_bytes + 8 + 4
                nbytes += int(sent[0, l, j]) * per + (int(sent[1, l, j]) * per if l else 0)
        st = EpochStats(len(self.history), eps, loss, acc, self.mean_acc, int(sent[0].sum()), int(sent[1, 1:].sum()),
                        self.rows_fwd, self.rows_bwd, nbytes)
        self.history.append(st)
        return st

    def accuracy_all(self) -> float:
        """Accuracy of the current logits over every vertex (train and held-out rows alike)."""
        scratch = torch.empty_like(self.dlogits)
        ls = torch.zeros(1, device=self.device)
        cn = torch.zeros(2, dtype=torch.int32, device=self.device)
        B.cdf_softmax_xent(self.logits, self.labels_all, 0.0, scratch, ls, cn, self.ws)
        c = cn.tolist()
        return c[0] / max(c[1], 1)
