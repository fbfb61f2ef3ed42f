"""TEST INFRASTRUCTURE ONLY - slow reference of training in the paper's own vertex-cut framing:
every device holds a subgraph with master and mirror replicas (Sec. 3.2), computes partial
pre-activations and partial gradients for all its replicas (Sec. 3.1), and the replicas are
reconciled by Alg. 2 in full: mirrors test their partial value against what they last sent and
send the difference to the master; the master adds incoming differences and its own to the
cached total and marks the vertex active; the totals of active vertices go back to the mirrors.
Composed of this package's routines; messages are array copies.

Pinned by tests/test_oracle_pins.py against dense full-graph training (threshold 0, loss-less
messages) and by the consistency invariant total = sum of the replicas' cached partials.
"""
import numpy as np

from . import (COMMIT_CUR, COMMIT_NONE, EPS_DEFAULTS, NORM_LINF, Q_MINMAX, Q_NONE, adam_step, cache_filter, dense_bwd,
               dense_fwd, dequantize, eps_update, quantize, row_bytes, softmax_xent, spmm)


class Part:
    def __init__(self, n_master, n_mirror, vertices, A, mirror_master_dev, mirror_master_row):
        self.n_master, self.n_mirror = int(n_master), int(n_mirror)
        self.n = self.n_master + self.n_mirror
        self.vertices = np.asarray(vertices, np.int64)
        self.A = A
        self.mdev = np.asarray(mirror_master_dev, np.int64)
        self.mrow = np.asarray(mirror_master_row, np.int64)
        self.index = None     # position of this device in the list, set by the trainer

    def tot_row(self, st, row):
        """The cached total this device holds in local row `row` of exchange state `st`."""
        return st.tot[self.index][row]


class _Sync:
    """Cache state of one exchanged quantity (a layer's partial Z, or a layer's partial gradient)."""

    def __init__(self, parts, dim):
        self.zc = [np.zeros((P.n, dim), np.float32) for P in parts]    # what each replica last contributed
        self.tot = [np.zeros((P.n, dim), np.float32) for P in parts]   # master rows: cached total; mirror rows: its copy


class Trainer:
    def __init__(self, parts, dims, x0, labels, train, W, eps, lr=0.01, adaptive=True, eps_params=EPS_DEFAULTS,
                 swap=False, norm=NORM_LINF, bits=8, qs=Q_MINMAX, qs_scatter=None):
        self.parts, self.dims, self.L = parts, dims, len(dims)
        for i, P in enumerate(parts):
            P.index = i
        self.n = x0.shape[0]
        self.x0 = [np.ascontiguousarray(x0[P.vertices], np.float32) for P in parts]
        lab = np.where(train, labels, -1).astype(np.int32)
        self.lab_all = [np.ascontiguousarray(lab[P.vertices]) for P in parts]             # every replica
        self.lab_master = [np.where(np.arange(P.n) < P.n_master, lab[P.vertices], -1).astype(np.int32) for P in parts]
        self.n_train = int(train.sum())
        self.W = [np.array(w, np.float32, order="C") for w in W]
        self.m = [np.zeros_like(w) for w in self.W]
        self.v = [np.zeros_like(w) for w in self.W]
        self.eps, self.lr, self.adaptive, self.eps_params, self.swap = float(eps), lr, adaptive, eps_params, swap
        self.norm, self.bits, self.qs = norm, bits, qs
        self.qs_scatter = qs if qs_scatter is None else qs_scatter
        self.zs = [_Sync(parts, g) for _, g in dims]                   # forward: partial Z of layer l
        self.ds = [None] + [_Sync(parts, f) for f, _ in dims[1:]]      # backward: partial gradient of layer l's input
        self.mean_acc, self.t = 0.0, 0
        self.history = []
        self.stats = None

    # ---- Alg. 2 -----------------------------------------------------------------------------
    def sync(self, st, part):
        """part[i]: this epoch's partial rows of device i (masters first). Returns the combined rows
        every device works with afterwards (st.tot)."""
        parts, eps = self.parts, self.eps
        dim = part[0].shape[1]
        active = [np.zeros(P.n_master, bool) for P in parts]
        msgs = []
        for i, P in enumerate(parts):                                   # mirrors: test, send difference, commit
            cur, cached = part[i][P.n_master:], st.zc[i][P.n_master:]
            _, idx = cache_filter(cur, cached, eps, self.norm)
            codes, meta = quantize(cur, cached, idx, self.bits, self.qs, COMMIT_CUR, True)
            msgs.append((idx, codes, meta))
            self.stats["gather"] += len(idx)
            self.stats["bytes"] += len(idx) * (row_bytes(dim, self.bits, self.qs) + 12)
        self.stats["mirror_rows"] += sum(P.n_mirror for P in parts)
        for i, P in enumerate(parts):                                   # masters: add the differences received
            idx, codes, meta = msgs[i]
            for j, Q in enumerate(parts):
                sel = P.mdev[idx] == j
                if sel.any():
                    rows = P.mrow[idx][sel].astype(np.int32)
                    dequantize(codes[sel], meta[sel], rows, st.tot[j], self.bits, self.qs, accumulate=True)
                    active[j][rows] = True
        for j, Q in enumerate(parts):                                   # masters: own value
            cur, cached = part[j][:Q.n_master], st.zc[j][:Q.n_master]
            _, idx = cache_filter(cur, cached, eps, self.norm)
            codes, meta = quantize(cur, cached, idx, self.bits, Q_NONE, COMMIT_CUR, True)   # local: exact difference
            dequantize(codes, meta, idx, st.tot[j], self.bits, Q_NONE, accumulate=True)
            active[j][idx] = True
            self.stats["master_updates"] += len(idx)
        for i, P in enumerate(parts):                                   # scatter: totals of active vertices
            if P.n_mirror == 0:
                continue
            on = np.array([active[d][r] for d, r in zip(P.mdev, P.mrow)], bool)
            idx = np.nonzero(on)[0].astype(np.int32)
            fresh = np.stack([st.tot[d][r] for d, r in zip(P.mdev, P.mrow)]).astype(np.float32)
            codes, meta = quantize(fresh, None, idx, self.bits, self.qs_scatter, COMMIT_NONE, False)
            dequantize(codes, meta, idx, st.tot[i][P.n_master:], self.bits, self.qs_scatter, accumulate=False)
            self.stats["scatter"] += len(idx)
            self.stats["bytes"] += len(idx) * (row_bytes(dim, self.bits, self.qs_scatter) + 12)
        return st.tot

    # ---- one epoch (Alg. 1) ---------------------------------------------------------------------
    def epoch(self):
        parts, dims, L = self.parts, self.dims, self.L
        eps = self.eps
        self.stats = dict(gather=0, scatter=0, master_updates=0, mirror_rows=0, bytes=0)
        X = self.x0
        Ms, Zs = [], []
        for l, (f, g) in enumerate(dims):
            M = [spmm(P.A[0], P.A[1], P.A[2], P.n, x) for P, x in zip(parts, X)]
            zpart = [dense_fwd(m, self.W[l], relu=False)[0] for m in M]
            Z = self.sync(self.zs[l], zpart)
            Ms.append(M)
            Zs.append([z.copy() for z in Z])
            X = [np.maximum(z, np.float32(0)) for z in Z] if l + 1 < L else None
        scale = 1.0 / max(self.n_train, 1)
        loss = ncor = nlab = 0
        dH = []
        for i, P in enumerate(parts):
            dH.append(softmax_xent(Zs[-1][i], self.lab_all[i], scale)[1])      # every replica, from its own copy
            ls, _, c, k = softmax_xent(Zs[-1][i], self.lab_master[i], scale)   # counted once, at the master
            loss, ncor, nlab = loss + ls, ncor + c, nlab + k
        dW = [None] * L
        for l in reversed(range(L)):
            tot = None
            dpart = []
            for i, P in enumerate(parts):
                gW, dM = dense_bwd(Ms[l][i], self.W[l], Zs[l][i], dH[i], relu=l + 1 < L, need_dm=l > 0)
                tot = gW.copy() if tot is None else (tot + gW).astype(np.float32)
                if l > 0:
                    dpart.append(spmm(P.A[0], P.A[1], P.A[2], P.n, dM))      # A_i is symmetric
            dW[l] = tot
            if l > 0:
                dH = [d.copy() for d in self.sync(self.ds[l], dpart)]
        self.t += 1
        for l in range(L):
            adam_step(self.W[l], np.ascontiguousarray(dW[l], np.float32), self.m[l], self.v[l], self.lr, self.t)
        acc = ncor / max(nlab, 1)
        new_eps, self.mean_acc = eps_update(self.eps, acc, self.mean_acc, self.eps_params, self.swap)
        if self.adaptive:
            self.eps = new_eps
        logits = np.zeros((self.n, dims[-1][1]), np.float32)
        for P, z in zip(parts, Zs[-1]):
            logits[P.vertices[:P.n_master]] = z[:P.n_master]
        st = dict(epoch=len(self.history), eps=eps, loss=loss / max(nlab, 1), train_acc=acc, mean_acc=self.mean_acc,
                  logits=logits, dW=dW, **self.stats)
        self.history.append(st)
        return st
