"""TEST INFRASTRUCTURE ONLY - the slow reference of the training loop (Alg. 1 with Alg. 2,
Sec. 5 and the Sec. 4.1 controller): all partitions of a graph stepped one after another on the
host, every step through the functions of this package, messages handed over as plain array
copies. Only tests, the smoke check and the benchmark's CPU leg may use it.

Pinned by tests/test_oracle_pins.py: with eps = 0 and unquantised messages the loop must reproduce
full-graph GCN training written with a dense normalised adjacency.
"""
import numpy as np

from . import (COMMIT_CUR, EPS_DEFAULTS, NORM_LINF, Q_MINMAX, adam_step, dequantize, eps_update, layer_bwd,
               layer_fwd, row_bytes, softmax_xent)


class Part:
    """One partition: CSR of its adjacency rows and of the transpose, global ids of owned and halo rows."""

    def __init__(self, n_loc, n_halo, owned, halo, A, At):
        self.n_loc, self.n_halo = int(n_loc), int(n_halo)
        self.owned, self.halo = np.asarray(owned, np.int64), np.asarray(halo, np.int64)
        self.A, self.At = A, At


class Trainer:
    def __init__(self, parts, dims, x0, labels, train, W, eps, lr=0.01, adaptive=True, eps_params=EPS_DEFAULTS,
                 swap=False, norm=NORM_LINF, bits=8, qs=Q_MINMAX, commit=COMMIT_CUR):
        """parts: list of Part; dims: [(f_in, f_out), ...]; x0 [n, f0] fp32 by vertex id; labels int [n];
        train bool [n]; W: list of fp32 [f_in, f_out] (copied)."""
        self.parts, self.dims, self.L = parts, dims, len(dims)
        self.n = x0.shape[0]
        self.labels = np.where(train, labels, -1).astype(np.int32)
        self.n_train = int(train.sum())
        self.W = [np.array(w, np.float32, order="C") for w in W]
        self.m = [np.zeros_like(w) for w in self.W]
        self.v = [np.zeros_like(w) for w in self.W]
        self.eps, self.lr, self.adaptive, self.eps_params, self.swap = float(eps), lr, adaptive, eps_params, swap
        self.kw = dict(norm=norm, bits=bits, qs=qs, commit=commit, delta=True)
        self.bits, self.qs = bits, qs
        self.mean_acc, self.t = 0.0, 0
        f32 = np.float32
        # per partition and layer: the rows it aggregates with (local rows first), both caches
        self.xfull = [[np.zeros((P.n_loc + P.n_halo, f), f32) for f, _ in dims] for P in parts]
        self.cache = [[np.zeros((P.n_halo, f), f32) for f, _ in dims] for P in parts]
        self.gcache = [[np.zeros((P.n_halo, f), f32) for f, _ in dims] for P in parts]
        # owner-side totals of the gradient messages, by vertex id
        self.S = [np.zeros((self.n, f), f32) for f, _ in dims]
        for P, xf in zip(parts, self.xfull):
            xf[0][:P.n_loc] = x0[P.owned]
        self.history = []

    def epoch(self):
        parts, dims, L, eps = self.parts, self.dims, self.L, self.eps
        f32 = np.float32
        H = np.zeros((self.n, dims[0][0]), f32)           # current rows of every vertex, by id
        for P, xf in zip(parts, self.xfull):
            H[P.owned] = xf[0][:P.n_loc]
        saved = [[None] * L for _ in parts]
        sent_f = sent_b = nbytes = 0
        for l, (f, g) in enumerate(dims):
            Hn = np.zeros((self.n, g), f32)
            for j, P in enumerate(parts):
                xf = self.xfull[j][l]
                if l:
                    xf[:P.n_loc] = H[P.owned]
                fresh = np.ascontiguousarray(H[P.halo])   # what the owners hold now
                r = layer_fwd(P.A, P.n_loc, P.n_halo, xf, fresh, self.cache[j][l], self.W[l], eps,
                              relu=l + 1 < L, **self.kw)
                saved[j][l] = r
                Hn[P.owned] = r["H"]
                sent_f += len(r["idx"])
                nbytes += len(r["idx"]) * (row_bytes(f, self.bits, self.qs) + 12)
            H = Hn
        loss, dlog, ncor, nlab = softmax_xent(H, self.labels, 1.0 / max(self.n_train, 1))
        dH = dlog
        dW = [None] * L
        for l in reversed(range(L)):
            f, g = dims[l]
            dXown = np.zeros((self.n, f), f32)
            tot = None
            outs = []
            for j, P in enumerate(parts):
                r = saved[j][l]
                o = layer_bwd(P.At, P.n_loc, P.n_halo, r["M"], r["Z"], np.ascontiguousarray(dH[P.owned]), self.W[l],
                              self.gcache[j][l], eps, relu=l + 1 < L, need_dx=l > 0, **self.kw)
                outs.append(o)
                tot = o["dW"].copy() if tot is None else (tot + o["dW"]).astype(f32)
            dW[l] = tot
            if l == 0:
                break
            for j, P in enumerate(parts):                 # readers -> owners
                o = outs[j]
                gl = P.halo[o["idx"]].astype(np.int32)
                dequantize(o["codes"], o["meta"], gl, self.S[l], self.bits, self.qs, accumulate=True)
                sent_b += len(o["idx"])
                nbytes += len(o["idx"]) * (row_bytes(f, self.bits, self.qs) + 12)
            for j, P in enumerate(parts):
                dXown[P.owned] = (outs[j]["dxfull"][:P.n_loc] + self.S[l][P.owned]).astype(f32)
            dH = dXown
        self.t += 1
        for l in range(L):
            adam_step(self.W[l], np.ascontiguousarray(dW[l], f32), self.m[l], self.v[l], self.lr, self.t)
        acc = ncor / max(nlab, 1)
        new_eps, self.mean_acc = eps_update(self.eps, acc, self.mean_acc, self.eps_params, self.swap)
        if self.adaptive:
            self.eps = new_eps
        st = dict(epoch=len(self.history), eps=eps, loss=loss / max(nlab, 1), train_acc=acc, mean_acc=self.mean_acc,
                  sent_fwd=sent_f, sent_bwd=sent_b, message_bytes=nbytes, logits=H, dW=dW)
        self.history.append(st)
        return st
