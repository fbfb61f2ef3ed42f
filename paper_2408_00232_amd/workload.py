"""Wires a seeded workload (graph partition + dense inputs) into device buffers and C
argument blocks, and steps the whole model through the library: forward over all layers,
then backward over all layers, every layer as a generic one (halo gradients included).
Marshalling only - all arithmetic happens inside libcdf."""
import torch

from cdfgen import bench_inputs, configs

from . import binding as B
from .layer import DeviceCsr, LayerBuffers, TfLayerBuffers

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}
_QS = {"minmax": B.Q_MINMAX, "symmetric": B.Q_SYMMETRIC, "none": B.Q_NONE}
_NORM = {"linf": B.NORM_LINF, "l2": B.NORM_L2}


class Model:
    def __init__(self, w: configs.Workload, device="cuda:0", rho=0.37, phi=0.01, partition=None, order="auto"):
        """order: "aggregate" = every layer computes (A X) W; "auto" = a layer whose output is
        narrower than its input computes A (X W) instead (fp32 workloads only)."""
        self.w, self.device = w, device
        P = partition if partition is not None else configs.build_partition(w, device=device)
        self.P = P
        self.n_loc, self.n_halo, self.nnz = P.n_loc, P.n_halo, P.nnz
        self.A = DeviceCsr(P.n_loc, P.n_loc + P.n_halo, P.rowptr, P.colidx, P.vals, device)
        self.At = DeviceCsr(P.n_loc + P.n_halo, P.n_loc, P.t_rowptr, P.t_colidx, P.t_vals, device)
        dt = _TORCH_DT[w.dtype]
        self.layers, self.inputs, self.fwd, self.bwd, self.tf = [], [], [], [], []
        dims = w.layers()
        for li, (f_in, f_out) in enumerate(dims):
            relu = li + 1 < len(dims)
            tf = order == "auto" and w.dtype == "f32" and f_out < f_in
            self.tf.append(tf)
            if tf:
                L = TfLayerBuffers(self.A, self.At, P.n_loc, P.n_halo, f_in, f_out, bits=w.bits, qs=_QS[w.qscheme],
                                   device=device, need_dx=True, keep_z=False)
                I = bench_inputs.make_layer_inputs(w.seed, li, P.n_loc, P.n_halo, f_in, f_out, rho, phi, device, dt,
                                                   halo_width=f_out)
                L.x_local.copy_(I.x_local)
                I.x_local = None
                L.W.copy_(I.W)
                L.halo_fresh = None
                L.dH = None
                fa, ba = [], []
                for v in range(2):
                    a = L.fwd_args(w.eps, _NORM[w.norm], B.COMMIT_CUR, True, relu)
                    a.halo_fresh = I.fresh[v].data_ptr()
                    fa.append(a)
                    b = L.bwd_args(w.eps, _NORM[w.norm], B.COMMIT_CUR, True, relu)
                    b.dH = I.dH[v].data_ptr()
                    ba.append(b)
                self.layers.append(L)
                self.inputs.append(I)
                self.fwd.append(fa)
                self.bwd.append(ba)
                continue
            L = LayerBuffers(self.A, self.At, P.n_loc, P.n_halo, f_in, f_out, dtype=dt, bits=w.bits,
                             qs=_QS[w.qscheme], device=device, need_dx=True, keep_z=False)
            I = bench_inputs.make_layer_inputs(w.seed, li, P.n_loc, P.n_halo, f_in, f_out, rho, phi, device, dt)
            L.xfull[:P.n_loc] = I.x_local
            I.x_local = None
            L.W.copy_(I.W)
            L.halo_fresh = None   # the two versions below replace the single input buffer
            L.dH = None
            fa, ba = [], []
            for v in range(2):
                a = L.fwd_args(w.eps, _NORM[w.norm], B.COMMIT_CUR, True, relu)
                a.halo_fresh = I.fresh[v].data_ptr()
                fa.append(a)
                b = L.bwd_args(w.eps, _NORM[w.norm], B.COMMIT_CUR, True, relu)
                b.dH = I.dH[v].data_ptr()
                ba.append(b)
            self.layers.append(L)
            self.inputs.append(I)
            self.fwd.append(fa)
            self.bwd.append(ba)
        rows = max(P.n_loc + P.n_halo, 1)
        nbytes = B.cdf_workspace_bytes(rows, max(max(d) for d in dims), max(P.nnz, 1))
        self.ws = torch.zeros(nbytes, dtype=torch.uint8, device=device)

    def capture(self) -> None:
        """Record the step for both input versions as HIP graphs; `step` replays them from then on.
        The step allocates nothing and never synchronises, and the library clears its counters with
        kernels (no memset nodes), so the capture holds kernel launches only. Run a few eager steps
        first: capture records, it does not execute."""
        self.graphs = []
        for v in range(2):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self._launch(v)
            self.graphs.append(g)

    def step(self, t: int) -> None:
        """One pass of the hot path: all layers forward, then all layers backward."""
        if getattr(self, "graphs", None):
            self.graphs[t & 1].replay()
        else:
            self._launch(t & 1)

    def _launch(self, v: int) -> None:
        for li in range(len(self.layers)):
            (B.cdf_gcn_layer_tf_fwd if self.tf[li] else B.cdf_gcn_layer_fwd)(self.fwd[li][v], self.ws)
        for li in reversed(range(len(self.layers))):
            (B.cdf_gcn_layer_tf_bwd if self.tf[li] else B.cdf_gcn_layer_bwd)(self.bwd[li][v], self.ws)

    def step_timed_per_layer(self, t: int):
        """One eager step with an event pair around every layer call: -> ([fwd ms per layer], [bwd ms per layer])."""
        v = t & 1
        ev = lambda: torch.cuda.Event(enable_timing=True)
        n = len(self.layers)
        fe = [(ev(), ev()) for _ in range(n)]
        be = [(ev(), ev()) for _ in range(n)]
        for li in range(n):
            fe[li][0].record()
            (B.cdf_gcn_layer_tf_fwd if self.tf[li] else B.cdf_gcn_layer_fwd)(self.fwd[li][v], self.ws)
            fe[li][1].record()
        for li in reversed(range(n)):
            be[li][0].record()
            (B.cdf_gcn_layer_tf_bwd if self.tf[li] else B.cdf_gcn_layer_bwd)(self.bwd[li][v], self.ws)
            be[li][1].record()
        torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in fe], [a.elapsed_time(b) for a, b in be]

    def spmm_widths(self):
        """Width of the rows each layer's aggregation gathers (f_out where the layer transforms first)."""
        return [g if tf else f for (f, g), tf in zip(self.w.layers(), self.tf)]

    def edges_per_step(self) -> int:
        return self.nnz * len(self.layers)

    def reset_caches(self) -> None:
        """Back to the state before the first step: sender caches, the receiver's halo rows and the
        gradient caches all zero (so the next step sends every non-zero row)."""
        n = self.n_loc
        for L, tf in zip(self.layers, self.tf):
            L.cache_sent.zero_()
            L.gcache_sent.zero_()
            (L.tfull if tf else L.xfull)[n:].zero_()

    def run_epochs(self, epochs: int, eta0: float = 0.2, kappa: float = 0.6):
        """`epochs` steps on drifting inputs from zero caches, the threshold fixed: every epoch the
        owners' halo rows and the upstream gradients are multiplied element-wise by 1 + eta_t u_r g
        (g ~ N(0,1), u_r log-uniform in [0.1, 10] per row, eta_t = eta0 kappa^t), so the updates shrink
        as they do when parameters settle and the cache hit rate rises from 0. The drift is input
        generation (torch, outside the timed region); the step is timed with events.
        -> [{epoch, ms, hit_rate_fwd [per layer], hit_rate_bwd [per layer]}]"""
        import math
        from cdfgen import rng
        dev, h, n = self.device, self.n_halo, self.n_loc
        self.reset_caches()
        gen = torch.Generator(device=dev)
        gen.manual_seed(self.w.seed * 7919 + 1)
        rates = []
        for li in range(len(self.layers)):
            lu_h = rng.uniform(self.w.seed, 500 + li, h, math.log(0.1), math.log(10.0), device=dev, dtype=torch.float64)
            lu_n = rng.uniform(self.w.seed, 600 + li, n, math.log(0.1), math.log(10.0), device=dev, dtype=torch.float64)
            rates.append((torch.exp(lu_h).float().view(-1, 1), torch.exp(lu_n).float().view(-1, 1)))
        out = []
        for t in range(epochs):
            if t > 0:
                eta = eta0 * kappa ** t
                for li in range(len(self.layers)):
                    I = self.inputs[li]
                    for buf, rate in ((I.fresh[0], rates[li][0]), (I.dH[0], rates[li][1])):
                        g = torch.randn(buf.shape, generator=gen, device=dev, dtype=torch.float32)
                        g.mul_(rate * eta).add_(1.0)
                        buf.copy_((buf.float() * g).to(buf.dtype))
                        del g
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            self._launch(0)
            b.record()
            torch.cuda.synchronize()
            out.append({"epoch": t, "ms": a.elapsed_time(b),
                        "hit_rate_fwd": [1.0 - int(L.n_sent.item()) / max(h, 1) for L in self.layers],
                        "hit_rate_bwd": [1.0 - int(L.gn_sent.item()) / max(h, 1) for L in self.layers]})
        return out
