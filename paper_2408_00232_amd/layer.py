"""Device-memory holders for one partition and one layer: they allocate torch
tensors and fill the C argument blocks. No arithmetic happens here."""
import ctypes

import torch

from . import binding as B


class DeviceCsr:
    """CSR arrays on the device plus the host struct that points at them (and, by default, the
    work-split table of the aggregation, built once here)."""

    def __init__(self, n_rows, n_cols, rowptr, colidx, vals, device="cuda:0", plan=True):
        self.rowptr = rowptr.to(device=device, dtype=torch.int64).contiguous()
        self.colidx = colidx.to(device=device, dtype=torch.int32).contiguous()
        self.vals = vals.to(device=device, dtype=torch.float32).contiguous()
        self.n_rows, self.n_cols, self.nnz = n_rows, n_cols, int(self.colidx.numel())
        self.struct = B.make_csr(n_rows, n_cols, self.rowptr, self.colidx, self.vals)
        self.plan = None
        if plan and self.rowptr.is_cuda:
            self.plan = torch.zeros(max(B.cdf_spmm_plan_bytes(self.nnz) // 4, 1), dtype=torch.int32, device=device)
            B.cdf_spmm_plan(self.struct, self.plan)


class LayerBuffers:
    """All device buffers of one layer (f_in -> f_out) on one partition."""

    def __init__(self, A: DeviceCsr, At: DeviceCsr, n_loc, n_halo, f_in, f_out, dtype=torch.float32,
                 bits=8, qs=B.Q_MINMAX, device="cuda:0", need_dx=True, keep_z=True):
        self.A, self.At = A, At
        self.n_loc, self.n_halo, self.f_in, self.f_out = n_loc, n_halo, f_in, f_out
        self.dtype, self.bits, self.qs, self.device, self.need_dx = dtype, bits, qs, device, need_dx
        z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=device)
        self.xfull = z(n_loc + n_halo, f_in, dt=dtype)
        self.halo_fresh = z(n_halo, f_in, dt=dtype)
        self.cache_sent = z(n_halo, f_in, dt=dtype)
        self.W = z(f_in, f_out)
        self.M = z(n_loc, f_in, dt=dtype)
        self.Z = z(n_loc, f_out) if keep_z else None
        self.H = z(n_loc, f_out)
        rb = B.cdf_code_row_bytes(f_in, bits, qs)
        self.row_bytes = rb
        self.mask = z(max(n_halo, 1), dt=torch.uint8)
        self.idx = z(max(n_halo, 1), dt=torch.int32)
        self.n_sent = z(1, dt=torch.int32)
        self.codes = z(max(n_halo * rb, 16), dt=torch.uint8)
        self.meta = z(max(n_halo, 1), 2)
        # backward
        self.dH = z(n_loc, f_out)
        self.dW = z(f_in, f_out)
        if need_dx:
            self.dM = z(n_loc, f_in, dt=dtype)
            self.dxfull = z(n_loc + n_halo, f_in, dt=dtype)
            self.gcache_sent = z(n_halo, f_in, dt=dtype)
            self.gmask = z(max(n_halo, 1), dt=torch.uint8)
            self.gidx = z(max(n_halo, 1), dt=torch.int32)
            self.gn_sent = z(1, dt=torch.int32)
            self.gcodes = z(max(n_halo * rb, 16), dt=torch.uint8)
            self.gmeta = z(max(n_halo, 1), 2)
        else:
            self.dM = self.dxfull = self.gcache_sent = None
            self.gmask = self.gidx = self.gn_sent = self.gcodes = self.gmeta = None

    def workspace_bytes(self) -> int:
        rows = max(self.n_loc + self.n_halo, 1)
        return B.cdf_workspace_bytes(rows, max(self.f_in, self.f_out), max(self.A.nnz, 1))

    def fwd_args(self, eps, norm=B.NORM_LINF, commit=B.COMMIT_CUR, delta=True, relu=True) -> B.cdf_layer_fwd_args:
        p = lambda t: None if t is None else t.data_ptr()
        return B.cdf_layer_fwd_args(
            ctypes.pointer(self.A.struct), self.n_loc, self.n_halo, self.f_in, self.f_out, B.dtype_of(self.xfull),
            1 if relu else 0, p(self.xfull), p(self.halo_fresh), p(self.cache_sent), p(self.W), eps, norm, self.bits,
            self.qs, commit, 1 if delta else 0, p(self.M), p(self.Z), p(self.H), p(self.mask), p(self.idx),
            p(self.n_sent), p(self.codes), p(self.meta))

    def bwd_args(self, eps, norm=B.NORM_LINF, commit=B.COMMIT_CUR, delta=True, relu=True) -> B.cdf_layer_bwd_args:
        p = lambda t: None if t is None else t.data_ptr()
        zs = self.Z if self.Z is not None else self.H
        return B.cdf_layer_bwd_args(
            ctypes.pointer(self.At.struct) if self.At is not None else None, self.n_loc, self.n_halo, self.f_in,
            self.f_out, B.dtype_of(self.M), 1 if relu else 0, 1 if self.need_dx else 0, p(self.dH), p(zs), p(self.M),
            p(self.W), p(self.dW), p(self.dM), p(self.dxfull), p(self.gcache_sent), eps, norm, self.bits, self.qs,
            commit, 1 if delta else 0, p(self.gmask), p(self.gidx), p(self.gn_sent), p(self.gcodes), p(self.gmeta))


class TfLayerBuffers:
    """Device buffers of one transform-first layer (fp32): the rows that cross the partition
    boundary are rows of T = X W, f_out wide."""

    def __init__(self, A: DeviceCsr, At: DeviceCsr, n_loc, n_halo, f_in, f_out, bits=8, qs=B.Q_MINMAX,
                 device="cuda:0", need_dx=True, keep_z=True):
        self.A, self.At = A, At
        self.n_loc, self.n_halo, self.f_in, self.f_out = n_loc, n_halo, f_in, f_out
        self.bits, self.qs, self.device, self.need_dx = bits, qs, device, need_dx
        z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=device)
        self.x_local = z(n_loc, f_in)
        self.W = z(f_in, f_out)
        self.tfull = z(n_loc + n_halo, f_out)
        self.halo_fresh = z(n_halo, f_out)
        self.cache_sent = z(n_halo, f_out)
        self.Z = z(n_loc, f_out) if keep_z else None
        self.H = z(n_loc, f_out)
        rb = B.cdf_code_row_bytes(f_out, bits, qs)
        self.row_bytes = rb
        self.mask = z(max(n_halo, 1), dt=torch.uint8)
        self.idx = z(max(n_halo, 1), dt=torch.int32)
        self.n_sent = z(1, dt=torch.int32)
        self.codes = z(max(n_halo * rb, 16), dt=torch.uint8)
        self.meta = z(max(n_halo, 1), 2)
        self.dH = z(n_loc, f_out)
        self.dZ = z(n_loc, f_out)
        self.dtfull = z(n_loc + n_halo, f_out)
        self.dW = z(f_in, f_out)
        self.dx_local = z(n_loc, f_in) if need_dx else None
        self.gcache_sent = z(n_halo, f_out)
        self.gmask = z(max(n_halo, 1), dt=torch.uint8)
        self.gidx = z(max(n_halo, 1), dt=torch.int32)
        self.gn_sent = z(1, dt=torch.int32)
        self.gcodes = z(max(n_halo * rb, 16), dt=torch.uint8)
        self.gmeta = z(max(n_halo, 1), 2)

    def workspace_bytes(self) -> int:
        rows = max(self.n_loc + self.n_halo, 1)
        return B.cdf_workspace_bytes(rows, max(self.f_in, self.f_out), max(self.A.nnz, 1))

    def fwd_args(self, eps, norm=B.NORM_LINF, commit=B.COMMIT_CUR, delta=True, relu=True):
        p = lambda t: None if t is None else t.data_ptr()
        return B.cdf_layer_tf_fwd_args(
            ctypes.pointer(self.A.struct), self.n_loc, self.n_halo, self.f_in, self.f_out, 1 if relu else 0,
            p(self.x_local), p(self.W), p(self.tfull), p(self.halo_fresh), p(self.cache_sent), eps, norm, self.bits,
            self.qs, commit, 1 if delta else 0, p(self.Z), p(self.H), p(self.mask), p(self.idx), p(self.n_sent),
            p(self.codes), p(self.meta))

    def bwd_args(self, eps, norm=B.NORM_LINF, commit=B.COMMIT_CUR, delta=True, relu=True):
        p = lambda t: None if t is None else t.data_ptr()
        zs = self.Z if self.Z is not None else self.H
        return B.cdf_layer_tf_bwd_args(
            ctypes.pointer(self.At.struct), self.n_loc, self.n_halo, self.f_in, self.f_out, 1 if relu else 0,
            p(self.dH), p(zs), p(self.x_local), p(self.W), p(self.dZ), p(self.dtfull), p(self.dW), p(self.dx_local),
            p(self.gcache_sent), eps, norm, self.bits, self.qs, commit, 1 if delta else 0, p(self.gmask),
            p(self.gidx), p(self.gn_sent), p(self.gcodes), p(self.gmeta))
