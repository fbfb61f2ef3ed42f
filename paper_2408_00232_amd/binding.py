"""Thin ctypes binding of libcdf.so: argument marshalling only.

Functions carry the names of the C entry points (include/cdf.h). Tensors are
torch CUDA tensors used as device memory; every step runs in the library's
kernels on the current torch stream. There is no fallback: if the library is
missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# CDF_LIB_SANITIZE=1 selects the build whose host code carries AddressSanitizer / UBSan instrumentation
# (paper_2408_00232_amd.build.build_lib(sanitize_host=True)); used by the CPU test suite only
LIB_PATH = os.path.join(_HERE, "libcdf_san.so" if os.environ.get("CDF_LIB_SANITIZE", "") not in ("", "0")
                        else "libcdf.so")

F32, BF16 = 0, 1
NORM_LINF, NORM_L2 = 0, 1
Q_MINMAX, Q_SYMMETRIC, Q_NONE = 0, 1, 2
COMMIT_NONE, COMMIT_CUR, COMMIT_DEQ = 0, 1, 2
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4

EXPORTS = ["cdf_profile_copy", "cdf_profile_enable", "cdf_profile_kernels", "cdf_profile_kernel_name", "cdf_profile_read", "cdf_profile_read_all",
           "cdf_last_error", "cdf_workspace_bytes", "cdf_code_row_bytes", "cdf_max_message_dim", "cdf_cache_filter", "cdf_cache_filter_static", "cdf_quantize", "cdf_cache_filter_quantize", "cdf_set_message_wait_limit",
           "cdf_dequantize", "cdf_spmm_plan_bytes", "cdf_spmm_plan", "cdf_spmm_fwd", "cdf_spmm_bwd", "cdf_spmm_dense_fwd", "cdf_dense_fwd", "cdf_dense_bwd",
           "cdf_gcn_layer_fwd", "cdf_gcn_layer_bwd", "cdf_gcn_layer_tf_fwd", "cdf_gcn_layer_tf_bwd",
           "cdf_softmax_xent", "cdf_adam_step", "cdf_accumulate", "cdf_gather_rows", "cdf_map_index",
           "cdf_mark_rows", "cdf_active_rows", "cdf_relu_fwd",
           "cdf_eps_update", "cdf_ebv_partition", "cdf_cut_statistics"]


class CdfError(RuntimeError):
    def __init__(self, fn, code, text):
        super().__init__(f"{fn} failed with status {code}: {text}")
        self.code = code


class cdf_csr(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int32), ("n_cols", ctypes.c_int32), ("nnz", ctypes.c_int64),
                ("rowptr", ctypes.c_void_p), ("colidx", ctypes.c_void_p), ("vals", ctypes.c_void_p),
                ("plan", ctypes.c_void_p)]


class cdf_layer_fwd_args(ctypes.Structure):
    _fields_ = [("A", ctypes.POINTER(cdf_csr)),
                ("n_loc", ctypes.c_int32), ("n_halo", ctypes.c_int32), ("f_in", ctypes.c_int32),
                ("f_out", ctypes.c_int32), ("dt", ctypes.c_int), ("relu", ctypes.c_int),
                ("xfull", ctypes.c_void_p), ("halo_fresh", ctypes.c_void_p), ("cache_sent", ctypes.c_void_p),
                ("W", ctypes.c_void_p), ("eps", ctypes.c_float), ("norm", ctypes.c_int), ("bits", ctypes.c_int),
                ("qs", ctypes.c_int), ("commit", ctypes.c_int), ("delta", ctypes.c_int),
                ("M", ctypes.c_void_p), ("Z", ctypes.c_void_p), ("H", ctypes.c_void_p),
                ("mask", ctypes.c_void_p), ("idx", ctypes.c_void_p), ("n_sent", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("meta", ctypes.c_void_p)]


class cdf_layer_bwd_args(ctypes.Structure):
    _fields_ = [("At", ctypes.POINTER(cdf_csr)),
                ("n_loc", ctypes.c_int32), ("n_halo", ctypes.c_int32), ("f_in", ctypes.c_int32),
                ("f_out", ctypes.c_int32), ("dt", ctypes.c_int), ("relu", ctypes.c_int), ("need_dx", ctypes.c_int),
                ("dH", ctypes.c_void_p), ("Zs", ctypes.c_void_p), ("M", ctypes.c_void_p), ("W", ctypes.c_void_p),
                ("dW", ctypes.c_void_p), ("dM", ctypes.c_void_p), ("dxfull", ctypes.c_void_p),
                ("gcache_sent", ctypes.c_void_p), ("eps", ctypes.c_float), ("norm", ctypes.c_int),
                ("bits", ctypes.c_int), ("qs", ctypes.c_int), ("commit", ctypes.c_int), ("delta", ctypes.c_int),
                ("mask", ctypes.c_void_p), ("idx", ctypes.c_void_p), ("n_sent", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("meta", ctypes.c_void_p)]


class cdf_layer_tf_fwd_args(ctypes.Structure):
    _fields_ = [("A", ctypes.POINTER(cdf_csr)),
                ("n_loc", ctypes.c_int32), ("n_halo", ctypes.c_int32), ("f_in", ctypes.c_int32),
                ("f_out", ctypes.c_int32), ("relu", ctypes.c_int),
                ("x_local", ctypes.c_void_p), ("W", ctypes.c_void_p), ("tfull", ctypes.c_void_p),
                ("halo_fresh", ctypes.c_void_p), ("cache_sent", ctypes.c_void_p),
                ("eps", ctypes.c_float), ("norm", ctypes.c_int), ("bits", ctypes.c_int),
                ("qs", ctypes.c_int), ("commit", ctypes.c_int), ("delta", ctypes.c_int),
                ("Z", ctypes.c_void_p), ("H", ctypes.c_void_p),
                ("mask", ctypes.c_void_p), ("idx", ctypes.c_void_p), ("n_sent", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("meta", ctypes.c_void_p)]


class cdf_layer_tf_bwd_args(ctypes.Structure):
    _fields_ = [("At", ctypes.POINTER(cdf_csr)),
                ("n_loc", ctypes.c_int32), ("n_halo", ctypes.c_int32), ("f_in", ctypes.c_int32),
                ("f_out", ctypes.c_int32), ("relu", ctypes.c_int),
                ("dH", ctypes.c_void_p), ("Zs", ctypes.c_void_p), ("x_local", ctypes.c_void_p), ("W", ctypes.c_void_p),
                ("dZ", ctypes.c_void_p), ("dtfull", ctypes.c_void_p), ("dW", ctypes.c_void_p),
                ("dx_local", ctypes.c_void_p), ("gcache_sent", ctypes.c_void_p),
                ("eps", ctypes.c_float), ("norm", ctypes.c_int), ("bits", ctypes.c_int),
                ("qs", ctypes.c_int), ("commit", ctypes.c_int), ("delta", ctypes.c_int),
                ("mask", ctypes.c_void_p), ("idx", ctypes.c_void_p), ("n_sent", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("meta", ctypes.c_void_p)]


class cdf_eps_params(ctypes.Structure):
    _fields_ = [("mu1", ctypes.c_float), ("mu2", ctypes.c_float), ("nu1", ctypes.c_float), ("nu2", ctypes.c_float),
                ("xi", ctypes.c_float), ("lambda1", ctypes.c_float), ("lambda2", ctypes.c_float),
                ("swap_conditions", ctypes.c_int)]


_lib = None


def load():
    """Load libcdf.so (built in-tree). Raises if it is absent: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2408_00232_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        lib.cdf_last_error.restype = ctypes.c_char_p
        lib.cdf_workspace_bytes.restype = ctypes.c_size_t
        lib.cdf_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int64]
        lib.cdf_code_row_bytes.restype = ctypes.c_size_t
        lib.cdf_spmm_plan_bytes.restype = ctypes.c_size_t
        lib.cdf_spmm_plan_bytes.argtypes = [ctypes.c_int64]
        lib.cdf_code_row_bytes.argtypes = [ctypes.c_int32, ctypes.c_int, ctypes.c_int]
        lib.cdf_profile_kernel_name.restype = ctypes.c_char_p
        lib.cdf_eps_update.restype = ctypes.c_float
        _lib = lib
    return _lib


def _check(fn, rc):
    if rc != 0:
        raise CdfError(fn, rc, load().cdf_last_error().decode())


def _ptr(t):
    if t is None:
        return ctypes.c_void_p(None)
    assert t.is_cuda, "device tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def dtype_of(t) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def _ld(t) -> int:
    assert t.dim() == 2 and t.stride(1) == 1
    return t.stride(0)


def make_csr(n_rows, n_cols, rowptr, colidx, vals) -> cdf_csr:
    """Host struct of device arrays (the tensors must outlive its use)."""
    assert rowptr.dtype == torch.int64 and colidx.dtype == torch.int32 and vals.dtype == torch.float32
    assert rowptr.numel() == n_rows + 1
    return cdf_csr(n_rows, n_cols, colidx.numel(), rowptr.data_ptr(), colidx.data_ptr(), vals.data_ptr(), None)


def cdf_spmm_plan_bytes(nnz: int) -> int:
    return int(load().cdf_spmm_plan_bytes(nnz))


def cdf_spmm_plan(A: cdf_csr, plan) -> None:
    """Fills `plan` (int32 device tensor of cdf_spmm_plan_bytes(A.nnz) bytes or more) and stores its
    address in A.plan; the tensor must outlive A's use."""
    assert plan.is_cuda and plan.dtype == torch.int32
    rc = load().cdf_spmm_plan(ctypes.byref(A), _ptr(plan), ctypes.c_size_t(plan.numel() * 4), _stream())
    _check("cdf_spmm_plan", rc)
    A.plan = plan.data_ptr()


def cdf_profile_enable(on: bool) -> None:
    _check("cdf_profile_enable", load().cdf_profile_enable(ctypes.c_int(1 if on else 0)))


def cdf_profile_kernels() -> int:
    return int(load().cdf_profile_kernels())


def cdf_profile_kernel_name(kernel: int) -> str:
    return load().cdf_profile_kernel_name(ctypes.c_int(kernel)).decode()


def cdf_profile_read(kernel: int, cap: int = 8192):
    """Durations (ms) of the recorded launches of one kernel, in launch order."""
    buf = (ctypes.c_float * cap)()
    n = load().cdf_profile_read(ctypes.c_int(kernel), buf, ctypes.c_int(cap))
    if n < 0:
        _check("cdf_profile_read", n)
    return [buf[i] for i in range(min(n, cap))]


def cdf_profile_read_all(cap: int = 8192):
    """[(kernel name, ms)] of every recorded launch, in launch order."""
    ids = (ctypes.c_int32 * cap)()
    ms = (ctypes.c_float * cap)()
    n = load().cdf_profile_read_all(ids, ms, ctypes.c_int(cap))
    if n < 0:
        _check("cdf_profile_read_all", n)
    names = [cdf_profile_kernel_name(k) for k in range(cdf_profile_kernels())]
    return [(names[ids[i]], ms[i]) for i in range(min(n, cap))]


def cdf_profile_copy(dst, src) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check("cdf_profile_copy", load().cdf_profile_copy(_ptr(dst), _ptr(src), ctypes.c_size_t(nbytes), _stream()))


def cdf_workspace_bytes(max_rows: int, max_dim: int, max_nnz: int) -> int:
    return int(load().cdf_workspace_bytes(max_rows, max_dim, max_nnz))


def cdf_code_row_bytes(dim: int, bits: int, qs: int) -> int:
    return int(load().cdf_code_row_bytes(dim, bits, qs))


def cdf_max_message_dim(dim: int, ld: int, dt: int) -> int:
    return int(load().cdf_max_message_dim(ctypes.c_int32(dim), ctypes.c_int64(ld), ctypes.c_int(dt)))


def cdf_cache_filter(cur, cached, eps, norm, mask, idx, n_sent, ws):
    rc = load().cdf_cache_filter(_ptr(cur), _ptr(cached), ctypes.c_int32(cur.shape[0]), ctypes.c_int32(cur.shape[1]),
                                 ctypes.c_int64(_ld(cur)), ctypes.c_int(dtype_of(cur)), ctypes.c_float(eps),
                                 ctypes.c_int(norm), _ptr(mask), _ptr(idx), _ptr(n_sent), _ptr(ws),
                                 ctypes.c_size_t(ws.numel() * ws.element_size()), _stream())
    _check("cdf_cache_filter", rc)


def cdf_cache_filter_static(cur, cached, eps, norm, mask, idx, n_sent):
    rc = load().cdf_cache_filter_static(_ptr(cur), _ptr(cached), ctypes.c_int32(cur.shape[0]),
                                        ctypes.c_int32(cur.shape[1]), ctypes.c_int64(_ld(cur)),
                                        ctypes.c_int(dtype_of(cur)), ctypes.c_float(eps), ctypes.c_int(norm),
                                        _ptr(mask), _ptr(idx), _ptr(n_sent), _stream())
    _check("cdf_cache_filter_static", rc)


def cdf_quantize(cur, cached, idx, n_sent, max_sent, bits, qs, commit, delta, codes, meta):
    rc = load().cdf_quantize(_ptr(cur), _ptr(cached), _ptr(idx), _ptr(n_sent), ctypes.c_int32(max_sent),
                             ctypes.c_int32(cur.shape[1]), ctypes.c_int64(_ld(cur)), ctypes.c_int(dtype_of(cur)),
                             ctypes.c_int(bits), ctypes.c_int(qs), ctypes.c_int(commit), ctypes.c_int(1 if delta else 0),
                             _ptr(codes), _ptr(meta), _stream())
    _check("cdf_quantize", rc)


def cdf_cache_filter_quantize(cur, cached, eps, norm, bits, qs, commit, delta, mask, idx, n_sent, codes, meta, ws):
    rc = load().cdf_cache_filter_quantize(_ptr(cur), _ptr(cached), ctypes.c_int32(cur.shape[0]), ctypes.c_int32(cur.shape[1]),
                                          ctypes.c_int64(_ld(cur)), ctypes.c_int(dtype_of(cur)), ctypes.c_float(eps),
                                          ctypes.c_int(norm), ctypes.c_int(bits), ctypes.c_int(qs), ctypes.c_int(commit),
                                          ctypes.c_int(1 if delta else 0), _ptr(mask), _ptr(idx), _ptr(n_sent), _ptr(codes),
                                          _ptr(meta), _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()), _stream())
    _check("cdf_cache_filter_quantize", rc)


def cdf_set_message_wait_limit(polls: int) -> None:
    _check("cdf_set_message_wait_limit", load().cdf_set_message_wait_limit(ctypes.c_int(polls)))


def cdf_dequantize(codes, meta, idx, n_sent, max_sent, bits, qs, dst, accumulate):
    rc = load().cdf_dequantize(_ptr(codes), _ptr(meta), _ptr(idx), _ptr(n_sent), ctypes.c_int32(max_sent),
                               ctypes.c_int32(dst.shape[1]), ctypes.c_int(bits), ctypes.c_int(qs), _ptr(dst),
                               ctypes.c_int64(_ld(dst)), ctypes.c_int(dtype_of(dst)),
                               ctypes.c_int(1 if accumulate else 0), _stream())
    _check("cdf_dequantize", rc)


def _spmm(name, A: cdf_csr, X, Y, ws):
    fn = getattr(load(), name)
    rc = fn(ctypes.byref(A), _ptr(X), ctypes.c_int64(_ld(X)), _ptr(Y), ctypes.c_int64(_ld(Y)),
            ctypes.c_int32(X.shape[1]), ctypes.c_int(dtype_of(X)), _ptr(ws),
            ctypes.c_size_t(ws.numel() * ws.element_size()), _stream())
    _check(name, rc)


def cdf_spmm_fwd(A: cdf_csr, X, Y, ws):
    _spmm("cdf_spmm_fwd", A, X, Y, ws)


def cdf_spmm_bwd(At: cdf_csr, dY, dX, ws):
    _spmm("cdf_spmm_bwd", At, dY, dX, ws)


def cdf_spmm_dense_fwd(A: cdf_csr, X, W, relu, M, Z, H, ws):
    rc = load().cdf_spmm_dense_fwd(ctypes.byref(A), _ptr(X), ctypes.c_int64(_ld(X)), ctypes.c_int(dtype_of(X)), _ptr(W),
                                   ctypes.c_int32(W.shape[0]), ctypes.c_int32(W.shape[1]), ctypes.c_int(1 if relu else 0),
                                   _ptr(M), ctypes.c_int64(_ld(M)), _ptr(Z), _ptr(H), _ptr(ws),
                                   ctypes.c_size_t(ws.numel() * ws.element_size()), _stream())
    _check("cdf_spmm_dense_fwd", rc)


def cdf_dense_fwd(M, W, relu, Z, H):
    rc = load().cdf_dense_fwd(_ptr(M), ctypes.c_int64(_ld(M)), ctypes.c_int(dtype_of(M)), _ptr(W),
                              ctypes.c_int32(M.shape[0]), ctypes.c_int32(W.shape[0]), ctypes.c_int32(W.shape[1]),
                              ctypes.c_int(1 if relu else 0), _ptr(Z), _ptr(H), _stream())
    _check("cdf_dense_fwd", rc)


def cdf_dense_bwd(M, W, Zs, dH, relu, dW, dM, ws):
    rc = load().cdf_dense_bwd(_ptr(M), ctypes.c_int64(_ld(M)), ctypes.c_int(dtype_of(M)), _ptr(W), _ptr(Zs), _ptr(dH),
                              ctypes.c_int32(M.shape[0]), ctypes.c_int32(W.shape[0]), ctypes.c_int32(W.shape[1]),
                              ctypes.c_int(1 if relu else 0), _ptr(dW), _ptr(dM),
                              ctypes.c_int64(_ld(dM) if dM is not None else W.shape[0]), _ptr(ws),
                              ctypes.c_size_t(ws.numel() * ws.element_size()), _stream())
    _check("cdf_dense_bwd", rc)


def cdf_gcn_layer_fwd(args: cdf_layer_fwd_args, ws):
    rc = load().cdf_gcn_layer_fwd(ctypes.byref(args), _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()),
                                  _stream())
    _check("cdf_gcn_layer_fwd", rc)


def cdf_gcn_layer_bwd(args: cdf_layer_bwd_args, ws):
    rc = load().cdf_gcn_layer_bwd(ctypes.byref(args), _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()),
                                  _stream())
    _check("cdf_gcn_layer_bwd", rc)


def cdf_gcn_layer_tf_fwd(args: cdf_layer_tf_fwd_args, ws):
    rc = load().cdf_gcn_layer_tf_fwd(ctypes.byref(args), _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()),
                                     _stream())
    _check("cdf_gcn_layer_tf_fwd", rc)


def cdf_gcn_layer_tf_bwd(args: cdf_layer_tf_bwd_args, ws):
    rc = load().cdf_gcn_layer_tf_bwd(ctypes.byref(args), _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()),
                                     _stream())
    _check("cdf_gcn_layer_tf_bwd", rc)


def cdf_softmax_xent(logits, labels, scale, dlogits, loss_sum, counts, ws):
    rc = load().cdf_softmax_xent(_ptr(logits), _ptr(labels), ctypes.c_int32(logits.shape[0]),
                                 ctypes.c_int32(logits.shape[1]), ctypes.c_float(scale), _ptr(dlogits), _ptr(loss_sum),
                                 _ptr(counts), _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()), _stream())
    _check("cdf_softmax_xent", rc)


def cdf_adam_step(W, dW, m, v, lr, t, beta1=0.9, beta2=0.999, eps=1e-8):
    rc = load().cdf_adam_step(_ptr(W), _ptr(dW), _ptr(m), _ptr(v), ctypes.c_int64(W.numel()), ctypes.c_float(lr),
                              ctypes.c_float(beta1), ctypes.c_float(beta2), ctypes.c_float(eps), ctypes.c_int32(t),
                              _stream())
    _check("cdf_adam_step", rc)


def cdf_accumulate(dst, src):
    assert dst.numel() == src.numel() and dst.is_contiguous() and src.is_contiguous()
    _check("cdf_accumulate", load().cdf_accumulate(_ptr(dst), _ptr(src), ctypes.c_int64(dst.numel()), _stream()))


def cdf_gather_rows(src, idx, dst):
    """dst[r] = src[idx[r]] for r < idx.numel(); 2-D row-major tensors of one element type."""
    assert src.dtype == dst.dtype and src.shape[1] == dst.shape[1] and idx.dtype == torch.int32
    assert dst.shape[0] >= idx.numel()
    rc = load().cdf_gather_rows(_ptr(src), ctypes.c_int64(_ld(src)), _ptr(idx), ctypes.c_int32(idx.numel()),
                                ctypes.c_int32(src.shape[1]), ctypes.c_int(dtype_of(src)), _ptr(dst),
                                ctypes.c_int64(_ld(dst)), _stream())
    _check("cdf_gather_rows", rc)


def cdf_map_index(idx, n_sent, mapping, out):
    assert idx.dtype == mapping.dtype == out.dtype == torch.int32 and out.numel() >= idx.numel()
    rc = load().cdf_map_index(_ptr(idx), _ptr(n_sent), ctypes.c_int32(idx.numel()), _ptr(mapping), _ptr(out), _stream())
    _check("cdf_map_index", rc)


def cdf_mark_rows(idx, n_sent, mapping, offset, flags):
    assert idx.dtype == torch.int32 and flags.dtype == torch.uint8
    rc = load().cdf_mark_rows(_ptr(idx), _ptr(n_sent), ctypes.c_int32(idx.numel()), _ptr(mapping), ctypes.c_int32(offset),
                              _ptr(flags), _stream())
    _check("cdf_mark_rows", rc)


def cdf_active_rows(flags, mapping, mask, idx, n_sent, ws):
    assert mapping.dtype == torch.int32 and flags.dtype == torch.uint8 and mask.numel() >= mapping.numel()
    rc = load().cdf_active_rows(_ptr(flags), _ptr(mapping), ctypes.c_int32(mapping.numel()), _ptr(mask), _ptr(idx),
                                _ptr(n_sent), _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size()), _stream())
    _check("cdf_active_rows", rc)


def cdf_relu_fwd(z, h):
    assert z.dtype == h.dtype == torch.float32 and z.numel() == h.numel() and z.is_contiguous() and h.is_contiguous()
    _check("cdf_relu_fwd", load().cdf_relu_fwd(_ptr(z), _ptr(h), ctypes.c_int64(z.numel()), _stream()))


def cdf_eps_update(eps, acc, mean_acc, params=None):
    """-> (new eps, new mean_acc); params: cdf_eps_params or None for the paper's defaults."""
    mean = ctypes.c_float(mean_acc)
    out = load().cdf_eps_update(ctypes.c_float(eps), ctypes.c_float(acc), ctypes.byref(mean),
                                ctypes.byref(params) if params is not None else None)
    return float(out), float(mean.value)


class cdf_ebv_params(ctypes.Structure):
    _fields_ = [("p", ctypes.c_int32), ("devices_per_host", ctypes.c_int32), ("alpha", ctypes.c_double),
                ("beta", ctypes.c_double), ("gamma", ctypes.c_double), ("sort_edges", ctypes.c_int)]


class cdf_cut_stats(ctypes.Structure):
    _fields_ = [("replication_factor", ctypes.c_double), ("edge_imbalance", ctypes.c_double),
                ("vertex_imbalance", ctypes.c_double), ("max_inner", ctypes.c_int64), ("max_outer", ctypes.c_int64),
                ("replicas_total", ctypes.c_int64)]


def _host_i64(t):
    assert not t.is_cuda and t.dtype == torch.int64 and t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def cdf_ebv_partition(n_vertices, eu, ev, p, devices_per_host=1, alpha=1.0, beta=1.0, gamma=0.1, sort_edges=True):
    """Host tensors eu, ev (int64, one entry per undirected edge) -> int32 [n_edges] device of every edge."""
    part = torch.zeros(eu.numel(), dtype=torch.int32)
    prm = cdf_ebv_params(p, devices_per_host, alpha, beta, gamma, 1 if sort_edges else 0)
    rc = load().cdf_ebv_partition(ctypes.c_int64(n_vertices), ctypes.c_int64(eu.numel()), _host_i64(eu), _host_i64(ev),
                                  ctypes.byref(prm), ctypes.c_void_p(part.data_ptr()))
    _check("cdf_ebv_partition", rc)
    return part


def cdf_cut_statistics(n_vertices, eu, ev, part, p, devices_per_host=1):
    """-> (cdf_cut_stats, master int32 [n_vertices]) for host tensors."""
    assert part.dtype == torch.int32 and not part.is_cuda and part.is_contiguous()
    master = torch.zeros(n_vertices, dtype=torch.int32)
    st = cdf_cut_stats()
    rc = load().cdf_cut_statistics(ctypes.c_int64(n_vertices), ctypes.c_int64(eu.numel()), _host_i64(eu), _host_i64(ev),
                                   ctypes.c_void_p(part.data_ptr()), ctypes.c_int32(p), ctypes.c_int32(devices_per_host),
                                   ctypes.c_void_p(master.data_ptr()), ctypes.byref(st))
    _check("cdf_cut_statistics", rc)
    return st, master
