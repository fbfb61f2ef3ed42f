"""Python face of the CPU oracle (test infrastructure only).

The arithmetic lives in cdf_oracle.c; this module compiles it with gcc, loads
it with ctypes, and composes its routines into the forward and backward layer
step in the order the method prescribes. Nothing here imports or is imported
by the GPU library. Arrays are numpy; bf16 data travels as uint16 bit patterns.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cdf_oracle.c")
# CDF_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (the process must then have gcc's libasan preloaded)
_SANITIZE = os.environ.get("CDF_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "libcdf_oracle_san.so" if _SANITIZE else "libcdf_oracle.so")

F32, BF16 = 0, 1
NORM_LINF, NORM_L2 = 0, 1
Q_MINMAX, Q_SYMMETRIC, Q_NONE = 0, 1, 2
COMMIT_NONE, COMMIT_CUR, COMMIT_DEQ = 0, 1, 2

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
               "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        if _SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
        subprocess.check_call(cmd)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_get_threads.restype = ctypes.c_int
    return _lib


def set_threads(n: int) -> None:
    lib().orc_set_threads(ctypes.c_int(n))


def get_threads() -> int:
    return int(lib().orc_get_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dt(a) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"unsupported element type {a.dtype}")


def _rowmajor(a):
    if a.ndim == 2 and a.size == 0:      # no rows (or no columns): any stride does
        return max(a.shape[1], 1)
    assert a.ndim == 2 and a.strides[1] == a.itemsize and a.strides[0] % a.itemsize == 0
    return a.strides[0] // a.itemsize


def row_bytes(dim: int, bits: int, qs: int) -> int:
    return dim * 4 if qs == Q_NONE else (dim * bits + 7) // 8


def cache_filter(cur, cached, eps: float, norm: int = NORM_LINF):
    """-> (mask uint8[R], idx int32[n_sent])"""
    R, F = cur.shape
    assert cached.shape == cur.shape and cached.dtype == cur.dtype
    ldm = _rowmajor(cur)
    assert _rowmajor(cached) == ldm
    mask = np.zeros(R, np.uint8)
    idx = np.zeros(max(R, 1), np.int32)
    n = ctypes.c_int32(0)
    rc = lib().orc_cache_filter(_p(cur), _p(cached), ctypes.c_int32(R), ctypes.c_int32(F),
                                ctypes.c_int64(ldm), ctypes.c_int(_dt(cur)), ctypes.c_float(eps),
                                ctypes.c_int(norm), _p(mask), _p(idx), ctypes.byref(n))
    assert rc == 0, rc
    return mask, idx[:n.value].copy()


def quantize(cur, cached, idx, bits: int = 8, qs: int = Q_MINMAX, commit: int = COMMIT_CUR,
             delta: bool = None):
    """-> (codes uint8[n_sent, row_bytes], meta float32[n_sent, 2]); `cached` is updated in place."""
    R, F = cur.shape
    ldm = _rowmajor(cur)
    if cached is not None:
        assert cached.shape == cur.shape and cached.dtype == cur.dtype and _rowmajor(cached) == ldm
    if delta is None:
        delta = cached is not None
    idx = np.ascontiguousarray(idx, np.int32)
    k = idx.size
    rb = row_bytes(F, bits, qs)
    codes = np.zeros((k, rb), np.uint8)
    meta = np.zeros((k, 2), np.float32)
    rc = lib().orc_quantize(_p(cur), _p(cached), _p(idx), ctypes.c_int32(k), ctypes.c_int32(F),
                            ctypes.c_int64(ldm), ctypes.c_int(_dt(cur)), ctypes.c_int(bits),
                            ctypes.c_int(qs), ctypes.c_int(commit), ctypes.c_int(1 if delta else 0),
                            _p(codes), _p(meta))
    assert rc == 0, rc
    return codes, meta


def dequantize(codes, meta, idx, dst, bits: int = 8, qs: int = Q_MINMAX, accumulate: bool = True):
    """Applies the messages to rows dst[idx[k]] in place."""
    F = dst.shape[1]
    idx = np.ascontiguousarray(idx, np.int32)
    k = idx.size
    codes = np.ascontiguousarray(codes)
    meta = np.ascontiguousarray(meta, np.float32)
    assert codes.size == k * row_bytes(F, bits, qs)
    rc = lib().orc_dequantize(_p(codes), _p(meta), _p(idx), ctypes.c_int32(k), ctypes.c_int32(F),
                              ctypes.c_int(bits), ctypes.c_int(qs), _p(dst), ctypes.c_int64(_rowmajor(dst)),
                              ctypes.c_int(_dt(dst)), ctypes.c_int(1 if accumulate else 0))
    assert rc == 0, rc


def spmm(rowptr, colidx, vals, n_cols: int, X, out_rows=None):
    """Y = A X for a CSR A with n_cols columns; Y has X's element type."""
    n_rows = rowptr.size - 1
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    colidx = np.ascontiguousarray(colidx, np.int32)
    vals = np.ascontiguousarray(vals, np.float32)
    assert X.shape[0] == n_cols
    F = X.shape[1]
    Y = np.zeros((n_rows, F), X.dtype)
    rc = lib().orc_spmm(ctypes.c_int32(n_rows), ctypes.c_int32(n_cols), _p(rowptr), _p(colidx), _p(vals),
                        _p(X), ctypes.c_int64(_rowmajor(X)), _p(Y), ctypes.c_int64(F), ctypes.c_int32(F),
                        ctypes.c_int(_dt(X)))
    assert rc == 0, rc
    return Y


def dense_fwd(M, W, relu: bool):
    """-> (Z, H) fp32"""
    n, f = M.shape
    g = W.shape[1]
    W = np.ascontiguousarray(W, np.float32)
    assert W.shape[0] == f
    Z = np.zeros((n, g), np.float32)
    H = np.zeros((n, g), np.float32)
    rc = lib().orc_dense_fwd(_p(M), ctypes.c_int64(_rowmajor(M)), ctypes.c_int(_dt(M)), _p(W),
                             ctypes.c_int32(n), ctypes.c_int32(f), ctypes.c_int32(g),
                             ctypes.c_int(1 if relu else 0), _p(Z), _p(H))
    assert rc == 0
    return Z, H


def dense_bwd(M, W, Z, dH, relu: bool, need_dm: bool = True):
    """-> (dW fp32 [f,g], dM [n,f] in M's type or None)"""
    n, f = M.shape
    g = W.shape[1]
    W = np.ascontiguousarray(W, np.float32)
    Z = np.ascontiguousarray(Z, np.float32)
    dH = np.ascontiguousarray(dH, np.float32)
    dW = np.zeros((f, g), np.float32)
    dM = np.zeros((n, f), M.dtype) if need_dm else None
    rc = lib().orc_dense_bwd(_p(M), ctypes.c_int64(_rowmajor(M)), ctypes.c_int(_dt(M)), _p(W), _p(Z), _p(dH),
                             ctypes.c_int32(n), ctypes.c_int32(f), ctypes.c_int32(g),
                             ctypes.c_int(1 if relu else 0), _p(dW), _p(dM), ctypes.c_int64(f))
    assert rc == 0
    return dW, dM


# ----------------------------------------------------------------------------
# The layer step, composed in the method's order.
# ----------------------------------------------------------------------------

def layer_fwd(A, n_loc, n_halo, xfull, halo_fresh, cache_sent, W, eps, norm=NORM_LINF, bits=8,
              qs=Q_MINMAX, commit=COMMIT_CUR, relu=True, delta=True):
    """Forward step of one layer on one partition.

    A = (rowptr, colidx, vals) of the n_loc x (n_loc+n_halo) normalised adjacency.
    1. cache test of the owners' fresh halo rows against what they last sent   (Alg. 2)
    2. difference, quantise, commit the sender cache                           (Sec. 5)
    3. recover and add to the halo rows the receiver aggregates with           (Alg. 2)
       (delta=False: messages carry the rows themselves and the receiver replaces)
    4. M = A^ Xfull ; Z = M W ; H = sigma(Z)                                   (Sec. 3.1)
    xfull's halo rows and cache_sent are updated in place.
    """
    mask, idx = cache_filter(halo_fresh, cache_sent, eps, norm)
    codes, meta = quantize(halo_fresh, cache_sent, idx, bits, qs, commit, delta)
    dequantize(codes, meta, idx, xfull[n_loc:], bits, qs, accumulate=delta)
    M = spmm(A[0], A[1], A[2], n_loc + n_halo, xfull)
    Z, H = dense_fwd(M, W, relu)
    return dict(mask=mask, idx=idx, codes=codes, meta=meta, M=M, Z=Z, H=H)


def layer_bwd(At, n_loc, n_halo, M, Z, dH, W, gcache_sent, eps, norm=NORM_LINF, bits=8, qs=Q_MINMAX,
              commit=COMMIT_CUR, relu=True, need_dx=True, delta=True):
    """Backward step of one layer on one partition.

    At = CSR of the transposed adjacency, (n_loc+n_halo) x n_loc.
    1. dZ = dH * sigma'(Z) ; dW = M^T dZ ; dM = dZ W^T                         (Sec. 3.1)
    2. dXfull = A^^T dM : rows [0, n_loc) are local input gradients, rows
       [n_loc, n_loc+n_halo) are partial gradients owed to the halo rows' owners
    3. cache test + quantise of those halo gradient rows (the same mechanism
       as for features)                                                         (Sec. 4.1)
    gcache_sent is updated in place.
    """
    dW, dM = dense_bwd(M, W, Z, dH, relu, need_dm=need_dx)
    out = dict(dW=dW, dM=dM)
    if need_dx:
        dx = spmm(At[0], At[1], At[2], n_loc, dM)
        mask, idx = cache_filter(dx[n_loc:], gcache_sent, eps, norm)
        codes, meta = quantize(dx[n_loc:], gcache_sent, idx, bits, qs, commit, delta)
        out.update(dxfull=dx, mask=mask, idx=idx, codes=codes, meta=meta)
    return out


def layer_tf_fwd(A, n_loc, n_halo, x_local, tfull, halo_fresh, cache_sent, W, eps, norm=NORM_LINF, bits=8,
                 qs=Q_MINMAX, commit=COMMIT_CUR, relu=True, delta=True):
    """Forward step with the transform applied first: Z = A^ (X W) (Sec. 3.1 leaves the order of
    the product A^ H W open). The rows exchanged are rows of T = X W.
    1. tfull[:n_loc] = x_local W
    2. cache test / message / commit on the owners' fresh T rows, recovery into tfull[n_loc:]
    3. Z = A^ tfull ; H = sigma(Z)
    """
    T, _ = dense_fwd(x_local, W, relu=False)
    tfull[:n_loc] = T
    mask, idx = cache_filter(halo_fresh, cache_sent, eps, norm)
    codes, meta = quantize(halo_fresh, cache_sent, idx, bits, qs, commit, delta)
    dequantize(codes, meta, idx, tfull[n_loc:], bits, qs, accumulate=delta)
    Z = spmm(A[0], A[1], A[2], n_loc + n_halo, tfull)
    H = np.maximum(Z, np.float32(0)) if relu else Z.copy()
    return dict(mask=mask, idx=idx, codes=codes, meta=meta, Z=Z, H=H)


def layer_tf_bwd(At, n_loc, n_halo, x_local, Zs, dH, W, gcache_sent, eps, norm=NORM_LINF, bits=8, qs=Q_MINMAX,
                 commit=COMMIT_CUR, relu=True, need_dx=True, delta=True):
    """Backward of the transform-first step.
    1. dZ = dH * sigma'(Zs)
    2. dtfull = A^^T dZ : rows [0, n_loc) = dT of local rows, the rest = halo gradient rows
    3. cache test + message build on the halo gradient rows
    4. dW = x_local^T dT_local ; dx_local = dT_local W^T
    """
    dZ = np.where(Zs > 0, dH, np.float32(0)).astype(np.float32) if relu else np.ascontiguousarray(dH, np.float32)
    dt = spmm(At[0], At[1], At[2], n_loc, dZ)
    mask, idx = cache_filter(dt[n_loc:], gcache_sent, eps, norm)
    codes, meta = quantize(dt[n_loc:], gcache_sent, idx, bits, qs, commit, delta)
    dW, dX = dense_bwd(x_local, W, np.zeros((n_loc, W.shape[1]), np.float32), dt[:n_loc], relu=False,
                       need_dm=need_dx)
    return dict(dZ=dZ, dtfull=dt, mask=mask, idx=idx, codes=codes, meta=meta, dW=dW, dx_local=dX)


# ----------------------------------------------------------------------------
# Training-loop pieces (loss, optimiser, threshold controller)
# ----------------------------------------------------------------------------
EPS_DEFAULTS = (0.001, 0.02, 0.3, 0.001, 0.01, 1.05, 0.9)   # mu1, mu2, nu1, nu2, xi, lambda1, lambda2 (Sec. 4.1)


def softmax_xent(logits, labels, scale: float = 1.0):
    """-> (loss_sum float, dlogits fp32, n_correct, n_labelled); rows with label < 0 are skipped."""
    logits = np.ascontiguousarray(logits, np.float32)
    labels = np.ascontiguousarray(labels, np.int32)
    n, c = logits.shape
    d = np.zeros_like(logits)
    loss = ctypes.c_double(0)
    nc, nl = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = lib().orc_softmax_xent(_p(logits), _p(labels), ctypes.c_int32(n), ctypes.c_int32(c), ctypes.c_float(scale),
                                _p(d), ctypes.byref(loss), ctypes.byref(nc), ctypes.byref(nl))
    assert rc == 0
    return loss.value, d, nc.value, nl.value


def adam_step(W, dW, m, v, lr, t, beta1=0.9, beta2=0.999, eps=1e-8):
    """In place on W, m, v (fp32 arrays)."""
    for a in (W, dW, m, v):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    rc = lib().orc_adam_step(_p(W), _p(dW), _p(m), _p(v), ctypes.c_int64(W.size), ctypes.c_float(lr),
                             ctypes.c_float(beta1), ctypes.c_float(beta2), ctypes.c_float(eps), ctypes.c_int32(t))
    assert rc == 0


def eps_update(eps, acc, mean_acc, params=EPS_DEFAULTS, swap=False):
    """-> (new eps, new mean_acc)"""
    fn = lib().orc_eps_update
    fn.restype = ctypes.c_float
    arr = (ctypes.c_float * 7)(*params)
    mean = ctypes.c_float(mean_acc)
    out = fn(ctypes.c_float(eps), ctypes.c_float(acc), ctypes.byref(mean), arr, ctypes.c_int(1 if swap else 0))
    return float(out), float(mean.value)
