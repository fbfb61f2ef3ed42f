"""Shared test helpers: independent dense references and the float tolerance."""
import numpy as np
import torch


def dense_norm_adj(g):
    """D^-1/2 (A+I) D^-1/2 as a dense float64 matrix, straight from the edge list."""
    n = g.n
    lo = g.lo.cpu().numpy()
    hi = g.hi.cpu().numpy()
    A = np.zeros((n, n), np.float64)
    A[lo, hi] = 1.0
    A[hi, lo] = 1.0
    A[np.arange(n), np.arange(n)] = 1.0
    d = A.sum(1)
    s = 1.0 / np.sqrt(d)
    return A * s[:, None] * s[None, :]


def csr_np(p, transposed=False):
    if transposed:
        return (p.t_rowptr.cpu().numpy(), p.t_colidx.cpu().numpy(), p.t_vals.cpu().numpy())
    return (p.rowptr.cpu().numpy(), p.colidx.cpu().numpy(), p.vals.cpu().numpy())


def csr_dense(rowptr, colidx, vals, n_cols):
    n = rowptr.size - 1
    D = np.zeros((n, n_cols), np.float64)
    for i in range(n):
        for k in range(rowptr[i], rowptr[i + 1]):
            D[i, colidx[k]] += float(vals[k])
    return D


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> bf16 bit patterns (uint16) using torch's cast."""
    t = torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def assert_rows_close(got, want, rel=1e-4, frob=1e-5, what=""):
    """Row-scaled bound: every row's largest error <= rel * the row's largest
    reference magnitude; plus a global Frobenius-relative bound."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if got.size == 0:
        return
    err = np.abs(got - want).reshape(got.shape[0], -1).max(1)
    ref = np.maximum(np.abs(want).reshape(want.shape[0], -1).max(1), 1e-30)
    worst = int(np.argmax(err / ref))
    assert (err <= rel * ref).all(), f"{what}: row {worst} err {err[worst]:.3e} ref {ref[worst]:.3e}"
    fn = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
    assert fn <= frob, f"{what}: frobenius rel {fn:.3e}"


def oracle_parts(parts):
    """cdfgen partitions -> the oracle training loop's partition records."""
    from oracle import training
    return [training.Part(P.n_loc, P.n_halo, P.owned.cpu().numpy(), P.halo.cpu().numpy(), csr_np(P), csr_np(P, True))
            for P in parts]


def oracle_vc_parts(parts):
    """cdfgen vertex-cut partitions -> the oracle's records."""
    from oracle import vc_training
    return [vc_training.Part(P.n_master, P.n_mirror, P.vertices.numpy(),
                             (P.rowptr.numpy(), P.colidx.numpy(), P.vals.numpy()),
                             P.mirror_master_dev.numpy(), P.mirror_master_row.numpy()) for P in parts]
