"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.
Integer outputs (masks, index lists, codes) and the fp32 sequences the method fixes must
be bit-equal; aggregated floats within 1e-4 of the row's largest reference magnitude."""
import numpy as np
import pytest
import torch

from cdfgen import configs, features
from helpers import assert_rows_close, bf16_to_f32, csr_np

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def cdf():
    import paper_2408_00232_amd as m
    m.binding.load()
    assert torch.cuda.is_available()
    return m


def to_np(t):
    """Device tensor -> numpy (bf16 as uint16 bit patterns)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def as_f64(a):
    return bf16_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


def assert_bf16_close(got, want, what=""):
    """bf16 outputs: within one bf16 step of the oracle's correctly rounded value, plus the
    fp32-accumulation allowance (1e-4 of the row's largest magnitude) where sums cancel."""
    g, o = as_f64(got), as_f64(want)
    rowmax = np.maximum(np.abs(o).max(1, keepdims=True), 1e-30)
    bad = np.abs(g - o) > np.abs(o) * 2.0 ** -7 + 1e-4 * rowmax
    assert not bad.any(), f"{what}: {int(bad.sum())} elements off"


def make_pair(R, F, ld, dtype, seed, frac_same=0.3, drift=0.08):
    """cached ~ N(0,1); cur = cached * (1 + drift_r * g), some rows untouched, some cached rows zero."""
    g = torch.Generator().manual_seed(seed)
    cached = torch.randn(R, ld, generator=g)
    rate = torch.rand(R, 1, generator=g) * drift
    cur = cached * (1 + rate * torch.randn(R, ld, generator=g))
    same = torch.rand(R, generator=g) < frac_same
    cur[same] = cached[same]
    zero = torch.rand(R, generator=g) < 0.05
    cached[zero] = 0
    cur, cached = cur.to(dtype), cached.to(dtype)
    return cur, cached


def ws_for(cdf, rows, dim, nnz=1):
    return torch.zeros(cdf.cdf_workspace_bytes(max(rows, 1), dim, max(nnz, 1)), dtype=torch.uint8, device=DEV)


FILTER_SHAPES = [(1000, 128, 128), (1000, 256, 256), (777, 100, 100), (1000, 602, 602), (515, 16, 16),
                 (300, 1024, 1024), (300, 37, 37), (300, 1, 1), (300, 3, 5), (400, 126, 130), (260, 2000, 2000),
                 (64, 700, 701)]


@pytest.mark.parametrize("R,F,ld", FILTER_SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("norm", [0, 1])
def test_cache_filter(cdf, oracle, R, F, ld, dtype, norm):
    cur, cached = make_pair(R, F, ld, dtype, seed=R * 31 + F)
    dcur, dcached = cur.to(DEV), cached.to(DEV)
    mask = torch.full((R,), 7, dtype=torch.uint8, device=DEV)
    idx = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    n_sent = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    ws = ws_for(cdf, R, F)
    ncur, ncached = to_np(cur)[:, :F], to_np(cached)[:, :F]
    for eps in (0.0, 0.05, 0.5):
        cdf.cdf_cache_filter(dcur[:, :F], dcached[:, :F], eps, norm, mask, idx, n_sent, ws)
        torch.cuda.synchronize()
        omask, oidx = oracle.cache_filter(ncur, ncached, eps, norm)
        n = int(n_sent.item())
        assert n == oidx.size
        np.testing.assert_array_equal(to_np(mask), omask)
        np.testing.assert_array_equal(to_np(idx)[:n], oidx)
    assert 0 < oidx.size < R or R < 10


@pytest.mark.parametrize("R", [64 * 8192, 64 * 8192 * 3, 64 * 8192 * 2 + 64 * 5 + 17, 64 * 8192 - 1, 64 * 8192 * 4 + 1])
def test_cache_filter_many_rows(cdf, oracle, R):
    """Row counts whose per-block counts fill one or several whole passes of the scan (8192 counts
    each, read as vectors), exactly or with a ragged rest, through the two-launch route and the
    one-pass route; narrow rows keep the oracle quick."""
    F = 4
    cur, cached = make_pair(R, F, F, torch.float32, seed=R % 1000 + 5, frac_same=0.5)
    dcur, dcached = cur.to(DEV), cached.to(DEV)
    mask = torch.full((R,), 7, dtype=torch.uint8, device=DEV)
    idx = torch.full((R,), -1, dtype=torch.int32, device=DEV)
    n_sent = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    ws = ws_for(cdf, R, F)
    omask, oidx = oracle.cache_filter(to_np(cur), to_np(cached), 0.05, 0)
    assert 0 < oidx.size < R
    cdf.cdf_cache_filter(dcur, dcached, 0.05, 0, mask, idx, n_sent, ws)
    torch.cuda.synchronize()
    assert int(n_sent.item()) == oidx.size
    np.testing.assert_array_equal(to_np(mask), omask)
    np.testing.assert_array_equal(to_np(idx)[:oidx.size], oidx)
    # one-pass route (same scan, counts written by the fused kernel)
    rb = cdf.cdf_code_row_bytes(F, 8, cdf.Q_MINMAX)
    codes = torch.zeros(R * rb, dtype=torch.uint8, device=DEV)
    meta = torch.zeros(R, 2, device=DEV)
    mask.fill_(7); idx.fill_(-1); n_sent.fill_(-1)
    cdf.cdf_cache_filter_quantize(dcur, dcached.clone(), 0.05, 0, 8, cdf.Q_MINMAX, cdf.COMMIT_CUR, True, mask, idx, n_sent,
                                  codes, meta, ws)
    torch.cuda.synchronize()
    assert int(n_sent.item()) == oidx.size
    np.testing.assert_array_equal(to_np(mask), omask)
    np.testing.assert_array_equal(to_np(idx)[:oidx.size], oidx)
    ocodes, ometa = oracle.quantize(to_np(cur), to_np(cached).copy(), oidx, 8, 0, 1, True)
    np.testing.assert_array_equal(to_np(codes)[:oidx.size * rb].reshape(-1, rb), ocodes.reshape(-1, rb))
    np.testing.assert_array_equal(to_np(meta)[:oidx.size], ometa)


def test_cache_filter_edges(cdf, oracle):
    ws = ws_for(cdf, 1024, 64)
    n_sent = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    # empty input: count defined, nothing else touched
    e = torch.zeros(0, 64, device=DEV)
    cdf.cdf_cache_filter(e, e, 0.1, 0, None, None, n_sent, ws)
    torch.cuda.synchronize()
    assert int(n_sent.item()) == 0
    # all rows sent / none sent, exactly one block and one block plus one row
    for R in (256, 257):
        cur = torch.randn(R, 64, device=DEV)
        mask = torch.zeros(R, dtype=torch.uint8, device=DEV)
        idx = torch.zeros(R, dtype=torch.int32, device=DEV)
        cdf.cdf_cache_filter(cur, torch.zeros_like(cur), 0.1, 0, mask, idx, n_sent, ws)
        torch.cuda.synchronize()
        assert int(n_sent.item()) == R and torch.equal(idx.cpu(), torch.arange(R, dtype=torch.int32))
        cdf.cdf_cache_filter(cur, cur.clone(), 0.0, 0, mask, idx, n_sent, ws)
        torch.cuda.synchronize()
        assert int(n_sent.item()) == 0 and int(mask.sum().item()) == 0


def test_nan_rows_follow_the_stated_rule(cdf, oracle):
    """Non-finite input: the kernels take the decisions the header states and the oracle pins (maxima drop
    NaN elements, L2 sums turn NaN and the row stays), in the separate calls and in the one-pass call."""
    from test_oracle_pins import nan_rows
    cur, cached = nan_rows()
    reps = 40                                   # several blocks of rows
    cur, cached = np.tile(cur, (reps, 1)), np.tile(cached, (reps, 1))
    R, F = cur.shape
    dcur, dcached = torch.from_numpy(cur).to(DEV), torch.from_numpy(cached).to(DEV)
    mask = torch.zeros(R, dtype=torch.uint8, device=DEV)
    idx = torch.zeros(R, dtype=torch.int32, device=DEV)
    n_sent = torch.zeros(1, dtype=torch.int32, device=DEV)
    ws = ws_for(cdf, R, F)
    for norm in (0, 1):
        cdf.cdf_cache_filter(dcur, dcached, 0.05, norm, mask, idx, n_sent, ws)
        torch.cuda.synchronize()
        omask, oidx = oracle.cache_filter(cur, cached, 0.05, norm)
        np.testing.assert_array_equal(to_np(mask), omask)
        assert int(n_sent.item()) == oidx.size
    omask, oidx = oracle.cache_filter(cur, cached, 0.05, 0)
    assert oidx.size == 2 * reps
    ocodes, ometa = oracle.quantize(cur, cached.copy(), oidx, 8, 0, 0, True)
    codes = torch.zeros(R * F, dtype=torch.uint8, device=DEV)
    meta = torch.zeros(R, 2, device=DEV)
    cdf.cdf_cache_filter_quantize(dcur, dcached, 0.05, 0, 8, 0, 0, True, mask, idx, n_sent, codes, meta, ws)
    torch.cuda.synchronize()
    n = int(n_sent.item())
    assert n == oidx.size
    np.testing.assert_array_equal(to_np(idx)[:n], oidx)
    np.testing.assert_array_equal(to_np(codes)[:n * F].reshape(n, F), ocodes)
    np.testing.assert_array_equal(to_np(meta)[:n], ometa)


def test_argument_errors(cdf):
    ws = ws_for(cdf, 64, 64)
    cur = torch.randn(8, 16, device=DEV)
    mask = torch.zeros(8, dtype=torch.uint8, device=DEV)
    idx = torch.zeros(8, dtype=torch.int32, device=DEV)
    n = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(cdf.binding.CdfError) as e:
        cdf.cdf_cache_filter(cur, cur, float("inf"), 0, mask, idx, n, ws)
    assert e.value.code == cdf.ERR_INVALID_ARG
    with pytest.raises(cdf.binding.CdfError) as e:
        cdf.cdf_cache_filter(cur, cur, 0.1, 0, mask, idx, n, ws[:8])
    assert e.value.code == cdf.ERR_WORKSPACE
    codes = torch.zeros(8 * 16, dtype=torch.uint8, device=DEV)
    meta = torch.zeros(8, 2, device=DEV)
    with pytest.raises(cdf.binding.CdfError) as e:
        cdf.cdf_quantize(cur, cur.clone(), idx, n, 8, 3, 0, 1, True, codes, meta)
    assert e.value.code == cdf.ERR_UNSUPPORTED
    with pytest.raises(cdf.binding.CdfError) as e:
        cdf.cdf_quantize(cur, None, idx, n, 8, 8, 0, 1, True, codes, meta)
    assert e.value.code == cdf.ERR_INVALID_ARG
    torch.cuda.synchronize()


QUANT_SHAPES = [(500, 128, 128), (300, 256, 256), (300, 100, 100), (200, 602, 602), (300, 16, 16),
                (100, 1024, 1024), (200, 37, 37), (200, 1, 1), (200, 3, 5), (100, 2048, 2048), (150, 126, 130)]


@pytest.mark.parametrize("R,F,ld", QUANT_SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bits,qs", [(8, 0), (4, 0), (8, 1), (4, 1), (8, 2)])
def test_quantize_dequantize(cdf, oracle, R, F, ld, dtype, bits, qs):
    cur, cached = make_pair(R, F, ld, dtype, seed=R * 17 + F + bits)
    g = torch.Generator().manual_seed(5)
    sel = torch.nonzero(torch.rand(R, generator=g) < 0.6).flatten().to(torch.int32)
    n = sel.numel()
    rb = cdf.cdf_code_row_bytes(F, bits, qs)
    for commit, delta in ((1, True), (2, True), (0, False), (2, False)):
        dcur, dcached = cur.to(DEV), cached.to(DEV)
        idx = torch.zeros(R, dtype=torch.int32, device=DEV)
        idx[:n] = sel.to(DEV)
        n_sent = torch.tensor([n], dtype=torch.int32, device=DEV)
        codes = torch.full((R * rb + 16,), 0xAB, dtype=torch.uint8, device=DEV)
        meta = torch.full((R, 2), -7.0, device=DEV)
        cdf.cdf_quantize(dcur[:, :F], dcached[:, :F], idx, n_sent, R, bits, qs, commit, delta, codes, meta)
        dst0 = torch.randn(R, ld, generator=g).to(dtype)
        ddst = dst0.to(DEV)
        cdf.cdf_dequantize(codes, meta, idx, n_sent, R, bits, qs, ddst[:, :F], accumulate=delta)
        torch.cuda.synchronize()
        ncur, ncached = to_np(cur), to_np(cached)
        ocodes, ometa = oracle.quantize(ncur[:, :F], ncached[:, :F], sel.numpy(), bits, qs, commit, delta)
        gcodes = to_np(codes)
        np.testing.assert_array_equal(gcodes[:n * rb].reshape(n, rb), ocodes)
        assert (gcodes[n * rb:] == 0xAB).all()                      # nothing written past the last message
        np.testing.assert_array_equal(to_np(meta)[:n], ometa)       # -0.0 == 0.0 here, by value
        np.testing.assert_array_equal(to_np(dcached), ncached)      # commit, including untouched rows / padding
        ndst = to_np(dst0)
        oracle.dequantize(ocodes, ometa, sel.numpy(), ndst[:, :F], bits, qs, accumulate=delta)
        np.testing.assert_array_equal(to_np(ddst), ndst)


def test_quantize_zero_rows(cdf):
    """*n_sent == 0 on the device: nothing is written."""
    cur = torch.randn(10, 32, device=DEV)
    cached = torch.zeros_like(cur)
    idx = torch.zeros(10, dtype=torch.int32, device=DEV)
    n_sent = torch.zeros(1, dtype=torch.int32, device=DEV)
    codes = torch.full((10 * 32,), 9, dtype=torch.uint8, device=DEV)
    meta = torch.full((10, 2), 3.0, device=DEV)
    cdf.cdf_quantize(cur, cached, idx, n_sent, 10, 8, 0, 1, True, codes, meta)
    cdf.cdf_dequantize(codes, meta, idx, n_sent, 10, 8, 0, cur, True)
    cdf.cdf_quantize(cur, cached, idx, n_sent, 0, 8, 0, 1, True, codes, meta)
    torch.cuda.synchronize()
    assert int((codes != 9).sum().item()) == 0 and int((cached != 0).sum().item()) == 0


def run_spmm(cdf, rowptr, colidx, vals, n_cols, X, bwd=False):
    n_rows = rowptr.numel() - 1
    A = cdf.DeviceCsr(n_rows, n_cols, rowptr, colidx, vals, DEV)
    ws = ws_for(cdf, n_rows, X.shape[1], colidx.numel())
    dX = X.to(DEV)
    Y = torch.full((n_rows, X.shape[1]), 3.0, dtype=X.dtype, device=DEV)
    (cdf.cdf_spmm_bwd if bwd else cdf.cdf_spmm_fwd)(A.struct, dX, Y, ws)
    torch.cuda.synchronize()
    return Y


# widths: whole 128-byte lines (column slices), rows of at most 32 lane-vectors (lane groups of 2 ... 32 lanes,
# exact and partial), odd widths (narrow lanes, whole wavefront per entry), several passes per row
@pytest.mark.parametrize("dim", [128, 256, 100, 602, 16, 37, 1, 1024, 3000, 4, 8, 12, 20, 28, 36, 64, 96, 120, 160])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_spmm_tiny_partition(cdf, oracle, dim, dtype):
    P = configs.build_partition(configs.TINY)
    X = features.normal_matrix(3, dim, P.n_loc + P.n_halo, dim).to(dtype)
    Y = run_spmm(cdf, P.rowptr, P.colidx, P.vals, P.n_loc + P.n_halo, X)
    want = oracle.spmm(*csr_np(P), P.n_loc + P.n_halo, to_np(X))
    if dtype == torch.float32:
        assert_rows_close(to_np(Y), want, what="Y")
    else:
        assert_bf16_close(to_np(Y), want, "Y")
        assert (to_np(Y) == want).mean() > 0.98
    dY = features.normal_matrix(4, dim, P.n_loc, dim).to(dtype)
    dXg = run_spmm(cdf, P.t_rowptr, P.t_colidx, P.t_vals, P.n_loc, dY, bwd=True)
    wantT = oracle.spmm(*csr_np(P, True), P.n_loc, to_np(dY))
    if dtype == torch.float32:
        assert_rows_close(to_np(dXg), wantT, what="dX")
    else:
        assert_bf16_close(to_np(dXg), wantT, "dX")


def test_spmm_long_and_empty_rows(cdf, oracle):
    """Rows of 0, 1, 255, 256, 257 and several thousand entries, empty rows at the start, at the
    end and exactly on chunk borders; run twice for bit-reproducibility."""
    rs = np.random.default_rng(21)
    lens = [0, 0, 1, 255, 0, 256, 0, 0, 257, 3, 5000, 0, 254, 2, 1, 1, 700, 0, 0, 1280, 0, 31, 0, 0]
    n_cols = 4000
    rowptr = np.zeros(len(lens) + 1, np.int64)
    rowptr[1:] = np.cumsum(lens)
    colidx = np.concatenate([np.sort(rs.choice(n_cols, l, replace=l > n_cols)) for l in lens]).astype(np.int32)
    vals = rs.standard_normal(colidx.size).astype(np.float32)
    for dim in (128, 100, 602):
        X = torch.from_numpy(rs.standard_normal((n_cols, dim)).astype(np.float32))
        args = (torch.from_numpy(rowptr), torch.from_numpy(colidx), torch.from_numpy(vals), n_cols, X)
        Y1 = run_spmm(cdf, *args)
        Y2 = run_spmm(cdf, *args)
        assert torch.equal(Y1, Y2)
        want = oracle.spmm(rowptr, colidx, vals, n_cols, X.numpy())
        assert_rows_close(to_np(Y1), want, what=f"Y dim {dim}")
        assert int((Y1[[0, 1, 4, 6, 7, 11, 17, 18, 20, 22, 23]] != 0).sum().item()) == 0
    # a matrix with no entries at all
    Y = run_spmm(cdf, torch.zeros(6, dtype=torch.int64), torch.zeros(0, dtype=torch.int32),
                 torch.zeros(0), n_cols, X)
    assert int((Y != 0).sum().item()) == 0


def run_spmm_padded(cdf, rowptr, colidx, vals, n_cols, X, ldx, ldy, bwd=False):
    """Same product with row pitches ldx / ldy larger than the width; returns (Y, padding of Y)."""
    n_rows = rowptr.numel() - 1
    dim = X.shape[1]
    A = cdf.DeviceCsr(n_rows, n_cols, rowptr, colidx, vals, DEV)
    ws = ws_for(cdf, n_rows, dim, colidx.numel())
    Xp = torch.full((X.shape[0], ldx), 7.0, dtype=X.dtype, device=DEV)    # padding must never be read into sums
    Xp[:, :dim] = X.to(DEV)
    Yp = torch.full((n_rows, ldy), 3.0, dtype=X.dtype, device=DEV)
    (cdf.cdf_spmm_bwd if bwd else cdf.cdf_spmm_fwd)(A.struct, Xp[:, :dim], Yp[:, :dim], ws)
    torch.cuda.synchronize()
    return Yp[:, :dim], Yp[:, dim:]


@pytest.mark.parametrize("nnz_target", [3000, 500_000, 560_000, 1_020_000, 1_100_000])
@pytest.mark.parametrize("dim", [32, 20])
def test_spmm_chunk_size_tiers_and_plan(cdf, oracle, nnz_target, dim):
    """The entries per wavefront step up with the matrix size (64, 128, 256, ...); matrices on both sides of
    the steps, with and without the work-split table computed ahead (cdf_spmm_plan): same bits either way,
    same values as the oracle."""
    rs = np.random.default_rng(nnz_target + dim)
    n_rows, n_cols = 3000, 5000
    lens = rs.zipf(1.6, n_rows).astype(np.int64)
    lens = np.minimum(lens * 20, 4 * n_cols)
    lens = (lens * (nnz_target / lens.sum())).astype(np.int64)
    lens[rs.integers(0, n_rows, 50)] = 0
    rowptr = np.zeros(n_rows + 1, np.int64)
    rowptr[1:] = np.cumsum(lens)
    nnz = int(rowptr[-1])
    colidx = np.concatenate([np.sort(rs.integers(0, n_cols, l)) for l in lens]).astype(np.int32)
    vals = rs.standard_normal(nnz).astype(np.float32)
    X = torch.from_numpy(rs.standard_normal((n_cols, dim)).astype(np.float32))
    t = (torch.from_numpy(rowptr), torch.from_numpy(colidx), torch.from_numpy(vals))
    ws = ws_for(cdf, n_rows, dim, nnz)
    dX = X.to(DEV)
    outs = []
    for plan in (True, False):
        A = cdf.DeviceCsr(n_rows, n_cols, *t, DEV, plan=plan)
        assert (A.struct.plan is not None) == plan
        Y = torch.full((n_rows, dim), 3.0, device=DEV)
        cdf.cdf_spmm_fwd(A.struct, dX, Y, ws)
        torch.cuda.synchronize()
        outs.append(Y)
    assert torch.equal(outs[0], outs[1])
    want = oracle.spmm(rowptr, colidx, vals, n_cols, X.numpy())
    assert_rows_close(to_np(outs[0]), want, what="Y")


# (dim, ldx, ldy): 16-byte vectors kept (pitch a multiple of 4 / 8 elements) on the column-sliced and the
# whole-row kernel, pitches that force 8-byte and single-element lanes, different pitches in and out
PADDED = [(128, 132, 132), (128, 160, 128), (256, 260, 288), (64, 68, 72), (100, 104, 108), (100, 101, 103),
          (602, 606, 608), (37, 41, 37), (16, 18, 16), (1, 3, 2), (1024, 1032, 1040), (96, 98, 96)]


@pytest.mark.parametrize("dim,ldx,ldy", PADDED)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_spmm_padded_pitch(cdf, oracle, dim, ldx, ldy, dtype):
    """cdf_spmm_fwd / cdf_spmm_bwd with leading dimensions above the width: same values as the oracle,
    bit-equal to the contiguous call where the lane-vector width is unchanged, padding untouched."""
    P = configs.build_partition(configs.TINY)
    X = features.normal_matrix(3, dim, P.n_loc + P.n_halo, dim).to(dtype)
    dY = features.normal_matrix(4, dim, P.n_loc, dim).to(dtype)
    for bwd, (rp, ci, va), n_cols, src in ((False, (P.rowptr, P.colidx, P.vals), P.n_loc + P.n_halo, X),
                                            (True, (P.t_rowptr, P.t_colidx, P.t_vals), P.n_loc, dY)):
        Y, pad = run_spmm_padded(cdf, rp, ci, va, n_cols, src, ldx, ldy, bwd)
        assert int((pad != 3.0).sum().item()) == 0, "padding of the output was written"
        want = oracle.spmm(rp.numpy(), ci.numpy(), va.numpy(), n_cols, to_np(src))
        if dtype == torch.float32:
            assert_rows_close(to_np(Y.contiguous()), want, what=f"Y bwd={bwd}")
        else:
            assert_bf16_close(to_np(Y.contiguous()), want, f"Y bwd={bwd}")
        # the order of the sums depends on the lane-vector width only, not on the pitch itself
        def lane_vector(*lds):
            v = 8 if dtype == torch.bfloat16 else 4
            while v > 1 and any(x % v for x in lds):
                v //= 2
            return v
        if lane_vector(dim, ldx, ldy) == lane_vector(dim):
            Yc = run_spmm(cdf, rp, ci, va, n_cols, src, bwd=bwd)
            assert torch.equal(Y.contiguous(), Yc)


def test_spmm_padded_pitch_long_rows(cdf, oracle):
    """Padded pitches on a matrix whose rows straddle chunk borders (the fix-up kernel writes those rows)."""
    rs = np.random.default_rng(22)
    lens = [0, 700, 0, 256, 1, 5000, 0, 3, 1280, 0, 31, 0]
    n_cols = 3000
    rowptr = np.zeros(len(lens) + 1, np.int64)
    rowptr[1:] = np.cumsum(lens)
    colidx = np.concatenate([np.sort(rs.choice(n_cols, l, replace=l > n_cols)) for l in lens]).astype(np.int32)
    vals = rs.standard_normal(colidx.size).astype(np.float32)
    for dim, ldx, ldy in ((128, 132, 136), (100, 101, 100), (256, 256, 264)):
        X = torch.from_numpy(rs.standard_normal((n_cols, dim)).astype(np.float32))
        Y, pad = run_spmm_padded(cdf, torch.from_numpy(rowptr), torch.from_numpy(colidx), torch.from_numpy(vals), n_cols,
                                 X, ldx, ldy)
        assert int((pad != 3.0).sum().item()) == 0
        want = oracle.spmm(rowptr, colidx, vals, n_cols, X.numpy())
        assert_rows_close(to_np(Y.contiguous()), want, what=f"Y dim {dim}")


@pytest.mark.parametrize("f_in,f_out", [(128, 16), (16, 8), (256, 41), (256, 47), (100, 47), (512, 24), (1024, 12),
                                        (64, 64), (4, 1), (256, 64), (128, 70), (37, 8)])
@pytest.mark.parametrize("relu", [True, False])
def test_spmm_dense_fwd_one_kernel(cdf, oracle, f_in, f_out, relu):
    """Aggregation with the dense transform in its row epilogue (narrow outputs) and its two-launch
    fall-back (256 x 64 needs more LDS than a block has, 70 columns are too many, 37 is not a multiple of
    four): M, Z, H against the oracle's aggregation followed by its transform; two runs bit-equal."""
    P = configs.build_partition(configs.TINY)
    n, nc = P.n_loc, P.n_loc + P.n_halo
    X = features.normal_matrix(5, f_in, nc, f_in)
    W = features.glorot(5, f_out, f_in, f_out)
    A = cdf.DeviceCsr(n, nc, P.rowptr, P.colidx, P.vals, DEV)
    ws = ws_for(cdf, nc, max(f_in, f_out), P.nnz)
    outs = []
    for _ in range(2):
        M = torch.full((n, f_in), 3.0, device=DEV)
        Z = torch.full((n, f_out), 3.0, device=DEV)
        H = torch.full((n, f_out), 3.0, device=DEV)
        cdf.cdf_spmm_dense_fwd(A.struct, X.to(DEV), W.to(DEV), relu, M, Z, H, ws)
        torch.cuda.synchronize()
        outs.append((M, Z, H))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    oM = oracle.spmm(*csr_np(P), nc, X.numpy())
    oZ, oH = oracle.dense_fwd(oM, W.numpy(), relu)
    M, Z, H = outs[0]
    assert_rows_close(to_np(M), oM, what="M")
    assert_rows_close(to_np(Z), oZ, what="Z")
    assert_rows_close(to_np(H), oH, what="H")
    # H alone (the layer step keeps no Z)
    H2 = torch.full((n, f_out), 3.0, device=DEV)
    cdf.cdf_spmm_dense_fwd(A.struct, X.to(DEV), W.to(DEV), relu, M, None, H2, ws)
    torch.cuda.synchronize()
    assert torch.equal(H2, H)


def test_spmm_dense_fwd_long_and_empty_rows(cdf, oracle):
    """Rows that straddle chunk borders take the fix-up route of the one-kernel call; empty rows give zeros."""
    rs = np.random.default_rng(23)
    lens = [0, 0, 1, 255, 0, 64, 0, 65, 3, 5000, 0, 63, 2, 1, 700, 0, 0, 1280, 0, 31, 0]
    n_cols = 4000
    rowptr = np.zeros(len(lens) + 1, np.int64)
    rowptr[1:] = np.cumsum(lens)
    colidx = np.concatenate([np.sort(rs.choice(n_cols, l, replace=l > n_cols)) for l in lens]).astype(np.int32)
    vals = rs.standard_normal(colidx.size).astype(np.float32)
    for f_in, f_out in ((128, 16), (256, 47), (512, 8)):
        X = torch.from_numpy(rs.standard_normal((n_cols, f_in)).astype(np.float32))
        W = torch.from_numpy((rs.standard_normal((f_in, f_out)) * 0.1).astype(np.float32))
        A = cdf.DeviceCsr(len(lens), n_cols, torch.from_numpy(rowptr), torch.from_numpy(colidx), torch.from_numpy(vals), DEV)
        ws = ws_for(cdf, n_cols, f_in, colidx.size)
        M = torch.full((len(lens), f_in), 3.0, device=DEV)
        Z = torch.full((len(lens), f_out), 3.0, device=DEV)
        H = torch.full((len(lens), f_out), 3.0, device=DEV)
        cdf.cdf_spmm_dense_fwd(A.struct, X.to(DEV), W.to(DEV), True, M, Z, H, ws)
        torch.cuda.synchronize()
        oM = oracle.spmm(rowptr, colidx, vals, n_cols, X.numpy())
        oZ, oH = oracle.dense_fwd(oM, W.numpy(), True)
        assert_rows_close(to_np(M), oM, what="M")
        assert_rows_close(to_np(Z), oZ, what="Z")
        assert_rows_close(to_np(H), oH, what="H")
        empty = [i for i, l in enumerate(lens) if l == 0]
        assert int((Z[empty] != 0).sum().item()) == 0 and int((H[empty] != 0).sum().item()) == 0


DENSE_SHAPES = [(1000, 100, 47), (300, 602, 256), (513, 16, 8), (700, 128, 256), (257, 256, 41), (130, 64, 64),
                (5000, 128, 16), (64, 33, 130), (4096, 128, 256), (2048, 256, 64), (1024, 64, 128),
                # aligned rows with ragged tiles: a reduction tail in the forward and dM products, a last
                # slab of dW that ends inside a tile, fewer columns than a tile
                (1000, 100, 48), (515, 36, 20), (300, 260, 132)]


@pytest.mark.parametrize("n,f,g", DENSE_SHAPES)
@pytest.mark.parametrize("relu", [True, False])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_dense_fwd_bwd(cdf, oracle, n, f, g, relu, dtype):
    M = features.normal_matrix(7, n + f, n, f).to(dtype)
    W = features.glorot(7, g, f, g)
    dH = features.normal_matrix(8, n + g, n, g)
    dM_, dW_, dH_, W_ = M.to(DEV), None, dH.to(DEV), W.to(DEV)
    Z = torch.zeros(n, g, device=DEV)
    H = torch.zeros(n, g, device=DEV)
    cdf.cdf_dense_fwd(dM_, W_, relu, Z, H)
    torch.cuda.synchronize()
    oZ, oH = oracle.dense_fwd(to_np(M), W.numpy(), relu)
    assert_rows_close(to_np(Z), oZ, what="Z")
    assert_rows_close(to_np(H), oH, rel=1e-4, frob=1e-5, what="H")
    # backward from the oracle's own Z (an input of this entry point), so the sign test is shared
    Zs = torch.from_numpy(oZ).to(DEV)
    dW = torch.zeros(f, g, device=DEV)
    dM = torch.zeros(n, f, dtype=dtype, device=DEV)
    ws = ws_for(cdf, n, max(f, g))
    cdf.cdf_dense_bwd(dM_, W_, Zs, dH_, relu, dW, dM, ws)
    dW2 = torch.zeros(f, g, device=DEV)
    cdf.cdf_dense_bwd(dM_, W_, Zs, dH_, relu, dW2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW2)
    odW, odM = oracle.dense_bwd(to_np(M), W.numpy(), oZ, dH.numpy(), relu)
    assert_rows_close(to_np(dW), odW, what="dW")
    if dtype == torch.float32:
        assert_rows_close(to_np(dM), odM, what="dM")
    else:
        assert_bf16_close(to_np(dM), odM, "dM")


@pytest.mark.parametrize("n,f,g", [(131072 + 77, 256, 192), (131072, 128, 128)])
def test_dense_bf16_many_row_tiles(cdf, oracle, n, f, g):
    """bf16 activations, more than a thousand row tiles: the 1-D grids of the forward and dM products
    (row tiles dealt to the XCDs in groups of eight, column blocks of a tile side by side) with a
    ragged last row tile, a last group of fewer than eight tiles and a half-filled last column block
    in the first shape."""
    M = features.normal_matrix(17, n + f, n, f).to(torch.bfloat16)
    W = features.glorot(17, g, f, g)
    dH = features.normal_matrix(18, n + g, n, g)
    M_, dH_, W_ = M.to(DEV), dH.to(DEV), W.to(DEV)
    Z = torch.zeros(n, g, device=DEV)
    H = torch.zeros(n, g, device=DEV)
    ws = ws_for(cdf, n, max(f, g))
    cdf.cdf_dense_fwd(M_, W_, True, Z, H)
    torch.cuda.synchronize()
    oZ, oH = oracle.dense_fwd(to_np(M), W.numpy(), True)
    assert_rows_close(to_np(Z), oZ, what="Z")
    assert_rows_close(to_np(H), oH, rel=1e-4, frob=1e-5, what="H")
    Zs = torch.from_numpy(oZ).to(DEV)
    dW = torch.zeros(f, g, device=DEV)
    dM = torch.zeros(n, f, dtype=torch.bfloat16, device=DEV)
    cdf.cdf_dense_bwd(M_, W_, Zs, dH_, True, dW, dM, ws)
    torch.cuda.synchronize()
    odW, odM = oracle.dense_bwd(to_np(M), W.numpy(), oZ, dH.numpy(), True)
    assert_rows_close(to_np(dW), odW, what="dW")
    assert_bf16_close(to_np(dM), odM, "dM")


@pytest.mark.parametrize("n,f,g", [(200, 40, 8), (200, 136, 8)])
def test_dense_bwd_bf16_weight_split_in_block_or_beforehand(cdf, oracle, n, f, g):
    """bf16 activations: with room in the workspace dM's weight operand is split into its bf16 parts once,
    otherwise in every workgroup. A workspace of exactly the slab partials (f*g*4 bytes here, less than
    the two split copies need after their 256-byte rounding) takes the second route; both give the same
    bits and match the oracle."""
    M = features.normal_matrix(27, n + f, n, f).to(torch.bfloat16)
    W = features.glorot(27, g, f, g)
    dH = features.normal_matrix(28, n + g, n, g)
    oZ, _ = oracle.dense_fwd(to_np(M), W.numpy(), True)
    M_, dH_, W_, Zs = M.to(DEV), dH.to(DEV), W.to(DEV), torch.from_numpy(oZ).to(DEV)
    outs = []
    for ws in (ws_for(cdf, n, max(f, g)), torch.zeros(f * g * 4, dtype=torch.uint8, device=DEV)):
        assert ws.numel() % 256 == 0
        dW = torch.zeros(f, g, device=DEV)
        dM = torch.zeros(n, f, dtype=torch.bfloat16, device=DEV)
        cdf.cdf_dense_bwd(M_, W_, Zs, dH_, True, dW, dM, ws)
        torch.cuda.synchronize()
        outs.append((dW, dM))
    assert 2 * ((f * g * 2 + 255) // 256 * 256) > f * g * 4      # the small workspace cannot hold the split copies
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    odW, odM = oracle.dense_bwd(to_np(M), W.numpy(), oZ, dH.numpy(), True)
    assert_rows_close(to_np(outs[1][0]), odW, what="dW")
    assert_bf16_close(to_np(outs[1][1]), odM, "dM")


def lockstep_messages(oracle, rows, cache0, L, h, eps, norm, bits, qs, commit, delta):
    """The cache test and the message build of a backward step, redone by the oracle on the halo gradient
    rows the GPU step itself produced (`rows`) against the cache the step started from (`cache0`): mask,
    row list, codes, meta and the committed cache must be equal bit for bit. Returns the sent fraction."""
    cache = cache0.copy()
    omask, oidx = oracle.cache_filter(rows, cache, eps, norm)
    ocodes, ometa = oracle.quantize(rows, cache, oidx, bits, qs, commit, delta)
    gn = int(L.gn_sent.item())
    assert gn == oidx.size
    np.testing.assert_array_equal(to_np(L.gmask)[:h], omask)
    np.testing.assert_array_equal(to_np(L.gidx)[:gn], oidx)
    np.testing.assert_array_equal(to_np(L.gcodes)[:gn * L.row_bytes].reshape(gn, -1), ocodes)
    np.testing.assert_array_equal(to_np(L.gmeta)[:gn], ometa)          # by value: -0.0 == 0.0
    np.testing.assert_array_equal(to_np(L.gcache_sent), cache)
    return gn / max(h, 1)


def layer_case(cdf, oracle, P, f_in, f_out, eps, norm, bits, qs, commit, delta, relu, epochs, dtype=torch.float32,
               seed=1):
    """Forward + backward of one layer for several epochs, oracle run beside it from the same
    inputs. The halo stream is an input, so the forward cache state stays bit-equal."""
    A = cdf.DeviceCsr(P.n_loc, P.n_loc + P.n_halo, P.rowptr, P.colidx, P.vals, DEV)
    At = cdf.DeviceCsr(P.n_loc + P.n_halo, P.n_loc, P.t_rowptr, P.t_colidx, P.t_vals, DEV)
    L = cdf.LayerBuffers(A, At, P.n_loc, P.n_halo, f_in, f_out, dtype=dtype, bits=bits, qs=qs, device=DEV)
    ws = torch.zeros(L.workspace_bytes(), dtype=torch.uint8, device=DEV)
    x_loc = features.normal_matrix(seed, 1, P.n_loc, f_in).to(dtype)
    W = features.glorot(seed, 2, f_in, f_out)
    stream = features.HaloStream(seed, P.n_halo, f_in)
    L.xfull[:P.n_loc] = x_loc.to(DEV)
    L.W.copy_(W)
    o_x = np.concatenate([to_np(x_loc), np.zeros((P.n_halo, f_in), to_np(x_loc).dtype)])
    o_sent = np.zeros_like(o_x[P.n_loc:])
    An, Atn = csr_np(P), csr_np(P, True)
    rates = []
    for t in range(epochs):
        fresh = stream.value().to(dtype)
        dH = features.normal_matrix(seed, 50 + t, P.n_loc, f_out)
        L.halo_fresh.copy_(fresh)
        L.dH.copy_(dH)
        cdf.cdf_gcn_layer_fwd(L.fwd_args(eps, norm, commit, delta, relu), ws)
        torch.cuda.synchronize()
        of = oracle.layer_fwd(An, P.n_loc, P.n_halo, o_x, to_np(fresh), o_sent, W.numpy(), eps, norm, bits, qs,
                              commit, relu, delta)
        n = int(L.n_sent.item())
        rates.append(n / max(P.n_halo, 1))
        assert n == of["idx"].size
        np.testing.assert_array_equal(to_np(L.mask)[:P.n_halo], of["mask"])
        np.testing.assert_array_equal(to_np(L.idx)[:n], of["idx"])
        np.testing.assert_array_equal(to_np(L.codes)[:n * L.row_bytes].reshape(n, -1), of["codes"])
        np.testing.assert_array_equal(to_np(L.meta)[:n], of["meta"])
        np.testing.assert_array_equal(to_np(L.cache_sent), o_sent)
        np.testing.assert_array_equal(to_np(L.xfull), o_x)
        if dtype == torch.float32:
            assert_rows_close(to_np(L.M), of["M"], what="M")
            assert_rows_close(to_np(L.Z), of["Z"], what="Z")
            assert_rows_close(to_np(L.H), of["H"], what="H")
        else:
            # bf16 storage: M within one bf16 step of the oracle's correctly rounded sums (and mostly
            # equal to them); the step's own Z follows its own M, so it is held to the fp32 bound
            # against the oracle's transform of those very rows, and the oracle's M through the
            # library's transform against the oracle's Z
            assert_bf16_close(to_np(L.M), of["M"], "M")
            assert (to_np(L.M) == of["M"]).mean() > 0.98
            oZ_own, oH_own = oracle.dense_fwd(to_np(L.M), W.numpy(), relu)
            assert_rows_close(to_np(L.Z), oZ_own, what="Z of the step's own M")
            assert_rows_close(to_np(L.H), oH_own, what="H of the step's own M")
            Mo = torch.from_numpy(of["M"].view(np.int16)).view(torch.bfloat16).to(DEV)
            Z2 = torch.zeros(P.n_loc, f_out, device=DEV)
            H2 = torch.zeros(P.n_loc, f_out, device=DEV)
            cdf.cdf_dense_fwd(Mo, L.W, relu, Z2, H2)
            torch.cuda.synchronize()
            assert_rows_close(to_np(Z2), of["Z"], what="Z")
            assert_rows_close(to_np(H2), of["H"], what="H")
        # backward: fed with the oracle's forward results and a gradient cache built from the
        # oracle's halo gradients so that every row sits well away from the threshold
        ob0 = oracle.dense_bwd(of["M"], W.numpy(), of["Z"], dH.numpy(), relu)
        odx = oracle.spmm(*Atn, P.n_loc, ob0[1])
        gh = as_f64(odx[P.n_loc:])
        rs = np.random.default_rng(seed + t)
        keep = rs.random(P.n_halo) < (0.5 if eps > 0 else -1.0)   # threshold 0: any difference is sent
        factor = np.where(keep, 1.0 + eps * 0.25, 1.0 + eps * 4.0 + 0.5)[:, None]
        gsent = torch.from_numpy((gh * factor).astype(np.float32)).to(dtype)
        L.M.copy_(torch.from_numpy(of["M"]).view(L.M.dtype) if dtype == torch.float32 else
                  torch.from_numpy(of["M"].view(np.int16)).view(torch.bfloat16))
        L.Z.copy_(torch.from_numpy(of["Z"]))
        L.gcache_sent.copy_(gsent)
        cdf.cdf_gcn_layer_bwd(L.bwd_args(eps, norm, commit, delta, relu), ws)
        torch.cuda.synchronize()
        o_gsent = to_np(gsent)
        ob = oracle.layer_bwd(Atn, P.n_loc, P.n_halo, of["M"], of["Z"], dH.numpy(), W.numpy(), o_gsent, eps, norm,
                              bits, qs, commit, relu, True, delta)
        assert_rows_close(to_np(L.dW), ob["dW"], what="dW")
        if dtype == torch.float32:
            assert_rows_close(to_np(L.dM), ob["dM"], what="dM")
            assert_rows_close(to_np(L.dxfull), ob["dxfull"], what="dxfull")
        else:
            assert_bf16_close(to_np(L.dM), ob["dM"], "dM")
            # the aggregation of the step's own dM rows (they differ from the oracle's by rounding steps)
            assert_bf16_close(to_np(L.dxfull), oracle.spmm(*Atn, P.n_loc, to_np(L.dM)), "dxfull")
        gn = int(L.gn_sent.item())
        # free-running comparison: every row was placed far from the threshold, so the decisions agree
        # although the gradients differ in their last bits
        np.testing.assert_array_equal(to_np(L.gmask)[:P.n_halo], ob["mask"])
        np.testing.assert_array_equal(to_np(L.gidx)[:gn], ob["idx"])
        if eps > 0:
            nz = np.abs(gh).max(1) > 0
            np.testing.assert_array_equal(ob["mask"][nz], (~keep[nz]).astype(np.uint8))
        lockstep_messages(oracle, to_np(L.dxfull)[P.n_loc:], to_np(gsent), L, P.n_halo, eps, norm, bits, qs, commit,
                          delta)
        # a second backward step on a cache that puts the rows on both sides of the threshold, densely
        # around it (checked in lock-step only: there the decision depends on the last bits)
        if eps > 0:
            own = as_f64(to_np(L.dxfull)[P.n_loc:])
            near = 1.0 + eps * rs.uniform(0.0, 2.2, P.n_halo)[:, None]
            gsent2 = torch.from_numpy((own * near).astype(np.float32)).to(dtype)
            L.gcache_sent.copy_(gsent2)
            cdf.cdf_gcn_layer_bwd(L.bwd_args(eps, norm, commit, delta, relu), ws)
            torch.cuda.synchronize()
            frac = lockstep_messages(oracle, to_np(L.dxfull)[P.n_loc:], to_np(gsent2), L, P.n_halo, eps, norm, bits,
                                     qs, commit, delta)
            assert 0.2 < frac < 0.8, frac
        stream.advance()
    return rates


def test_layer_tiny_paper_setting(cdf, oracle):
    w = configs.TINY
    P = configs.build_partition(w)
    rates = layer_case(cdf, oracle, P, 128, 16, w.eps, 0, 8, 0, 1, True, True, epochs=3)
    assert rates[0] > 0.99 and rates[-1] < rates[0]
    layer_case(cdf, oracle, P, 16, 8, w.eps, 0, 8, 0, 1, True, False, epochs=3)


def test_layer_tiny_l2_symmetric(cdf, oracle):
    P = configs.build_partition(configs.TINY)
    layer_case(cdf, oracle, P, 128, 16, 0.05, 1, 8, 1, 1, True, True, epochs=3)


@pytest.mark.parametrize("part", [1, 3])
def test_layer_tiny_other_partitions_4bit_deq_commit(cdf, oracle, part):
    P = configs.build_partition(configs.TINY, part=part)
    layer_case(cdf, oracle, P, 128, 16, 0.05, 0, 4, 0, 2, True, True, epochs=3)


def test_layer_eps_zero_is_uncached(cdf, oracle):
    """Threshold 0 with value messages: the halo rows the aggregation reads are bit-equal to
    the fresh rows, so the step equals the uncached one on the same kernels."""
    P = configs.build_partition(configs.TINY)
    rates = layer_case(cdf, oracle, P, 128, 16, 0.0, 0, 8, 2, 1, False, True, epochs=3)
    assert all(r > 0.99 for r in rates)


def test_layer_mid_shrunk(cdf, oracle):
    w = configs.shrink(configs.MID, 12000)
    P = configs.build_partition(w)
    assert P.nnz > 30000 and P.n_halo > 2000
    layer_case(cdf, oracle, P, 602, 256, 0.01, 0, 8, 0, 1, True, True, epochs=2)
    layer_case(cdf, oracle, P, 256, 41, 0.1, 0, 8, 0, 1, True, False, epochs=2)


def test_layer_large_shrunk_bfs(cdf, oracle):
    w = configs.shrink(configs.LARGE, 20000)
    P = configs.build_partition(w)
    layer_case(cdf, oracle, P, 100, 256, 0.05, 0, 8, 0, 1, True, True, epochs=2)
    layer_case(cdf, oracle, P, 256, 47, 0.05, 0, 8, 0, 1, True, False, epochs=1)


def test_layer_wide_shrunk_bf16_4bit(cdf, oracle):
    w = configs.shrink(configs.WIDE, 4096)
    P = configs.build_partition(w)
    layer_case(cdf, oracle, P, 1024, 512, 0.05, 0, 4, 0, 1, True, True, epochs=2, dtype=torch.bfloat16)


def tf_layer_case(cdf, oracle, P, f_in, f_out, eps, bits, qs, commit, relu, epochs, seed=2):
    """Transform-first layer against the oracle: forward for several epochs from the same input
    stream; backward on the oracle's forward results with a gradient cache that keeps every row
    well away from the threshold."""
    n, h = P.n_loc, P.n_halo
    A = cdf.DeviceCsr(n, n + h, P.rowptr, P.colidx, P.vals, DEV)
    At = cdf.DeviceCsr(n + h, n, P.t_rowptr, P.t_colidx, P.t_vals, DEV)
    L = cdf.TfLayerBuffers(A, At, n, h, f_in, f_out, bits=bits, qs=qs, device=DEV)
    ws = torch.zeros(L.workspace_bytes(), dtype=torch.uint8, device=DEV)
    x_loc = features.normal_matrix(seed, 1, n, f_in)
    W = features.glorot(seed, 2, f_in, f_out)
    stream = features.HaloStream(seed, h, f_out)
    L.x_local.copy_(x_loc)
    L.W.copy_(W)
    o_t = np.zeros((n + h, f_out), np.float32)
    o_sent = np.zeros((h, f_out), np.float32)
    An, Atn = csr_np(P), csr_np(P, True)
    for t in range(epochs):
        fresh = stream.value()
        dH = features.normal_matrix(seed, 50 + t, n, f_out)
        L.halo_fresh.copy_(fresh)
        L.dH.copy_(dH)
        cdf.cdf_gcn_layer_tf_fwd(L.fwd_args(eps, 0, commit, True, relu), ws)
        torch.cuda.synchronize()
        of = oracle.layer_tf_fwd(An, n, h, x_loc.numpy(), o_t, fresh.numpy().copy(), o_sent, W.numpy(), eps, 0, bits,
                                 qs, commit, relu, True)
        ns = int(L.n_sent.item())
        assert ns == of["idx"].size
        np.testing.assert_array_equal(to_np(L.mask)[:h], of["mask"])
        np.testing.assert_array_equal(to_np(L.idx)[:ns], of["idx"])
        np.testing.assert_array_equal(to_np(L.codes)[:ns * L.row_bytes].reshape(ns, -1), of["codes"])
        np.testing.assert_array_equal(to_np(L.meta)[:ns], of["meta"])
        np.testing.assert_array_equal(to_np(L.cache_sent), o_sent)
        np.testing.assert_array_equal(to_np(L.tfull)[n:], o_t[n:])
        assert_rows_close(to_np(L.tfull)[:n], o_t[:n], what="T local")
        assert_rows_close(to_np(L.Z), of["Z"], what="Z")
        assert_rows_close(to_np(L.H), of["H"], what="H")
        # backward
        dZ = np.where(of["Z"] > 0, dH.numpy(), np.float32(0)) if relu else dH.numpy()
        odt = oracle.spmm(*Atn, n, np.ascontiguousarray(dZ, np.float32))
        gh = odt[n:].astype(np.float64)
        rs = np.random.default_rng(seed + t)
        keep = rs.random(h) < (0.5 if eps > 0 else -1.0)
        factor = np.where(keep, 1.0 + eps * 0.25, 1.0 + eps * 4.0 + 0.5)[:, None]
        gsent = torch.from_numpy((gh * factor).astype(np.float32))
        L.Z.copy_(torch.from_numpy(of["Z"]))
        L.gcache_sent.copy_(gsent)
        cdf.cdf_gcn_layer_tf_bwd(L.bwd_args(eps, 0, commit, True, relu), ws)
        torch.cuda.synchronize()
        o_g = gsent.numpy().copy()
        ob = oracle.layer_tf_bwd(Atn, n, h, x_loc.numpy(), of["Z"], dH.numpy(), W.numpy(), o_g, eps, 0, bits, qs,
                                 commit, relu, True, True)
        assert_rows_close(to_np(L.dtfull), ob["dtfull"], what="dtfull")
        assert_rows_close(to_np(L.dW), ob["dW"], what="dW")
        assert_rows_close(to_np(L.dx_local), ob["dx_local"], what="dx_local")
        gn = int(L.gn_sent.item())
        np.testing.assert_array_equal(to_np(L.gmask)[:h], ob["mask"])
        np.testing.assert_array_equal(to_np(L.gidx)[:gn], ob["idx"])
        lockstep_messages(oracle, to_np(L.dtfull)[n:], gsent.numpy(), L, h, eps, 0, bits, qs, commit, True)
        if eps > 0:
            near = 1.0 + eps * rs.uniform(0.0, 2.2, h)[:, None]
            gsent2 = torch.from_numpy((to_np(L.dtfull)[n:].astype(np.float64) * near).astype(np.float32))
            L.gcache_sent.copy_(gsent2)
            cdf.cdf_gcn_layer_tf_bwd(L.bwd_args(eps, 0, commit, True, relu), ws)
            torch.cuda.synchronize()
            frac = lockstep_messages(oracle, to_np(L.dtfull)[n:], gsent2.numpy(), L, h, eps, 0, bits, qs, commit, True)
            assert 0.2 < frac < 0.8, frac
        stream.advance()


def test_tf_layer_tiny(cdf, oracle):
    P = configs.build_partition(configs.TINY)
    tf_layer_case(cdf, oracle, P, 128, 16, 0.05, 8, 0, 1, True, epochs=3)
    tf_layer_case(cdf, oracle, P, 16, 8, 0.05, 4, 0, 2, False, epochs=2)


def test_tf_layer_mid_shrunk(cdf, oracle):
    P = configs.build_partition(configs.shrink(configs.MID, 12000))
    tf_layer_case(cdf, oracle, P, 256, 41, 0.1, 8, 0, 1, False, epochs=2)
    tf_layer_case(cdf, oracle, P, 602, 256, 0.01, 8, 0, 1, True, epochs=1)


def test_tf_layer_large_shrunk(cdf, oracle):
    P = configs.build_partition(configs.shrink(configs.LARGE, 20000))
    tf_layer_case(cdf, oracle, P, 256, 64, 0.05, 8, 0, 1, True, epochs=2)


@pytest.mark.parametrize("n,classes", [(1000, 8), (777, 41), (300, 64), (130, 47), (64, 1), (500, 200)])
def test_softmax_xent(cdf, oracle, n, classes):
    g = torch.Generator().manual_seed(n + classes)
    logits = torch.randn(n, classes, generator=g) * 3
    logits[5] = logits[5, 0]                                    # an all-equal row: ties go to class 0
    labels = torch.randint(-1, classes, (n,), generator=g, dtype=torch.int32)
    labels[5] = 0
    d = torch.full((n, classes), 9.0, device=DEV)
    loss = torch.zeros(1, device=DEV)
    counts = torch.zeros(2, dtype=torch.int32, device=DEV)
    ws = ws_for(cdf, n, classes)
    cdf.cdf_softmax_xent(logits.to(DEV), labels.to(DEV), 0.25, d, loss, counts, ws)
    torch.cuda.synchronize()
    ol, od, oc, on = oracle.softmax_xent(logits.numpy(), labels.numpy(), 0.25)
    assert counts.tolist() == [oc, on]
    assert abs(float(loss.item()) - ol) <= 1e-5 * max(abs(ol), 1.0)
    np.testing.assert_allclose(to_np(d), od, rtol=0, atol=2e-6)


def test_adam_and_accumulate(cdf, oracle):
    g = torch.Generator().manual_seed(9)
    count = 602 * 256 + 3
    W = torch.randn(count, generator=g)
    m = torch.zeros(count)
    v = torch.zeros(count)
    dW, dm, dv = W.to(DEV), m.to(DEV), v.to(DEV)
    oW, om, ov = W.numpy().copy(), m.numpy().copy(), v.numpy().copy()
    for t in range(1, 6):
        grad = torch.randn(count, generator=g) * (10.0 ** torch.randint(-4, 2, (count,), generator=g).float())
        cdf.cdf_adam_step(dW, grad.to(DEV), dm, dv, 0.01, t)
        oracle.adam_step(oW, grad.numpy().copy(), om, ov, 0.01, t)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_np(dW), oW, rtol=0, atol=2e-6)
    np.testing.assert_allclose(to_np(dm), om, rtol=2e-6, atol=1e-6 * np.abs(om).max())   # sums that cancel
    np.testing.assert_allclose(to_np(dv), ov, rtol=2e-6, atol=1e-6 * np.abs(ov).max())
    a = torch.randn(count, generator=g)
    b = torch.randn(count, generator=g)
    da = a.to(DEV)
    cdf.cdf_accumulate(da, b.to(DEV))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(da), (a + b).numpy())


@pytest.mark.parametrize("dtype,f_in,bits,qs", [("f32", 128, 8, "minmax"), ("f32", 100, 4, "minmax"),
                                                 ("bf16", 64, 4, "symmetric"), ("f32", 7, 8, "symmetric"),
                                                 ("bf16", 256, 8, "minmax"), ("f32", 1024, 8, "minmax")])
@pytest.mark.parametrize("delta,commit", [(True, "cur"), (False, "deq")])
def test_one_pass_message_build_equals_the_two_entry_points(dtype, f_in, bits, qs, delta, commit):
    """With a workspace of cdf_workspace_bytes the layer step tests and codes the halo rows in one pass;
    cdf_cache_filter followed by cdf_quantize is the two-pass route. Mask, row list, codes, meta and the
    committed cache must be bit-identical between the two."""
    from paper_2408_00232_amd import binding as B
    from paper_2408_00232_amd.layer import DeviceCsr, LayerBuffers
    w = configs.shrink(configs.TINY, 1500)
    P = configs.build_partition(w)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    QS = {"minmax": B.Q_MINMAX, "symmetric": B.Q_SYMMETRIC}[qs]
    CM = {"cur": B.COMMIT_CUR, "deq": B.COMMIT_DEQ}[commit]
    A = DeviceCsr(P.n_loc, P.n_loc + P.n_halo, P.rowptr, P.colidx, P.vals)
    L = LayerBuffers(A, None, P.n_loc, P.n_halo, f_in, 16, dtype=tdt, bits=bits, qs=QS, need_dx=False)
    g = torch.Generator().manual_seed(7)
    L.xfull.copy_(torch.randn(P.n_loc + P.n_halo, f_in, generator=g).to(tdt))
    cache0 = torch.randn(P.n_halo, f_in, generator=g)
    cache0[::17] = 0                                            # zero cached rows: sent on any difference
    amp = 0.04 * torch.rand(P.n_halo, 1, generator=g)           # per-row change: roughly half the rows pass the test
    fresh = cache0 * (1 + amp * torch.randn(P.n_halo, f_in, generator=g))
    fresh[::17] = torch.randn(fresh[::17].shape, generator=g)
    fresh[5::23] = cache0[5::23]                                # unchanged rows: never sent
    L.cache_sent.copy_(cache0.to(tdt))
    L.halo_fresh.copy_(fresh.to(tdt))
    L.W.copy_(torch.randn(f_in, 16, generator=g) * 0.1)
    # two-pass route on copies
    cache2 = L.cache_sent.clone()
    mask2 = torch.zeros_like(L.mask); idx2 = torch.zeros_like(L.idx); n2 = torch.zeros_like(L.n_sent)
    codes2 = torch.zeros_like(L.codes); meta2 = torch.zeros_like(L.meta)
    ws = torch.zeros(L.workspace_bytes(), dtype=torch.uint8, device="cuda")
    B.cdf_cache_filter(L.halo_fresh, cache2, 0.05, B.NORM_LINF, mask2, idx2, n2, ws)
    B.cdf_quantize(L.halo_fresh, cache2, idx2, n2, P.n_halo, bits, QS, CM, delta, codes2, meta2)
    B.cdf_gcn_layer_fwd(L.fwd_args(0.05, commit=CM, delta=delta), ws)
    torch.cuda.synchronize()
    n = int(L.n_sent.item())
    assert 0 < n < P.n_halo and n == int(n2.item())
    assert torch.equal(L.mask, mask2) and torch.equal(L.idx[:n], idx2[:n])
    assert torch.equal(L.codes[:n * L.row_bytes], codes2[:n * L.row_bytes])
    assert torch.equal(L.meta[:n].view(torch.int32), meta2[:n].view(torch.int32))
    it = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(L.cache_sent.view(it), cache2.view(it))


def test_captured_step_replays_like_the_eager_step():
    """The whole step (all layers forward and backward) captured as HIP graphs: every replay - with
    eager library work and synchronisations between the replays - must leave exactly the buffers
    the eager run leaves after the same step."""
    from paper_2408_00232_amd import binding as B
    from paper_2408_00232_amd.workload import Model
    w = configs.shrink(configs.MID, 3000)

    def snapshot(m):
        out = []
        for L in m.layers:
            out += [L.H.clone(), L.dW.clone(), L.n_sent.clone(), L.gn_sent.clone(), L.codes.clone(), L.gcodes.clone(),
                    L.cache_sent.clone(), L.gcache_sent.clone(), L.idx.clone()]
        return out

    eager = Model(w)
    want = []
    for t in range(8):
        eager.step(t)
        torch.cuda.synchronize()
        want.append(snapshot(eager))
    m = Model(w)
    for t in range(2):
        m.step(t)
    torch.cuda.synchronize()
    m.capture()
    a = torch.randn(100, 64, device="cuda")
    b = torch.zeros_like(a)
    for t in range(2, 8):
        m.step(t)
        B.cdf_relu_fwd(a, b)                      # unrelated eager work on the same stream
        torch.cuda.synchronize()
        got = snapshot(m)
        for x, y in zip(got, want[t]):
            assert torch.equal(x, y), f"replay of step {t} differs from the eager step"
        _ = (a @ a.t()).sum().item()              # a library call and a host read-back between replays


@pytest.mark.parametrize("dtype,dim,bits,qs,norm", [("f32", 128, 8, "minmax", "linf"), ("bf16", 96, 4, "symmetric", "linf"),
                                                     ("f32", 33, 8, "minmax", "linf"), ("f32", 64, 8, "minmax", "l2"),
                                                     ("f32", 1024, 8, "minmax", "l2"), ("f32", 602, 8, "symmetric", "l2"),
                                                     ("f32", 301, 4, "minmax", "l2"), ("bf16", 1024, 4, "minmax", "l2"),
                                                     ("bf16", 130, 8, "symmetric", "l2"), ("f32", 3, 8, "minmax", "l2"),
                                                     ("f32", 1, 8, "minmax", "l2"), ("f32", 64, 8, "none", "linf")])
def test_cache_filter_quantize_equals_the_two_calls(dtype, dim, bits, qs, norm):
    """cdf_cache_filter_quantize against cdf_cache_filter + cdf_quantize on copies of the same state:
    bit-identical outputs on its one-pass route (either norm; the L2 cases cover lane vectors of 4, 2
    and 1 elements, rows shorter and longer than a wavefront) and on the cases it hands to the two
    calls (unquantised messages, a workspace without room for the scratch)."""
    from paper_2408_00232_amd import binding as B
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    QS = {"minmax": B.Q_MINMAX, "symmetric": B.Q_SYMMETRIC, "none": B.Q_NONE}[qs]
    NM = {"linf": B.NORM_LINF, "l2": B.NORM_L2}[norm]
    R = 4321
    g = torch.Generator().manual_seed(11)
    cached0 = torch.randn(R, dim, generator=g)
    # per-row change sized so that about half the rows fail the test (the L2 ratio has no max over elements)
    amp = (0.04 if norm == "linf" else 0.1) * torch.rand(R, 1, generator=g)
    cur = (cached0 * (1 + amp * torch.randn(R, dim, generator=g))).to(tdt).cuda()
    rb = B.cdf_code_row_bytes(dim, bits, QS)
    full = B.cdf_workspace_bytes(R, dim, 0)
    for ws_bytes in (full, 4096):
        outs = []
        for one_call in (True, False):
            cached = cached0.to(tdt).cuda()
            mask = torch.zeros(R, dtype=torch.uint8, device="cuda")
            idx = torch.zeros(R, dtype=torch.int32, device="cuda")
            n = torch.zeros(1, dtype=torch.int32, device="cuda")
            codes = torch.zeros(R * rb, dtype=torch.uint8, device="cuda")
            meta = torch.zeros(R, 2, device="cuda")
            ws = torch.zeros(ws_bytes if one_call else full, dtype=torch.uint8, device="cuda")
            if one_call:
                B.cdf_cache_filter_quantize(cur, cached, 0.05, NM, bits, QS, B.COMMIT_CUR, True, mask, idx, n, codes, meta, ws)
            else:
                B.cdf_cache_filter(cur, cached, 0.05, NM, mask, idx, n, ws)
                B.cdf_quantize(cur, cached, idx, n, R, bits, QS, B.COMMIT_CUR, True, codes, meta)
            torch.cuda.synchronize()
            k = int(n.item())
            it = torch.int16 if dtype == "bf16" else torch.int32
            outs.append((k, mask.cpu(), idx[:k].cpu(), codes[:k * rb].cpu(), meta[:k].view(torch.int32).cpu(),
                         cached.view(it).cpu()))
        assert 0 < outs[0][0] < R
        for a, b in zip(*outs):
            assert (a == b) if isinstance(a, int) else torch.equal(a, b)


def test_look_back_wait_is_bounded(cdf, oracle):
    """The small-input route of cdf_cache_filter_quantize waits for its predecessors a bounded number of
    polls. With the bound forced down to one poll a call either completes as usual or reports -1 in
    *n_sent; it terminates either way, and with the default bound restored the same call is exact again."""
    R, F = 40000, 64
    cur, cached = make_pair(R, F, F, torch.float32, seed=77)
    dcur = cur.to(DEV)
    omask, oidx = oracle.cache_filter(to_np(cur), to_np(cached), 0.05, 0)
    ws = ws_for(cdf, R, F)
    rb = cdf.cdf_code_row_bytes(F, 8, 0)
    try:
        for limit in (1, 0):
            cdf.cdf_set_message_wait_limit(limit)
            for _ in range(3):
                dcached = cached.to(DEV)
                mask = torch.zeros(R, dtype=torch.uint8, device=DEV)
                idx = torch.zeros(R, dtype=torch.int32, device=DEV)
                n_sent = torch.full((1,), -7, dtype=torch.int32, device=DEV)
                codes = torch.zeros(R * rb, dtype=torch.uint8, device=DEV)
                meta = torch.zeros(R, 2, device=DEV)
                cdf.cdf_cache_filter_quantize(dcur, dcached, 0.05, 0, 8, 0, 1, True, mask, idx, n_sent, codes, meta, ws)
                torch.cuda.synchronize()
                n = int(n_sent.item())
                assert n == oidx.size or (limit == 1 and n == -1), n
                np.testing.assert_array_equal(to_np(mask), omask)       # the test itself never waits
                if n >= 0:
                    np.testing.assert_array_equal(to_np(idx)[:n], oidx)
                # a consumer sees "no messages" when the count is -1: nothing is applied, nothing faults
                dst = torch.zeros(R, F, device=DEV)
                cdf.cdf_dequantize(codes, meta, idx, n_sent, R, 8, 0, dst, True)
                torch.cuda.synchronize()
                if n < 0:
                    assert int((dst != 0).sum().item()) == 0
    finally:
        cdf.cdf_set_message_wait_limit(0)


@pytest.mark.parametrize("bits,qs", [(8, 0), (4, 0), (8, 1)])
def test_subnormal_and_extreme_rows_are_bit_exact(cdf, oracle, bits, qs):
    """fp32 subnormals are not flushed and extreme ranges take the same path on both sides: rows
    whose values, differences or min-max range are subnormal (so the reciprocal overflows), rows
    near the largest finite value, constant rows and single-outlier rows - masks, codes, meta,
    committed cache and recovered rows equal the oracle's bit for bit."""
    R, F = 96, 64
    g = torch.Generator().manual_seed(23)
    base = torch.randn(R, F, generator=g)
    scale = torch.ones(R, 1)
    scale[0:16] = 1e-40                      # subnormal values
    scale[16:32] = 3e-39                     # around the smallest normal
    scale[32:48] = 1e38                      # near overflow (differences may overflow to inf)
    scale[48:56] = 1e-30
    cur = base * scale
    cached = cur * (1 + 0.3 * torch.randn(R, F, generator=g))
    cached[56:64] = 0                        # zero cache
    cur[64:72] = 2.5e-41                     # constant subnormal rows (range 0)
    cached[64:72] = 0
    cur[72:80] = cached[72:80]               # unchanged rows
    cur[80:88] = 0
    cached[80:88] = 0
    cur[80:88, 7] = 1e-44                    # a single subnormal outlier against a zero cache
    cur, cached = cur.contiguous(), cached.contiguous()
    ncur, ncached = cur.numpy().copy(), cached.numpy().copy()
    dcur, dcached = cur.to(DEV), cached.to(DEV)
    mask = torch.zeros(R, dtype=torch.uint8, device=DEV)
    idx = torch.zeros(R, dtype=torch.int32, device=DEV)
    n_sent = torch.zeros(1, dtype=torch.int32, device=DEV)
    ws = ws_for(cdf, R, F)
    for norm in (0, 1):
        cdf.cdf_cache_filter(dcur, dcached, 0.05, norm, mask, idx, n_sent, ws)
        torch.cuda.synchronize()
        omask, oidx = oracle.cache_filter(ncur, ncached, 0.05, norm)
        np.testing.assert_array_equal(to_np(mask), omask)
    cdf.cdf_cache_filter(dcur, dcached, 0.05, 0, mask, idx, n_sent, ws)
    omask, oidx = oracle.cache_filter(ncur, ncached, 0.05, 0)
    n = oidx.size
    assert 40 < n < R
    rb = cdf.cdf_code_row_bytes(F, bits, qs)
    codes = torch.zeros(R * rb, dtype=torch.uint8, device=DEV)
    meta = torch.zeros(R, 2, device=DEV)
    cdf.cdf_quantize(dcur, dcached, idx, n_sent, R, bits, qs, 2, True, codes, meta)      # commit = recovered value
    dst = torch.zeros(R, F, device=DEV)
    cdf.cdf_dequantize(codes, meta, idx, n_sent, R, bits, qs, dst, accumulate=False)
    torch.cuda.synchronize()
    ocodes, ometa = oracle.quantize(ncur, ncached, oidx, bits, qs, 2, True)
    np.testing.assert_array_equal(to_np(codes)[:n * rb].reshape(n, rb), ocodes)
    np.testing.assert_array_equal(to_np(meta)[:n].view(np.uint32), ometa.view(np.uint32))
    np.testing.assert_array_equal(to_np(dcached).view(np.uint32), ncached.view(np.uint32))
    odst = np.zeros((R, F), np.float32)
    oracle.dequantize(ocodes, ometa, oidx, odst, bits, qs, accumulate=False)
    np.testing.assert_array_equal(to_np(dst).view(np.uint32), odst.view(np.uint32))
