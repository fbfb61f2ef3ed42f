"""Pins for the CPU oracle: each test fixes a piece of it to something other than
itself - a dense brute force from the edge list, finite differences, closed
forms of the quantiser, hand-built threshold rows, invariants of the cache.
"""
import os

import numpy as np
import pytest

from cdfgen import configs, features, graphs
from helpers import (assert_rows_close, bf16_bits, bf16_to_f32, csr_dense, csr_np, dense_norm_adj)

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def small_graph(n=200, seed=11):
    w = configs.shrink(configs.TINY, n)
    w.seed = seed
    return w, configs.build_graph(w)


def f32(a):
    return np.ascontiguousarray(a, np.float32)


# --------------------------------------------------------------------------
# Aggregation + transform against the dense definition (Sec. 3.1, Z = A^ H W)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("parts", [1, 4])
def test_forward_matches_dense_definition(oracle, parts):
    w, g = small_graph(256)
    Ad = dense_norm_adj(g)
    rs = np.random.default_rng(1)
    X = rs.standard_normal((g.n, 24))
    W = rs.standard_normal((24, 7)) * 0.3
    Zd = Ad @ X @ W
    for p in range(parts):
        P = graphs.extract_partition(g, graphs.range_mask(g.n, parts, p))
        own, halo = P.owned.numpy(), P.halo.numpy()
        xfull = f32(np.concatenate([X[own], X[halo]]))
        M = oracle.spmm(*csr_np(P), P.n_loc + P.n_halo, xfull)
        Z, H = oracle.dense_fwd(M, f32(W), relu=True)
        assert_rows_close(M, (Ad @ X)[own], rel=2e-6, frob=1e-6, what="M")
        assert_rows_close(Z, Zd[own], rel=2e-6, frob=1e-6, what="Z")
        np.testing.assert_array_equal(H, np.maximum(Z, 0))


def test_partition_blocks_are_the_dense_rows():
    """CSR block and its transpose reproduce the owned rows of the dense matrix."""
    w, g = small_graph(128)
    Ad = dense_norm_adj(g)
    P = graphs.extract_partition(g, graphs.range_mask(g.n, 4, 1))
    own, halo = P.owned.numpy(), P.halo.numpy()
    cols = np.concatenate([own, halo])
    D = csr_dense(*csr_np(P), P.n_loc + P.n_halo)
    np.testing.assert_allclose(D, Ad[np.ix_(own, cols)], rtol=1e-7, atol=0)
    # every non-zero of the owned rows is covered
    rest = np.setdiff1d(np.arange(g.n), cols)
    assert np.count_nonzero(Ad[np.ix_(own, rest)]) == 0
    Dt = csr_dense(*csr_np(P, True), P.n_loc)
    np.testing.assert_array_equal(Dt, D.T.astype(np.float32).astype(np.float64))


def test_adjoint_identity(oracle):
    w, g = small_graph(256)
    P = graphs.extract_partition(g, graphs.range_mask(g.n, 4, 0))
    rs = np.random.default_rng(2)
    X = f32(rs.standard_normal((P.n_loc + P.n_halo, 9)))
    Y = f32(rs.standard_normal((P.n_loc, 9)))
    AX = oracle.spmm(*csr_np(P), P.n_loc + P.n_halo, X)
    AtY = oracle.spmm(*csr_np(P, True), P.n_loc, Y)
    lhs = float((AX.astype(np.float64) * Y).sum())
    rhs = float((X.astype(np.float64) * AtY).sum())
    assert abs(lhs - rhs) <= 1e-5 * max(abs(lhs), 1.0)


def test_spmm_empty_rows_and_bf16_rounding(oracle):
    rowptr = np.array([0, 0, 2, 2, 3], np.int64)
    colidx = np.array([0, 2, 1], np.int32)
    vals = np.array([0.5, 0.25, 3.0], np.float32)
    X = f32([[1, 2], [3, 4], [5, 6]])
    Y = oracle.spmm(rowptr, colidx, vals, 3, X)
    np.testing.assert_array_equal(Y, f32([[0, 0], [1.75, 2.5], [0, 0], [9, 12]]))
    # bf16 storage: result is the exactly accumulated sum rounded once, ties to even (torch's cast)
    rs = np.random.default_rng(3)
    Xf = f32(rs.standard_normal((3, 33)))
    Xb = bf16_bits(Xf)
    Yb = oracle.spmm(rowptr, colidx, vals, 3, Xb)
    exact = csr_dense(rowptr, colidx, vals, 3) @ bf16_to_f32(Xb).astype(np.float64)
    np.testing.assert_array_equal(Yb, bf16_bits(exact.astype(np.float32)))


# --------------------------------------------------------------------------
# Back-propagation against central finite differences (chain rule of Sec. 3.1)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("relu", [False, True])
def test_backward_matches_finite_differences(oracle, relu):
    w, g = small_graph(96, seed=5)
    P = graphs.extract_partition(g, graphs.range_mask(g.n, 3, 1))
    nf = P.n_loc + P.n_halo
    Ad = csr_dense(*csr_np(P), nf)
    rs = np.random.default_rng(4)
    f, gdim = 6, 5
    X = f32(rs.standard_normal((nf, f))).astype(np.float64)
    W = f32(rs.standard_normal((f, gdim)) * 0.5).astype(np.float64)
    T = f32(rs.standard_normal((P.n_loc, gdim))).astype(np.float64)

    def loss(Xv, Wv):
        Z = Ad @ Xv @ Wv
        return float(((np.maximum(Z, 0) if relu else Z) * T).sum())

    h = 1e-6
    gW = np.zeros_like(W)
    for i in range(f):
        for j in range(gdim):
            Wp, Wm = W.copy(), W.copy()
            Wp[i, j] += h
            Wm[i, j] -= h
            gW[i, j] = (loss(X, Wp) - loss(X, Wm)) / (2 * h)
    gX = np.zeros_like(X)
    for i in range(nf):
        for j in range(f):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, j] += h
            Xm[i, j] -= h
            gX[i, j] = (loss(Xp, W) - loss(Xm, W)) / (2 * h)

    M = oracle.spmm(*csr_np(P), nf, f32(X))
    Z, H = oracle.dense_fwd(M, f32(W), relu)
    zero_cache = np.zeros((P.n_halo, f), np.float32)
    out = oracle.layer_bwd(csr_np(P, True), P.n_loc, P.n_halo, M, Z, f32(T), f32(W), zero_cache,
                           eps=0.0, relu=relu)
    assert_rows_close(out["dW"], gW, rel=2e-5, frob=1e-5, what="dW")
    # row-scaled with an absolute floor: rows whose gradient is exactly zero stay zero
    np.testing.assert_allclose(out["dxfull"], gX, rtol=0, atol=2e-5 * max(1.0, np.abs(gX).max()))


# --------------------------------------------------------------------------
# Cache test (Alg. 2): hand-built threshold rows, monotonicity, staleness bound
# --------------------------------------------------------------------------
def test_cache_test_threshold_rows(oracle):
    F = 8
    cached = np.zeros((7, F), np.float32)
    cur = np.zeros((7, F), np.float32)
    eps = np.float32(0.25)
    # row 0: both zero -> nothing to send
    # row 1: cached zero, any difference -> send (product form: D > eps*0)
    cur[1, 3] = 1e-30
    # row 2: D == eps*C exactly -> strict '>' keeps it cached
    cached[2, 0] = 4.0
    cur[2, :] = cached[2, :]
    cur[2, 5] = 1.0
    # row 3: one ulp above the threshold -> send
    cached[3, 0] = 4.0
    cur[3, :] = cached[3, :]
    cur[3, 5] = np.nextafter(np.float32(1.0), np.float32(2.0))
    # row 4: the largest |cached| element is negative; difference on that element
    cached[4, 2] = -8.0
    cur[4, 2] = -10.5          # D = 2.5 > 0.25*8 = 2 -> send
    # row 5: same, D = 1.5 < 2 -> keep
    cached[5, 2] = -8.0
    cur[5, 2] = -6.5
    # row 6: many small differences, none above threshold (L-inf ignores their number)
    cached[6, :] = 1.0
    cur[6, :] = 1.2
    mask, idx = oracle.cache_filter(cur, cached, float(eps), oracle.NORM_LINF)
    np.testing.assert_array_equal(mask, [0, 1, 0, 1, 1, 0, 0])
    np.testing.assert_array_equal(idx, [1, 3, 4])
    # L2 on row 6: ||d||^2 = 8*0.04 = 0.32 > eps^2 * 8 = 0.5 ? no -> keep; with eps = 0.15 -> 0.18 -> send
    m2, _ = oracle.cache_filter(cur[6:7], cached[6:7], 0.25, oracle.NORM_L2)
    m3, _ = oracle.cache_filter(cur[6:7], cached[6:7], 0.15, oracle.NORM_L2)
    assert m2[0] == 0 and m3[0] == 1


def test_cache_test_monotone_and_eps_zero(oracle):
    rs = np.random.default_rng(6)
    cached = f32(rs.standard_normal((500, 37)))
    cur = cached * f32(1 + rs.standard_normal((500, 1)) * 0.1 * rs.standard_normal((500, 37)))
    cur[::7] = cached[::7]                       # untouched rows
    prev = None
    for norm in (oracle.NORM_LINF, oracle.NORM_L2):
        prev = None
        for eps in (0.0, 0.01, 0.05, 0.2, 1.0):
            mask, idx = oracle.cache_filter(cur, cached, eps, norm)
            np.testing.assert_array_equal(idx, np.nonzero(mask)[0])
            if prev is not None:
                assert (mask <= prev).all()      # larger threshold never adds rows
            else:
                np.testing.assert_array_equal(mask, (cur != cached).any(1))
            prev = mask


def test_cache_linf_permutation_invariant_and_l2_matches_double(oracle):
    rs = np.random.default_rng(7)
    R, F = 2000, 300
    cached = f32(rs.standard_normal((R, F)))
    cur = f32(cached + rs.standard_normal((R, F)) * rs.uniform(0, 0.2, (R, 1)))
    perm = rs.permutation(F)
    m1, _ = oracle.cache_filter(cur, cached, 0.1, oracle.NORM_LINF)
    m2, _ = oracle.cache_filter(f32(cur[:, perm]), f32(cached[:, perm]), 0.1, oracle.NORM_LINF)
    np.testing.assert_array_equal(m1, m2)
    assert 0 < m1.sum() < R
    eps = 0.1
    d = (cur - cached).astype(np.float64)
    D2 = (d * d).sum(1)
    C2 = (cached.astype(np.float64) ** 2).sum(1)
    thr = (eps * eps) * C2
    ml2, _ = oracle.cache_filter(cur, cached, eps, oracle.NORM_L2)
    band = np.abs(D2 - thr) <= 1e-5 * thr
    np.testing.assert_array_equal(ml2[~band], (D2 > thr)[~band])
    assert band.mean() < 0.01 and 0 < ml2.sum() < R


def test_l2_summation_order_is_the_stated_one(oracle):
    """Values chosen so that the order of additions changes the fp32 sum.
    d has 4096 on chain 0 (square 2^24), ones on chains 1..255 and one more one on
    chain 0 (j = 256). Chain 0: fma(1, 1, 2^24) ties to even -> 2^24. Butterfly stride 1:
    2^24 + 1 -> 2^24 again, every other pair gives 2; from stride 2 on all sums are even
    and exact. D2 = 2^24 + 2*127 = 2^24 + 254. A left-to-right sum would give 2^24.
    The cached row's squares (on chains 44..49, far from the d entries) add exactly to
    2^24 + 254 or 2^24 + 252, and eps = 1, so the test reads D2 back to the last bit."""
    F = 512
    d = np.zeros(F, np.float32)
    d[0] = 4096.0
    d[1:257] = 1.0
    for extra, sent in (((15.0, 5.0, 2.0, 0.0), 0),        # 225 + 25 + 4      = 254 : D2 == C2
                        ((14.0, 6.0, 4.0, 2.0), 1)):       # 196 + 36 + 16 + 4 = 252 : D2 >  C2
        cached = np.zeros((1, F), np.float32)
        cached[0, 300] = 4096.0
        cached[0, 302:306] = extra
        cur = cached + d[None, :]
        np.testing.assert_array_equal(cur - cached, d[None, :])
        m, _ = oracle.cache_filter(cur, cached, 1.0, oracle.NORM_L2)
        assert m[0] == sent


def nan_rows():
    """Rows with NaN elements, hand-built: what the row maxima must make of them."""
    nan = np.float32(np.nan)
    cached = np.array([[1, 2, 4, -3], [1, 2, 4, -3], [1, 2, 4, -3], [0, 0, 0, 0], [1, nan, 4, -3]], np.float32)
    cur = cached.copy()
    cur[0] = [1, nan, 4, -3]          # only change is a NaN: the finite elements are unchanged -> not sent
    cur[1] = [1.5, nan, 4, -3]        # finite change 0.5 > 0.05 * 4 -> sent
    cur[2] = [nan, nan, nan, nan]     # nothing finite -> difference maximum stays 0 -> not sent
    cur[3] = [nan, 0, 0, 1e-3]        # zero cache: the finite difference decides -> sent
    cur[4] = [1, 2, 4, -3]            # NaN in the cache: dropped from both maxima, the rest is unchanged -> not sent
    return cur, cached


def test_nan_elements_are_dropped_by_the_row_maxima(oracle):
    """The stated behaviour for non-finite input (IEEE maxNum / minNum drop a NaN operand): LINF judges a
    row by its other elements; L2 sums become NaN and the row is not sent; the quantiser scales by the
    finite elements and gives a NaN element code 0."""
    cur, cached = nan_rows()
    mask, idx = oracle.cache_filter(cur, cached, 0.05, oracle.NORM_LINF)
    assert mask.tolist() == [0, 1, 0, 1, 0] and idx.tolist() == [1, 3]
    mask2, _ = oracle.cache_filter(cur, cached, 0.05, oracle.NORM_L2)
    assert mask2.tolist() == [0, 0, 0, 0, 0]
    codes, meta = oracle.quantize(cur, cached.copy(), idx, 8, oracle.Q_MINMAX, oracle.COMMIT_NONE, True)
    # row 1: m = (0.5, NaN, 0, 0) -> lo 0, hi 0.5; codes 255, 0 (NaN), 0, 0
    assert meta[0].tolist() == [0.0, 0.5] and codes[0].tolist() == [255, 0, 0, 0]
    # row 3: m = (NaN, 0, 0, 1e-3) -> lo 0, hi 1e-3; codes 0 (NaN), 0, 0, 255
    assert codes[1].tolist() == [0, 0, 0, 255] and meta[1, 0] == 0.0 and meta[1, 1] == np.float32(1e-3)


def test_staleness_bound_after_commits(oracle):
    """After test + commit, every row obeys ||cur - cached|| <= eps ||cached|| (premise of Lemma 2)."""
    rs = np.random.default_rng(8)
    R, F, eps = 300, 20, 0.08
    cached = np.zeros((R, F), np.float32)
    cur = f32(rs.standard_normal((R, F)))
    for t in range(6):
        mask, idx = oracle.cache_filter(cur, cached, eps)
        oracle.quantize(cur, cached, idx, qs=oracle.Q_NONE, commit=oracle.COMMIT_CUR)
        np.testing.assert_array_equal(cached[idx], cur[idx])
        D = np.abs(cur - cached).max(1)
        C = np.abs(cached).max(1)
        assert (D <= np.float32(eps) * C).all()
        again, _ = oracle.cache_filter(cur, cached, eps)
        assert again.sum() == 0
        cur = f32(cur * (1 + 0.1 * 0.5 ** t * rs.standard_normal((R, F))))


# --------------------------------------------------------------------------
# Quantiser (Sec. 5): closed forms, packing, error bound, message size
# --------------------------------------------------------------------------
def read_golden(name):
    rows = []
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line)
    return rows


def test_quantizer_hand_worked_cases(oracle):
    """Cases worked by hand from the two equations of Sec. 5 (levels 2^B - 1)."""
    cases = read_golden("quantizer_cases.txt")
    assert len(cases) >= 5
    for line in cases:
        bits, scheme, vals, want_codes, want_meta, want_deq = [s.strip() for s in line.split("|")]
        bits = int(bits)
        qs = {"minmax": oracle.Q_MINMAX, "symmetric": oracle.Q_SYMMETRIC}[scheme]
        m = f32([[float(v) for v in vals.split()]])
        codes, meta = oracle.quantize(m, None, np.array([0], np.int32), bits, qs, oracle.COMMIT_NONE)
        np.testing.assert_array_equal(codes[0], [int(b, 16) for b in want_codes.split()])
        np.testing.assert_array_equal(meta[0], f32([float(v) for v in want_meta.split()]))
        dst = np.zeros_like(m)
        oracle.dequantize(codes, meta, np.array([0], np.int32), dst, bits, qs, accumulate=False)
        np.testing.assert_array_equal(dst[0], f32([float(v) for v in want_deq.split()]))


@pytest.mark.parametrize("bits", [8, 4])
def test_quantizer_grid_rows_are_lossless(oracle, bits):
    """m_j = lo + k_j * 2^-e : codes are k_j and the round trip is exact."""
    rs = np.random.default_rng(9)
    Lv = (1 << bits) - 1
    for e in (0, 3, 10):
        F = 77
        k = rs.integers(0, Lv + 1, F)
        k[0], k[1] = 0, Lv
        lo = -3.0
        scale = 2.0 ** -e
        m = f32([lo + k * scale])
        # the per-row reciprocal Lv / range is not a power of two, so the product may miss
        # the integer by an ulp before +0.5 and floor; the codes must still be k exactly
        codes, meta = oracle.quantize(m, None, np.array([0], np.int32), bits, oracle.Q_MINMAX,
                                      oracle.COMMIT_NONE)
        got = codes[0] if bits == 8 else np.stack([codes[0] & 15, codes[0] >> 4], 1).ravel()[:F]
        np.testing.assert_array_equal(got, k)
        np.testing.assert_array_equal(meta[0], f32([lo, lo + Lv * scale]))
        dst = np.zeros_like(m)
        oracle.dequantize(codes, meta, np.array([0], np.int32), dst, bits, oracle.Q_MINMAX, False)
        np.testing.assert_array_equal(dst, m)


@pytest.mark.parametrize("bits,qs", [(8, 0), (4, 0), (8, 1), (4, 1)])
def test_quantizer_round_trip_error_bound(oracle, bits, qs):
    """|recover(quantise(m)) - m| <= scale/2 (Sec. 5's bound with 2^B - 1 levels)."""
    rs = np.random.default_rng(10)
    R, F = 400, 130
    m = f32(rs.standard_normal((R, F)) * np.exp(rs.uniform(-8, 8, (R, 1))))
    m[5] = 0.75                                    # constant row
    m[6] = 0.0
    idx = np.arange(R, dtype=np.int32)
    codes, meta = oracle.quantize(m, None, idx, bits, qs, oracle.COMMIT_NONE)
    assert codes.shape == (R, (F * bits + 7) // 8)  # B*L bits, + 2T bits of meta
    dst = np.zeros_like(m)
    oracle.dequantize(codes, meta, idx, dst, bits, qs, accumulate=False)
    if qs == 0:
        scale = (meta[:, 1].astype(np.float64) - meta[:, 0]) / ((1 << bits) - 1)
        np.testing.assert_array_equal(meta[:, 0], m.min(1))
        np.testing.assert_array_equal(meta[:, 1], m.max(1))
        mag = np.maximum(np.abs(meta[:, 0]), np.abs(meta[:, 1])).astype(np.float64)
    else:
        scale = meta[:, 0].astype(np.float64)
        mag = np.abs(m).max(1).astype(np.float64)
    err = np.abs(dst.astype(np.float64) - m).max(1)
    slack = scale / 2 * (1 + 2.0 ** -10) + 2 * np.spacing(mag.astype(np.float32)).astype(np.float64)
    assert (err <= slack).all()
    np.testing.assert_array_equal(dst[5], m[5])
    np.testing.assert_array_equal(dst[6], m[6])
    # the same rule evaluated exactly (double) obeys the bound without slack on a sample
    if qs == 0:
        for r in range(0, R, 50):
            lo, hi = float(m[r].min()), float(m[r].max())
            if hi == lo:
                continue
            Lv = (1 << bits) - 1
            q = np.floor(Lv * (m[r].astype(np.float64) - lo) / (hi - lo) + 0.5)
            back = (hi - lo) / Lv * q + lo
            assert np.abs(back - m[r]).max() <= (hi - lo) / Lv / 2 * (1 + 1e-12)


def test_message_size_matches_paper_formula(oracle):
    """B*L + 2T bits per vertex (T = 32): ceil(L*B/8) code bytes + 8 bytes of (min, max)."""
    for F in (1, 7, 100, 602):
        for bits in (4, 8):
            m = np.ones((1, F), np.float32)
            codes, meta = oracle.quantize(m, None, np.array([0], np.int32), bits, 0, 0)
            assert codes.nbytes == (F * bits + 7) // 8 and meta.nbytes == 8


def test_commit_modes(oracle):
    rs = np.random.default_rng(12)
    cur = f32(rs.standard_normal((10, 16)))
    idx = np.array([1, 4, 7], np.int32)
    base = f32(rs.standard_normal((10, 16)))
    c1 = base.copy()
    codes, meta = oracle.quantize(cur, c1, idx, 8, 0, oracle.COMMIT_CUR)
    np.testing.assert_array_equal(c1[idx], cur[idx])
    rest = np.setdiff1d(np.arange(10), idx)
    np.testing.assert_array_equal(c1[rest], base[rest])
    # DEQ: the sender's cache moves by exactly what a receiver adds
    c2 = base.copy()
    codes2, meta2 = oracle.quantize(cur, c2, idx, 8, 0, oracle.COMMIT_DEQ)
    np.testing.assert_array_equal(codes, codes2)
    recv = base.copy()
    oracle.dequantize(codes2, meta2, idx, recv, 8, 0, accumulate=True)
    np.testing.assert_array_equal(recv, c2)
    c3 = base.copy()
    oracle.quantize(cur, c3, idx, 8, 0, oracle.COMMIT_NONE)
    np.testing.assert_array_equal(c3, base)


def test_bf16_cache_and_quantizer(oracle):
    """bf16 storage widens exactly to fp32; commits store bf16 rows unchanged."""
    rs = np.random.default_rng(13)
    cur = bf16_bits(f32(rs.standard_normal((50, 40))))
    cached = bf16_bits(f32(rs.standard_normal((50, 40))))
    cached[::2] = cur[::2]
    mask, idx = oracle.cache_filter(cur, cached, 0.0)
    np.testing.assert_array_equal(idx, np.arange(1, 50, 2))
    mf, _ = oracle.cache_filter(bf16_to_f32(cur), bf16_to_f32(cached), 0.3)
    mb, idxb = oracle.cache_filter(cur, cached, 0.3)
    np.testing.assert_array_equal(mf, mb)
    cf = bf16_to_f32(cached).copy()
    codes_f, meta_f = oracle.quantize(bf16_to_f32(cur), cf, idxb, 4, 0, oracle.COMMIT_CUR)
    codes_b, meta_b = oracle.quantize(cur, cached, idxb, 4, 0, oracle.COMMIT_CUR)
    np.testing.assert_array_equal(codes_f, codes_b)
    np.testing.assert_array_equal(meta_f, meta_b)
    np.testing.assert_array_equal(cached[idxb], cur[idxb])


# --------------------------------------------------------------------------
# Invariant: threshold 0 with loss-less messages reproduces uncached training
# --------------------------------------------------------------------------
def test_eps_zero_equals_uncached(oracle):
    w, g = configs.TINY, configs.build_graph(configs.TINY)
    P = configs.build_partition(w, graph=g)
    A = csr_np(P)
    f_in, f_out = 32, 8
    local = features.normal_matrix(1, 1, P.n_loc, f_in).numpy()
    W = features.glorot(1, 2, f_in, f_out).numpy()
    stream = features.HaloStream(1, P.n_halo, f_in)
    xfull = np.concatenate([local, np.zeros((P.n_halo, f_in), np.float32)])
    xacc = xfull.copy()
    sent = np.zeros((P.n_halo, f_in), np.float32)
    sent2 = sent.copy()
    for t in range(4):
        fresh = stream.value().numpy().copy()
        if t == 2:
            fresh[::3] = sent[::3]               # some rows do not change: nothing is sent for them
        out = oracle.layer_fwd(A, P.n_loc, P.n_halo, xfull, fresh, sent, W, eps=0.0,
                               qs=oracle.Q_NONE, delta=False)
        ref_x = np.concatenate([local, fresh])
        M = oracle.spmm(*A, P.n_loc + P.n_halo, ref_x)
        Z, H = oracle.dense_fwd(M, W, True)
        np.testing.assert_array_equal(xfull, ref_x)
        np.testing.assert_array_equal(out["M"], M)
        np.testing.assert_array_equal(out["H"], H)
        if t == 2:
            assert out["mask"][::3].sum() == 0
        # delta-accumulate form: z~ + (z - z~) equals z only up to rounding
        out2 = oracle.layer_fwd(A, P.n_loc, P.n_halo, xacc, fresh, sent2, W, eps=0.0,
                                qs=oracle.Q_NONE, delta=True)
        np.testing.assert_array_equal(out2["mask"], out["mask"])
        assert_rows_close(xacc, ref_x, rel=4e-7, frob=1e-6)
        stream.advance()


def test_partitioned_training_step_equals_single_device():
    """Sec. 3.1's closing claim: with the halo exchanges done, parameter gradients of the
    partitioned run equal those of the single-device full-batch run. Two layers, four
    partitions stepped in turn, oracle routines only; compared with a dense float64 run."""
    import oracle as orc
    w, g = configs.TINY, configs.build_graph(configs.TINY)
    Ad = dense_norm_adj(g)
    n = g.n
    rs = np.random.default_rng(14)
    dims = [12, 10, 5]
    X = f32(rs.standard_normal((n, dims[0])))
    Ws = [f32(rs.standard_normal((dims[i], dims[i + 1])) * 0.4) for i in range(2)]
    T = f32(rs.standard_normal((n, dims[2])))
    # dense reference: loss = sum(H2 * T), H1 = relu(A X W0), H2 = A H1 W1
    M1 = Ad @ X
    Z1 = M1 @ Ws[0]
    H1 = np.maximum(Z1, 0)
    M2 = Ad @ H1
    dW1 = M2.T @ T
    dH1 = Ad.T @ (T @ Ws[1].T.astype(np.float64))
    dW0 = M1.T @ (dH1 * (Z1 > 0))

    parts = [graphs.extract_partition(g, graphs.range_mask(n, w.parts, p)) for p in range(w.parts)]
    # layer 1 forward on every partition (exact halo rows: threshold 0, loss-less, replace)
    H1p = np.zeros((n, dims[1]), np.float32)
    saved = []
    for P in parts:
        own, halo = P.owned.numpy(), P.halo.numpy()
        xfull = np.concatenate([X[own], np.zeros((P.n_halo, dims[0]), np.float32)])
        sent = np.zeros((P.n_halo, dims[0]), np.float32)
        o = orc.layer_fwd(csr_np(P), P.n_loc, P.n_halo, xfull, X[halo].copy(), sent, Ws[0], 0.0,
                          qs=orc.Q_NONE, delta=False)
        H1p[own] = o["H"]
        saved.append(o)
    saved2 = []
    for P in parts:
        own, halo = P.owned.numpy(), P.halo.numpy()
        xfull = np.concatenate([H1p[own], np.zeros((P.n_halo, dims[1]), np.float32)])
        sent = np.zeros((P.n_halo, dims[1]), np.float32)
        o = orc.layer_fwd(csr_np(P), P.n_loc, P.n_halo, xfull, H1p[halo].copy(), sent, Ws[1], 0.0,
                          qs=orc.Q_NONE, delta=False, relu=False)
        saved2.append(o)
    # backward layer 2: halo gradient rows travel to their owners as loss-less messages
    dH1p = np.zeros((n, dims[1]), np.float32)
    dW1p = np.zeros_like(dW1)
    for P, o in zip(parts, saved2):
        own, halo = P.owned.numpy(), P.halo.numpy()
        gsent = np.zeros((P.n_halo, dims[1]), np.float32)
        b = orc.layer_bwd(csr_np(P, True), P.n_loc, P.n_halo, o["M"], o["Z"], T[own], Ws[1], gsent, 0.0,
                          qs=orc.Q_NONE, relu=False)
        dW1p += b["dW"]
        dH1p[own] += b["dxfull"][:P.n_loc]
        recv = np.zeros((P.n_halo, dims[1]), np.float32)
        orc.dequantize(b["codes"], b["meta"], b["idx"], recv, qs=orc.Q_NONE, accumulate=True)
        dH1p[halo] += recv
    dW0p = np.zeros_like(dW0)
    for P, o in zip(parts, saved):
        own = P.owned.numpy()
        gsent = np.zeros((P.n_halo, dims[0]), np.float32)
        b = orc.layer_bwd(csr_np(P, True), P.n_loc, P.n_halo, o["M"], o["Z"], dH1p[own], Ws[0], gsent, 0.0,
                          qs=orc.Q_NONE, relu=True, need_dx=False)
        dW0p += b["dW"]
    assert_rows_close(H1p, H1, rel=1e-5, frob=1e-6, what="H1")
    assert_rows_close(dW1p, dW1, rel=1e-5, frob=2e-6, what="dW1")
    assert_rows_close(dH1p, dH1, rel=2e-5, frob=2e-6, what="dH1")
    assert_rows_close(dW0p, dW0, rel=2e-5, frob=5e-6, what="dW0")


# --------------------------------------------------------------------------
# Transform-first order: Z = A^ (X W)
# --------------------------------------------------------------------------
def test_transform_first_matches_dense_and_aggregate_first(oracle):
    """With exact halo rows both orders give the dense A^ X W, and their parameter gradients obey
    dW_aggregate_first = X_local^T dT_local + X_halo^T dT_halo (the same sum, regrouped)."""
    w, g = small_graph(256)
    Ad = dense_norm_adj(g)
    rs = np.random.default_rng(31)
    f, gd = 20, 6
    X = f32(rs.standard_normal((g.n, f)))
    W = f32(rs.standard_normal((f, gd)) * 0.3)
    R = f32(rs.standard_normal((g.n, gd)))
    Zd = Ad @ X.astype(np.float64) @ W.astype(np.float64)
    for p in range(4):
        P = graphs.extract_partition(g, graphs.range_mask(g.n, 4, p))
        own, halo = P.owned.numpy(), P.halo.numpy()
        tfull = np.zeros((P.n_loc + P.n_halo, gd), np.float32)
        T_halo, _ = oracle.dense_fwd(X[halo], W, relu=False)
        sent = np.zeros((P.n_halo, gd), np.float32)
        o = oracle.layer_tf_fwd(csr_np(P), P.n_loc, P.n_halo, X[own], tfull, T_halo, sent, W, 0.0,
                                qs=oracle.Q_NONE, delta=False, relu=True)
        assert_rows_close(o["Z"], Zd[own], rel=5e-6, frob=2e-6, what="Z transform-first")
        np.testing.assert_array_equal(o["H"], np.maximum(o["Z"], 0))
        np.testing.assert_array_equal(tfull[P.n_loc:], T_halo)
        # aggregate-first on the same partition
        xfull = np.concatenate([X[own], np.zeros((P.n_halo, f), np.float32)])
        sent2 = np.zeros((P.n_halo, f), np.float32)
        a = oracle.layer_fwd(csr_np(P), P.n_loc, P.n_halo, xfull, X[halo].copy(), sent2, W, 0.0,
                             qs=oracle.Q_NONE, delta=False, relu=True)
        assert_rows_close(o["Z"], a["Z"], rel=5e-6, frob=2e-6, what="orders agree")
        # backward: same upstream gradient, mask from the aggregate-first Z for both
        gs = np.zeros((P.n_halo, gd), np.float32)
        bt = oracle.layer_tf_bwd(csr_np(P, True), P.n_loc, P.n_halo, X[own], a["Z"], R[own], W, gs, 0.0,
                                 qs=oracle.Q_NONE, relu=True)
        gs2 = np.zeros((P.n_halo, f), np.float32)
        ba = oracle.layer_bwd(csr_np(P, True), P.n_loc, P.n_halo, a["M"], a["Z"], R[own], W, gs2, 0.0,
                              qs=oracle.Q_NONE, relu=True)
        dW_regrouped = bt["dW"].astype(np.float64) + X[halo].astype(np.float64).T @ bt["dtfull"][P.n_loc:]
        assert_rows_close(dW_regrouped, ba["dW"], rel=2e-5, frob=5e-6, what="dW regrouped")
        # dx_local of the transform-first step equals the local rows of dXfull
        assert_rows_close(bt["dx_local"], ba["dxfull"][:P.n_loc], rel=2e-5, frob=5e-6, what="dx_local")


@pytest.mark.parametrize("relu", [False, True])
def test_transform_first_backward_matches_finite_differences(oracle, relu):
    w, g = small_graph(96, seed=7)
    P = graphs.extract_partition(g, graphs.range_mask(g.n, 3, 2))
    n, h = P.n_loc, P.n_halo
    Ad = csr_dense(*csr_np(P), n + h)
    rs = np.random.default_rng(32)
    f, gd = 5, 4
    X = f32(rs.standard_normal((n, f))).astype(np.float64)
    W = f32(rs.standard_normal((f, gd)) * 0.5).astype(np.float64)
    Th = f32(rs.standard_normal((h, gd))).astype(np.float64)
    R = f32(rs.standard_normal((n, gd))).astype(np.float64)

    def loss(Xv, Wv, Tv):
        Z = Ad @ np.concatenate([Xv @ Wv, Tv])
        return float(((np.maximum(Z, 0) if relu else Z) * R).sum())

    def fd(arr, which):
        out = np.zeros_like(arr)
        for i in range(arr.shape[0]):
            for j in range(arr.shape[1]):
                a, b = arr.copy(), arr.copy()
                a[i, j] += 1e-6
                b[i, j] -= 1e-6
                args_a = {"X": X, "W": W, "T": Th}
                args_b = dict(args_a)
                args_a[which], args_b[which] = a, b
                out[i, j] = (loss(args_a["X"], args_a["W"], args_a["T"]) -
                             loss(args_b["X"], args_b["W"], args_b["T"])) / 2e-6
        return out

    tfull = np.zeros((n + h, gd), np.float32)
    sent = np.zeros((h, gd), np.float32)
    o = oracle.layer_tf_fwd(csr_np(P), n, h, f32(X), tfull, f32(Th), sent, f32(W), 0.0, qs=oracle.Q_NONE,
                            delta=False, relu=relu)
    gs = np.zeros((h, gd), np.float32)
    b = oracle.layer_tf_bwd(csr_np(P, True), n, h, f32(X), o["Z"], f32(R), f32(W), gs, 0.0, qs=oracle.Q_NONE,
                            relu=relu)
    tol = lambda ref: 2e-5 * max(1.0, np.abs(ref).max())
    gW, gX, gT = fd(W, "W"), fd(X, "X"), fd(Th, "T")
    np.testing.assert_allclose(b["dW"], gW, rtol=0, atol=tol(gW))
    np.testing.assert_allclose(b["dx_local"], gX, rtol=0, atol=tol(gX))
    np.testing.assert_allclose(b["dtfull"][n:], gT, rtol=0, atol=tol(gT))


# --------------------------------------------------------------------------
# Training-loop pieces: loss, optimiser, threshold controller
# --------------------------------------------------------------------------
def test_softmax_xent_closed_forms_and_gradient(oracle):
    # uniform logits: loss = ln C per row; gradient = (1/C - onehot)
    C = 7
    z = np.zeros((3, C), np.float32)
    y = np.array([0, 3, -1], np.int32)
    loss, d, nc, nl = oracle.softmax_xent(z, y)
    assert abs(loss - 2 * np.log(C)) < 1e-12 and nl == 2
    assert nc == 1                      # ties: the lowest index wins, so only label 0 counts as correct
    np.testing.assert_allclose(d[1], np.full(C, 1 / C) - np.eye(C)[3], atol=1e-7)
    assert not d[2].any()
    # a dominant logit: loss -> 0, gradient -> 0
    z = np.full((1, C), -50.0, np.float32)
    z[0, 2] = 50.0
    loss, d, nc, nl = oracle.softmax_xent(z, np.array([2], np.int32))
    assert loss < 1e-30 and np.abs(d).max() < 1e-30 and nc == 1
    # finite differences of the summed loss
    rs = np.random.default_rng(41)
    z = f32(rs.standard_normal((5, C)) * 2)
    y = np.array([1, 0, 6, -1, 3], np.int32)
    _, d, _, _ = oracle.softmax_xent(z, y, scale=0.5)
    for r in range(5):
        for c in range(C):
            zp, zm = z.astype(np.float64).copy(), z.astype(np.float64).copy()
            zp[r, c] += 1e-5
            zm[r, c] -= 1e-5

            def tot(a):
                m = a.max(1, keepdims=True)
                lse = np.log(np.exp(a - m).sum(1)) + m[:, 0]
                return sum(lse[i] - a[i, y[i]] for i in range(5) if y[i] >= 0)
            fd = 0.5 * (tot(zp) - tot(zm)) / 2e-5
            assert abs(d[r, c] - fd) < 2e-6


def test_adam_first_steps(oracle):
    """Step 1 moves every weight by lr * g / (|g| + eps): lr in magnitude when |g| >> eps."""
    g = f32([0.5, -2.0, 1e-3, 0.0])
    W = f32([1.0, 1.0, 1.0, 1.0])
    m = np.zeros(4, np.float32)
    v = np.zeros(4, np.float32)
    oracle.adam_step(W, g, m, v, lr=0.01, t=1)
    np.testing.assert_allclose(W, [0.99, 1.01, 1.0 - 0.01 * 1e-3 / (1e-3 + 1e-8), 1.0], rtol=0, atol=1e-7)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-6)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=3e-5)   # beta2 is the fp32 value nearest 0.999
    # second step with the same gradient: bias-corrected moments still equal g and g^2
    oracle.adam_step(W, g, m, v, lr=0.01, t=2)
    np.testing.assert_allclose(W[:2], [0.98, 1.02], rtol=0, atol=2e-7)


def test_eps_controller_hand_worked(oracle):
    rows = read_golden("eps_controller_cases.txt")
    assert len(rows) >= 8
    for line in rows:
        eps, acc, mean, want_eps, want_mean = [float(x) for x in line.split("|")]
        got_eps, got_mean = oracle.eps_update(eps, acc, mean)
        assert abs(got_eps - want_eps) < 2e-7 and abs(got_mean - want_mean) < 2e-7, line
    # the swapped reading exchanges the two actions
    e, _ = oracle.eps_update(0.05, 0.60, 0.50, swap=True)
    assert abs(e - 0.0525) < 2e-7
    e, _ = oracle.eps_update(0.05, 0.40, 0.50, swap=True)
    assert abs(e - 0.045) < 2e-7


# --------------------------------------------------------------------------
# The training loop (Alg. 1) around the layer step
# --------------------------------------------------------------------------
def _dense_gcn_training(Ad, X, y, train, Ws, lr, epochs):
    """Full-graph two-layer GCN, softmax cross-entropy on the train rows, Adam; float64 throughout."""
    Ws = [w.astype(np.float64) for w in Ws]
    m = [np.zeros_like(w) for w in Ws]
    v = [np.zeros_like(w) for w in Ws]
    rows = np.nonzero(train)[0]
    out = []
    for t in range(1, epochs + 1):
        M1 = Ad @ X
        Z1 = M1 @ Ws[0]
        H1 = np.maximum(Z1, 0)
        M2 = Ad @ H1
        Z2 = M2 @ Ws[1]
        zz = Z2[rows] - Z2[rows].max(1, keepdims=True)
        P = np.exp(zz) / np.exp(zz).sum(1, keepdims=True)
        loss = -np.log(P[np.arange(rows.size), y[rows]]).mean()
        acc = (Z2[rows].argmax(1) == y[rows]).mean()
        dZ2 = np.zeros_like(Z2)
        P[np.arange(rows.size), y[rows]] -= 1
        dZ2[rows] = P / rows.size
        dW1 = M2.T @ dZ2
        dH1 = Ad.T @ (dZ2 @ Ws[1].T)
        dW0 = M1.T @ (dH1 * (Z1 > 0))
        for k, gW in enumerate((dW0, dW1)):
            m[k] = 0.9 * m[k] + 0.1 * gW
            v[k] = 0.999 * v[k] + 0.001 * gW * gW
            Ws[k] = Ws[k] - lr * (m[k] / (1 - 0.9 ** t)) / (np.sqrt(v[k] / (1 - 0.999 ** t)) + 1e-8)
        out.append(dict(loss=loss, acc=acc, W=[w.copy() for w in Ws], logits=Z2, dW=[dW0, dW1]))
    return out


def test_training_loop_without_cache_equals_full_graph_training(oracle):
    """Sec. 3.1's equivalence, over whole epochs: with threshold 0 and loss-less difference messages
    the partitioned loop (forward, loss, backward with gradient messages to the owners, Adam)
    follows full-graph training on the dense normalised adjacency."""
    from cdfgen import labels as labelgen
    from helpers import oracle_parts
    from oracle import training
    w, g = small_graph(240, seed=5)
    n, classes, f0, f1 = g.n, 5, 12, 9
    Ad = dense_norm_adj(g)
    y = labelgen.planted_labels(g, classes, 77)
    X = labelgen.planted_features(y, f0, 77, signal=0.5).numpy()
    tm = labelgen.train_mask(n, 77).numpy()
    y = y.numpy()
    Ws = [features.glorot(77, 70, f0, f1).numpy(), features.glorot(77, 71, f1, classes).numpy()]
    parts = [graphs.extract_partition(g, graphs.range_mask(n, 3, p)) for p in range(3)]
    tr = training.Trainer(oracle_parts(parts), [(f0, f1), (f1, classes)], X, y, tm, Ws, eps=0.0, lr=0.01,
                          adaptive=False, qs=oracle.Q_NONE)
    ref = _dense_gcn_training(Ad, X.astype(np.float64), y, tm, Ws, 0.01, 4)
    halo_rows = sum(P.n_halo for P in parts)
    for t in range(4):
        st = tr.epoch()
        assert abs(st["loss"] - ref[t]["loss"]) < 2e-6 * max(1.0, ref[t]["loss"])
        assert st["train_acc"] == pytest.approx(ref[t]["acc"], abs=1.5 / tm.sum())
        assert_rows_close(st["logits"], ref[t]["logits"], rel=2e-4, frob=2e-5, what=f"logits {t}")
        for k in range(2):
            assert_rows_close(st["dW"][k], ref[t]["dW"][k], rel=5e-4, frob=5e-5, what=f"dW{k} epoch {t}")
            np.testing.assert_allclose(tr.W[k], ref[t]["W"][k], rtol=0, atol=2e-4)
        # layer-0 rows never change: after the first epoch only layer 1 sends in the forward pass
        assert st["sent_fwd"] <= (2 if t == 0 else 1) * halo_rows
    assert tr.history[1]["sent_fwd"] <= halo_rows


def test_training_loop_cache_reduces_messages_and_still_learns(oracle):
    """Alg. 2 inside the loop: a positive threshold sends fewer rows than threshold 0, the rows
    each reader aggregates with stay within the threshold of the owners' rows (product form of
    the test), and the loss still falls."""
    from cdfgen import labels as labelgen
    from helpers import oracle_parts
    from oracle import training
    w, g = small_graph(240, seed=6)
    n, classes, f0, f1 = g.n, 4, 10, 8
    y = labelgen.planted_labels(g, classes, 78)
    X = labelgen.planted_features(y, f0, 78, signal=0.6).numpy()
    tm = labelgen.train_mask(n, 78).numpy()
    Ws = [features.glorot(78, 70, f0, f1).numpy(), features.glorot(78, 71, f1, classes).numpy()]
    parts = [graphs.extract_partition(g, graphs.range_mask(n, 3, p)) for p in range(3)]
    runs = {}
    for eps in (0.0, 0.1):
        tr = training.Trainer(oracle_parts(parts), [(f0, f1), (f1, classes)], X, y.numpy(), tm, Ws, eps=eps, lr=0.02,
                              adaptive=False, qs=oracle.Q_NONE)
        hist = [tr.epoch() for _ in range(12)]
        runs[eps] = (tr, hist)
    sent0 = sum(h["sent_fwd"] + h["sent_bwd"] for h in runs[0.0][1])
    sent1 = sum(h["sent_fwd"] + h["sent_bwd"] for h in runs[0.1][1])
    assert sent1 < 0.8 * sent0
    tr, hist = runs[0.1]
    assert hist[-1]["loss"] < 0.9 * hist[0]["loss"]
    # staleness of the reader's copy of layer-1 inputs after the last epoch: <= eps * |cached row|
    for P, xf, c in zip(tr.parts, tr.xfull, tr.cache):
        np.testing.assert_allclose(xf[1][P.n_loc:], c[1], rtol=0, atol=1e-5)   # reader copy == sender cache


# --------------------------------------------------------------------------
# The paper's own framing: vertex-cut, master / mirror replicas, Alg. 2 in full
# --------------------------------------------------------------------------
def _vc_task(n, seed, p, classes, f0, f1, signal=0.5):
    from cdfgen import labels as labelgen, vertex_cut as vcut
    w, g = small_graph(n, seed=seed)
    y = labelgen.planted_labels(g, classes, seed)
    X = labelgen.planted_features(y, f0, seed, signal=signal).numpy()
    tm = labelgen.train_mask(g.n, seed).numpy()
    Ws = [features.glorot(seed, 70, f0, f1).numpy(), features.glorot(seed, 71, f1, classes).numpy()]
    part = vcut.hashed_edge_cut(g, p, seed)
    parts = vcut.extract_vertex_cut(g, part, vcut.choose_masters(g, part, p), p)
    return g, y.numpy(), X, tm, Ws, parts


def test_vertex_cut_blocks_sum_to_the_normalised_adjacency():
    from cdfgen import vertex_cut as vcut
    w, g = small_graph(150, seed=9)
    part = vcut.hashed_edge_cut(g, 3, 9)
    master = vcut.choose_masters(g, part, 3)
    parts = vcut.extract_vertex_cut(g, part, master, 3)
    A = np.zeros((g.n, g.n))
    owners = np.zeros(g.n, int)
    for i, P in enumerate(parts):
        v = P.vertices.numpy()
        A[np.ix_(v, v)] += csr_dense(P.rowptr.numpy(), P.colidx.numpy(), P.vals.numpy(), P.n)
        owners[v[:P.n_master]] += 1
        assert (master[P.vertices[:P.n_master]] == i).all() and (master[P.vertices[P.n_master:]] != i).all()
        md, mr = P.mirror_master_dev.numpy(), P.mirror_master_row.numpy()
        for k in range(P.n_mirror):                        # the mirror's record points at the same vertex
            assert parts[md[k]].vertices[mr[k]] == P.vertices[P.n_master + k] and mr[k] < parts[md[k]].n_master
    np.testing.assert_allclose(A, dense_norm_adj(g), atol=1e-7)
    assert (owners == 1).all()                             # every vertex has exactly one master


def test_vertex_cut_training_without_cache_equals_full_graph_training(oracle):
    """Sec. 3.2's claim: after gather and scatter the replicas hold what sequential training would.
    Threshold 0 and loss-less messages, four epochs against dense float64 training."""
    from helpers import oracle_vc_parts
    from oracle import vc_training
    g, y, X, tm, Ws, parts = _vc_task(240, 5, 3, 5, 12, 9)
    tr = vc_training.Trainer(oracle_vc_parts(parts), [(12, 9), (9, 5)], X, y, tm, Ws, eps=0.0, lr=0.01, adaptive=False,
                             qs=oracle.Q_NONE)
    ref = _dense_gcn_training(dense_norm_adj(g), X.astype(np.float64), y, tm, Ws, 0.01, 4)
    for t in range(4):
        st = tr.epoch()
        assert abs(st["loss"] - ref[t]["loss"]) < 2e-6 * max(1.0, ref[t]["loss"])
        assert_rows_close(st["logits"], ref[t]["logits"], rel=2e-4, frob=2e-5, what=f"logits {t}")
        for k in range(2):
            assert_rows_close(st["dW"][k], ref[t]["dW"][k], rel=5e-4, frob=5e-5, what=f"dW{k} epoch {t}")
            np.testing.assert_allclose(tr.W[k], ref[t]["W"][k], rtol=0, atol=2e-4)


def test_alg2_invariants_with_a_positive_threshold(oracle):
    """With loss-less messages and threshold 0.1, after every exchange: (a) the master's cached total
    equals the sum of the cached partial values of all replicas of the vertex; (b) every mirror's copy
    equals its master's total (any change activates the vertex and is scattered); and fewer rows
    travel than with threshold 0."""
    from helpers import oracle_vc_parts
    from oracle import vc_training
    g, y, X, tm, Ws, parts = _vc_task(240, 6, 3, 4, 10, 8, signal=0.6)
    oparts = oracle_vc_parts(parts)
    sent = {}
    for eps in (0.0, 0.1):
        tr = vc_training.Trainer(oparts, [(10, 8), (8, 4)], X, y, tm, Ws, eps=eps, lr=0.02, adaptive=False,
                                 qs=oracle.Q_NONE)
        hist = [tr.epoch() for _ in range(10)]
        sent[eps] = sum(h["gather"] + h["scatter"] for h in hist)
        for st in tr.zs + tr.ds[1:]:
            dim = st.zc[0].shape[1]
            total = np.zeros((g.n, dim))
            for P, zc in zip(oparts, st.zc):
                np.add.at(total, P.vertices, zc.astype(np.float64))
            for P, tot in zip(oparts, st.tot):
                scale = np.abs(total[P.vertices]).max() + 1e-30
                np.testing.assert_allclose(tot[:P.n_master], total[P.vertices[:P.n_master]], rtol=0, atol=3e-5 * scale)
                for k in range(P.n_mirror):
                    assert np.array_equal(tot[P.n_master + k], oparts[P.mdev[k]].tot_row(st, P.mrow[k]))
        assert hist[-1]["loss"] < 0.9 * hist[0]["loss"]
    assert sent[0.1] < 0.8 * sent[0.0]
