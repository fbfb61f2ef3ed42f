"""Self-checks of the seeded input generators (input data only)."""
import numpy as np
import torch

from cdfgen import configs, features, graphs, rng


def test_streams_are_deterministic_and_distinct():
    c = torch.arange(1000, dtype=torch.int64)
    a = rng.bits64(5, 1, c)
    assert torch.equal(a, rng.bits64(5, 1, c))
    assert not torch.equal(a, rng.bits64(5, 2, c))
    assert not torch.equal(a, rng.bits64(6, 1, c))
    # batching does not change values
    assert torch.equal(a[500:], rng.bits64(5, 1, c[500:]))
    u = rng.uniform01(5, 1, torch.arange(200000, dtype=torch.int64))
    assert 0.0 < float(u.min()) and float(u.max()) < 1.0
    assert abs(float(u.mean()) - 0.5) < 5e-3
    z = rng.normal(5, 3, 200000)
    assert abs(float(z.mean())) < 1e-2 and abs(float(z.std()) - 1.0) < 1e-2


def test_tiny_graph_shape_and_normalisation():
    w = configs.TINY
    g = configs.build_graph(w)
    assert g.n == 2048 and int((g.lo >= g.hi).sum()) == 0
    assert torch.unique(g.lo * g.n + g.hi).numel() == g.lo.numel()
    total = 0
    seen = torch.zeros(g.n, dtype=torch.bool)
    for p in range(w.parts):
        P = configs.build_partition(w, part=p, graph=g)
        assert P.n_loc == 512 and not seen[P.owned].any()
        seen[P.owned] = True
        total += P.nnz
        rp, ci, v = P.rowptr.numpy(), P.colidx.numpy(), P.vals.numpy()
        assert rp[0] == 0 and rp[-1] == P.nnz and (np.diff(rp) >= 1).all()      # self-loop in every row
        for i in range(0, P.n_loc, 37):
            row = ci[rp[i]:rp[i + 1]]
            assert (np.diff(row) > 0).all() and i in row
            assert rp[i + 1] - rp[i] == int(g.deg[P.owned[i]])
        # weights: 1/sqrt(d_u d_v) with global degrees
        allid = torch.cat([P.owned, P.halo])
        rows = np.repeat(np.arange(P.n_loc), np.diff(rp))
        du = g.deg[P.owned].numpy()[rows].astype(np.float64)
        dv = g.deg[allid].numpy()[ci].astype(np.float64)
        np.testing.assert_array_equal(v, (1.0 / np.sqrt(du * dv)).astype(np.float32))
        # halo columns are exactly the non-owned neighbours; transpose has the same entries
        assert set(np.unique(ci[ci >= P.n_loc]) - P.n_loc) == set(range(P.n_halo))
        assert P.t_rowptr[-1] == P.nnz and P.t_colidx.max() < P.n_loc
    assert seen.all() and total == g.nnz


def test_bfs_partition_is_balanced_and_total():
    w = configs.shrink(configs.LARGE, 6000)
    g = configs.build_graph(w)
    own = graphs.bfs_grown_owner(g, w.parts, w.seed)
    cnt = torch.bincount(own, minlength=w.parts)
    assert int(own.min()) >= 0 and int(cnt.max()) <= -(-g.n // w.parts) and int(cnt.sum()) == g.n
    assert torch.equal(own, graphs.bfs_grown_owner(g, w.parts, w.seed))


def test_halo_stream_drift_shrinks():
    s = features.HaloStream(3, 400, 16)
    prev = s.value().clone()
    steps = []
    for _ in range(5):
        cur = s.advance()
        steps.append(float(((cur - prev).abs().amax(1) / prev.abs().amax(1)).median()))
        prev = cur.clone()
    assert all(a > b for a, b in zip(steps, steps[1:]))
