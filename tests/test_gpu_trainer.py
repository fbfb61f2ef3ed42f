"""The training loop on the device (all partitions of a workload stepped on one GPU through
libcdf) against the oracle's training loop on the same seeded task."""
import numpy as np
import pytest
import torch

from cdfgen import configs
from helpers import assert_rows_close, oracle_parts

pytestmark = pytest.mark.gpu


def _pair(w, oracle, **kw):
    from oracle import training
    from paper_2408_00232_amd import binding as B
    from paper_2408_00232_amd.trainer import Trainer
    qname = kw.pop("qscheme", w.qscheme)
    tr = Trainer(w, device="cuda:0", keep_inputs=True, qscheme=qname, **kw)
    I = tr.inputs
    qs = {"minmax": oracle.Q_MINMAX, "symmetric": oracle.Q_SYMMETRIC, "none": oracle.Q_NONE}[qname]
    ref = training.Trainer(oracle_parts(tr.parts), w.layers(), I["x0"].numpy(), I["labels"].numpy(),
                           I["train"].numpy(), [W.cpu().numpy() for W in tr.W], eps=tr.eps, lr=tr.lr,
                           adaptive=tr.adaptive, qs=qs, bits=tr.bits)
    return tr, ref


def _logits_by_vertex(tr):
    out = np.zeros((tr.n, tr.classes), np.float32)
    out[tr.vertex_of_slot.numpy()] = tr.logits.cpu().numpy()
    return out


@pytest.mark.parametrize("n", [600, 2048])
def test_uncached_lossless_epochs_follow_the_oracle(oracle, n):
    """Threshold 0, unquantised difference messages: every epoch within the float tolerance."""
    w = configs.shrink(configs.TINY, n) if n != configs.TINY.n_vertices else configs.TINY
    tr, ref = _pair(w, oracle, eps0=0.0, adaptive=False, qscheme="none")
    for t in range(4):
        st, rs = tr.epoch(), ref.epoch()
        assert st.sent_fwd == rs["sent_fwd"] or t > 0
        assert abs(st.loss - rs["loss"]) <= 1e-5 * max(1.0, rs["loss"])
        assert abs(st.train_acc - rs["train_acc"]) <= 2.0 / tr.n_train
        assert_rows_close(_logits_by_vertex(tr), rs["logits"], rel=2e-4, frob=2e-5, what=f"logits epoch {t}")
        for l in range(tr.L):
            assert_rows_close(tr.pl[0][l].dW.cpu().numpy(), rs["dW"][l], rel=5e-4, frob=5e-5, what=f"dW{l} epoch {t}")
            np.testing.assert_allclose(tr.W[l].cpu().numpy(), ref.W[l], rtol=0, atol=1e-4)


def test_first_epoch_with_cache_and_quantiser_is_exact_where_it_must_be(oracle):
    """Epoch 0 from identical state: the sent-row counts of every layer and partition are equal
    (all caches start at zero, so every nonzero row is sent), and values agree to tolerance."""
    w = configs.shrink(configs.TINY, 900)
    tr, ref = _pair(w, oracle, eps0=0.05, adaptive=False)
    st, rs = tr.epoch(), ref.epoch()
    assert st.sent_fwd == rs["sent_fwd"]
    assert abs(st.sent_bwd - rs["sent_bwd"]) <= 2          # a gradient row that is exactly zero on one side only
    assert abs(st.message_bytes - rs["message_bytes"]) <= 2 * 64
    # Layer-1 inputs differ in the last bits between the two sides (fp32 MFMA vs the oracle's
    # double accumulation), which moves a few 8-bit codes by one step = (hi - lo) / 255 of their row:
    # the bound below is a handful of such steps, far under what a wrong step would cause.
    assert_rows_close(_logits_by_vertex(tr), rs["logits"], rel=1e-2, frob=5e-4, what="logits")
    for l in range(tr.L):
        assert_rows_close(tr.pl[0][l].dW.cpu().numpy(), rs["dW"][l], rel=1e-2, frob=1e-3, what=f"dW{l}")


def test_adaptive_run_tracks_the_oracle_and_saves_messages(oracle):
    """Free-running adaptive training (8-bit messages, controller on): threshold and hit-rate
    curves stay close to the oracle's, messages fall well below the uncached count, and the loss
    falls. Trajectories are compared loosely: one flipped cache decision changes later epochs."""
    w = configs.TINY
    tr, ref = _pair(w, oracle, eps0=0.01, adaptive=True, lr=0.02)
    E = 25
    for t in range(E):
        st, rs = tr.epoch(), ref.epoch()
        assert abs(st.eps - rs["eps"]) <= 0.0101, (t, st.eps, rs["eps"])
        assert abs(st.loss - rs["loss"]) <= 0.02 * max(1.0, rs["loss"]), (t, st.loss, rs["loss"])
        assert abs(st.train_acc - rs["train_acc"]) <= 0.03
        tot = st.rows_fwd + st.rows_bwd
        assert abs((st.sent_fwd + st.sent_bwd) - (rs["sent_fwd"] + rs["sent_bwd"])) <= 0.05 * tot
    h = tr.history
    assert h[-1].loss < 0.9 * h[0].loss
    assert sum(x.sent_fwd + x.sent_bwd for x in h[1:]) < 0.9 * sum(x.rows_fwd + x.rows_bwd for x in h[1:])
    assert 0.0 <= tr.accuracy_all() <= 1.0


def test_gather_rows_and_map_index():
    from paper_2408_00232_amd import binding as B
    g = torch.Generator().manual_seed(3)
    for dt, dim in ((torch.float32, 128), (torch.float32, 7), (torch.bfloat16, 10), (torch.bfloat16, 5),
                    (torch.float32, 2)):
        src = torch.randn(1000, dim, generator=g).to(dt).cuda()
        idx = torch.randint(0, 1000, (777,), generator=g, dtype=torch.int32).cuda()
        dst = torch.zeros(780, dim, dtype=dt, device="cuda")
        B.cdf_gather_rows(src, idx, dst)
        torch.cuda.synchronize()
        assert torch.equal(dst[:777].cpu(), src.cpu()[idx.cpu().long()])
        assert not dst[777:].any()
    wide = torch.randn(500, 64, generator=g).cuda()
    view = wide[:, 8:40]                                   # leading dimension above the row width
    idx = torch.randint(0, 500, (300,), generator=g, dtype=torch.int32).cuda()
    dst = torch.zeros(300, 32, device="cuda")
    B.cdf_gather_rows(view, idx, dst)
    assert torch.equal(dst.cpu(), view.cpu()[idx.cpu().long()])
    mp = torch.randint(0, 10**6, (1000,), generator=g, dtype=torch.int32).cuda()
    out = torch.full((777,), -1, dtype=torch.int32, device="cuda")
    ns = torch.tensor([500], dtype=torch.int32, device="cuda")
    idx = torch.randint(0, 1000, (777,), generator=g, dtype=torch.int32).cuda()
    B.cdf_map_index(idx, ns, mp, out)
    assert torch.equal(out[:500].cpu(), mp.cpu()[idx[:500].cpu().long()])
    assert (out[500:] == -1).all()
    B.cdf_gather_rows(view, idx[:0], dst)                  # empty list: nothing happens


def test_single_partition_has_no_halo_and_still_trains(oracle):
    """Degenerate case: one partition owns everything, there is nothing to exchange."""
    from dataclasses import replace
    w = replace(configs.shrink(configs.TINY, 500), parts=1)
    tr, ref = _pair(w, oracle, eps0=0.05, adaptive=False)
    assert tr.parts[0].n_halo == 0
    for t in range(3):
        st, rs = tr.epoch(), ref.epoch()
        assert st.sent_fwd == st.sent_bwd == 0 and st.hit_rate == 1.0
        assert abs(st.loss - rs["loss"]) <= 1e-5 * max(1.0, rs["loss"])
        assert_rows_close(_logits_by_vertex(tr), rs["logits"], rel=2e-4, frob=2e-5, what=f"logits epoch {t}")


def test_streams_do_not_change_the_result(oracle):
    """The partitions' layer steps of a phase spread over four streams: every buffer equals the
    single-stream run bit for bit (the partitions do not touch each other's rows, sums keep their order)."""
    from paper_2408_00232_amd.trainer import Trainer
    w = configs.shrink(configs.TINY, 1500)
    a = Trainer(w, eps0=0.05, adaptive=True, lr=0.02)
    b = Trainer(w, eps0=0.05, adaptive=True, lr=0.02, streams=4)
    for t in range(6):
        sa, sb = a.epoch(), b.epoch()
        assert (sa.sent_fwd, sa.sent_bwd, sa.eps, sa.loss) == (sb.sent_fwd, sb.sent_bwd, sb.eps, sb.loss)
        assert torch.equal(a.logits, b.logits)
        for l in range(a.L):
            assert torch.equal(a.W[l], b.W[l])
