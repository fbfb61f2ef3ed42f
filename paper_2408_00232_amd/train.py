"""Train all partitions of a seeded workload on one GPU and print the per-epoch curves the
paper plots for its cache (Sec. 7, hit rate and threshold over epochs): threshold, cache hit
rate, message volume, loss and train accuracy.

    python -m paper_2408_00232_amd.train --workload mid --epochs 100
    python -m paper_2408_00232_amd.train --workload mid --epochs 100 --eps0 0 --fixed --qscheme none   # no cache, fp32 messages
    python -m paper_2408_00232_amd.train --workload mid --epochs 100 --framing vertex-cut             # Alg. 2 in full, EBV partition
"""
import argparse
import json
import time

import torch

from cdfgen import configs

from . import binding as B
from .trainer import Trainer
from .vc_trainer import VcTrainer


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="tiny", choices=sorted(configs.ALL))
    ap.add_argument("--vertices", type=int, default=0, help="shrink the workload to this many vertices")
    ap.add_argument("--epochs", type=int, default=50)
    ap.add_argument("--eps0", type=float, default=None, help="starting threshold (default: the workload's)")
    ap.add_argument("--fixed", action="store_true", help="keep the threshold fixed (controller off)")
    ap.add_argument("--swap-conditions", action="store_true",
                    help="controller follows the prose of Sec. 4.1 instead of its printed case equation")
    ap.add_argument("--qscheme", default=None, choices=["minmax", "symmetric", "none"])
    ap.add_argument("--bits", type=int, default=None, choices=[4, 8])
    ap.add_argument("--lr", type=float, default=0.01)
    ap.add_argument("--every", type=int, default=1, help="print every k-th epoch")
    ap.add_argument("--framing", default="halo", choices=["halo", "vertex-cut"],
                    help="halo: owned rows + halo rows per partition; vertex-cut: master / mirror replicas (Sec. 3.2)")
    ap.add_argument("--devices-per-host", type=int, default=0, help="vertex-cut: hosts for the partitioner's gamma term")
    ap.add_argument("--gamma", type=float, default=0.1)
    ap.add_argument("--streams", type=int, default=1, help="halo framing: streams the partitions of a phase are spread over")
    ap.add_argument("--gen-device", default="cpu", help="where the seeded inputs are generated (cpu or cuda:0)")
    ap.add_argument("--json", action="store_true", help="one JSON object per printed epoch")
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        raise SystemExit("train: no GPU visible - the training loop runs in libcdf's kernels only")
    w = configs.ALL[a.workload]
    if a.vertices:
        w = configs.shrink(w, a.vertices)
    params = None
    if a.swap_conditions:
        params = B.cdf_eps_params(0.001, 0.02, 0.3, 0.001, 0.01, 1.05, 0.9, 1)
    t0 = time.time()
    vc = a.framing == "vertex-cut"
    if vc:
        g = configs.build_graph(w)
        dph = a.devices_per_host or w.parts
        part = B.cdf_ebv_partition(g.n, g.lo.contiguous(), g.hi.contiguous(), w.parts, dph, 1.0, 1.0, a.gamma, True)
        st, _ = B.cdf_cut_statistics(g.n, g.lo.contiguous(), g.hi.contiguous(), part, w.parts, dph)
        tr = VcTrainer(w, eps0=a.eps0, lr=a.lr, adaptive=not a.fixed, eps_params=params, qscheme=a.qscheme, bits=a.bits,
                       edge_part=part, graph=g)
        torch.cuda.synchronize()
        print(f"# {w.name}: {tr.n} vertices on {tr.p} devices ({dph} per host), layers {w.dims}, {tr.n_train} train rows, "
              f"replication factor {st.replication_factor:.3f}, edge imbalance {st.edge_imbalance:.4f}, "
              f"{sum(P.n_mirror for P in tr.parts)} mirrors, set-up {time.time() - t0:.1f} s", flush=True)
    else:
        tr = Trainer(w, eps0=a.eps0, lr=a.lr, adaptive=not a.fixed, eps_params=params, qscheme=a.qscheme, bits=a.bits,
                     gen_device=a.gen_device, streams=a.streams)
        torch.cuda.synchronize()
        print(f"# {w.name}: {tr.n} vertices, {tr.p} partitions, layers {w.dims}, {tr.n_train} train rows, "
              f"{sum(P.n_halo for P in tr.parts)} halo rows, set-up {time.time() - t0:.1f} s", flush=True)
    if not a.json:
        print("# epoch     eps  hit_rate   " + ("gather   scatter" if vc else "sent_fwd  sent_bwd") +
              "     MB_sent      loss  train_acc   ms")
    total_bytes = 0
    for e in range(a.epochs):
        torch.cuda.synchronize()
        t1 = time.time()
        st = tr.epoch()
        torch.cuda.synchronize()
        ms = (time.time() - t1) * 1e3
        total_bytes += st.message_bytes
        if e % a.every and e + 1 != a.epochs:
            continue
        c1, c2 = (st.gather, st.scatter) if vc else (st.sent_fwd, st.sent_bwd)
        if a.json:
            print(json.dumps(dict(epoch=e, eps=st.eps, hit_rate=st.hit_rate, sent_a=c1, sent_b=c2,
                                  message_bytes=st.message_bytes, loss=st.loss, train_acc=st.train_acc, ms=ms)),
                  flush=True)
        else:
            print(f"{e:7d} {st.eps:7.4f} {st.hit_rate:9.4f} {c1:9d} {c2:9d} "
                  f"{st.message_bytes / 1e6:11.3f} {st.loss:9.5f} {st.train_acc:10.4f} {ms:6.1f}", flush=True)
    tail = "" if vc else f"accuracy over all vertices {tr.accuracy_all():.4f}; "
    print(f"# {tail}messages {total_bytes / 1e6:.1f} MB in {a.epochs} epochs", flush=True)


if __name__ == "__main__":
    main()
