"""Partition a seeded workload graph with the hierarchical EBV vertex-cut (Sec. 6) and print the
statistics of the paper's partition table (Sec. 7 ablation): inner / outer connections, replication
factor, edge imbalance. CPU only.

    python -m paper_2408_00232_amd.partition --workload mid --hosts 2 --devices-per-host 4
"""
import argparse
import time

import torch

from cdfgen import configs, rng

from . import binding as B


def hashed_edge_cut(g, p, seed):
    """Baseline: every edge to a hashed device (random vertex-cut)."""
    return (rng.uniform01(seed, 90, torch.arange(g.lo.numel(), dtype=torch.int64)) * p).to(torch.int32).clamp_(0, p - 1)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="mid", choices=sorted(configs.ALL))
    ap.add_argument("--vertices", type=int, default=0, help="shrink the workload to this many vertices")
    ap.add_argument("--hosts", type=int, default=2)
    ap.add_argument("--devices-per-host", type=int, default=4)
    ap.add_argument("--alpha", type=float, default=1.0)
    ap.add_argument("--beta", type=float, default=1.0)
    ap.add_argument("--gammas", type=float, nargs="+", default=[0.0, 0.1])
    ap.add_argument("--listed-order", action="store_true", help="do not sort the edges by degree sum")
    a = ap.parse_args(argv)
    w = configs.ALL[a.workload]
    if a.vertices:
        w = configs.shrink(w, a.vertices)
    g = configs.build_graph(w)
    p, dph = a.hosts * a.devices_per_host, a.devices_per_host
    eu, ev = g.lo.contiguous(), g.hi.contiguous()
    print(f"# {w.name}: |V| = {g.n}, |E| = {eu.numel()} undirected edges, {a.hosts} hosts x {dph} devices")
    print("# method            inner      outer       RF   edge_IF  vertex_IF   seconds")
    rows = []
    for gamma in a.gammas:
        t0 = time.time()
        part = B.cdf_ebv_partition(g.n, eu, ev, p, dph, a.alpha, a.beta, gamma, not a.listed_order)
        dt = time.time() - t0
        st, _ = B.cdf_cut_statistics(g.n, eu, ev, part, p, dph)
        rows.append((f"EBV gamma={gamma:g}", st, dt))
    t0 = time.time()
    part = hashed_edge_cut(g, p, w.seed)
    st, _ = B.cdf_cut_statistics(g.n, eu, ev, part, p, dph)
    rows.append(("hashed edges", st, time.time() - t0))
    for name, st, dt in rows:
        print(f"{name:<16} {st.max_inner:9d} {st.max_outer:10d} {st.replication_factor:8.4f} {st.edge_imbalance:9.4f} "
              f"{st.vertex_imbalance:10.4f} {dt:9.2f}")


if __name__ == "__main__":
    main()
