#!/usr/bin/env python3
"""Benchmark of the per-partition GCN layer step on one MI355X.

A step = the whole hot path over the model of the chosen workload: for every layer the
forward step (cache test, message build, recovery, aggregation, dense transform) and the
backward step (dense gradients, transposed aggregation, cache test and message build on the
halo gradients). value = edges traversed per second = layers * nnz / step time, inputs
resident in HBM. One JSON line on stdout; progress on stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def spmm_bytes(rows_out, rows_in, nnz, dim, esz):
    """Algorithmic bytes of one aggregation launch: the CSR arrays, every needed input row once,
    every output row once (compulsory traffic), and the same with no reuse of input rows."""
    csr = 8 * (rows_out + 1) + 8 * nnz
    out = rows_out * dim * esz
    return csr + out + rows_in * dim * esz, csr + out + nnz * dim * esz


def cpu_baseline(model, budget_edges=12_000_000):
    """The oracle, as it stands, on a bounded sample of the same workload: every k-th local row of
    the partition (with all columns those rows touch), one stationary step of all layers."""
    import numpy as np
    import torch
    import oracle

    P, w = model.P, model.w
    oracle.build()
    cores = min(os.cpu_count() or 1, 16)
    oracle.set_threads(cores)
    stride = max(1, int(round(P.nnz / budget_edges)))
    rows = torch.arange(0, P.n_loc, stride, device=P.rowptr.device)
    lens = (P.rowptr[rows + 1] - P.rowptr[rows])
    ptr = torch.zeros(rows.numel() + 1, dtype=torch.int64, device=rows.device)
    torch.cumsum(lens, 0, out=ptr[1:])
    nnz_s = int(ptr[-1])
    seg = torch.repeat_interleave(torch.arange(rows.numel(), device=rows.device), lens)
    pos = torch.arange(nnz_s, device=rows.device) - ptr[seg] + P.rowptr[rows][seg]
    cols = P.colidx[pos].long()
    vals = P.vals[pos]
    # local ids: sampled rows first (they stay "local"), every other touched column is halo
    n_s = rows.numel()
    lid = torch.full((P.n_loc + P.n_halo,), -1, dtype=torch.int64, device=rows.device)
    lid[rows] = torch.arange(n_s, device=rows.device)
    other = torch.unique(cols[lid[cols] < 0])
    lid[other] = n_s + torch.arange(other.numel(), device=rows.device)
    h_s = other.numel()
    lc = lid[cols]
    order = torch.argsort(seg * (n_s + h_s) + lc)
    A = (ptr.cpu().numpy(), lc[order].to(torch.int32).cpu().numpy(), vals[order].cpu().numpy())
    order_t = torch.argsort(lc * n_s + seg)
    tptr = torch.zeros(n_s + h_s + 1, dtype=torch.int64, device=rows.device)
    torch.cumsum(torch.bincount(lc, minlength=n_s + h_s), 0, out=tptr[1:])
    At = (tptr.cpu().numpy(), seg[order_t].to(torch.int32).cpu().numpy(), vals[order_t].cpu().numpy())
    qs = {"minmax": oracle.Q_MINMAX, "symmetric": oracle.Q_SYMMETRIC, "none": oracle.Q_NONE}[w.qscheme]
    norm = {"linf": oracle.NORM_LINF, "l2": oracle.NORM_L2}[w.norm]

    def host(t):
        t = t.detach().cpu()
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).numpy().view(np.uint16).copy()
        return t.numpy().copy()

    # inputs of the sample: local rows from xfull, "halo" rows from the full xfull rows the sample
    # touches; their two alternating versions are the same matrix (local part) or the fresh versions
    state = []
    for li, L in enumerate(model.layers):
        I = model.inputs[li]
        if model.tf[li]:
            # transform-first layer: the exchanged rows are rows of T = X W. Columns of the sample
            # that are local rows of the partition get their T row from the oracle's own transform.
            is_h = other >= P.n_loc
            Wn = host(L.W)
            t_loc, _ = oracle.dense_fwd(host(L.x_local[other[~is_h]]), Wn, relu=False)
            fresh = []
            for v in range(2):
                fr = np.zeros((other.numel(), L.f_out), np.float32)
                fr[host(~is_h)] = t_loc
                fr[host(is_h)] = host(I.fresh[v][other[is_h] - P.n_loc])
                fresh.append(fr)
            state.append(dict(tf=True, x=host(L.x_local[rows]), t=np.zeros((n_s + h_s, L.f_out), np.float32),
                              fresh=fresh, sent=np.zeros_like(fresh[0]), gsent=np.zeros_like(fresh[0]), W=Wn,
                              dH=[host(I.dH[v][rows]) for v in range(2)]))
            continue
        full = [torch.cat([L.xfull[:P.n_loc], I.fresh[v]]) for v in range(2)]
        fresh = [host(f[other]) for f in full]
        x = np.concatenate([host(L.xfull[rows]), np.zeros_like(fresh[0])])
        state.append(dict(tf=False, x=x, fresh=fresh, sent=np.zeros_like(fresh[0]), gsent=np.zeros_like(fresh[0]),
                          W=host(L.W), dH=[host(I.dH[v][rows]) for v in range(2)]))
        del full
    nl = len(model.layers)

    def step(v):
        outs = []
        for li in range(nl):
            s = state[li]
            if s["tf"]:
                outs.append(oracle.layer_tf_fwd(A, n_s, h_s, s["x"], s["t"], s["fresh"][v], s["sent"], s["W"], w.eps,
                                                norm, w.bits, qs, oracle.COMMIT_CUR, li + 1 < nl, True))
                continue
            outs.append(oracle.layer_fwd(A, n_s, h_s, s["x"], s["fresh"][v], s["sent"], s["W"], w.eps, norm,
                                         w.bits, qs, oracle.COMMIT_CUR, li + 1 < nl, True))
        for li in reversed(range(nl)):
            s = state[li]
            if s["tf"]:
                oracle.layer_tf_bwd(At, n_s, h_s, s["x"], outs[li]["H"], s["dH"][v], s["W"], s["gsent"], w.eps, norm,
                                    w.bits, qs, oracle.COMMIT_CUR, li + 1 < nl, True, True)
                continue
            oracle.layer_bwd(At, n_s, h_s, outs[li]["M"], outs[li]["H"], s["dH"][v], s["W"], s["gsent"], w.eps,
                             norm, w.bits, qs, oracle.COMMIT_CUR, li + 1 < nl, True, True)

    step(0)                       # fills the caches (everything is sent once), not timed
    t0 = time.perf_counter()
    step(1)
    dt = time.perf_counter() - t0
    return {"value": nl * nnz_s / dt / 1e9, "unit": "GE/s", "cores": oracle.get_threads(), "kind": "oracle",
            "sample": f"every {stride}th local row of the partition: {n_s} rows, {h_s} other columns, "
                      f"{nnz_s} edges, all {nl} layers fwd+bwd, one stationary step in {dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="share", help="tiny | mid | large | wide | share")
    ap.add_argument("--rho", type=float, default=0.37, help="fraction of halo rows refreshed per step")
    ap.add_argument("--phi", type=float, default=0.01, help="fraction of local rows whose gradient changes")
    ap.add_argument("--order", default="auto", choices=["auto", "aggregate"],
                    help="auto: layers with f_out < f_in compute A (X W); aggregate: every layer computes (A X) W")
    ap.add_argument("--graph", action="store_true",
                    help="also time the same steps replayed from captured HIP graphs (reported beside the eager figures)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run the library's plain copy kernel on 1 GiB (for scaling hardware counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1")
        sys.exit(2)

    import torch
    from cdfgen import configs
    import paper_2408_00232_amd as cdf
    from paper_2408_00232_amd.workload import Model

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cdf.binding.load()
    dev = "cuda:0"
    w = configs.ALL[args.workload]
    t_setup = time.time()
    log(f"[bench] building workload '{w.name}' on {dev} ...")
    model = Model(w, dev, rho=args.rho, phi=args.phi, order=args.order)
    torch.cuda.synchronize()
    log(f"[bench] partition: n_loc={model.n_loc} n_halo={model.n_halo} nnz={model.nnz} "
        f"layers={w.layers()} setup {time.time() - t_setup:.1f}s "
        f"mem {torch.cuda.memory_allocated() / 2**30:.1f} GiB")

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.zeros_like(src)
        for _ in range(3):
            cdf.cdf_profile_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    for t in range(args.warmup):
        model.step(t)
    torch.cuda.synchronize()
    log("[bench] warmup done")

    cdf.cdf_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup, args.warmup + args.steps):
        model.step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    cdf.cdf_profile_enable(False)

    ms_per_step = elapsed / args.steps * 1e3
    ges = model.edges_per_step() / (elapsed / args.steps) / 1e9

    # per layer shape: forward and backward time of the generic layer step (a separate, untimed pass
    # of the same steps with an event pair around every layer call), median over the passes
    import statistics
    fw, bw = [], []
    for t in range(args.warmup + args.steps, args.warmup + args.steps + max(4, min(args.steps, 10))):
        a_ms, b_ms = model.step_timed_per_layer(t)
        fw.append(a_ms)
        bw.append(b_ms)
    per_layer = []
    for li, (f_in, f_out) in enumerate(w.layers()):
        tf_ms = statistics.median(x[li] for x in fw)
        tb_ms = statistics.median(x[li] for x in bw)
        per_layer.append({"f_in": f_in, "f_out": f_out, "order": "transform-first" if model.tf[li] else "aggregate-first",
                          "fwd_ms": tf_ms, "bwd_ms": tb_ms, "GE_per_s": model.nnz / ((tf_ms + tb_ms) * 1e-3) / 1e9})

    graph_replay = None
    if args.graph:
        # launch-bound workloads (tiny, mid): the same steps as two captured graphs, one per input version
        model.capture()
        t_next = args.warmup + args.steps
        for t in range(t_next, t_next + 2):
            model.step(t)
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for t in range(t_next + 2, t_next + 2 + args.steps):
            model.step(t)
        torch.cuda.synchronize()
        eg = time.perf_counter() - tg
        graph_replay = {"ms_per_step": eg / args.steps * 1e3, "value": model.edges_per_step() / (eg / args.steps) / 1e9,
                        "unit": "GE/s"}

    # per-kernel durations from the events recorded inside the timed region
    kernels = {}
    for k in range(cdf.cdf_profile_kernels()):
        ms = cdf.cdf_profile_read(k)
        if ms:
            name = cdf.cdf_profile_kernel_name(k)
            kernels[name] = {"launches": len(ms), "avg_ms": sum(ms) / len(ms),
                             "ms_per_step": sum(ms) / args.steps, "_ms": ms}
    # dominant kernel: the aggregation. Launch order within a step: forward layers 0..L-1 on A,
    # then backward layers L-1..0 on A^T; algorithmic bytes differ per launch (feature width).
    esz = 2 if w.dtype == "bf16" else 4
    n, h, nnz = model.n_loc, model.n_halo, model.nnz
    widths = model.spmm_widths()
    per_step = [spmm_bytes(n, n + h, nnz, f, esz) for f in widths] + \
               [spmm_bytes(n + h, n, nnz, f, esz) for f in reversed(widths)]
    nl = len(per_step)
    # which launch of a step runs which aggregation kernel (the library slices the columns when the
    # width is a whole number of 128-byte lines and rows average 8+ entries)
    line = 64 if w.dtype == "bf16" else 32
    rows_of = [n] * len(widths) + [n + h] * len(widths)
    wid_of = list(widths) + list(reversed(widths))
    kern_of = ["spmm_sliced_kernel" if wd % line == 0 and nnz >= 8 * r else "spmm_kernel"
               for wd, r in zip(wid_of, rows_of)]
    times = {k: list(kernels[k]["_ms"]) for k in ("spmm_kernel", "spmm_sliced_kernel") if k in kernels}
    pos_ms = [[] for _ in range(nl)]
    ok = all(sum(1 for k in kern_of if k == name) * args.steps == len(ms) for name, ms in times.items())
    if ok:
        cursor = {k: 0 for k in times}
        for _ in range(args.steps):
            for i, k in enumerate(kern_of):
                pos_ms[i].append(times[k][cursor[k]])
                cursor[k] += 1
    roof = None
    if ok and all(pos_ms):
        spmm_name = max(times, key=lambda k: sum(times[k]))
        sel = [i for i, k in enumerate(kern_of) if k == spmm_name]
        bmin = sum(per_step[i][0] for i in sel) / len(sel)
        bmax = sum(per_step[i][1] for i in sel) / len(sel)
        avg_s = sum(times[spmm_name]) / len(times[spmm_name]) / 1e3
        # achieved: the aggregation's algorithmic bytes - per stored entry 8 bytes of CSR plus one
        # feature row (dim * element size), plus row pointers and the output rows - over the
        # average launch time. compulsory_*: the same with every input row counted once only.
        roof = {"kernel": spmm_name, "bound": "hbm", "achieved": bmax / avg_s / 1e9, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": bmax / avg_s / 1e9 / HBM_PEAK_GBS, "traffic": None,
                "avg_launch_ms": avg_s * 1e3, "algorithmic_bytes_per_launch": bmax,
                "compulsory_bytes_per_launch": bmin, "compulsory_GBps": bmin / avg_s / 1e9,
                "launches_per_step": len(sel),
                "aggregation_ms_by_position": [sum(x) / len(x) for x in pos_ms],
                "aggregation_kernel_by_position": kern_of,
                "aggregation_width_by_position": wid_of,
                "algorithmic_GBps_by_position": [per_step[i][1] / (sum(pos_ms[i]) / len(pos_ms[i])) / 1e6
                                                 for i in range(nl)]}
        tfile = os.path.join(ROOT, "profiles", f"traffic_{w.name}.txt")
        if os.path.exists(tfile):
            for line in open(tfile):
                if line.startswith(spmm_name + " ="):
                    f_b, w_b = line.split("=")[1].split()
                    roof["traffic"] = float(f_b) + float(w_b)

    # every HBM-bound kernel against its own algorithmic bytes, every dense kernel against the fp32
    # matrix-core peak (per-launch averages over the timed region; widths differ between layers)
    def avg(xs):
        return sum(xs) / len(xs)
    lay = [(f, g) for f, g in zip(widths, [g for _, g in w.layers()])]   # (width of the halo rows, f_out)
    sent_f = [int(L.n_sent.item()) for L in model.layers]
    sent_b = [int(L.gn_sent.item()) for L in model.layers]
    rb = [L.row_bytes for L in model.layers]
    alg = {
        "filter_kernel": avg([h * (2 * f * esz + 1) + 4 * sent_f[i] for i, (f, _) in enumerate(lay)] +
                             [h * (2 * f * esz + 1) + 4 * sent_b[i] for i, (f, _) in enumerate(lay)]),
        "quantize_kernel": avg([sent_f[i] * (3 * f * esz + rb[i] + 12) for i, (f, _) in enumerate(lay)] +
                               [sent_b[i] * (3 * f * esz + rb[i] + 12) for i, (f, _) in enumerate(lay)]),
        "dequantize_kernel": avg([sent_f[i] * (2 * f * esz + rb[i] + 12) for i, (f, _) in enumerate(lay)]),
        # one-pass test + message build: every row read once, sent rows committed and coded
        "test_encode_kernel": avg([h * (2 * f * esz + 1) + sn[i] * (f * esz + rb[i] + 8)
                                   for sn in (sent_f, sent_b) for i, (f, _) in enumerate(lay)]),
        "gather_codes_kernel": avg([sn[i] * (2 * rb[i] + 16 + 4)
                                    for sn in (sent_f, sent_b) for i, (f, _) in enumerate(lay)]),
    }
    flops = avg([2.0 * n * f * g for f, g in w.layers()])
    per_kernel = {}
    for name, b in alg.items():
        if name in kernels:
            gbs = b / (kernels[name]["avg_ms"] * 1e-3) / 1e9
            per_kernel[name] = {"bound": "hbm", "algorithmic_bytes_per_launch": b, "achieved_GBps": gbs,
                                "frac": gbs / HBM_PEAK_GBS}
    for name in ("gemm_kernel<FWD>", "gemm_kernel<DW>", "gemm_kernel<DM>"):
        if name in kernels:
            tf = flops / (kernels[name]["avg_ms"] * 1e-3) / 1e12
            per_kernel[name] = {"bound": "mfma", "flops_per_launch": flops, "achieved_TFLOPs": tf,
                                "frac": tf / 157.3}
    # measured streaming ceiling: the library's plain copy kernel on 1 GiB (read + write bytes)
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.zeros_like(src)
    cdf.cdf_profile_copy(dst, src)
    torch.cuda.synchronize()
    tc = time.perf_counter()
    for _ in range(10):
        cdf.cdf_profile_copy(dst, src)
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * (1 << 30) / (time.perf_counter() - tc) / 1e9
    del src, dst

    rho_f = [int(L.n_sent.item()) / max(h, 1) for L in model.layers]
    rho_b = [int(L.gn_sent.item()) / max(h, 1) for L in model.layers]

    for v in kernels.values():
        v.pop("_ms", None)
    out = {
        "metric": "GCN layer fwd+bwd edges/sec (GE/s) per partition; % of HBM roofline",
        "value": ges, "unit": "GE/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.kind} graph, {w.n_vertices} vertices, partition {w.part} of "
                               f"{w.parts} ({w.partitioner}), n_loc={n}, n_halo={h}, nnz={nnz}, layers "
                               f"{'-'.join(str(d) for d in w.dims)}, {w.bits}-bit {w.qscheme} messages, "
                               f"eps={w.eps} ({w.norm})",
                   "order_per_layer": ["transform-first" if t else "aggregate-first" for t in model.tf],
                   "edges_per_step": model.edges_per_step(), "send_fraction_fwd": rho_f,
                   "send_fraction_bwd": rho_b},
        "roofline": roof,
        "kernels": kernels,
        "kernel_rooflines": per_kernel,
        "per_layer": per_layer,
        "copy_ceiling_GBps": copy_gbs,
        "graph_replay": graph_replay,
    }
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a sample ...")
        out["cpu_baseline"] = cpu_baseline(model)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
