"""Microbenchmarks of the three message kernels at forced send fractions: the cache test
(cdf_cache_filter), the message build (cdf_quantize) and the recovery (cdf_dequantize), on the
halo rows of a workload's partition, every layer width, rho in {0, 0.1, 0.5, 1}.

    python -m paper_2408_00232_amd.microbench --workload share

The commit is switched off (CDF_COMMIT_NONE) so that every repetition sees the same rows fail;
the commit write (F*s bytes per sent row) is therefore not part of these figures.
"""
import argparse
import json

import torch

from cdfgen import configs, rng

from . import binding as B

_QS = {"minmax": B.Q_MINMAX, "symmetric": B.Q_SYMMETRIC, "none": B.Q_NONE}
_NORM = {"linf": B.NORM_LINF, "l2": B.NORM_L2}


def _time(fn, reps):
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="share", choices=sorted(configs.ALL))
    ap.add_argument("--rows", type=int, default=0, help="halo rows (default: the workload partition's)")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        raise SystemExit("microbench: no GPU visible")
    w = configs.ALL[a.workload]
    dev = "cuda:0"
    R = a.rows or configs.build_partition(w, device=dev).n_halo
    dt = torch.float32 if w.dtype == "f32" else torch.bfloat16
    esz = 4 if w.dtype == "f32" else 2
    qs, norm = _QS[w.qscheme], _NORM[w.norm]
    widths = sorted({f for f, _ in w.layers()})
    ws = torch.zeros(B.cdf_workspace_bytes(R, max(widths), 1), dtype=torch.uint8, device=dev)
    if not a.json:
        print(f"# {w.name}: {R} halo rows, {w.dtype}, {w.bits}-bit {w.qscheme}, eps {w.eps}")
        print("# width   rho   sent      filter ms   GB/s   quantize ms   GB/s   dequantize ms   GB/s")
    out = []
    for F in widths:
        g = torch.Generator(device=dev).manual_seed(w.seed + F)
        cached = torch.randn(R, F, device=dev, generator=g).to(dt)
        rb = B.cdf_code_row_bytes(F, w.bits, qs)
        mask = torch.zeros(R, dtype=torch.uint8, device=dev)
        idx = torch.zeros(R, dtype=torch.int32, device=dev)
        ns = torch.zeros(1, dtype=torch.int32, device=dev)
        codes = torch.zeros(R * rb, dtype=torch.uint8, device=dev)
        meta = torch.zeros(R, 2, device=dev)
        dst = torch.zeros(R, F, dtype=dt, device=dev)
        u = rng.uniform01(w.seed, 95, torch.arange(R, dtype=torch.int64, device=dev))
        for rho in (0.0, 0.1, 0.5, 1.0):
            fail = (u < rho).view(R, 1)
            # failing rows move by 50 %, the others by 0.1 % (far below the threshold)
            cur = (cached.float() * torch.where(fail, 1.5, 1.001)).to(dt)
            f_ms = _time(lambda: B.cdf_cache_filter(cur, cached, w.eps, norm, mask, idx, ns, ws), a.reps)
            n = int(ns.item())
            q_ms = _time(lambda: B.cdf_quantize(cur, cached, idx, ns, R, w.bits, qs, B.COMMIT_NONE, True, codes, meta),
                         a.reps)
            d_ms = _time(lambda: B.cdf_dequantize(codes, meta, idx, ns, R, w.bits, qs, dst, True), a.reps)
            fb = R * (2 * F * esz + 1) + 4 * n
            qb = n * (2 * F * esz + rb + 12)
            db = n * (2 * F * esz + rb + 12)
            rec = dict(width=F, rho=rho, sent=n, filter_ms=f_ms, filter_GBps=fb / f_ms / 1e6, quantize_ms=q_ms,
                       quantize_GBps=qb / q_ms / 1e6 if n else 0.0, dequantize_ms=d_ms,
                       dequantize_GBps=db / d_ms / 1e6 if n else 0.0)
            out.append(rec)
            if not a.json:
                print(f"{F:7d} {rho:5.1f} {n:9d} {f_ms:11.3f} {rec['filter_GBps']:7.0f} {q_ms:12.3f} "
                      f"{rec['quantize_GBps']:7.0f} {d_ms:14.3f} {rec['dequantize_GBps']:7.0f}", flush=True)
    if a.json:
        print(json.dumps(out))


if __name__ == "__main__":
    main()
