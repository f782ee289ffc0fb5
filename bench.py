#!/usr/bin/env python3
"""Benchmark of the FM pass on one MI355X.

A step is one full-gradient epoch (forward, multipliers, gradient, update:
fm_sgd_epoch) over the click-style workload (config 4: N=1e7, D=1e6, 39 nnz/row,
K=16), inputs resident in HBM.  Prints ONE JSON line with the throughput in
nonzeros/s, the roofline figures of the dominant kernel (timed with HIP events on
the launch stream) and the oracle's CPU baseline on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(N, D, K, counts, seg=256, tile_rows=512, tile_min=8, tile_seg=256):
    """Bytes each kernel must move if every array is streamed once and every gather is served
    from cache (fp32 values, int32 indices, int64 pointers).  Columns are classed as the library
    classes them: empty / short (<= seg entries) -> cols; dense-ish (>= tile_min entries per row
    tile on average) -> cols_tile; the other long columns -> cols_long; partial sums of the long
    columns are added by cols_finish.  The compulsory read of r and G (4N(K+1) bytes) is shared
    between the three accumulation kernels in proportion to the entries they process."""
    import numpy as np
    nnz = int(counts.sum())
    ntiles = (N + tile_rows - 1) // tile_rows
    tile_thr = max(tile_min * ntiles, seg + 1) if ntiles >= 2 and tile_min > 0 else np.iinfo(np.int64).max
    short = counts <= seg
    tiled = counts >= tile_thr
    longc = ~short & ~tiled
    nnz_s, nnz_t, nnz_l = int(counts[short].sum()), int(counts[tiled].sum()), int(counts[longc].sum())
    items_l = int(((counts[longc] + seg - 1) // seg).sum())
    items_t = int(np.maximum(ntiles, (counts[tiled] + tile_seg - 1) // tile_seg).sum())
    nlong = int((~short).sum())
    aux = 4 * N * (K + 1)
    fwd = 8 * nnz + 8 * (N + 1) + 4 * N + 4 * D * (K + 1) + aux
    share = lambda e: aux * (e / max(nnz, 1))
    cols = 8 * nnz_s + 8 * (D + 1) + 4 * int((short & (counts > 0)).sum()) + share(nnz_s) + 8 * int(short.sum()) * (K + 1)
    cols_long = 8 * nnz_l + 16 * items_l + share(nnz_l) + 4 * items_l * (K + 2)
    cols_tile = 8 * nnz_t + 16 * items_t + share(nnz_t) + 4 * items_t * (K + 2)
    cols_finish = 4 * (items_l + items_t) * (K + 2) + 12 * nlong + 8 * nlong * (K + 1)
    return {"rows_forward": fwd, "cols": cols, "cols_long": cols_long, "cols_tile": cols_tile,
            "cols_finish": cols_finish,
            "epoch": 16 * nnz + 8 * N * (K + 1) + 12 * D * (K + 1) + 12 * N + 8 * D,
            "classes": {"nnz_short": nnz_s, "nnz_long": nnz_l, "nnz_tile": nnz_t, "items_long": items_l,
                        "items_tile": items_t, "long_columns": nlong}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--cpu-rows", type=int, default=10_000_000, help="rows of the workload the oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stratified", action="store_true", help="also time fm_stratified_epoch (reported in extra)")
    ap.add_argument("--parts", action="store_true",
                    help="also time fm_forward and fm_gradient on their own (reported in extra)")
    ap.add_argument("--minibatch", type=int, default=0, metavar="B",
                    help="also time fm_minibatch_epoch over B row batches (reported in extra)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain 1 GiB device copy three times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); nothing here uses a second device")

    import numpy as np
    import torch
    from paper_2004_13940_amd import binding as B
    from paper_2004_13940_amd.workloads import make_config

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    t0 = time.time()
    wl = make_config(args.workload, scale=args.scale)
    t_gen = time.time() - t0
    print(f"[bench] workload {wl.name}: N={wl.N} D={wl.D} nnz={wl.nnz} K={wl.K} generated in {t_gen:.1f}s",
          file=sys.stderr, flush=True)
    t0 = time.time()
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    t_up = time.time() - t0
    t0 = time.time()
    m.fm_build_csc()
    torch.cuda.synchronize()
    t_csc = time.time() - t0
    print(f"[bench] upload {t_up:.2f}s, CSC build {t_csc:.2f}s", file=sys.stderr, flush=True)

    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0)
    w0 = torch.tensor([float(wl.w0)], device="cuda")
    w = torch.from_numpy(wl.w).cuda()
    V = torch.from_numpy(wl.V).cuda().reshape(-1)
    y = torch.from_numpy(wl.y).cuda()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        m.fm_sgd_epoch(p, y, w0, w, V)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        m.fm_sgd_epoch(p, y, w0, w, V)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    value = wl.nnz * args.steps / dt
    print(f"[bench] {ms_per_step:.3f} ms/epoch, {value:.4g} nnz/s", file=sys.stderr, flush=True)

    # per-kernel durations from HIP events on the launch stream, over the same number of steps
    m.fm_profile_enable(True)
    for _ in range(args.steps):
        m.fm_sgd_epoch(p, y, w0, w, V)
    prof = m.fm_profile_read()
    m.fm_profile_enable(False)
    counts = np.bincount(wl.col, minlength=wl.D).astype(np.int64)
    ab = algorithmic_bytes(wl.N, wl.D, wl.K, counts)
    kern = {k: {"launches": n, "avg_ms": ms / n} for k, (n, ms) in prof.items() if n > 0}
    dominant = max(kern, key=lambda k: kern[k]["avg_ms"] * kern[k]["launches"])
    dom_ms = kern[dominant]["avg_ms"]
    achieved = ab[dominant] / (dom_ms * 1e-3) / 1e9
    traffic = None
    epoch_traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl.name}.json")
    if args.scale == 1.0 and os.path.exists(tpath):
        tj = json.load(open(tpath))
        traffic = tj.get(dominant, {}).get("hbm_bytes_per_launch")
        epoch_traffic = sum(v["hbm_bytes_per_launch"] for k, v in tj.items() if isinstance(v, dict))
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "algorithmic_bytes_per_launch": ab[dominant], "avg_launch_ms": dom_ms,
                "epoch_algorithmic_GBs": ab["epoch"] / (ms_per_step * 1e-3) / 1e9,
                "epoch_frac": ab["epoch"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                # counted HBM bytes (rocprofv3 summary under profiles/) over the durations measured here:
                # what the memory system actually moved, misses of the gathers included
                "traffic_GBs": None if traffic is None else traffic / (dom_ms * 1e-3) / 1e9,
                "traffic_frac": None if traffic is None else traffic / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "epoch_traffic": epoch_traffic,
                "epoch_traffic_frac": None if epoch_traffic is None
                else epoch_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "kernels": {k: {"avg_ms": v["avg_ms"], "algorithmic_GBs": ab[k] / (v["avg_ms"] * 1e-3) / 1e9}
                            for k, v in kern.items() if k in ab}}

    # ceiling of the traffic these kernels are bound by: random 128-byte line reads from a buffer of the
    # size of the aggregates, measured here; beside it the lines per second the dominant kernel moves
    # according to the committed counter summary
    try:
        from paper_2004_13940_amd import bench_probe
        line_peak = bench_probe.gather_rate(max(1 << 20, min(wl.N * 128, 8 << 30)), 128)
    except Exception as e:  # a failed calibration must not lose the measurement
        print(f"[bench] gather calibration failed: {e}", file=sys.stderr, flush=True)
        line_peak = None
    roofline["random_line_reads_per_s"] = line_peak
    roofline["lines_per_s"] = None if traffic is None else traffic / 128.0 / (dom_ms * 1e-3)
    roofline["line_frac"] = None if (traffic is None or not line_peak) else roofline["lines_per_s"] / line_peak

    extra = {"column_classes": ab["classes"], "gen_s": t_gen, "upload_s": t_up, "csc_build_s": t_csc, "sha256": wl.sha256()[:16]}
    if args.stratified:
        m.fm_partition(wl.P)
        m.fm_stratified_epoch(p, y, w0, w, V)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        m.fm_stratified_epoch(p, y, w0, w, V)
        torch.cuda.synchronize()
        ts = time.perf_counter() - t0
        extra["stratified_ms_per_epoch"] = 1e3 * ts
        extra["stratified_nnz_per_s"] = wl.nnz / ts
        extra["P"] = wl.P

    if args.parts:
        # the two halves of the pass through their own entry points (dense caller-side arrays)
        yhat = torch.empty(wl.N, device="cuda")
        a = torch.empty(wl.N, device="cuda")
        q = torch.empty(wl.N, device="cuda")
        r = torch.empty(wl.N, device="cuda")
        G = torch.empty(wl.N * wl.K, device="cuda")
        gw = torch.empty(wl.D, device="cuda")
        gV = torch.empty(wl.D * wl.K, device="cuda")
        gw0 = torch.empty(1, device="cuda")
        for name, fn in (("forward", lambda: m.fm_forward(p, y, w0, w, V, yhat=yhat, a=a, G=G, q=q, r=r)),
                         ("gradient", lambda: m.fm_gradient(p, r, G, w, V, gw0, gw, gV))):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            tp = (time.perf_counter() - t0) / args.steps
            extra[f"{name}_ms"] = 1e3 * tp
            extra[f"{name}_nnz_per_s"] = wl.nnz / tp
        del yhat, a, q, r, G, gw, gV

    if args.minibatch > 0:
        m.fm_partition_batches(args.minibatch)
        m.fm_minibatch_epoch(p, y, w0, w, V)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        m.fm_minibatch_epoch(p, y, w0, w, V)
        torch.cuda.synchronize()
        tb = time.perf_counter() - t0
        extra["minibatch_ms_per_epoch"] = 1e3 * tb
        extra["minibatch_nnz_per_s"] = wl.nnz / tb
        extra["B"] = args.minibatch

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fm_oracle as O
        n = min(wl.N, args.cpu_rows)
        e = int(wl.rowptr[n])
        X = O.make_matrix(n, wl.D, wl.rowptr[:n + 1], wl.col[:e], wl.val[:e])
        kw = dict(loss=wl.loss, s=wl.loss_scale, lambda_w=wl.lambda_w, lambda_v=wl.lambda_v, eta=wl.eta,
                  update_w0=bool(wl.update_w0))
        ow0, ow, oV = float(wl.w0), wl.w, wl.V
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            ow0, ow, oV, _ = O.full_epoch(X, wl.y[:n], ow0, ow, oV, **kw)
        tc = (time.perf_counter() - t0) / reps
        cpu = {"value": e / tc, "unit": "nnz/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"first {n} rows ({e} nnz) of {wl.name}, {reps} full-gradient epochs, fp64, {tc:.2f} s/epoch"}

    out = {"metric": "FM epoch (fwd+grad+update) nonzeros/sec at K=16", "value": value, "unit": "nnz/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{wl.name} scale={args.scale}", "N": wl.N, "D": wl.D, "nnz": wl.nnz, "K": wl.K,
                      "loss": "logistic" if wl.loss == 1 else "squared"},
           "roofline": roofline, "cpu_baseline": cpu, "extra": extra}
    print(json.dumps(out))
    m.close()


if __name__ == "__main__":
    main()
