#!/usr/bin/env python3
"""Benchmark of the FM pass on one MI355X.

A step is one full-gradient epoch (forward, multipliers, gradient, update: fm_sgd_epoch) over the click-style
workload (config 4: N=1e7, D=1e6, 39 entries per row, K=16), inputs resident in HBM.  Prints ONE JSON line:
throughput in nonzeros/s over exactly --steps epochs (wall clock between two device synchronisations; the
parameters are restored from a device copy before every epoch, so that all repetitions do the same work),
per-epoch HIP-event times (median, min), the roofline figures of the dominant kernel (timed with HIP events on
the launch stream by the library), the oracle's CPU baseline, and in extra.per_config the same protocol on all
five workloads (forward, gradient, full-gradient epoch, stratified epoch).

`bench.py --traffic-from FETCH.csv WRITE.csv` does not run the benchmark: it turns two rocprofv3 counter files
(FETCH_SIZE and WRITE_SIZE, each from a run of `bench.py --copy-calibration`) into profiles/traffic_<workload>.json,
stamped with a hash of the kernel sources; the benchmark only reports those figures while the hash still matches.
"""
import argparse
import csv
import glob
import hashlib
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
COPY_BYTES = 1 << 30  # the calibration copy: 1 GiB read and 1 GiB written
TRAFFIC_KIND = ("L2-miss side: bytes requested from / written to the fabric behind the L2 (FETCH_SIZE and WRITE_SIZE, "
                "each scaled by what the same counter reads for a plain 1 GiB copy); hits in the memory-side cache are "
                "included, rocprofv3 exposes no counter behind it, so this is an upper bound of the HBM bytes")


def csrc_sha256():
    """Hash of everything the library is built from (the counter figures are only valid for these sources)."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2004_13940_amd", "csrc", "fm_*")) +
                   [os.path.join(ROOT, "include", "fm.h")])
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


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
            "gradient": 8 * nnz + 8 * D + 4 * N * (K + 1) + 8 * D * (K + 1),
            "epoch": 16 * nnz + 8 * N * (K + 1) + 12 * D * (K + 1) + 12 * N + 8 * D,
            "classes": {"nnz_short": nnz_s, "nnz_long": nnz_l, "nnz_tile": nnz_t, "items_long": items_l,
                        "items_tile": items_t, "long_columns": nlong}}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


# ----------------------------------------------------------------- timing ----

class Timed:
    """HIP events around repetitions of a call on torch's current stream (the one the binding launches on)."""

    def __init__(self, torch):
        self.torch = torch

    def run(self, fn, reps, before=None):
        """Times fn() reps times; before() (untimed by the events) runs ahead of every repetition.  Returns the
        per-repetition milliseconds and the wall-clock seconds of the whole loop between two synchronisations."""
        torch = self.torch
        a = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        b = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(reps):
            if before is not None:
                before()
            a[i].record()
            fn()
            b[i].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return [a[i].elapsed_time(b[i]) for i in range(reps)], wall


def stats(ms):
    s = sorted(ms)
    n = len(s)
    med = s[n // 2] if n % 2 else 0.5 * (s[n // 2 - 1] + s[n // 2])
    return {"median_ms": med, "min_ms": s[0], "mean_ms": sum(s) / n, "reps": n}


def device_state(torch, wl):
    w0 = torch.tensor([float(wl.w0)], device="cuda")
    w = torch.from_numpy(wl.w).cuda()
    V = torch.from_numpy(wl.V).cuda().reshape(-1)
    y = torch.from_numpy(wl.y).cuda()
    init = (w0.clone(), w.clone(), V.clone())

    def restore():
        w0.copy_(init[0])
        w.copy_(init[1])
        V.copy_(init[2])

    return w0, w, V, y, restore


def oracle_epoch_time(wl, rows, reps=1):
    """Seconds per full-gradient epoch of the fp64 oracle on the first `rows` rows, all OpenMP threads."""
    from oracle import fm_oracle as O
    n = min(wl.N, rows)
    e = int(wl.rowptr[n])
    X = O.make_matrix(n, wl.D, wl.rowptr[:n + 1], wl.col[:e], wl.val[:e])
    kw = dict(loss=wl.loss, s=wl.loss_scale, lambda_w=wl.lambda_w, lambda_v=wl.lambda_v, eta=wl.eta,
              update_w0=bool(wl.update_w0))
    ow0, ow, oV = float(wl.w0), wl.w, wl.V
    t0 = time.perf_counter()
    for _ in range(reps):
        ow0, ow, oV, _ = O.full_epoch(X, wl.y[:n], ow0, ow, oV, **kw)
    return (time.perf_counter() - t0) / reps, n, e, O.threads()


def oracle_single_thread(index, scale):
    """The same oracle epoch with one OpenMP thread, in a child process (the thread count is fixed when the
    oracle's library is loaded); the child touches no GPU."""
    code = ("import sys, time, json; sys.path.insert(0, %r)\n"
            "from paper_2004_13940_amd.workloads import make_config\n"
            "from oracle import fm_oracle as O\n"
            "wl = make_config(%d, scale=%r)\n"
            "X = O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)\n"
            "kw = dict(loss=wl.loss, s=wl.loss_scale, lambda_w=wl.lambda_w, lambda_v=wl.lambda_v, eta=wl.eta, update_w0=bool(wl.update_w0))\n"
            "t0 = time.perf_counter(); O.full_epoch(X, wl.y, float(wl.w0), wl.w, wl.V, **kw); t = time.perf_counter() - t0\n"
            "print(json.dumps({'s_per_epoch': t, 'nnz': wl.nnz, 'rows': wl.N, 'threads': O.threads()}))\n" % (ROOT, index, scale))
    env = dict(os.environ, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=300)
    if r.returncode != 0:
        raise RuntimeError(r.stderr[-500:])
    return json.loads(r.stdout.strip().splitlines()[-1])


def permuted_columns(wl, seed=13940):
    """The same matrix with its column ids sent through a random permutation (rows re-sorted): spreads the head of
    a Zipf law that is not permuted by its recipe over all column blocks."""
    import numpy as np
    from dataclasses import replace
    perm = np.random.default_rng(seed).permutation(wl.D).astype(np.int64)
    rows = np.repeat(np.arange(wl.N, dtype=np.int64), np.diff(wl.rowptr))
    order = np.argsort(rows * wl.D + perm[wl.col], kind="stable")
    return replace(wl, name=wl.name + "_permuted", col=perm[wl.col][order].astype(np.int32), val=wl.val[order],
                   notes=dict(wl.notes, permuted=True))


def time_config(torch, B, wl, reps, oracle_rows):
    """Forward, gradient, full-gradient epoch and stratified epoch of one workload: median/min of HIP-event times,
    nonzeros/s, algorithmic bytes over time against the 8 TB/s peak; the oracle's epoch on a bounded sample."""
    T = Timed(torch)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0)
    w0, w, V, y, restore = device_state(torch, wl)
    N, D, K, nnz = wl.N, wl.D, wl.K, wl.nnz
    b_fwd = 8 * nnz + 8 * (N + 1) + 4 * N + 4 * D * (K + 1) + 4 * N * (K + 1)
    b_grad = 8 * nnz + 8 * D + 4 * N * (K + 1) + 8 * D * (K + 1)
    b_epoch = 16 * nnz + 8 * N * (K + 1) + 12 * D * (K + 1) + 12 * N + 8 * D
    out = {"N": N, "D": D, "nnz": nnz, "K": K, "P": wl.P, "reps": reps, "sha256": wl.sha256()[:16]}

    def entry(ms, nbytes):
        st = stats(ms)
        gbs = nbytes / (st["median_ms"] * 1e-3) / 1e9 if nbytes else None
        return {"median_ms": st["median_ms"], "min_ms": st["min_ms"], "nnz_per_s": nnz / (st["median_ms"] * 1e-3),
                "algorithmic_GBs": gbs, "algorithmic_frac_of_hbm_peak": None if gbs is None else gbs / HBM_PEAK_GBS,
                "counted_GBs": None}

    for _ in range(2):
        restore()
        m.fm_sgd_epoch(p, y, w0, w, V)
    ms, _ = T.run(lambda: m.fm_sgd_epoch(p, y, w0, w, V), reps, before=restore)
    out["epoch"] = entry(ms, b_epoch)
    yhat, a, q, r = (torch.empty(N, device="cuda") for _ in range(4))
    G = torch.empty(N * K, device="cuda")
    gw, gV, gw0 = torch.empty(D, device="cuda"), torch.empty(D * K, device="cuda"), torch.empty(1, device="cuda")
    restore()
    fwd = lambda: m.fm_forward(p, y, w0, w, V, yhat=yhat, a=a, G=G, q=q, r=r)
    grad = lambda: m.fm_gradient(p, r, G, w, V, gw0, gw, gV)
    fwd(), grad()
    ms, _ = T.run(fwd, reps)
    out["forward"] = entry(ms, b_fwd)
    ms, _ = T.run(grad, reps)
    out["gradient"] = entry(ms, b_grad)
    if K % 4 == 0:  # the same forward and epoch with the V rows gathered from the half-precision copy (not the headline)
        ph = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0, half_gather=1)
        fwd_h = lambda: m.fm_forward(ph, y, w0, w, V, yhat=yhat, a=a, G=G, q=q, r=r)
        fwd_h()
        ms, _ = T.run(fwd_h, reps)
        out["forward_half_gather"] = entry(ms, None)
        ms, _ = T.run(lambda: m.fm_sgd_epoch(ph, y, w0, w, V), reps, before=restore)
        out["epoch_half_gather"] = entry(ms, None)
    if nnz == N * D and D in (32, 64) and K in (32, 64):
        # every row stores all columns: the figures above are those of the dense (matrix-core) kernels, which
        # do not read the column indices (they move 4 of the 8 bytes per entry that the algorithmic count
        # holds); the same calls through the general sparse kernels, for comparison
        out["kernels"] = "dense rows: fp32 MFMA contractions (column indices not read)"
        m.fm_set_option(B.FM_OPT_DENSE_ROWS, 0)
        fwd(), grad()
        ms, _ = T.run(fwd, reps)
        out["forward_sparse_kernels"] = entry(ms, b_fwd)
        ms, _ = T.run(grad, reps)
        out["gradient_sparse_kernels"] = entry(ms, b_grad)
        restore()
        m.fm_sgd_epoch(p, y, w0, w, V)
        ms, _ = T.run(lambda: m.fm_sgd_epoch(p, y, w0, w, V), reps, before=restore)
        out["epoch_sparse_kernels"] = entry(ms, b_epoch)
        m.fm_set_option(B.FM_OPT_DENSE_ROWS, 1)
    del yhat, a, q, r, G, gw, gV
    torch.cuda.empty_cache()
    t0 = time.perf_counter()
    free0 = torch.cuda.mem_get_info()[0]
    m.fm_partition(wl.P)
    torch.cuda.synchronize()
    out["partition_s"] = time.perf_counter() - t0
    out["partition_device_bytes"] = free0 - torch.cuda.mem_get_info()[0]  # the two re-ordered copies are 16 B per entry
    restore()
    m.fm_stratified_epoch(p, y, w0, w, V)
    ms, _ = T.run(lambda: m.fm_stratified_epoch(p, y, w0, w, V), reps, before=restore)
    out["stratified"] = entry(ms, None)  # its extra traffic (aggregates of every touched row per stratum) is inherent
    m.close()
    del w0, w, V, y
    torch.cuda.empty_cache()
    if oracle_rows > 0:
        tc, n, e, th = oracle_epoch_time(wl, oracle_rows)
        out["oracle"] = {"s_per_epoch": tc, "nnz_per_s": e / tc, "threads": th, "sample": f"first {n} rows ({e} nnz), 1 epoch"}
    return out


# ------------------------------------------------------- counter files ----

def traffic_from(fetch_csv, write_csv, name):
    """profiles/traffic_<name>.json from two rocprofv3 counter CSVs (FETCH_SIZE, WRITE_SIZE; KiB per dispatch)."""
    def per_kernel(path, counter):
        acc = {}
        for row in csv.DictReader(open(path)):
            if row["Counter_Name"] != counter:
                continue
            k = re.sub(r"\(anonymous namespace\)::", "", row["Kernel_Name"])
            k = re.sub(r"^void ", "", k)
            acc.setdefault(k, []).append(float(row["Counter_Value"]))
        return {k: sum(v) / len(v) for k, v in acc.items()}
    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    copy = [k for k in fetch if "k_probe_copy" in k]
    if not copy:
        sys.exit("no k_probe_copy dispatch in the counter file: run bench.py with --copy-calibration")
    f_scale = (COPY_BYTES / 1024.0) / fetch[copy[0]]
    w_scale = (COPY_BYTES / 1024.0) / write[copy[0]]
    groups = {"rows_forward": r"^k_rows<.*, 0>", "cols": r"^k_cols(_empty)?<", "cols_long": r"^k_cols_long<",
              "cols_tile": r"^k_cols_tile<", "cols_finish": r"^k_cols_finish_", "reduce": r"^k_reduce", "bias": r"^k_bias"}
    out = {"_kind": TRAFFIC_KIND, "_csrc_sha256": csrc_sha256(), "_fetch_scale": f_scale, "_write_scale": w_scale,
           "_copy_reads_KiB": fetch[copy[0]], "_copy_writes_KiB": write[copy[0]]}
    for g, pat in groups.items():
        ks = [k for k in fetch if re.search(pat, k)]
        out[g] = {"l2_miss_bytes_per_launch": sum(1024.0 * (fetch[k] * f_scale + write.get(k, 0.0) * w_scale) for k in ks),
                  "fetch_KiB": sum(fetch[k] for k in ks), "write_KiB": sum(write.get(k, 0.0) for k in ks), "kernels": ks}
    path = os.path.join(ROOT, "profiles", f"traffic_{name}.json")
    json.dump(out, open(path, "w"), indent=1)
    print("wrote", path)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--cpu-rows", type=int, default=10_000_000, help="rows of the workload the oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the table over all five workloads")
    ap.add_argument("--minibatch", type=int, default=0, metavar="B",
                    help="also time fm_minibatch_epoch over B row batches (reported in extra)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain 1 GiB device copy three times (reference for the byte counters)")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"))
    ap.add_argument("--only-config", type=int, default=0, metavar="IDX",
                    help="time workload IDX alone with the per-config protocol and print its entry (for kernel traces)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); nothing here uses a second device")

    import numpy as np
    from paper_2004_13940_amd.workloads import make_config
    if args.traffic_from:
        names = {1: "cfg1_tiny_binary", 2: "cfg2_dense_regression", 3: "cfg3_textlike_sparse", 4: "cfg4_click_onehot",
                 5: "cfg5_hashed_stress"}
        traffic_from(args.traffic_from[0], args.traffic_from[1], names[args.workload])
        return

    import torch
    from paper_2004_13940_amd import bench_probe
    from paper_2004_13940_amd import binding as B
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    T = Timed(torch)
    if args.only_config:
        cw = make_config(args.only_config, scale=args.scale)
        print(json.dumps({cw.name: time_config(torch, B, cw, 5, 0)}))
        return
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
    w0, w, V, y, restore = device_state(torch, wl)

    if args.copy_calibration:
        src = torch.ones(COPY_BYTES // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        bench_probe.copy(src, dst, reps=3)
        torch.cuda.synchronize()
        del src, dst
    epoch = lambda: m.fm_sgd_epoch(p, y, w0, w, V)
    for _ in range(args.warmup):
        restore()
        epoch()
    ev_ms, wall = T.run(epoch, args.steps, before=restore)
    ms_per_step = 1e3 * wall / args.steps
    value = wl.nnz * args.steps / wall
    ev = stats(ev_ms)
    print(f"[bench] {ms_per_step:.3f} ms/epoch by the wall clock (restores included), events: median {ev['median_ms']:.3f} "
          f"min {ev['min_ms']:.3f} ms; {value:.4g} nnz/s", file=sys.stderr, flush=True)

    # per-kernel durations from HIP events on the launch stream, over the same number of steps
    m.fm_profile_enable(True)
    for _ in range(args.steps):
        restore()
        epoch()
    prof = m.fm_profile_read()
    m.fm_profile_enable(False)
    counts = np.bincount(wl.col, minlength=wl.D).astype(np.int64)
    ab = algorithmic_bytes(wl.N, wl.D, wl.K, counts)
    kern = {k: {"launches": n, "avg_ms": ms / n} for k, (n, ms) in prof.items() if n > 0}
    dominant = max((k for k in kern if k in ab), key=lambda k: kern[k]["avg_ms"] * kern[k]["launches"])
    dom_ms = kern[dominant]["avg_ms"]
    achieved = ab[dominant] / (dom_ms * 1e-3) / 1e9
    # counter figures: only while the sources they were taken with are the ones that run now
    now = csrc_sha256()
    traffic = epoch_traffic = None
    source = {"file": None, "csrc_sha256_now": now[:16], "csrc_sha256_recorded": None, "match": False}
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl.name}.json")
    tj = {}
    if args.scale == 1.0 and os.path.exists(tpath):
        tj = json.load(open(tpath))
        source.update(file=os.path.relpath(tpath, ROOT), csrc_sha256_recorded=str(tj.get("_csrc_sha256"))[:16],
                      match=tj.get("_csrc_sha256") == now)
        if source["match"]:
            traffic = tj.get(dominant, {}).get("l2_miss_bytes_per_launch")
            epoch_traffic = sum(v["l2_miss_bytes_per_launch"] for v in tj.values() if isinstance(v, dict))
    ep_ms = ev["median_ms"]
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_kind": TRAFFIC_KIND,
                "traffic_source": source,
                "algorithmic_bytes_per_launch": ab[dominant], "avg_launch_ms": dom_ms,
                "traffic_over_algorithmic": None if traffic is None else traffic / ab[dominant],
                "epoch_algorithmic_bytes": ab["epoch"], "epoch_algorithmic_GBs": ab["epoch"] / (ep_ms * 1e-3) / 1e9,
                "epoch_frac": ab["epoch"] / (ep_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "epoch_l2_miss_bytes": epoch_traffic,
                "kernels": {k: {"avg_ms": v["avg_ms"], "algorithmic_GBs": ab[k] / (v["avg_ms"] * 1e-3) / 1e9,
                                "l2_miss_bytes_per_launch": (tj.get(k, {}).get("l2_miss_bytes_per_launch")
                                                             if source["match"] else None)}
                            for k, v in kern.items() if k in ab}}
    # ceiling of the traffic these kernels are bound by: random 128-byte line reads from a buffer of the size of the
    # aggregates, measured here; beside it the lines per second the dominant kernel requests by the counter summary
    try:
        line_peak = bench_probe.gather_rate(max(1 << 20, min(wl.N * 128, 8 << 30)), 128)
    except Exception as e:  # a failed calibration must not lose the measurement
        print(f"[bench] gather calibration failed: {e}", file=sys.stderr, flush=True)
        line_peak = None
    roofline["random_line_reads_per_s"] = line_peak
    roofline["l2_miss_lines_per_s"] = None if traffic is None else traffic / 128.0 / (dom_ms * 1e-3)
    roofline["l2_miss_lines_over_random_line_rate"] = (None if (traffic is None or not line_peak)
                                                        else roofline["l2_miss_lines_per_s"] / line_peak)

    extra = {"events": ev, "column_classes": ab["classes"], "gen_s": t_gen, "upload_s": t_up, "csc_build_s": t_csc,
             "sha256": wl.sha256()[:16], "timing": "value = nnz*steps / wall clock of the loop (one device copy of the "
             "parameters per step restores them inside it); events = HIP events around each epoch alone"}
    if args.minibatch > 0:
        m.fm_partition_batches(args.minibatch)
        restore()
        m.fm_minibatch_epoch(p, y, w0, w, V)
        ms, _ = T.run(lambda: m.fm_minibatch_epoch(p, y, w0, w, V), 3, before=restore)
        extra["minibatch"] = dict(stats(ms), B=args.minibatch, nnz_per_s=wl.nnz / (stats(ms)["median_ms"] * 1e-3))
    m.close()
    del w0, w, V, y
    torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu_baseline:
        tc, n, e, th = oracle_epoch_time(wl, args.cpu_rows, reps=2)
        cpu = {"value": e / tc, "unit": "nnz/s", "cores": th, "kind": "oracle",
               "sample": f"first {n} rows ({e} nnz) of {wl.name}, 2 full-gradient epochs, fp64, {tc:.2f} s/epoch",
               "nproc": os.cpu_count(), "cpu_model": cpu_model()}
        try:
            st = oracle_single_thread(args.workload, min(args.scale, 0.1))
            cpu["single_thread"] = {"value": st["nnz"] / st["s_per_epoch"], "unit": "nnz/s", "cores": st["threads"],
                                    "sample": f"{st['rows']} rows ({st['nnz']} nnz) of the same recipe, 1 epoch, "
                                              f"{st['s_per_epoch']:.2f} s"}
        except Exception as ex:
            print(f"[bench] single-thread oracle run failed: {ex}", file=sys.stderr, flush=True)

    if not args.no_per_config and args.scale == 1.0:
        per = {}
        plan = [(1, 10, 2000), (2, 10, 200_000), (3, 10, 50_000), (4, 10, 0), (5, 5, 100_000)]
        for idx, reps, orows in plan:
            if args.no_cpu_baseline:
                orows = 0
            t0 = time.time()
            cw = wl if idx == args.workload else make_config(idx)
            per[cw.name] = time_config(torch, B, cw, reps, orows)
            print(f"[bench] {cw.name}: epoch {per[cw.name]['epoch']['median_ms']:.3f} ms, stratified "
                  f"{per[cw.name]['stratified']['median_ms']:.3f} ms ({time.time() - t0:.0f}s)", file=sys.stderr, flush=True)
            if idx == 5:
                pw = permuted_columns(cw)
                per[pw.name] = time_config(torch, B, pw, reps, 0)
                print(f"[bench] {pw.name}: epoch {per[pw.name]['epoch']['median_ms']:.3f} ms, stratified "
                      f"{per[pw.name]['stratified']['median_ms']:.3f} ms", file=sys.stderr, flush=True)
                del pw
            if idx != args.workload:
                del cw
        if source["match"] and wl.name in per:  # the counted figure exists for the workload the counters were taken on
            e = per[wl.name]["epoch"]
            e["counted_GBs"] = epoch_traffic / (e["median_ms"] * 1e-3) / 1e9
            f = per[wl.name]["forward"]
            f["counted_GBs"] = tj["rows_forward"]["l2_miss_bytes_per_launch"] / (f["median_ms"] * 1e-3) / 1e9
        if cpu is not None and wl.name in per:
            per[wl.name]["oracle"] = {"s_per_epoch": wl.nnz / cpu["value"], "nnz_per_s": cpu["value"], "threads": cpu["cores"],
                                      "sample": cpu["sample"]}
        extra["per_config"] = per
        extra["per_config_note"] = ("algorithmic_GBs = bytes of the floor formulas (every array streamed once, gathers cached) "
                                    "over the median time; counted_GBs = L2-miss side bytes of the committed counter summary "
                                    "over the same time, only where one exists for the sources that ran")

    out = {"metric": "FM epoch (fwd+grad+update) nonzeros/sec at K=16", "value": value, "unit": "nnz/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{wl.name} scale={args.scale}", "N": wl.N, "D": wl.D, "nnz": wl.nnz, "K": wl.K,
                      "loss": "logistic" if wl.loss == 1 else "squared"},
           "roofline": roofline, "cpu_baseline": cpu, "extra": extra}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
