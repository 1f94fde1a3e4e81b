"""Benchmark of the SGD matrix-factorization hot path on one MI355X.

A step is one epoch of the paper's Algorithm 1 over the whole training set of the workload
(rating fetch, gather, dot, update, scatter, stratum scheduling) in HOGWILD mode, followed by the
held-out RMSE.  The rating matrix is partitioned and resident in HBM before the timed region.
Prints one JSON line: metric, value (updates per second over the timed steps), ms_per_step, config,
`roofline` (algorithmic bytes per launch of the dominant kernel over its measured duration, against
the 8 TB/s HBM peak; `traffic` = memory-side bytes per launch from the rocprofv3 counter passes) and
`cpu_baseline` (the CPU oracle timed on the same workload).
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

# Launch configuration per workload: grid, split rule, scale of the initial factors.  The default
# workload is the largest fp32 one (the Yahoo!Music shape of the paper's Table 1), where the
# factors (833 MB) exceed every cache and the HBM roofline binds.
WORKLOAD_DEFAULTS = {
    "tiny": ("16x16", 1, 0.1),
    "medium": ("256x256", 1, 0.1),
    "large": ("224x224", 1, 0.1),
    "xlarge": ("256x2048", 2, 1.25),
    "stress": ("256x2560", 2, 0.1),
}
# grids of the deterministic mode's side figures (more block rows: its workgroups are single wavefronts)
DET_GRIDS = {"medium": "512x512", "large": "1024x1024", "xlarge": "1024x6144", "stress": "2048x8192"}
CPU_SAMPLE = 16_000_000     # ratings of the workload the CPU oracle is timed on


def profiled_traffic(key):
    """Memory-side bytes per launch of the dominant kernel for this exact configuration, from the
    rocprofv3 counter passes summarised under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by
    what the same counter reads for a plain device copy of known size).  Counters cannot be read
    from inside this process; a summary carries a line `bench-key: <key> traffic_bytes_per_launch=<n>`.
    Returns (bytes, file name) or (None, None)."""
    folder = os.path.join(ROOT, "profiles")
    try:
        names = sorted(os.listdir(folder))
    except OSError:
        return None, None
    for name in names:
        if not name.endswith(".md"):
            continue
        with open(os.path.join(folder, name)) as fh:
            for line in fh:
                if line.startswith("bench-key:") and f" {key} " in line + " ":
                    for word in line.split():
                        if word.startswith("traffic_bytes_per_launch="):
                            return float(word.split("=", 1)[1]), name
    return None, None


def load_dataset(name, factor):
    import workloads

    return workloads.load(name, factor, keep=False)


def cpu_baseline(ds, gr, gc, k, split, scale):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload: the
    first CPU_SAMPLE training ratings in the data's own (seeded, unsorted) order, partitioned by
    the oracle on the same grid and split rule, whole epochs with the independent blocks of every
    stratum on OpenMP threads (bit-identical to the serial order), and the serial oracle on the
    sample's first stratum."""
    import oracle

    cfg = ds.cfg
    take = min(CPU_SAMPLE, ds.rows.size)
    rows, cols, vals = ds.rows[:take], ds.cols[:take], ds.vals[:take]
    perm, bp, _, _ = oracle.partition(rows, cols, cfg.m, cfg.n, gr, gc, split)
    P = oracle.init_factors(cfg.m * k, 1, 0, scale).reshape(cfg.m, k)
    Q = oracle.init_factors(cfg.n * k, 1, 1, scale).reshape(cfg.n, k)
    # whole epochs over the sample until about ten seconds have passed (at least one, at most 64)
    epochs = 0
    t0 = time.perf_counter()
    while epochs < 64 and (epochs == 0 or time.perf_counter() - t0 < 10.0):
        oracle.sgd_epoch_omp(P, Q, rows, cols, vals, perm, bp, gr, gc, cfg.lr, cfg.lam)
        epochs += 1
    t_omp = (time.perf_counter() - t0) / epochs
    # serial: the sample's first strata, about a million ratings
    strata = 1
    while strata < gc and bp[strata * gr] < 1_000_000:
        strata += 1
    bp1 = bp[: strata * gr + 1].copy()
    n1 = int(bp1[-1])
    t0 = time.perf_counter()
    oracle.sgd_epoch(P, Q, rows, cols, vals, perm, bp1, gr, strata, cfg.lr, cfg.lam)
    t_ser = time.perf_counter() - t0
    threads = min(oracle.num_threads(), gr)
    what = "the whole training set" if take == ds.rows.size else f"the first {take} of {ds.rows.size} training ratings (seeded order)"
    return {"value": take / t_omp, "unit": "updates/s", "cores": threads, "kind": "oracle",
            "sample": f"{epochs} epochs over {what}, grid {gr}x{gc}, split {split}, fp64 oracle, "
                      f"independent blocks of each stratum on {threads} OpenMP threads",
            "serial_value": n1 / max(t_ser, 1e-9), "serial_cores": 1,
            "serial_sample": f"the first {strata} strata of the same sample ({n1} updates) on one core",
            "host_cores": len(os.sched_getaffinity(0))}


def epochs_in_one_call(mf, torch, model, cfg, mode, nnz, together=8):
    """`together` epochs in ONE call of mf_sgd_epochs (one launch where an epoch is one launch;
    no RMSE between them), by the wall clock."""
    model.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    model.sgd_epochs(cfg.lr, cfg.lam, mode, together)
    model.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    bytes_per_update = 12 + 4 * cfg.k * (4 if cfg.storage == "f32" else 2)
    value = nnz * together / elapsed
    return {"epochs": together, "value": value, "unit": "updates/s", "ms_per_epoch": elapsed * 1e3 / together,
            "algorithmic_frac_of_hbm_peak": value * bytes_per_update / 1e9 / HBM_PEAK_GBS}


def det_rate(mf, torch, ds, name, steps=3, warmup=1, together=8):
    """Deterministic-mode throughput of a configuration at full size on its grid of DET_GRIDS (side
    figure: epochs alone, by the wall clock)."""
    _, split, scale = WORKLOAD_DEFAULTS[name]
    grid = DET_GRIDS[name]
    gr, gc = (int(x) for x in grid.split("x"))
    cfg = ds.cfg
    model = mf.MatrixFactorization(cfg.m, cfg.n, cfg.k, cfg.storage, seed=1, scale=scale)
    coo = [torch.from_numpy(x).to(model.P.device) for x in (ds.rows, ds.cols, ds.vals)]
    model.load_blocks_device(coo[0], coo[1], coo[2], gr, gc, split)
    del coo
    plan = model.epoch_plan(mf.MF_MODE_DET)
    for i in range(warmup + steps):
        if i == warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        model.sgd_epoch(cfg.lr, cfg.lam, mf.MF_MODE_DET)
    model.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    nnz = ds.rows.size
    one_call = epochs_in_one_call(mf, torch, model, cfg, mf.MF_MODE_DET, nnz, together)
    model.close()
    bytes_per_update = 12 + 4 * cfg.k * (4 if cfg.storage == "f32" else 2)
    value = nnz * steps / elapsed
    return {"workload": f"{cfg.name}: m={cfg.m} n={cfg.n} nnz_train={nnz} k={cfg.k} {cfg.storage}", "mode": "det",
            "grid": grid, "split": split, "steps": steps, "value": value, "unit": "updates/s",
            "ms_per_step": elapsed * 1e3 / steps,
            "algorithmic_frac_of_hbm_peak": value * bytes_per_update / 1e9 / HBM_PEAK_GBS,
            "kernel": plan["kernel"], "waves_per_workgroup": plan["waves"], "launches_per_epoch": plan["launches"],
            "epochs_in_one_call": one_call}


def quick_rate(mf, torch, name, steps=5, warmup=2):
    """Hogwild throughput of another configuration at full size on its grid of WORKLOAD_DEFAULTS (a
    few steps of epoch + held-out RMSE by the wall clock; these are side figures, the line's
    `value` is timed separately)."""
    grid, split, scale = WORKLOAD_DEFAULTS[name]
    gr, gc = (int(x) for x in grid.split("x"))
    ds = load_dataset(name, 1.0)
    cfg = ds.cfg
    model = mf.MatrixFactorization(cfg.m, cfg.n, cfg.k, cfg.storage, seed=1, scale=scale)
    coo = [torch.from_numpy(x).to(model.P.device) for x in (ds.rows, ds.cols, ds.vals)]
    model.load_blocks_device(coo[0], coo[1], coo[2], gr, gc, split)
    del coo
    test = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    plan = model.epoch_plan(mf.MF_MODE_HOGWILD)
    rmse = float("nan")
    for i in range(warmup + steps):
        if i == warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        model.sgd_epoch(cfg.lr, cfg.lam, mf.MF_MODE_HOGWILD)
        rmse = model.rmse(*test)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    nnz = ds.rows.size
    one_call = epochs_in_one_call(mf, torch, model, cfg, mf.MF_MODE_HOGWILD, nnz)
    model.close()
    bytes_per_update = 12 + 4 * cfg.k * (4 if cfg.storage == "f32" else 2)
    value = nnz * steps / elapsed
    return [{"workload": f"{cfg.name}: m={cfg.m} n={cfg.n} nnz_train={nnz} k={cfg.k} {cfg.storage}", "mode": "hogwild",
             "grid": grid, "split": split, "steps": steps, "value": value, "unit": "updates/s",
             "ms_per_step": elapsed * 1e3 / steps, "bytes_per_update": bytes_per_update,
             "algorithmic_frac_of_hbm_peak": value * bytes_per_update / 1e9 / HBM_PEAK_GBS,
             "kernel": plan["kernel"], "waves_per_workgroup": plan["waves"], "held_out_rmse": rmse,
             "epochs_in_one_call": one_call},
            det_rate(mf, torch, ds, name)]


def block_size_curve(args, mf, ds):
    """--curve: kernel time per launch against ratings per launch, on random subsets of the
    workload at a fixed grid, for one launch per stratum and for one launch per epoch (the
    analogue of the paper's Fig. 3a / Fig. 7), with least-squares fits of the two forms of the
    paper's kernel cost model (Section 5.3): T = a|R| + b, and T = |R| / (a log|R| + b).
    Prints the markdown tables of profiles/block_size_curve_<workload>.md."""
    import numpy as np

    cfg = ds.cfg
    rng = np.random.Generator(np.random.Philox(7))
    fractions = (0.01, 0.02, 0.05, 0.1, 0.2, 0.35, 0.5, 0.75, 1.0)
    print(f"# Kernel time against ratings per launch: {cfg.name}, k={cfg.k} {cfg.storage}, Hogwild, LDS kernels")
    print(f"\nCommand: `python bench.py --curve --workload {args.workload} --steps {args.steps}`"
          " (times: HIP events around every launch, MF_OPT_PROFILE).\n")
    for grid, ring in ((128, 0), (224, 1)):
        pts = []
        for frac in fractions:
            keep = rng.random(ds.rows.size) < frac
            rows, cols, vals = (np.ascontiguousarray(x[keep]) for x in (ds.rows, ds.cols, ds.vals))
            model = mf.MatrixFactorization(cfg.m, cfg.n, cfg.k, cfg.storage, scale=args.init_scale,
                                           options={mf.MF_OPT_PROFILE: 1, mf.MF_OPT_RING: ring,
                                                    mf.MF_OPT_HOGWILD_KERNEL: mf.MF_HOGWILD_LDS})
            model.load_blocks(rows, cols, vals, grid, grid, mf.MF_SPLIT_NNZ_BALANCED)
            model.sgd_epoch(cfg.lr, cfg.lam, mf.MF_MODE_HOGWILD)
            mf.binding.mf_profile_read(model.ctx)
            for _ in range(args.steps):
                model.sgd_epoch(cfg.lr, cfg.lam, mf.MF_MODE_HOGWILD)
            ms, launches = mf.binding.mf_profile_read(model.ctx)
            model.close()
            pts.append((rows.size * args.steps / launches, ms / launches * 1e3))
        size = np.array([p[0] for p in pts])
        us = np.array([p[1] for p in pts])
        a1, b1 = np.polyfit(size, us, 1)
        rate = size / us                                     # ratings per microsecond = a log|R| + b
        a2, b2 = np.polyfit(np.log(size), rate, 1)
        fit1, fit2 = a1 * size + b1, size / (a2 * np.log(size) + b2)
        what = "one launch per epoch" if ring else "one launch per stratum"
        print(f"## {what}, {grid} x {grid} grid: |R| = ratings per launch\n")
        print("| ratings |R| | kernel us | G updates/s | affine fit us | log-model fit us |\n|---|---|---|---|---|")
        for i in range(size.size):
            print(f"| {size[i]:.0f} | {us[i]:.2f} | {size[i] / us[i] / 1e3:.3f} | {fit1[i]:.2f} | {fit2[i]:.2f} |")
        e1, e2 = np.abs(fit1 - us) / us, np.abs(fit2 - us) / us
        print(f"\nT = a|R| + b: a = {a1 * 1e3:.4f} ns per rating, b = {b1:.2f} us; mean relative error {e1.mean() * 100:.1f} %, "
              f"max {e1.max() * 100:.1f} %; asymptotic rate {1e-3 / a1:.2f} G updates/s.")
        print(f"T = |R| / (a log|R| + b): a = {a2:.2f}, b = {b2:.2f} (ratings per us); mean relative error "
              f"{e2.mean() * 100:.1f} %, max {e2.max() * 100:.1f} %.\n")


def rmse_kernel_bench(args, mf, model, nnz, k, elt):
    """--rmse-bench: the RMSE kernel alone over the loaded training ratings (packed order)."""
    import torch

    model.rmse()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        value = model.rmse()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    per_entry = 12 + 2 * k * elt                 # rating record + read of p_u and q_v
    print(json.dumps({"rmse_kernel": True, "entries": nnz, "ms_per_call": dt * 1e3, "entries_per_s": nnz / dt,
                      "bytes_per_entry": per_entry, "algorithmic_gbs": nnz * per_entry / dt / 1e9,
                      "frac_of_hbm_peak": nnz * per_entry / dt / 1e9 / HBM_PEAK_GBS, "train_rmse": value}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="xlarge", choices=sorted(WORKLOAD_DEFAULTS))
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (testing only)")
    ap.add_argument("--init-scale", type=float, default=None,
                    help="initial factors are uniform in [0, this); default: the workload's (WORKLOAD_DEFAULTS)")
    ap.add_argument("--mode", default="hogwild", choices=["hogwild", "det"])
    ap.add_argument("--grid", default=None, help="GRxGC; default: the workload's (WORKLOAD_DEFAULTS)")
    ap.add_argument("--hogwild-kernel", default="auto", choices=["auto", "global_atomics", "lds"])
    ap.add_argument("--lds-chunk", type=int, default=0)
    ap.add_argument("--lds-waves", type=int, default=0, help="0: the library's choice")
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--affinity", type=int, default=1)
    ap.add_argument("--split", type=int, default=None,
                    help="0 equal width, 1 ratings balanced, 2 ratings and width balanced; default: the workload's")
    ap.add_argument("--ring", type=int, default=1, help="1: one launch per epoch (workgroups hand the strips round)")
    ap.add_argument("--epochs-per-call", type=int, default=1,
                    help="more than 1: a step is that many epochs in one call of mf_sgd_epochs, then the held-out RMSE")
    ap.add_argument("--stratum-seed", type=int, default=0,
                    help="nonzero: every epoch visits the strata in a seeded random order (mf_stratum_order)")
    ap.add_argument("--pack-strips", type=int, default=1, help="0: the LDS kernels always keep whole strips; 2: packed strips wherever possible")
    ap.add_argument("--load", default="device", choices=["host", "device"],
                    help="partition on the host (mf_load_blocks) or on the GPU (mf_load_blocks_device); outside the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the side figures for the other full-size configurations (default run only)")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--curve", action="store_true",
                    help="print the block-size curve of the workload (subsampled, both launch schemes) and exit")
    ap.add_argument("--rmse-bench", action="store_true",
                    help="time mf_rmse over the loaded training ratings --steps times and exit")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of this many MiB five times (a kernel of known "
                         "traffic, used to scale the profiler's FETCH_SIZE / WRITE_SIZE readings) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2006_15980_amd as mf

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(3)
    if args.copy_calibration > 0:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_mib": args.copy_calibration, "bytes_read": n * 4, "bytes_written": n * 4,
                          "launches": 5}))
        return
    d_grid, d_split, d_scale = WORKLOAD_DEFAULTS[args.workload]
    args.grid = args.grid or d_grid
    args.split = d_split if args.split is None else args.split
    args.init_scale = d_scale if args.init_scale is None else args.init_scale
    t0 = time.perf_counter()
    ds = load_dataset(args.workload, args.scale)
    t_generate = time.perf_counter() - t0
    cfg = ds.cfg
    if args.curve:
        block_size_curve(args, mf, ds)
        return
    gr, gc = (int(x) for x in args.grid.split("x"))
    mode = mf.MF_MODE_HOGWILD if args.mode == "hogwild" else mf.MF_MODE_DET
    k = cfg.k
    elt = 4 if cfg.storage == "f32" else 2
    bytes_per_update = 12 + 4 * k * elt      # rating record + read and write of p_u and q_v

    which = {"auto": mf.MF_HOGWILD_AUTO, "global_atomics": mf.MF_HOGWILD_GLOBAL_ATOMICS,
             "lds": mf.MF_HOGWILD_LDS}[args.hogwild_kernel]
    opts = {mf.MF_OPT_HOGWILD_CHUNK: args.chunk, mf.MF_OPT_XCD_AFFINITY: args.affinity,
            mf.MF_OPT_HOGWILD_KERNEL: which,
            mf.MF_OPT_LDS_CHUNK: args.lds_chunk, mf.MF_OPT_RING: args.ring, mf.MF_OPT_PACK_STRIPS: args.pack_strips}
    if args.lds_waves:
        opts[mf.MF_OPT_LDS_WAVES] = args.lds_waves
    model = mf.MatrixFactorization(cfg.m, cfg.n, k, cfg.storage, seed=1, scale=args.init_scale, options=opts)
    if args.load == "device":
        import torch
        coo = [torch.from_numpy(x).to(model.P.device) for x in (ds.rows, ds.cols, ds.vals)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        model.load_blocks_device(coo[0], coo[1], coo[2], gr, gc, args.split)
        model.sync()
        t_load = time.perf_counter() - t0
        del coo
    else:
        t0 = time.perf_counter()
        model.load_blocks(ds.rows, ds.cols, ds.vals, gr, gc, args.split)
        model.sync()
        t_load = time.perf_counter() - t0
    tr, tc, tv = model.to_device(ds.test_rows, ds.test_cols, ds.test_vals)
    nnz = ds.rows.size * max(1, args.epochs_per_call)     # updates per step
    if args.rmse_bench:
        rmse_kernel_bench(args, mf, model, nnz, k, elt)
        model.close()
        return
    plan = model.epoch_plan(mode)     # the kernel the library launches for this mode and grid
    print(f"bench: {cfg.name} generated in {t_generate:.1f} s, loaded in {t_load:.2f} s; {plan['note']}",
          file=sys.stderr, flush=True)

    epochs_run = [0]

    def run_steps(count):
        last = float("nan")
        for _ in range(count):
            order = None
            if args.stratum_seed:
                order = mf.binding.mf_stratum_order(args.stratum_seed, epochs_run[0], gc)
            if args.epochs_per_call > 1:
                model.sgd_epochs(cfg.lr, cfg.lam, mode, args.epochs_per_call)
            else:
                model.sgd_epoch(cfg.lr, cfg.lam, mode, stratum_order=order)
            epochs_run[0] += args.epochs_per_call
            last = model.rmse(tr, tc, tv)
        return last

    # timed region: K steps, no per-launch instrumentation
    mf.binding.mf_set_option(model.ctx, mf.MF_OPT_PROFILE, 0)
    run_steps(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    rmse = run_steps(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # the same K steps once more with every SGD kernel launch bracketed by HIP events on the
    # library's stream (the brackets cost about as much as the launches they time, so they are
    # kept out of the region above); gives the kernel's average duration for the roofline
    kernel_ms, launches, elapsed_events = 0.0, 0, 0.0
    if not args.no_kernel_events:
        mf.binding.mf_set_option(model.ctx, mf.MF_OPT_PROFILE, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rmse = run_steps(args.steps)
        torch.cuda.synchronize()
        elapsed_events = time.perf_counter() - t0
        kernel_ms, launches = mf.binding.mf_profile_read(model.ctx)
    # the default run adds side figures (the profiles' commands, with --no-cpu-baseline, do not)
    default_run = (args.workload == "xlarge" and args.scale == 1.0 and args.mode == "hogwild" and args.grid == d_grid
                   and args.split == d_split and not args.no_cpu_baseline and args.stratum_seed == 0
                   and args.epochs_per_call == 1)
    one_call = None
    if default_run and not args.no_per_config:
        mf.binding.mf_set_option(model.ctx, mf.MF_OPT_PROFILE, 0)
        one_call = epochs_in_one_call(mf, torch, model, cfg, mode, nnz)
    model.close()

    value = nnz * args.steps / elapsed
    roofline = None
    if launches > 0:
        avg_s = kernel_ms * 1e-3 / launches
        bytes_per_launch = bytes_per_update * nnz * args.steps / launches
        achieved = bytes_per_launch / avg_s / 1e9
        # `achieved` counts ALGORITHMIC bytes (12 + 4*k*sizeof(storage) per update): what the path
        # would move without any reuse.  The kernel keeps column strips in LDS and rows in the
        # L2s, so it can exceed what the memory really carried; `traffic` is that real figure,
        # taken from the counter passes summarised in `traffic_source`, not measured in this run.
        key = (f"workload={args.workload} scale={args.scale:g} mode={args.mode} grid={args.grid} split={args.split} "
               f"kernel={plan['kernel']} waves={plan['waves']}")
        traffic, source = profiled_traffic(key)
        if args.lds_chunk != 0 or args.chunk != 0 or not args.affinity or args.pack_strips != 1 or args.stratum_seed != 0 or args.epochs_per_call != 1:
            traffic, source = None, None
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                    "traffic_source": None if source is None else "profiles/" + source,
                    "kernel": "%s<%s,%d>" % (plan["kernel"], "float" if cfg.storage == "f32" else "__half", k),
                    "waves_per_workgroup": plan["waves"],
                    "avg_launch_us": avg_s * 1e6, "launches_per_step": launches / args.steps,
                    "updates_per_launch": nnz * args.steps / launches,
                    "bytes_per_update": bytes_per_update,
                    "traffic_gbs": None if traffic is None else traffic / avg_s / 1e9,
                    "traffic_frac_of_peak": None if traffic is None else traffic / avg_s / 1e9 / HBM_PEAK_GBS,
                    "profile_key": key,
                    "ms_per_step_with_event_brackets": elapsed_events * 1e3 / args.steps}
    mode_name = "HOGWILD" if args.mode == "hogwild" else "deterministic"
    out = {"metric": f"SGD updates/s at k={k} ({mode_name} epoch + held-out RMSE per step)", "value": value,
           "unit": "updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": elapsed * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32" if cfg.storage == "f32" else "f16 storage / f32 math",
           "data": "synthetic",
           "config": {"workload": f"{cfg.name}: m={cfg.m} n={cfg.n} nnz_train={nnz} k={k} {cfg.storage}",
                      "mode": args.mode, "grid": args.grid, "split": args.split, "init_scale": args.init_scale,
                      "hogwild_kernel": args.hogwild_kernel,
                      "lds_chunk": args.lds_chunk, "lds_waves": args.lds_waves, "ring": args.ring,
                      "pack_strips": args.pack_strips, "stratum_seed": args.stratum_seed, "epochs_per_call": args.epochs_per_call,
                      "chunk": args.chunk,
                      "xcd_affinity": args.affinity,
                      "lr": cfg.lr, "lambda": cfg.lam},
           "final_test_rmse": rmse, "generate_s": t_generate, "load_blocks_s": t_load, "load_path": args.load,
           "algorithmic_gbs": value * bytes_per_update / 1e9,
           "hbm_roofline_frac": value * bytes_per_update / 1e9 / HBM_PEAK_GBS,
           "roofline": roofline}
    if one_call:
        # side figure: epochs without the RMSE between them, in one call (never `value`)
        out["epochs_in_one_call"] = one_call
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(ds, gr, gc, k, args.split, args.init_scale)
    if default_run and not args.no_per_config:
        # side figures: this configuration in deterministic mode, then the other configurations at
        # full size on their grids in both modes
        out["per_config"] = [det_rate(mf, torch, ds, "xlarge")]
        del ds
        import workloads
        workloads.forget()
        for name in ("medium", "large", "stress"):
            out["per_config"] += quick_rate(mf, torch, name)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
