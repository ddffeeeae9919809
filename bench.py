"""Benchmark of the DistGrid training hot path on one MI355X.

One "step" is one forward + backward pass of every hot-path stage (ray/box segments, distribution,
sampling, direction encoding, hash-grid encode, MLPs, segment compositing, merge, loss seeds and
all their backward passes, including zeroing the gradient buffers) over one batch of synthetic
rays that is already resident in HBM.  The headline workload is the largest single-GPU
configuration: one GPU's share of a 2 x 4 tiling (c5_share: 2^20 rays x 64 samples, L=16, F=2,
T=2^24, all eight boxes traced, one sub-model resident, the other boxes' partials synthetic).
The other paper-scale configurations are timed after it and reported as blocks of the same
line (`also`).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5_share] [--also c4_big,c3_2x2,c2_ngp,c1_tiny]
                    [--no-cpu-baseline] [--no-optimizer] [--no-peaks]

--workload c7_occ runs c2's scene with occupancy-guided sampling (Sec. 3.2, Sec. 5.1) instead of 64 stratified
samples per segment, and also times the occupancy refresh.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA, published
LINE_BYTES = 128               # what one L2 miss fetches

# HBM-side bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (scaled by a plain copy kernel of known size), summed
# over the kernels an entry point launches: (fetched, written).  Measured once per workload with the kernels as they
# stand; the runs, their commands and the calibration are in profiles/<workload>_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = {
    "c5_share": {"dg_hashgrid_encode_fwd": (283.1e9, 4.295e9), "dg_hashgrid_encode_bwd": (71.77e9, 55.86e9), "dg_mlp_fwd": (4.368e9, 1.074e9),
                 "dg_mlp_bwd": (11.96e9, 10.82e9)},
    "c4_big": {"dg_hashgrid_encode_fwd": (82.81e9, 1.275e9), "dg_hashgrid_encode_bwd": (19.05e9, 14.98e9), "dg_mlp_fwd": (1.456e9, 0.3168e9),
               "dg_mlp_bwd": (3.939e9, 3.247e9)},
    "c2_ngp": {"dg_hashgrid_encode_fwd": (6.503e9, 0.854e9), "dg_hashgrid_encode_bwd": (10.91e9, 6.764e9), "dg_mlp_fwd": (0.8681e9, 0.2135e9),
               "dg_mlp_bwd": (2.44e9, 2.214e9)},
}


def algorithmic_work(entry, L, F, n_samples, mlp_flops_fwd):
    """(bound, units of work per launch) for an entry point; bytes for HBM-bound ones, flops for the MLPs.

    encode fwd : 12 B coordinates + L*8 corners*F*4 B table reads + L*F*2 B fp16 features per sample
    encode bwd : 12 B coordinates + L*F*4 B feature gradient + L*8*F*4 B of atomic adds per sample
    MLP fwd    : useful multiply-adds of both networks x 2;  MLP bwd: twice that again (dgrad + wgrad)
                 plus the recomputed forward
    """
    gather = L * 8 * F * 4
    if entry == "dg_hashgrid_encode_fwd":
        return "hbm", n_samples * (12 + gather + L * F * 2)
    if entry == "dg_hashgrid_encode_bwd":
        return "hbm", n_samples * (12 + L * F * 4 + gather)
    if entry == "dg_mlp_fwd":
        return "mfma", n_samples * mlp_flops_fwd
    if entry == "dg_mlp_bwd":
        return "mfma", n_samples * mlp_flops_fwd * 3
    return "hbm", None


def workload_config(name):
    """The configuration with the partition set the benchmark traces and the partitions whose sub-models are resident."""
    import dg_inputs as di
    cfg = di.config(name)
    P = cfg["parts"].shape[0]
    resident = [cfg["resident"]] if "resident" in cfg else list(range(P))
    return cfg, resident


# ------------------------------------------------------------------------------------------------ CPU baseline
def _oracle_pass(job):
    """One forward + backward pass of the oracle over rays [lo, hi) of the batch (runs in a forked worker or in place)."""
    import oracle.step as ostep
    lo, hi = job
    cfg, hm, ho, app, resident, o, d, Cgt = _ORACLE_STATE
    t = time.perf_counter()
    ostep.run_step(cfg, hm, o[lo:hi], d[lo:hi], Cgt[lo:hi], seed=0, lambda1=1e-3, loss_scale=65536.0, resident=resident, occ=ho,
                   appearance=None if app is None else (app[0], app[1][lo:hi]))
    return time.perf_counter() - t


_ORACLE_STATE = None


def cpu_baseline(name, rays_per_core):
    """The oracle as it stands on this machine's host cores: first on one core, then one process per core, each over
    its own `rays_per_core` rays of the same batch with the full-size tables (forked after the tables are built, so the
    workers share them).  Must run before anything initialises the GPU: the workers are forks of this process."""
    global _ORACLE_STATE
    import multiprocessing as mp
    import dg_inputs as di
    import oracle.step as ostep
    cfg, resident = workload_config(name)
    R = cfg["R"]
    o, d = di.make_rays(cfg, seed=0)
    Cgt = di.make_targets(R, seed=0)
    hm = ostep.make_models(dict(cfg, resident_list=resident), seed=0)
    ho = ostep.make_occupancy(cfg, seed=0) if "occ" in cfg else None
    app = di.make_appearance(cfg["n_images"], cfg["mlp"]["n_app"], R, seed=0) if cfg["mlp"].get("n_app") else None
    _ORACLE_STATE = (cfg, hm, ho, app, resident, o, d, Cgt)
    Rc = min(rays_per_core, R)
    single_s = _oracle_pass((0, Rc))
    # the box gives this job 16 cores whatever the machine reports
    cores = max(1, min(16, os.cpu_count() or 1, R // Rc))
    jobs = [(k * Rc, (k + 1) * Rc) for k in range(cores)]
    t = time.perf_counter()
    with mp.get_context("fork").Pool(cores) as pool:
        pool.map(_oracle_pass, jobs)
    all_s = time.perf_counter() - t
    _ORACLE_STATE = None
    model = ""
    try:
        model = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
    except (OSError, StopIteration):
        pass
    return {"value": round(cores * Rc / all_s, 2), "unit": "rays/s", "cores": cores, "kind": "oracle",
            "sample": "%d rays per core of the same batch (%s), full-size tables, one fwd+bwd pass, one process per core, %.1f s"
                      % (Rc, name, all_s),
            "single_core": {"value": round(Rc / single_s, 2), "unit": "rays/s", "cores": 1,
                            "sample": "first %d rays, %.1f s" % (Rc, single_s)},
            "nproc": os.cpu_count(), "cpu_model": model}


# ------------------------------------------------------------------------------------------------ one workload on the GPU
def run_workload(name, steps, warmup, peaks, with_optimiser=True, with_evaluation=True):
    import numpy as np
    import torch
    import dg_inputs as di
    from paper_2405_04416_amd import binding as B
    from paper_2405_04416_amd.step import Occupancy, SubModel, TrainStep, split_appearance_columns

    dev = torch.device("cuda:0")
    cfg, resident = workload_config(name)
    g, m = cfg["grid"], cfg["mlp"]
    R, S, k_max = cfg["R"], cfg["S"], cfg["k_max"]
    P = cfg["parts"].shape[0]
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # seeded synthetic inputs, moved to HBM before anything is timed
    o, d = di.make_rays(cfg, seed=0)
    Cgt = di.make_targets(R, seed=0)
    n_feat = g["L"] * g["F"]
    models = {}
    for p in resident:
        gp = di.grid_params(cfg, p)            # the coarse level of a cascade has its own table length
        growth = gp.get("growth") or B.dg_growth_factor(gp["n_min"], gp["n_max"], gp["L"])
        grid = B.dg_grid_desc_init(gp["L"], gp["F"], gp["log2_T"], gp["n_min"], growth, di.box_extent(cfg["parts"][p]))
        mlp = B.dg_mlp_desc(n_feat, m["n_hidden_d"], m["n_geo"], m["sh_degree"] ** 2, m["n_hidden_c"], m["n_layers_c"], 1,
                            m.get("n_app", 0))
        table = to_dev(di.make_table(grid.n_entries, gp["F"], cfg["table_range"], seed=1000 * p))
        weights = to_dev(split_appearance_columns(di.make_mlp_weights(n_feat, m, seed=1000 * p), mlp))
        models[p] = SubModel(grid, mlp, table, weights)
    od, dd, Cd = to_dev(o), to_dev(d), to_dev(Cgt)
    occupancy, extra = None, {}
    if "occ" in cfg:
        # occupancy-guided sampling: seeded stand-in densities per cell, thresholded by the library into the bit field
        occupancy = {}
        for p in resident:
            ext = di.box_extent(cfg["parts"][p])
            desc = B.dg_occ_desc_init(cfg["occ"]["res"], ext)
            density = to_dev(di.make_cell_densities(list(desc.res), seed=1000 * p))
            bits = torch.zeros((desc.n_cells + 31) // 32, dtype=torch.int32, device=dev)
            occupancy[p] = Occupancy(desc, density, bits, np.float32(float(ext.max()) * np.sqrt(3.0) / 1024), cfg["occ"]["max_steps"])
            B.dg_occ_bits(density, 0.6, bits, occupancy[p].n_set)
        extra = dict(occupancy=occupancy, max_samples=R * 32)
    if m.get("n_app"):
        # appearance vectors per image as further colour-net inputs (Sec. 4.4.3): seeded stand-ins, every ray in a random image
        app_host = di.make_appearance(cfg["n_images"], m["n_app"], R, seed=0)
        extra["appearance"] = (to_dev(app_host[0]), to_dev(app_host[1].view(np.int32)))
    # room for the resident sub-models' segments: a ray crosses a box once (twice where the box has a hole)
    max_segments = R * min(k_max, 4) if len(resident) == P else R * len(resident)
    step = TrainStep(to_dev(cfg["parts"]), models, resident, R, S, k_max, m["sh_degree"], loss_scale=65536.0,
                     lambda1=1e-3, seed=0, holes=to_dev(cfg["holes"]) if "holes" in cfg else None,
                     max_segments=max_segments, foreign_prefilled=len(resident) < P, encode_ws_cap=72 << 30, **extra)
    if len(resident) < P:
        # partial results of the boxes whose sub-models live on other GPUs: synthetic (colour, transmittance) in every
        # slot, written once -- the local rendering overwrites the slots of the resident box's segments every step, the
        # merge reads the first seg_count[r] slots of a ray
        fC, fT = di.make_foreign_partials(R, k_max, seed=0)
        step.Ck.copy_(to_dev(fC)); step.Tk.copy_(to_dev(fT))

    for w in range(warmup):
        step.seed = w
        step.step(od, dd, Cd)
    torch.cuda.synchronize()
    step.timings = {}
    t0 = time.perf_counter()
    for k in range(steps):
        step.seed = warmup + k                 # fresh jitter every step, drawn inside the sampling kernel
        step.step(od, dd, Cd)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / steps
    n_seg = sum(step.offsets[p + 1] - step.offsets[p] for p in resident)
    n_samples = n_seg * S if occupancy is None else sum(n for _, n in step.samples.values())
    per_call = step.timing_summary()           # HIP events on the launch stream, inside the timed region
    seg_hist = torch.bincount(step.seg_count, minlength=k_max + 1).cpu().tolist()

    # the count sweep that TrainStep runs ahead on its second stream, timed alone (it is hidden inside the step)
    count_ahead_ms = None
    if step.side is not None and occupancy is None:
        p0 = resident[0]
        n0 = (step.offsets[p0 + 1] - step.offsets[p0]) * S
        if n0 and B.dg_hashgrid_encode_bwd_workspace_bytes(models[p0].grid, n0) <= step.ws_enc.numel() * 4:
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            B.dg_hashgrid_encode_bwd_count(models[p0].grid, step.u[:n0], n0, step.ws_enc)
            ev[0].record()
            for _ in range(3):
                B.dg_hashgrid_encode_bwd_count(models[p0].grid, step.u[:n0], n0, step.ws_enc)
            ev[1].record()
            ev[1].synchronize()
            count_ahead_ms = ev[0].elapsed_time(ev[1]) / 3

    # the occupancy refresh (every 16th iteration, Sec. 5.1), measured apart from the metric, in both of its forms
    refresh = None
    if occupancy is not None:
        cells = sum(q.desc.n_cells for q in occupancy.values())
        refresh = {"cells": cells, "occupied_fraction": round(sum(int(q.n_set.item()) for q in occupancy.values()) / cells, 4)}
        for label, it in (("warmup_all_cells", 16), ("half_uniform_half_occupied", 4112)):
            saved = {p: (q.density.clone(), q.bits.clone()) for p, q in occupancy.items()}
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            step.timings = None
            step.refresh_occupancy(it)
            torch.cuda.synchronize()
            refresh[label] = {"ms": round(1e3 * (time.perf_counter() - t1), 3),
                              "candidates": sum(q.desc.n_cells // (1 if it < 4096 else 2) for q in occupancy.values())}
            for p, q in occupancy.items():         # the random-weight field is no scene: put the stand-in grid back
                q.density.copy_(saved[p][0]); q.bits.copy_(saved[p][1])

    # the optimiser sweep (Sec. 5.1: Adam), measured apart from the metric: `value` stays the forward+backward rate
    optimiser = None
    if with_optimiser:
        n_param = sum(models[p].table.numel() for p in resident)
        touched = sum(int(torch.count_nonzero(models[p].dtable)) for p in resident)
        step.timings = {}
        for k in range(3):
            if k:
                step.step(od, dd, Cd)                      # fresh gradients for every sweep
            step.optimiser_step(k)
        calls, total_ms = step.timing_summary()["dg_adam_step"]
        ms = total_ms / 3
        moved = touched * 32 + (n_param - touched) * 4     # touched: value, gradient, 2 moments read and written; else the gradient read
        optimiser = {"entry": "dg_adam_step", "ms_per_step": round(ms, 4), "parameters": n_param,
                     "touched_fraction": round(touched / n_param, 4), "algorithmic_bytes": moved,
                     "GB/s": round(moved / (ms * 1e-3) / 1e9, 1), "frac_hbm": round(moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # evaluation rendering (forward only: colour, depth, transmittance; Sec. 4.4.2), apart from the metric
    evaluation = None
    if with_evaluation:
        step.timings = None
        step.render(od, dd)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(3):
            step.render(od, dd)
        torch.cuda.synchronize()
        ev_ms = 1e3 * (time.perf_counter() - t1) / 3
        evaluation = {"ms_per_batch": round(ev_ms, 4), "rays_per_s": round(R / (ev_ms * 1e-3), 1), "outputs": "colour, depth, transmittance"}

    shapes = di.mlp_layer_shapes(n_feat, m)
    mlp_flops_fwd = 2 * sum(no * ni for no, ni in shapes)
    breakdown = {k: round(ms / steps, 4) for k, (n, ms) in sorted(per_call.items(), key=lambda kv: -kv[1][1])}
    per_launch_samples = n_samples / max(len(resident), 1)
    traffic = MEASURED_TRAFFIC_BYTES.get(name, {})
    copy_peak = (peaks or {}).get("stream_copy_GBps")
    gather_peak = (peaks or {}).get("random_gather_16B_1024MiB_Gps")
    atomic_peak = (peaks or {}).get("random_atomic_add_f32_1024MiB_Gps")
    mfma_peak = (peaks or {}).get("mfma_f16_32x32x16_TFLOPs")

    # every headline entry point: time per launch, algorithmic rate against the datasheet peak, the rate by measured HBM
    # traffic where a profile of this workload exists, and the rate against the yardstick measured in this run
    kernels = {}
    for entry in ("dg_hashgrid_encode_fwd", "dg_hashgrid_encode_bwd", "dg_mlp_fwd", "dg_mlp_bwd"):
        if entry not in per_call:
            continue
        c, t = per_call[entry]
        k = {"avg_launch_ms": round(t / c, 4)}
        if entry == "dg_hashgrid_encode_bwd" and count_ahead_ms is not None:
            # the count sweep of the first sub-model's pass runs on a second stream beside the forward gather, so it is not
            # inside this entry point's events; its stand-alone time is part of the pass all the same and is added before
            # any rate is formed
            k["count_sweep_on_second_stream_ms"] = round(count_ahead_ms, 4)
            t += count_ahead_ms * steps
        sec = t / c * 1e-3
        bound, work = algorithmic_work(entry, g["L"], g["F"], per_launch_samples, mlp_flops_fwd)
        if bound == "hbm":
            k["algorithmic_GBps"] = round(work / sec / 1e9, 1)
            k["algorithmic_frac_of_hbm_peak"] = round(work / sec / 1e9 / HBM_PEAK_GBS, 4)
            if entry in traffic:
                fetched, written = traffic[entry]
                k["hbm_traffic_bytes"] = fetched + written
                k["hbm_GBps_by_counters"] = round((fetched + written) / sec / 1e9, 1)
                k["counters_frac_of_hbm_peak"] = round((fetched + written) / sec / 1e9 / HBM_PEAK_GBS, 4)
                k["traffic_over_algorithmic"] = round((fetched + written) / work, 2)
                if copy_peak:
                    k["counters_frac_of_measured_copy"] = round((fetched + written) / sec / 1e9 / copy_peak, 3)
                if entry == "dg_hashgrid_encode_fwd" and gather_peak:
                    lines = fetched / LINE_BYTES / sec / 1e9
                    k["lines_fetched_Gps"] = round(lines, 2)
                    k["frac_of_measured_random_gather"] = round(lines / gather_peak, 3)
            if entry == "dg_hashgrid_encode_bwd":
                adds = per_launch_samples * g["L"] * 8 * g["F"] / sec / 1e9
                k["scatter_adds_Gps"] = round(adds, 1)
                if atomic_peak:
                    k["vs_measured_atomic_add"] = round(adds / atomic_peak, 2)
        else:
            k["TFLOPs"] = round(work / sec / 1e12, 2)
            k["frac_of_mfma_peak"] = round(work / sec / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)
            if mfma_peak:
                k["frac_of_measured_mfma_loop"] = round(work / sec / 1e12 / mfma_peak, 4)
        kernels[entry] = k

    dominant = next(iter(breakdown))
    calls, total_ms = per_call[dominant]
    avg_ms = total_ms / calls
    bound, work = algorithmic_work(dominant, g["L"], g["F"], per_launch_samples, mlp_flops_fwd)
    moved = sum(traffic[dominant]) if dominant in traffic else None
    if work is None:
        roofline = {"kernel": dominant, "bound": bound, "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": None, "traffic": None, "avg_launch_ms": round(avg_ms, 4)}
    elif bound == "hbm":
        ach = work / (avg_ms * 1e-3) / 1e9
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": moved, "algorithmic_bytes": work,
                    "avg_launch_ms": round(avg_ms, 4)}
        if moved:
            # what the memory system actually moved for this launch, as a rate: a random 8-byte gather out of tables that no
            # cache holds fetches a whole 128-byte line per miss, so this rate, not the algorithmic one, is what HBM sees
            roofline["achieved_by_traffic"] = round(moved / (avg_ms * 1e-3) / 1e9, 1)
            roofline["frac_by_traffic"] = round(moved / (avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    else:
        ach = work / (avg_ms * 1e-3) / 1e12
        roofline = {"kernel": dominant, "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_F16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / MFMA_F16_PEAK_TFLOPS, 4), "traffic": moved,
                    "avg_launch_ms": round(avg_ms, 4)}

    out = {
        "value": round(R / (ms_per_step * 1e-3), 1), "ms_per_step": round(ms_per_step, 4), "steps": steps, "warmup": warmup,
        "config": {"workload": name, "rays": R,
                   "samples_per_segment": S if occupancy is None else round(n_samples / max(n_seg, 1), 2), "segments": n_seg,
                   "segments_per_ray_histogram": seg_hist,
                   "sampling": "stratified" if occupancy is None else "occupancy-guided, resolution %d" % cfg["occ"]["res"],
                   "samples": n_samples, "levels": g["L"], "features": g["F"], "log2_T": g["log2_T"],
                   "partitions_traced": P, "partitions_resident": len(resident), "mlp_operands": "f16, f32 accumulate"},
        "samples_per_s": round(n_samples / (ms_per_step * 1e-3), 1),
        "roofline": roofline, "kernels": kernels, "ms_per_call": breakdown, "optimiser": optimiser, "occupancy_refresh": refresh,
        "evaluation": evaluation,
    }
    del step, models
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5_share")
    ap.add_argument("--also", default=None, help="comma-separated workloads timed after the headline one and reported as blocks of the "
                                                 "same line (default: the other four configurations when the headline is c5_share, else none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rays", type=int, default=8192, help="rays per host core of the oracle's pass")
    ap.add_argument("--no-optimizer", action="store_true", help="skip the separate timing of the Adam sweep")
    ap.add_argument("--no-peaks", action="store_true", help="skip the yardstick kernels (stream copy, random gather, atomics, MFMA loop)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, stream 1 GiB through one elementwise kernel (known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not available. "
                 "value is the one GPU's throughput." % args.gpus)
    also = args.also if args.also is not None else ("c4_big,c3_2x2,c2_ngp,c1_tiny" if args.workload == "c5_share" else "")
    also = [w for w in also.split(",") if w and w != args.workload]

    # the oracle on the host cores first: its workers are forks, which must exist before this process touches the GPU
    cpu = None if args.no_cpu_baseline else cpu_baseline(args.workload, args.cpu_rays)

    import torch
    from paper_2405_04416_amd import binding as B
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.lib()                                    # fail loudly if the HIP library is not built
    peaks = None
    if not args.no_peaks:
        from paper_2405_04416_amd import peaks as P
        peaks = P.measure("cuda:0")
        torch.cuda.empty_cache()

    head = run_workload(args.workload, args.steps, args.warmup, peaks, with_optimiser=not args.no_optimizer)
    others = {w: run_workload(w, max(1, min(args.steps, 10)), min(args.warmup, 3), peaks, with_optimiser=False, with_evaluation=False)
              for w in also}

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)           # 1 GiB read + 1 GiB written by one plain elementwise kernel
        torch.cuda.synchronize()

    out = {
        "metric": "training rays/s (fwd+bwd)", "value": head["value"], "unit": "rays/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": head["config"], "samples_per_s": head["samples_per_s"], "roofline": head["roofline"],
        "kernels": head["kernels"], "ms_per_call": head["ms_per_call"], "optimiser": head["optimiser"],
        "occupancy_refresh": head["occupancy_refresh"], "evaluation": head["evaluation"],
        "peaks_measured": peaks, "peaks_datasheet": {"hbm_GBps": HBM_PEAK_GBS, "mfma_f16_TFLOPs": MFMA_F16_PEAK_TFLOPS},
        "also": others, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
