"""Benchmark of the DistGrid training hot path on one MI355X.

One "step" is one forward + backward pass of every hot-path stage (ray/box segments, distribution,
sampling, direction encoding, hash-grid encode, MLPs, segment compositing, merge, loss seeds and
all their backward passes, including zeroing the gradient buffers) over one batch of synthetic
rays that is already resident in HBM.  The workload is the Instant-NGP-scale single-partition
configuration (2^18 rays x 64 samples, L=16, F=2, T=2^19).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_ngp] [--no-cpu-baseline] [--no-optimizer]

--workload c7_occ runs the same scene with occupancy-guided sampling (Sec. 3.2, Sec. 5.1) instead of 64 stratified
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

# HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (scaled by a known elementwise kernel), summed over the
# kernels an entry point launches; measured once per workload and recorded in profiles/<workload>_hbm_traffic.md
MEASURED_TRAFFIC_BYTES = {
    "c2_ngp": {"dg_hashgrid_encode_bwd": 17.5e9, "dg_hashgrid_encode_fwd": 7.33e9, "dg_mlp_fwd": 1.08e9, "dg_mlp_bwd": 4.6e9},
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_ngp")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rays", type=int, default=16384)
    ap.add_argument("--no-optimizer", action="store_true", help="skip the separate timing of the Adam sweep")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, stream 1 GiB through one elementwise kernel (known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not available. "
                 "value is the one GPU's throughput." % args.gpus)

    import numpy as np
    import torch
    import dg_inputs as di
    from paper_2405_04416_amd import binding as B
    from paper_2405_04416_amd.step import Occupancy, SubModel, TrainStep, split_appearance_columns

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.lib()                                    # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    cfg = di.config(args.workload)
    g, m = cfg["grid"], cfg["mlp"]
    R, S, k_max = cfg["R"], cfg["S"], cfg["k_max"]
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    foreign = None
    if "resident" in cfg:
        # one GPU's share of a larger tiling: only the resident box is traced; for a seeded fraction of the rays
        # 1..k_max-1 partials of other partitions are synthetic (colour, transmittance) pairs placed around the local one
        cfg["parts"] = cfg["parts"][cfg["resident"]:cfg["resident"] + 1]
        cfg["rays"] = "oblique"
        before, after, fC, fT = di.make_extra_partials(R, k_max, cfg["extra_fraction"], seed=0)
        before_d, total_d = to_dev(before.astype(np.int64)), to_dev((before + after + 1).astype(np.int32))
        fC_d, fT_d = to_dev(fC), to_dev(fT)

        def foreign(st):
            n = st.offsets[1]
            ray = st.seg_ray[:n].long()
            loc_c, loc_t = st.Ck[ray, 0].clone(), st.Tk[ray, 0].clone()
            st.Ck.copy_(fC_d); st.Tk.copy_(fT_d)
            st.Ck[ray, before_d[ray]] = loc_c; st.Tk[ray, before_d[ray]] = loc_t
            st.seg_slot[:n] = before_d[ray].int()
            st.seg_count.mul_(total_d)
    P = cfg["parts"].shape[0]
    resident = list(range(P))

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
    app_host = None
    if m.get("n_app"):
        # appearance vectors per image as further colour-net inputs (Sec. 4.4.3): seeded stand-ins, every ray in a random image
        app_host = di.make_appearance(cfg["n_images"], m["n_app"], R, seed=0)
        extra["appearance"] = (to_dev(app_host[0]), to_dev(app_host[1].view(np.int32)))
    step = TrainStep(to_dev(cfg["parts"]), models, resident, R, S, k_max, m["sh_degree"], loss_scale=65536.0,
                     lambda1=1e-3, seed=0, holes=to_dev(cfg["holes"]) if "holes" in cfg else None,
                     max_segments=R * min(k_max, 4), **extra)  # rays of these recipes average well under four segments

    for w in range(args.warmup):
        step.seed = w
        step.step(od, dd, Cd, None, foreign)
    torch.cuda.synchronize()
    step.timings = {}
    t0 = time.perf_counter()
    for k in range(args.steps):
        step.seed = args.warmup + k            # fresh jitter every step, drawn inside the sampling kernel
        step.step(od, dd, Cd, None, foreign)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / args.steps
    n_seg = sum(step.offsets[p + 1] - step.offsets[p] for p in resident)
    n_samples = n_seg * S if occupancy is None else sum(n for _, n in step.samples.values())
    per_call = step.timing_summary()           # HIP events on the launch stream, inside the timed region

    # the occupancy refresh (every 16th iteration, Sec. 5.1), measured apart from the metric, in both of its forms
    refresh = None
    if occupancy is not None:
        cells = sum(q.desc.n_cells for q in occupancy.values())
        refresh = {"cells": cells, "occupied_fraction": round(sum(int(q.n_set.item()) for q in occupancy.values()) / cells, 4)}
        for name, it in (("warmup_all_cells", 16), ("half_uniform_half_occupied", 4112)):
            saved = {p: (q.density.clone(), q.bits.clone()) for p, q in occupancy.items()}
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            step.timings = None
            step.refresh_occupancy(it)
            torch.cuda.synchronize()
            refresh[name] = {"ms": round(1e3 * (time.perf_counter() - t1), 3),
                             "candidates": sum(q.desc.n_cells // (1 if it < 4096 else 2) for q in occupancy.values())}
            for p, q in occupancy.items():         # the random-weight field is no scene: put the stand-in grid back
                q.density.copy_(saved[p][0]); q.bits.copy_(saved[p][1])

    # the optimiser sweep (Sec. 5.1: Adam), measured apart from the metric: `value` stays the forward+backward rate
    optimiser = None
    if not args.no_optimizer:
        n_param = sum(models[p].table.numel() for p in resident)
        touched = sum(int(torch.count_nonzero(models[p].dtable)) for p in resident)
        step.timings = {}
        for k in range(3):
            if k:
                step.step(od, dd, Cd, None, foreign)       # fresh gradients for every sweep
            step.optimiser_step(k)
        calls, total_ms = step.timing_summary()["dg_adam_step"]
        ms = total_ms / 3
        moved = touched * 32 + (n_param - touched) * 4     # touched: value, gradient, 2 moments read and written; else the gradient read
        optimiser = {"entry": "dg_adam_step", "ms_per_step": round(ms, 4), "parameters": n_param,
                     "touched_fraction": round(touched / n_param, 4), "algorithmic_bytes": moved,
                     "GB/s": round(moved / (ms * 1e-3) / 1e9, 1), "frac_hbm": round(moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # evaluation rendering (forward only: colour, depth, transmittance; Sec. 4.4.2), apart from the metric
    evaluation = None
    if foreign is None:
        step.timings = None
        step.render(od, dd)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(3):
            step.render(od, dd)
        torch.cuda.synchronize()
        ev_ms = 1e3 * (time.perf_counter() - t1) / 3
        evaluation = {"ms_per_batch": round(ev_ms, 4), "rays_per_s": round(R / (ev_ms * 1e-3), 1), "outputs": "colour, depth, transmittance"}

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)           # 1 GiB read + 1 GiB written by one plain elementwise kernel
        torch.cuda.synchronize()

    shapes = di.mlp_layer_shapes(n_feat, m)
    mlp_flops_fwd = 2 * sum(no * ni for no, ni in shapes)
    breakdown = {k: round(ms / args.steps, 4) for k, (n, ms) in sorted(per_call.items(), key=lambda kv: -kv[1][1])}
    dominant = next(iter(breakdown))
    calls, total_ms = per_call[dominant]
    avg_ms = total_ms / calls
    per_launch_samples = n_samples / max(len(resident), 1)
    bound, work = algorithmic_work(dominant, g["L"], g["F"], per_launch_samples, mlp_flops_fwd)
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload, {}).get(dominant)
    if work is None:
        roofline = {"kernel": dominant, "bound": bound, "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": None, "traffic": None, "avg_launch_ms": round(avg_ms, 4)}
    elif bound == "hbm":
        ach = work / (avg_ms * 1e-3) / 1e9
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic, "algorithmic_bytes": work,
                    "avg_launch_ms": round(avg_ms, 4)}
    else:
        ach = work / (avg_ms * 1e-3) / 1e12
        roofline = {"kernel": dominant, "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_F16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / MFMA_F16_PEAK_TFLOPS, 4), "traffic": traffic,
                    "avg_launch_ms": round(avg_ms, 4)}
    # the other headline kernels, same accounting
    others = {}
    for entry in ("dg_hashgrid_encode_fwd", "dg_hashgrid_encode_bwd", "dg_mlp_fwd", "dg_mlp_bwd"):
        if entry in per_call:
            c, t = per_call[entry]
            b, wk = algorithmic_work(entry, g["L"], g["F"], per_launch_samples, mlp_flops_fwd)
            rate = wk / (t / c * 1e-3)
            others[entry] = ({"GB/s": round(rate / 1e9, 1), "frac_hbm": round(rate / 1e9 / HBM_PEAK_GBS, 4)} if b == "hbm"
                             else {"TFLOP/s": round(rate / 1e12, 2), "frac_mfma": round(rate / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)})

    cpu = None
    if not args.no_cpu_baseline:
        import oracle.step as ostep            # the oracle, as it stands, on the host cores of this machine
        Rc = min(args.cpu_rays, R)
        hm = ostep.make_models(dict(cfg, resident_list=resident), seed=0)
        ho = ostep.make_occupancy(cfg, seed=0) if occupancy is not None else None     # built outside the timed call, like the tables
        t1 = time.perf_counter()
        ostep.run_step(cfg, hm, o[:Rc], d[:Rc], Cgt[:Rc], seed=0, lambda1=1e-3, loss_scale=65536.0, resident=resident, occ=ho,
                       appearance=None if app_host is None else (app_host[0], app_host[1][:Rc]))   # (without the synthetic foreign partials)
        cpu_s = time.perf_counter() - t1
        cpu = {"value": round(Rc / cpu_s, 2), "unit": "rays/s", "cores": 1, "kind": "oracle",
               "sample": "first %d rays of the same batch, full-size tables, one fwd+bwd pass, %.1f s" % (Rc, cpu_s)}

    out = {
        "metric": "training rays/s (fwd+bwd)", "value": round(R / (ms_per_step * 1e-3), 1), "unit": "rays/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "rays": R,
                   "samples_per_segment": S if occupancy is None else round(n_samples / max(n_seg, 1), 2), "segments": n_seg,
                   "sampling": "stratified" if occupancy is None else "occupancy-guided, resolution %d" % cfg["occ"]["res"],
                   "samples": n_samples, "levels": g["L"], "features": g["F"], "log2_T": g["log2_T"],
                   "partitions_resident": len(resident), "mlp_operands": "f16, f32 accumulate"},
        "samples_per_s": round(n_samples / (ms_per_step * 1e-3), 1),
        "roofline": roofline, "kernels": others, "ms_per_call": breakdown, "optimiser": optimiser, "occupancy_refresh": refresh, "evaluation": evaluation,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
