"""Oracle-side forward + backward pass of the whole hot path -- TEST INFRASTRUCTURE ONLY.

Chains the oracle's functions in the order of the paper's training procedure (Sec. 4.4.2, Fig. 2)
on host arrays.  Used by the parity tests, the smoke check and the benchmark's cpu-baseline leg.
"""
import numpy as np

import oracle as O


def make_models(cfg, seed=0):
    """Grid geometry, MLP descriptor and seeded parameters for every partition of a configuration."""
    import dg_inputs as di
    m = cfg["mlp"]
    models = {}
    for p in cfg.get("resident_list", range(cfg["parts"].shape[0])):
        g = di.grid_params(cfg, p)
        growth = g.get("growth") or O.growth_factor(g["n_min"], g["n_max"], g["L"])
        grid = O.grid_init(g["L"], g["F"], g["log2_T"], g["n_min"], growth, di.box_extent(cfg["parts"][p]))
        n_feat = g["L"] * g["F"]
        # appearance features (Sec. 4.4.3) are further inputs of the colour net, after the direction encoding
        mlp = O.mlp_desc(n_feat, m["n_hidden_d"], m["n_geo"], m["sh_degree"] ** 2 + m.get("n_app", 0), m["n_hidden_c"],
                         m["n_layers_c"], 1, 1)
        table = di.make_table(grid.n_entries, g["F"], cfg["table_range"], seed=seed + 1000 * p)
        weights = di.make_mlp_weights(n_feat, m, seed=seed + 1000 * p)
        models[p] = dict(grid=grid, mlp=mlp, table=table, weights=weights)
    return models


def make_occupancy(cfg, seed=0, threshold=0.6):
    """Occupancy grid of every partition (Sec. 3.2, Sec. 5.1) from seeded stand-in densities: geometry, densities,
    bits and the marching step (Instant-NGP's step of sqrt(3)/1024 for the unit cube, scaled to the box)."""
    import dg_inputs as di
    occ = {}
    for p in range(cfg["parts"].shape[0]):
        ext = di.box_extent(cfg["parts"][p])
        g = O.occ_init(cfg["occ"]["res"], ext)
        dens = di.make_cell_densities(list(g.shape), seed=seed + 1000 * p)
        bits, _ = O.occ_bits(dens, threshold)
        occ[p] = dict(grid=g, density=dens, bits=bits, dt=np.float32(float(ext.max()) * np.sqrt(3.0) / 1024),
                      max_steps=cfg["occ"]["max_steps"])
    return occ


def run_step(cfg, models, o, d, Cgt, jitter=None, seed=0, lambda1=0.0, loss_scale=65536.0, resident=None,
             foreign=None, want_bwd=True, occ=None, appearance=None):
    """Returns a dict of every intermediate the GPU path can be compared with.

    occ: None (fixed stratified samples per segment), or {partition: occupancy grid} from make_occupancy:
    occupancy-guided sampling, segments of different lengths.
    appearance: None, or (table [n_images, n_app], image_of_ray [R]): per-image vectors fed to the colour net."""
    parts, S, k_max = cfg["parts"], cfg["S"], cfg["k_max"]
    P, R = parts.shape[0], o.shape[0]
    deg = cfg["mlp"]["sh_degree"]
    resident = list(range(P)) if resident is None else list(resident)
    out = {}
    cnt, seg_t, seg_part, status = O.ray_aabb_segments(o, d, parts, 0.0, k_max, holes=cfg.get("holes"))
    off, seg_ray, seg_slot = O.bucket_segments(cnt, seg_part, P)
    out.update(seg_count=cnt, seg_t=seg_t, seg_part=seg_part, status=status, part_offset=off, seg_ray=seg_ray,
               seg_slot=seg_slot)
    Ck = np.zeros((R, k_max, 3)); Tk = np.ones((R, k_max))
    per = {}
    for p in resident:
        b, e = int(off[p]), int(off[p + 1])
        if e == b:
            continue
        m = models[p]
        if occ is None:
            jit = None if jitter is None else jitter[b * S:e * S]
            u, delta = O.sample_segments(o, d, seg_t, seg_ray, seg_slot, b, e, parts[p], S, seed=seed, jitter_arr=jit)
            dir_enc = O.sh(d[seg_ray[b:e]], deg)
            if appearance is not None:
                dir_enc = np.concatenate([dir_enc, appearance[0][appearance[1][seg_ray[b:e]]].astype(np.float64)], axis=1)
            first, S_mlp = None, S
        else:
            q = occ[p]
            first, u, delta, t, sample_ray = O.march_segments(o, d, seg_t, seg_ray, seg_slot, b, e, parts[p], q["grid"], q["bits"],
                                                              q["dt"], q["max_steps"], seed=seed)
            dir_enc = O.sh(d[sample_ray], deg)            # one direction row per sample
            if appearance is not None:
                dir_enc = np.concatenate([dir_enc, appearance[0][appearance[1][sample_ray]].astype(np.float64)], axis=1)
            S_mlp = 1
        feat = O.encode_fwd(m["grid"], m["table"], u)
        sigma, rgb = O.mlp_fwd(m["mlp"], m["weights"].astype(np.float64), feat, dir_enc, S_mlp)
        if occ is None:
            Cseg, Tseg = O.composite_fwd(sigma, rgb, delta.astype(np.float64), S)
        else:
            Cseg, Tseg = O.composite_fwd_ragged(sigma, rgb, delta.astype(np.float64), first)
        Ck[seg_ray[b:e], seg_slot[b:e]] = Cseg
        Tk[seg_ray[b:e], seg_slot[b:e]] = Tseg
        per[p] = dict(u=u, delta=delta, dir_enc=dir_enc, feat=feat, sigma=sigma, rgb=rgb, b=b, e=e, first=first, S_mlp=S_mlp)
    if foreign is not None:
        foreign(Ck, Tk, out)
        cnt = out["seg_count"]
    C, T = O.merge_fwd(Ck, Tk, cnt)
    loss, gC, gT = O.loss(C, T, Cgt, lambda1)
    out.update(Ck=Ck, Tk=Tk, C=C, T=T, loss=loss, gC=gC, gT=gT, per=per)
    if not want_bwd:
        return out
    gCk, gTk = O.merge_bwd(Ck, Tk, cnt, gC, gT)
    out.update(gCk=gCk, gTk=gTk)
    for p, q in per.items():
        b, e = q["b"], q["e"]
        m = models[p]
        if q["first"] is None:
            dsigma, drgb = O.composite_bwd(q["sigma"], q["rgb"], q["delta"].astype(np.float64), S,
                                           gCk[seg_ray[b:e], seg_slot[b:e]], gTk[seg_ray[b:e], seg_slot[b:e]])
        else:
            dsigma, drgb = O.composite_bwd_ragged(q["sigma"], q["rgb"], q["delta"].astype(np.float64), q["first"],
                                                  gCk[seg_ray[b:e], seg_slot[b:e]], gTk[seg_ray[b:e], seg_slot[b:e]])
        dfeat, dW = O.mlp_bwd(m["mlp"], m["weights"].astype(np.float64), q["feat"], q["dir_enc"], q["S_mlp"], dsigma, drgb,
                              loss_scale)
        dtable = O.encode_bwd(m["grid"], q["u"], dfeat)
        q.update(dsigma=dsigma, drgb=drgb, dfeat=dfeat, dW=dW, dtable=dtable)
    return out


def refresh_occupancy(models, occ, iteration, seed=0, tries=32, resident=None):
    """The occupancy refresh of Sec. 5.1 / Instant-NGP App. E.2 at one training iteration, in place on `occ`:
    decay, candidate cells (all cells during warm-up, afterwards n_cells/2 of which half uniform and half among the
    occupied ones), the field's density at a random point of each, maximum, new bits.  Returns False when the
    schedule asks for no refresh at this iteration."""
    update_now, warmup, decay, threshold = O.occ_schedule(iteration)
    if not update_now:
        return False
    for p in (occ if resident is None else resident):
        q, m = occ[p], models[p]
        g = q["grid"]
        O.occ_decay(q["density"], np.float32(decay))
        M = g.n_cells if warmup else g.n_cells // 2
        cell, u = O.occ_candidates(g, q["bits"], M, 0 if warmup else M // 2, warmup, seed, iteration, tries)
        feat = O.encode_fwd(m["grid"], m["table"], u)
        no_dir = np.zeros((M, m["mlp"].n_dir))                      # the density does not depend on the direction
        sigma, _ = O.mlp_fwd(m["mlp"], m["weights"].astype(np.float64), feat, no_dir, 1)
        O.occ_update(q["density"], cell, sigma.astype(np.float32))
        q["bits"], q["n_set"] = O.occ_bits(q["density"], threshold)
        q["last_sigma"], q["last_cell"] = sigma, cell
    return True
