"""Seeded synthetic inputs shaped like the paper's aerial workloads.

Shared by the tests, the benchmark and the smoke check.  This module holds none
of the method's arithmetic: it only draws random rays, boxes, table values,
weights, targets, jitter and stand-in cell densities, and names the workload configurations.  The
paper trains on drone oblique photography of flat scenes, rays drawn uniformly
at random over all images (DistGrid Sec. 4.4.1, Sec. 5.1); those datasets are
not available here, so the generators below stand in for them.
"""
import math

import numpy as np

# ---------------------------------------------------------------------------
# Workload configurations.  "grid" gives the hash-grid hyper-parameters, "mlp"
# the widths of the density / colour networks, "parts" the partition boxes.
# ---------------------------------------------------------------------------


def _tile(x_edges, y_edges, z0, z1):
    boxes = []
    for j in range(len(y_edges) - 1):
        for i in range(len(x_edges) - 1):
            boxes.append([x_edges[i], y_edges[j], z0, x_edges[i + 1], y_edges[j + 1], z1])
    return np.asarray(boxes, np.float32)


CONFIGS = {
    "c1_tiny": dict(
        parts=_tile([-1, 1], [-1, 1], -1, 1), rays="surface_inward", R=1024, S=32, k_max=1,
        grid=dict(L=4, F=2, log2_T=12, n_min=16, growth=1.5), table_range=0.1,
        mlp=dict(n_hidden_d=32, n_geo=16, sh_degree=2, n_hidden_c=32, n_layers_c=1)),
    "c2_ngp": dict(
        parts=_tile([-1, 1], [-1, 1], 0, 0.25), rays="aerial", cam_height=1.5, tilt_deg=30.0, R=1 << 18, S=64,
        k_max=1, grid=dict(L=16, F=2, log2_T=19, n_min=16, n_max=2048), table_range=1e-4,
        mlp=dict(n_hidden_d=64, n_geo=16, sh_degree=4, n_hidden_c=64, n_layers_c=2)),
    "c3_2x2": dict(
        parts=_tile([-2, 0, 2], [-2, 0, 2], 0, 0.25), rays="oblique", r_max=4.0, cam_height=1.5, R=1 << 18, S=64,
        k_max=4, grid=dict(L=16, F=2, log2_T=22, n_min=16, n_max=2048), table_range=1e-4,
        mlp=dict(n_hidden_d=64, n_geo=16, sh_degree=4, n_hidden_c=64, n_layers_c=2)),
    "c4_big": dict(
        parts=_tile([-1, 1], [-1, 1], 0, 0.2), rays="aerial", cam_height=1.5, tilt_deg=30.0, R=1 << 19, S=48,
        k_max=1, grid=dict(L=16, F=2, log2_T=24, n_min=16, n_max=8192), table_range=1e-4,
        mlp=dict(n_hidden_d=64, n_geo=16, sh_degree=4, n_hidden_c=64, n_layers_c=2)),
    # One GPU's share of a 2 x 4 tiling: all eight boxes are traced, only box `resident` has its sub-model here; the
    # partials of the other boxes' segments are synthetic.  r_max is set so that 60 % of the rays also cross 1..3 other boxes.
    "c5_share": dict(
        parts=_tile([-4, -2, 0, 2, 4], [-2, 0, 2], 0, 0.25), resident=1, rays="through_resident", r_max=3.35,
        cam_height=1.5, R=1 << 20, S=64, k_max=4,
        grid=dict(L=16, F=2, log2_T=24, n_min=16, n_max=8192), table_range=1e-4,
        mlp=dict(n_hidden_d=64, n_geo=16, sh_degree=4, n_hidden_c=64, n_layers_c=2)),
    # Two-level cascade of Sec. 4.2.2: fine sub-models tile the inner box, coarse sub-models (T = 2^19) tile the outer
    # box with the same split planes and cover it minus the inner box ("holes": the box subtracted from each partition).
    "c6_cascade": dict(
        parts=np.concatenate([_tile([-1, 0, 1], [-1, 0, 1], 0, 0.25), _tile([-3, 0, 3], [-3, 0, 3], 0, 0.5)]),
        holes=np.concatenate([np.zeros((4, 6), np.float32), _tile([-1, 0, 1], [-1, 0, 1], 0, 0.25)]),
        rays="through_inner", r_max=2.5, cam_height=1.5, R=1 << 18, S=64, k_max=10,
        grid=dict(L=16, F=2, log2_T=22, n_min=16, n_max=2048), grid_coarse=dict(L=16, F=2, log2_T=19, n_min=16, n_max=2048),
        coarse_from=4, table_range=1e-4,
        mlp=dict(n_hidden_d=64, n_geo=16, sh_degree=4, n_hidden_c=64, n_layers_c=2)),
    # Occupancy-guided sampling (Sec. 3.2, Sec. 5.1): the c2 scene and rays with an occupancy grid of resolution 512 along
    # the longest side; segments are cut into strata of Instant-NGP's marching step and only occupied cells are sampled.
    "c7_occ": dict(
        parts=_tile([-1, 1], [-1, 1], 0, 0.25), rays="aerial", cam_height=1.5, tilt_deg=30.0, R=1 << 18, S=64,
        k_max=1, grid=dict(L=16, F=2, log2_T=19, n_min=16, n_max=2048), table_range=1e-4,
        occ=dict(res=512, max_steps=1024),
        mlp=dict(n_hidden_d=64, n_geo=16, sh_degree=4, n_hidden_c=64, n_layers_c=2)),
    # Appearance features (Sec. 4.4.3): c2 with 48 further colour-net inputs, one fixed vector per image, 1000 images.
    "c8_app": dict(
        parts=_tile([-1, 1], [-1, 1], 0, 0.25), rays="aerial", cam_height=1.5, tilt_deg=30.0, R=1 << 18, S=64,
        k_max=1, grid=dict(L=16, F=2, log2_T=19, n_min=16, n_max=2048), table_range=1e-4, n_images=1000,
        mlp=dict(n_hidden_d=64, n_geo=16, sh_degree=4, n_hidden_c=64, n_layers_c=2, n_app=48)),
}


def grid_params(cfg, p):
    """Hash-grid hyper-parameters of partition p (the coarse level of a cascade has its own)."""
    return cfg["grid_coarse"] if "coarse_from" in cfg and p >= cfg["coarse_from"] else cfg["grid"]


def config(name, **overrides):
    cfg = dict(CONFIGS[name])
    cfg["name"] = name
    cfg.update(overrides)
    return cfg


def box_extent(box6):
    box6 = np.asarray(box6, np.float64)
    return box6[3:] - box6[:3]


# ---------------------------------------------------------------------------
# Rays
# ---------------------------------------------------------------------------


def _normalise(v):
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def rays_surface_inward(R, box6, rng):
    """Origins uniform on the surface of a box, directions Gaussian, flipped to point inward."""
    lo, hi = np.asarray(box6[:3], np.float64), np.asarray(box6[3:], np.float64)
    ext = hi - lo
    areas = np.array([ext[1] * ext[2], ext[0] * ext[2], ext[0] * ext[1]])
    axis = rng.choice(3, size=R, p=areas / areas.sum())
    side = rng.integers(0, 2, size=R)
    o = lo + rng.random((R, 3)) * ext
    o[np.arange(R), axis] = np.where(side == 1, hi[axis], lo[axis])
    d = _normalise(rng.standard_normal((R, 3)))
    outward = np.where(side == 1, 1.0, -1.0)
    flip = d[np.arange(R), axis] * outward > 0
    d[flip] *= -1.0
    return o.astype(np.float32), d.astype(np.float32)


def rays_aerial(R, scene6, cam_height, tilt_deg, rng):
    """Cameras at a fixed height above the scene footprint, looking down within a cone."""
    lo, hi = np.asarray(scene6[:3], np.float64), np.asarray(scene6[3:], np.float64)
    o = np.empty((R, 3))
    o[:, 0] = lo[0] + rng.random(R) * (hi[0] - lo[0])
    o[:, 1] = lo[1] + rng.random(R) * (hi[1] - lo[1])
    o[:, 2] = cam_height
    theta = np.deg2rad(tilt_deg) * rng.random(R)
    phi = 2.0 * math.pi * rng.random(R)
    d = np.stack([np.sin(theta) * np.cos(phi), np.sin(theta) * np.sin(phi), -np.cos(theta)], axis=1)
    return o.astype(np.float32), d.astype(np.float32)


def rays_oblique(R, scene6, cam_height, r_max, rng, through=None):
    """Oblique rays: enter through the top face, leave through the bottom at a lateral offset <= r_max.

    With `through` (a box) the entry point is drawn on that box's top face, so every ray crosses it.
    """
    lo, hi = np.asarray(scene6[:3], np.float64), np.asarray(scene6[3:], np.float64)
    elo, ehi = (lo, hi) if through is None else (np.asarray(through[:3], np.float64), np.asarray(through[3:], np.float64))
    top = np.empty((R, 3))
    top[:, 0] = elo[0] + rng.random(R) * (ehi[0] - elo[0])
    top[:, 1] = elo[1] + rng.random(R) * (ehi[1] - elo[1])
    top[:, 2] = hi[2]
    r = r_max * rng.random(R)
    phi = 2.0 * math.pi * rng.random(R)
    bottom = top + np.stack([r * np.cos(phi), r * np.sin(phi), np.full(R, lo[2] - hi[2])], axis=1)
    bottom[:, 0] = np.clip(bottom[:, 0], lo[0], hi[0])
    bottom[:, 1] = np.clip(bottom[:, 1], lo[1], hi[1])
    d = _normalise(bottom - top)
    o = top - d * ((cam_height - hi[2]) / -d[:, 2])[:, None]
    return o.astype(np.float32), d.astype(np.float32)


def make_rays(cfg, seed=0, R=None):
    rng = np.random.default_rng([seed, 11])
    R = cfg["R"] if R is None else R
    parts = cfg["parts"]
    scene = np.concatenate([parts[:, :3].min(0), parts[:, 3:].max(0)])
    kind = cfg["rays"]
    if kind == "surface_inward":
        return rays_surface_inward(R, scene, rng)
    if kind == "aerial":
        return rays_aerial(R, scene, cfg["cam_height"], cfg["tilt_deg"], rng)
    if kind == "oblique":
        return rays_oblique(R, scene, cfg["cam_height"], cfg["r_max"], rng)
    if kind == "through_inner":       # cameras look at the inner (fine) area of a cascade: entry points above it
        fine = parts[:cfg["coarse_from"]]
        return rays_oblique(R, scene, cfg["cam_height"], cfg["r_max"], rng, through=np.concatenate([fine[:, :3].min(0), fine[:, 3:].max(0)]))
    if kind == "through_resident":
        return rays_oblique(R, scene, cfg["cam_height"], cfg["r_max"], rng, through=parts[cfg["resident"]])
    raise ValueError(kind)


# ---------------------------------------------------------------------------
# Parameters, targets, jitter
# ---------------------------------------------------------------------------


def make_table(n_entries, F, value_range, seed=0):
    rng = np.random.default_rng([seed, 23])
    t = rng.random((n_entries, F), dtype=np.float32)
    t *= np.float32(2.0 * value_range)
    t -= np.float32(value_range)
    return t


def mlp_layer_shapes(n_feat, mlp):
    """[(out, in)] of the five (or four) weight matrices in packing order.  Appearance features (mlp["n_app"]) are
    further inputs of the first colour layer, after the direction encoding."""
    n_dir = mlp["sh_degree"] ** 2 + mlp.get("n_app", 0)
    shapes = [(mlp["n_hidden_d"], n_feat), (mlp["n_geo"], mlp["n_hidden_d"]),
              (mlp["n_hidden_c"], mlp["n_geo"] + n_dir)]
    if mlp["n_layers_c"] == 2:
        shapes.append((mlp["n_hidden_c"], mlp["n_hidden_c"]))
    shapes.append((3, mlp["n_hidden_c"]))
    return shapes


def make_mlp_weights(n_feat, mlp, seed=0, gain=1.0):
    """Uniform +-sqrt(6/(in+out)) per layer, rounded to fp16, packed layer after layer, each [out, in]."""
    rng = np.random.default_rng([seed, 37])
    chunks = []
    for (n_out, n_in) in mlp_layer_shapes(n_feat, mlp):
        a = gain * math.sqrt(6.0 / (n_in + n_out))
        chunks.append(((rng.random((n_out, n_in)) * 2.0 - 1.0) * a).astype(np.float16).ravel())
    return np.concatenate(chunks)


def make_appearance(n_images, n_app, R, seed=0):
    """Per-image appearance vectors (fp16, N(0,1): stand-ins for the PCA-reduced Gram features of Sec. 4.4.3) and the
    image every ray belongs to (rays are drawn uniformly over all images)."""
    rng = np.random.default_rng([seed, 97])
    table = rng.standard_normal((n_images, n_app)).astype(np.float16)
    image_of_ray = rng.integers(0, n_images, R).astype(np.uint32)
    return table, image_of_ray


def make_targets(R, seed=0):
    return np.random.default_rng([seed, 41]).random((R, 3), dtype=np.float32)


def make_jitter(n, seed=0):
    return np.random.default_rng([seed, 53]).random(n, dtype=np.float32)


def make_unit_coords(n, seed=0):
    return np.random.default_rng([seed, 67]).random((n, 3), dtype=np.float32)


def make_foreign_partials(R, k_max, seed=0):
    """Stand-ins for the partial results other GPUs would send: (colour, transmittance) ~ U[0,1] for every slot of
    every ray, Ck [R,k_max,3], Tk [R,k_max]; the slots of resident segments are overwritten by the local rendering."""
    rng = np.random.default_rng([seed, 71])
    return rng.random((R, k_max, 3), dtype=np.float32), rng.random((R, k_max), dtype=np.float32)


# ---------------------------------------------------------------------------
# Occupancy (for occupancy-guided sampling)
# ---------------------------------------------------------------------------


def make_cell_densities(shape, seed=0, shell=0.08, n_blocks=40, level=100.0, skin=3):
    """Per-cell densities of a scene shaped like an aerial capture, [shape_z, shape_y, shape_x] flattened (x fastest).

    A rolling ground surface (a few random sinusoids) of relative thickness `shell`, plus `n_blocks` box-shaped
    "buildings" standing on it; the surface cells of that solid get a density around `level` (log-uniform over two
    decades), all other cells 0.  These are stand-in numbers for the densities a trained field would report.
    """
    rng = np.random.default_rng([seed, 83])
    nx, ny, nz = (int(v) for v in shape)
    x = (np.arange(nx) + 0.5) / nx
    y = (np.arange(ny) + 0.5) / ny
    z = (np.arange(nz) + 0.5) / nz
    ground = np.full((ny, nx), 0.3)
    for _ in range(4):
        fx, fy = rng.integers(1, 5, size=2)
        ground += 0.06 * np.sin(2 * math.pi * (fx * x[None, :] + fy * y[:, None]) + rng.random() * 6.28)
    top = ground.copy()
    for _ in range(n_blocks):
        cx, cy = rng.random(2)
        wx, wy = 0.02 + 0.06 * rng.random(2)
        h = 0.1 + 0.4 * rng.random()
        inside = (np.abs(x[None, :] - cx) < wx) & (np.abs(y[:, None] - cy) < wy)
        top = np.where(inside, np.maximum(top, ground + h), top)
    solid = (z[:, None, None] <= top[None]) & (z[:, None, None] >= ground[None] - shell)
    # matter that cameras see is the surface of the solid: drop what lies more than `skin` cells inside
    deep = solid.copy()
    for _ in range(skin):
        core = deep.copy()
        core[1:] &= deep[:-1]; core[:-1] &= deep[1:]
        core[:, 1:] &= deep[:, :-1]; core[:, :-1] &= deep[:, 1:]
        core[:, :, 1:] &= deep[:, :, :-1]; core[:, :, :-1] &= deep[:, :, 1:]
        deep = core
    visible = solid & ~deep
    dens = np.where(visible, level * 10.0 ** (rng.random((nz, ny, nx)) * 2.0 - 1.0), 0.0)
    return dens.astype(np.float32).ravel()
