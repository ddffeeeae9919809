"""Pins for the oracle's occupancy grid and occupancy-guided sampling (CPU only).

Sources: DistGrid Sec. 3.2 (an occupancy grid records per-voxel density so that marching skips empty space),
Sec. 4.1 (the grid is deformable like the hash grid: ceil(a/s N) cells per axis), Sec. 5.1 (resolution 512, one
scale, plain storage order, decay 0.99 every 16 iterations, warm-up of 4096 iterations, bit threshold 0.6 before
iteration 10 000 and 60 afterwards); Instant-NGP App. E.2 for the refresh rule (decay, candidate cells, maximum,
threshold); the published splitmix64 test vector; numpy routines for maximum / packbits; invariants of Eq. 3.
"""
import numpy as np

import dg_inputs as di
import oracle


# ---------------------------------------------------------------- geometry
def test_deformable_shape_follows_the_hash_grid_rule():
    g = oracle.occ_init(8, (4.0, 2.0, 1.0))
    assert list(g.shape) == [8, 4, 2] and g.n_cells == 64                  # ceil(a/s N), Sec. 4.1
    g = oracle.occ_init(10, (1.0, 1.0, 0.25))
    assert list(g.shape) == [10, 10, 3] and g.n_cells == 300               # 2.5 rounds up: the top cell overhangs
    g = oracle.occ_init(512, (2.0, 2.0, 0.25))
    assert list(g.shape) == [512, 512, 64]
    # the same shape as a hash-grid level of that resolution
    grid = oracle.grid_init(1, 2, 19, 512, 1.0, (2.0, 2.0, 0.25))
    assert [int(v) for v in grid.shape[0]] == [512, 512, 64]


def test_cells_are_cubes_of_side_s_over_N_in_x_fastest_order():
    ext = np.array([3.0, 1.5, 0.7])
    N = 24
    g = oracle.occ_init(N, ext)
    side = ext.max() / N
    rng = np.random.default_rng(5)
    x = rng.random((4000, 3)) * ext                                         # world position relative to the box corner
    grid_pos = x / side
    clear = np.all(np.abs(grid_pos - np.round(grid_pos)) > 1e-4, axis=1)    # away from cell faces (fp32 rounding)
    c = np.floor(grid_pos).astype(np.int64)
    want = c[:, 0] + g.shape[0] * (c[:, 1] + g.shape[1] * c[:, 2])
    got = oracle.occ_cell(g, (x / ext).astype(np.float32))
    np.testing.assert_array_equal(got[clear], want[clear])
    # corners: first and last cell; coordinates outside [0,1] clamp
    assert oracle.occ_cell(g, [[0, 0, 0]])[0] == 0
    assert oracle.occ_cell(g, [[1, 1, 1]])[0] == g.n_cells - 1
    assert oracle.occ_cell(g, [[-3, 0.0, 0.0]])[0] == 0 and oracle.occ_cell(g, [[7, 9, 2]])[0] == g.n_cells - 1
    assert oracle.occ_cell(g, [[1.0 / 24 + 1e-4, 0, 0]])[0] == 1             # x is the fastest axis
    assert oracle.occ_cell(g, [[0, 2.0 / 24 * 3.0 / 1.5 * 0.5 + 1e-4, 0]])[0] == g.shape[0]


def test_schedule_is_the_papers():
    for it in range(0, 200):
        assert oracle.occ_schedule(it)[0] == (it % 16 == 0)                  # every 16 iterations
    assert oracle.occ_schedule(4095)[1] and not oracle.occ_schedule(4096)[1]  # warm-up of 4096 iterations
    assert abs(oracle.occ_schedule(7)[2] - 0.99) < 1e-7
    assert abs(oracle.occ_schedule(9999)[3] - 0.6) < 1e-7 and oracle.occ_schedule(10000)[3] == 60.0
    assert oracle.occ_schedule(300000)[3] == 60.0


def test_generator_matches_the_published_splitmix64_vector():
    # splitmix64 seeded with 0 produces these first outputs (reference implementation by Vigna)
    assert oracle.rand64(0, 0) == 0xE220A8397B1DCDAF
    assert oracle.rand64(0, 1) == 0x6E789E6AA1B965F4
    assert oracle.rand64(0, 2) == 0x06C45D188009454F


# ---------------------------------------------------------------- refresh
def test_warmup_candidates_are_all_cells_with_a_point_inside_each():
    g = oracle.occ_init(12, (1.0, 0.8, 0.3))
    bits = np.zeros((g.n_cells + 31) // 32, np.uint32)
    cell, u = oracle.occ_candidates(g, bits, g.n_cells, 0, True, seed=9, iteration=16)
    np.testing.assert_array_equal(cell, np.arange(g.n_cells))
    pos = u.astype(np.float64) * np.array(list(g.gain))
    idx = np.stack([cell % g.shape[0], (cell // g.shape[0]) % g.shape[1], cell // (g.shape[0] * g.shape[1])], 1)
    assert np.all(pos >= idx - 1e-5) and np.all(pos <= idx + 1 + 1e-5)
    off = pos - idx
    assert 0.45 < off.mean() < 0.55 and off.std() > 0.25                    # spread over the cell, not its corner
    cell2, u2 = oracle.occ_candidates(g, bits, g.n_cells, 0, True, seed=9, iteration=32)
    assert np.any(u2 != u)                                                  # a new point at every refresh


def test_later_candidates_half_uniform_half_occupied():
    g = oracle.occ_init(8, (1.0, 1.0, 0.5))                                 # 256 cells
    rng = np.random.default_rng(3)
    occupied = rng.random(g.n_cells) < 0.5
    bits = np.packbits(np.concatenate([occupied, np.zeros(-g.n_cells % 32, bool)]), bitorder="little").view(np.uint32)
    M = 51200
    cell, u = oracle.occ_candidates(g, bits, M, M // 2, False, seed=4, iteration=4112)
    assert cell.max() < g.n_cells
    first, second = cell[:M // 2], cell[M // 2:]
    # uniform half: every cell about M/2/256 = 100 times
    cnt = np.bincount(first, minlength=g.n_cells)
    assert cnt.min() > 50 and cnt.max() < 160
    # occupied half: only occupied cells (32 tries at 50 % occupancy never all fail), evenly
    assert np.all(occupied[second])
    cnt2 = np.bincount(second, minlength=g.n_cells)[occupied]
    assert cnt2.min() > 0.5 * cnt2.mean() and cnt2.max() < 1.6 * cnt2.mean()
    # the point lies in its cell
    pos = u.astype(np.float64) * np.array(list(g.gain))
    idx = np.stack([cell % g.shape[0], (cell // g.shape[0]) % g.shape[1], cell // (g.shape[0] * g.shape[1])], 1)
    assert np.all(pos >= idx - 1e-5) and np.all(pos <= idx + 1 + 1e-5)
    # with nothing occupied the rejection half still returns valid cells (the last draw)
    cell3, _ = oracle.occ_candidates(g, np.zeros_like(bits), 1000, 500, False, seed=4, iteration=4112)
    assert cell3.max() < g.n_cells and len(set(cell3[500:])) > 200
    # a refresh produced in pieces is the same refresh
    a, ua = oracle.occ_candidates(g, bits, 300, M // 2, False, seed=4, iteration=4112, i0=M // 2 - 100)
    np.testing.assert_array_equal(a, cell[M // 2 - 100:M // 2 + 200])
    np.testing.assert_array_equal(ua, u[M // 2 - 100:M // 2 + 200])
    # one try: the rejection half degenerates to uniform draws
    cell4, _ = oracle.occ_candidates(g, bits, 4000, 0, False, seed=4, iteration=4112, tries=1)
    assert 0.4 < occupied[cell4].mean() < 0.6


def test_decay_maximum_and_bits_against_numpy():
    rng = np.random.default_rng(8)
    n = 1000
    dens0 = (rng.random(n) * 100).astype(np.float32)
    dens = dens0.copy()
    for _ in range(10):
        oracle.occ_decay(dens, np.float32(0.99))
    np.testing.assert_allclose(dens, dens0.astype(np.float64) * 0.99 ** 10, rtol=2e-6)    # closed form
    cell = rng.integers(0, n, 5000).astype(np.uint32)                       # many duplicates
    sigma = (rng.random(5000) * 120).astype(np.float32)
    want = dens.copy()
    np.maximum.at(want, cell, sigma)
    oracle.occ_update(dens, cell, sigma)
    np.testing.assert_array_equal(dens, want)
    for thr in (0.6, 60.0):
        bits, n_set = oracle.occ_bits(dens, thr)
        mask = dens > np.float32(thr)
        want_bits = np.packbits(np.concatenate([mask, np.zeros(-n % 32, bool)]), bitorder="little").view(np.uint32)
        np.testing.assert_array_equal(bits, want_bits)
        assert n_set == int(mask.sum())
    # the threshold is strict
    bits, n_set = oracle.occ_bits(np.array([60.0, 60.000004], np.float32), 60.0)
    assert bits[0] == 2 and n_set == 1


# ---------------------------------------------------------------- marching
def _setup(R=300, N=32, seed=1):
    cfg = di.config("c2_ngp")
    box = cfg["parts"][0]
    o, d = di.make_rays(cfg, seed=seed, R=R)
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, 1)
    off, seg_ray, seg_slot = oracle.bucket_segments(cnt, part, 1)
    g = oracle.occ_init(N, di.box_extent(box))
    dens = di.make_cell_densities(list(g.shape), seed=seed)
    bits, n_set = oracle.occ_bits(dens, 0.6)
    assert 0.03 < n_set / g.n_cells < 0.5
    dt = float(di.box_extent(box).max()) * np.sqrt(3.0) / 1024          # Instant-NGP's step for the unit cube, scaled
    return cfg, box, o, d, seg_t, seg_ray, seg_slot, int(off[1]), g, bits, np.float32(dt)


def test_fully_occupied_grid_reduces_to_stratified_sampling():
    cfg, box, o, d, seg_t, seg_ray, seg_slot, n_seg, g, bits, dt = _setup()
    full = np.full_like(bits, 0xFFFFFFFF)
    first, u, delta, t, ray = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, full, dt, seed=3)
    lens = (seg_t[seg_ray[:n_seg], seg_slot[:n_seg], 1] - seg_t[seg_ray[:n_seg], seg_slot[:n_seg], 0]).astype(np.float64)
    ratio = lens / float(dt)
    clear = np.abs(ratio - np.round(ratio)) > 1e-3
    counts = np.diff(first.astype(np.int64))
    np.testing.assert_array_equal(counts[clear], np.ceil(ratio)[clear].astype(np.int64))   # strata no wider than dt
    assert counts.min() >= 1 and counts.max() > 64                          # several wavefront-widths long
    for j in (0, 7, n_seg - 1):
        S = int(counts[j])
        u1, d1, t1 = oracle.sample_segments(o, d, seg_t, seg_ray, seg_slot, j, j + 1, box, S, seed=3, want_t=True)
        sl = slice(first[j], first[j + 1])
        np.testing.assert_array_equal(u[sl], u1)
        np.testing.assert_array_equal(delta[sl], d1)
        np.testing.assert_array_equal(t[sl], t1)
        assert np.all(ray[sl] == seg_ray[j])
    # strata pave the segment
    total = np.add.reduceat(delta.astype(np.float64), first[:-1].astype(np.int64))
    np.testing.assert_allclose(total, lens, rtol=1e-5)


def test_empty_grid_gives_no_samples():
    cfg, box, o, d, seg_t, seg_ray, seg_slot, n_seg, g, bits, dt = _setup(R=50)
    first, u, delta, t, ray = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, np.zeros_like(bits), dt)
    assert u.shape[0] == 0 and np.all(first == 0) and first.size == n_seg + 1


def test_kept_samples_are_exactly_those_in_occupied_cells():
    cfg, box, o, d, seg_t, seg_ray, seg_slot, n_seg, g, bits, dt = _setup()
    full = np.full_like(bits, 0xFFFFFFFF)
    f_all, u_all, d_all, t_all, r_all = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, full, dt, seed=5)
    first, u, delta, t, ray = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, bits, dt, seed=5)
    cells = oracle.occ_cell(g, u_all)
    keep = ((bits[cells >> 5] >> (cells & 31)) & 1).astype(bool)
    assert 0.02 < keep.mean() < 0.6
    np.testing.assert_array_equal(u, u_all[keep])
    np.testing.assert_array_equal(delta, d_all[keep])
    np.testing.assert_array_equal(t, t_all[keep])
    np.testing.assert_array_equal(ray, r_all[keep])
    seg_of = np.repeat(np.arange(n_seg), np.diff(f_all.astype(np.int64)))
    np.testing.assert_array_equal(np.diff(first.astype(np.int64)), np.bincount(seg_of[keep], minlength=n_seg))
    assert np.any(np.diff(first.astype(np.int64)) == 0)                     # some segments see nothing


def test_skipping_empty_space_does_not_change_the_rendering():
    # a field whose density vanishes outside the occupied cells renders the same with and without skipping
    cfg, box, o, d, seg_t, seg_ray, seg_slot, n_seg, g, bits, dt = _setup()
    full = np.full_like(bits, 0xFFFFFFFF)
    f_all, u_all, d_all, t_all, _ = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, full, dt, seed=6)
    first, u, delta, t, _ = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, bits, dt, seed=6)
    cells = oracle.occ_cell(g, u_all)
    keep = ((bits[cells >> 5] >> (cells & 31)) & 1).astype(bool)
    rng = np.random.default_rng(2)
    sigma_all = np.where(keep, rng.random(keep.size) * 300.0, 0.0)
    rgb_all = rng.random((keep.size, 3))
    C_all, T_all = oracle.composite_fwd_ragged(sigma_all, rgb_all, d_all, f_all)
    D_all = oracle.composite_depth_ragged(sigma_all, d_all, t_all, f_all)
    C, T = oracle.composite_fwd_ragged(sigma_all[keep], rgb_all[keep], delta, first)
    D = oracle.composite_depth_ragged(sigma_all[keep], delta, t, first)
    np.testing.assert_allclose(C, C_all, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(T, T_all, rtol=1e-12)
    np.testing.assert_allclose(D, D_all, rtol=1e-12, atol=1e-15)
    assert T.min() < 0.5 and np.any(T == 1.0)


def test_step_limit_stretches_the_strata():
    cfg, box, o, d, seg_t, seg_ray, seg_slot, n_seg, g, bits, dt = _setup(R=40)
    full = np.full_like(bits, 0xFFFFFFFF)
    first, u, delta, t, _ = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, full, dt, max_steps=5)
    np.testing.assert_array_equal(np.diff(first.astype(np.int64)), 5)
    lens = (seg_t[seg_ray[:n_seg], seg_slot[:n_seg], 1] - seg_t[seg_ray[:n_seg], seg_slot[:n_seg], 0]).astype(np.float64)
    np.testing.assert_allclose(delta.reshape(n_seg, 5).sum(1), lens, rtol=1e-5)
    # a step longer than the segment: one stratum
    first, *_ = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, 0, n_seg, box, g, full, np.float32(100.0))
    np.testing.assert_array_equal(np.diff(first.astype(np.int64)), 1)


# ---------------------------------------------------------------- compositing segments of different lengths
def test_ragged_composite_equals_fixed_length_composite_when_lengths_agree():
    rng = np.random.default_rng(1)
    n_seg, S = 9, 13
    sigma, delta = rng.random(n_seg * S) * 30, rng.random(n_seg * S) * 0.1
    rgb, t = rng.random((n_seg * S, 3)), np.sort(rng.random((n_seg, S)), 1).ravel()
    first = np.arange(n_seg + 1, dtype=np.uint32) * S
    C1, T1 = oracle.composite_fwd(sigma, rgb, delta, S)
    C2, T2 = oracle.composite_fwd_ragged(sigma, rgb, delta, first)
    np.testing.assert_array_equal(C1, C2)
    np.testing.assert_array_equal(T1, T2)
    gC, gT = rng.standard_normal((n_seg, 3)), rng.standard_normal(n_seg)
    a = oracle.composite_bwd(sigma, rgb, delta, S, gC, gT)
    b = oracle.composite_bwd_ragged(sigma, rgb, delta, first, gC, gT)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    np.testing.assert_array_equal(oracle.composite_depth(sigma, delta, t, S), oracle.composite_depth_ragged(sigma, delta, t, first))


def test_ragged_composite_by_hand_and_by_finite_differences():
    rng = np.random.default_rng(4)
    first = np.array([0, 3, 3, 4, 10], np.uint32)                           # lengths 3, 0, 1, 6
    n = 10
    sigma, delta, rgb = rng.random(n) * 20, rng.random(n) * 0.1, rng.random((n, 3))
    C, T = oracle.composite_fwd_ragged(sigma, rgb, delta, first)
    assert np.all(C[1] == 0) and T[1] == 1.0                                # nothing sampled: transparent
    a = 1 - np.exp(-sigma * delta)
    np.testing.assert_allclose(C[2], a[3] * rgb[3], rtol=1e-12)             # one sample: alpha c
    np.testing.assert_allclose(T[2], 1 - a[3], rtol=1e-12)
    np.testing.assert_allclose(C[0], a[0] * rgb[0] + (1 - a[0]) * a[1] * rgb[1] + (1 - a[0]) * (1 - a[1]) * a[2] * rgb[2], rtol=1e-12)
    np.testing.assert_allclose(T[3], np.prod(1 - a[4:10]), rtol=1e-12)
    gC, gT = rng.standard_normal((4, 3)), rng.standard_normal(4)
    dsigma, drgb = oracle.composite_bwd_ragged(sigma, rgb, delta, first, gC, gT)

    def f(s, c):
        Cx, Tx = oracle.composite_fwd_ragged(s, c, delta, first)
        return float((Cx * gC).sum() + (Tx * gT).sum())
    for i in range(n):
        e = np.zeros(n); e[i] = 1e-6
        np.testing.assert_allclose(dsigma[i], (f(sigma + e, rgb) - f(sigma - e, rgb)) / 2e-6, rtol=1e-5, atol=1e-9)
        ec = np.zeros((n, 3)); ec[i, 1] = 1e-6
        np.testing.assert_allclose(drgb[i, 1], (f(sigma, rgb + ec) - f(sigma, rgb - ec)) / 2e-6, rtol=1e-5, atol=1e-9)
