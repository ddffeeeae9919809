"""Pins for the oracle's ray / box segments, bucketing, sampling and direction encoding (CPU only).

Sources: DistGrid Sec. 4.2.1 (closely-paved, non-overlapping boxes; ray/box
test gives start, end and boundary-crossing times and the order), Fig. 2 steps
2-3; textbook slab test values; the published splitmix64 test vector; the
orthonormality and addition theorem of spherical harmonics.
"""
import numpy as np

import dg_inputs as di
import oracle


def test_single_box_textbook_cases():
    box = np.array([[-1, -1, -1, 1, 1, 1]], np.float32)
    o = np.array([[-3, 0, 0], [0, 0, 5], [0.5, 0.5, 0.5], [-3, 2, 0], [3, 3, 3], [0, 0, 5]], np.float32)
    d = np.array([[1, 0, 0], [0, 0, -1], [0, 1, 0], [1, 0, 0], [-1, -1, -1], [0, 0, 1]], np.float32)
    cnt, seg_t, part, status = oracle.ray_aabb_segments(o, d, box, 0.0, 2)
    assert list(cnt) == [1, 1, 1, 0, 1, 0] and status == 0
    np.testing.assert_array_equal(seg_t[0, 0], [2, 4])
    np.testing.assert_array_equal(seg_t[1, 0], [4, 6])
    np.testing.assert_array_equal(seg_t[2, 0], [0, 0.5])          # origin inside: clipped at t_min
    np.testing.assert_array_equal(seg_t[4, 0], [2, 4])            # unnormalised diagonal
    assert part[0, 0] == 0 and part[3, 0] == -1
    # t_min moves the start
    cnt, seg_t, _, _ = oracle.ray_aabb_segments(o[:1], d[:1], box, 3.0, 1)
    np.testing.assert_array_equal(seg_t[0, 0], [3, 4])


def test_rays_in_a_shared_face_belong_to_one_box():
    parts = di.config("c3_2x2")["parts"]
    # a ray running inside the plane x = 0 (d_x = 0): half-open rule assigns it to the boxes with lo_x = 0
    o = np.array([[0.0, -3.0, 0.1]], np.float32)
    d = np.array([[0.0, 1.0, 0.0]], np.float32)
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, parts, 0.0, 4)
    assert cnt[0] == 2
    assert [int(p) for p in part[0, :2]] == [1, 3]                # the two boxes with x in [0, 2]
    np.testing.assert_array_equal(seg_t[0, :2], [[1, 3], [3, 5]])
    # a ray on the outer face x = 2 of the tiling is outside every box
    cnt, *_ = oracle.ray_aabb_segments(np.array([[2.0, -3.0, 0.1]], np.float32), d, parts, 0.0, 4)
    assert cnt[0] == 0


def _tiling_checks(cfg, R, seed):
    parts = cfg["parts"]
    P = parts.shape[0]
    o, d = di.make_rays(cfg, seed=seed, R=R)
    cnt, seg_t, part, status = oracle.ray_aabb_segments(o, d, parts, 0.0, 6)
    assert status == 0
    scene = np.concatenate([parts[:, :3].min(0), parts[:, 3:].max(0)])[None]
    wcnt, wt, _, _ = oracle.ray_aabb_segments(o, d, scene, 0.0, 1)
    for r in range(R):
        K = cnt[r]
        if K == 0:
            continue
        t = seg_t[r, :K]
        assert np.all(t[:, 1] > t[:, 0])
        # consecutive, with bit-identical shared boundaries (the boxes pave the scene)
        np.testing.assert_array_equal(t[1:, 0], t[:-1, 1])
        assert len(set(part[r, :K])) == K                 # a convex box is crossed at most once
        # the union is the ray's intersection with the whole scene box (up to fp32 rounding of the ends)
        if wcnt[r]:
            assert abs(t[0, 0] - wt[r, 0, 0]) <= 1e-5 * max(1.0, abs(wt[r, 0, 0]))
            assert abs(t[-1, 1] - wt[r, 0, 1]) <= 1e-5 * max(1.0, abs(wt[r, 0, 1]))
        # brute force: points along each segment lie in the claimed box and in no other
        for k in range(K):
            for frac in (0.02, 0.5, 0.98):
                x = o[r].astype(np.float64) + (t[k, 0] + frac * (float(t[k, 1]) - float(t[k, 0]))) * d[r].astype(np.float64)
                inside = [p for p in range(P) if np.all(x >= parts[p, :3] - 1e-6) and np.all(x <= parts[p, 3:] + 1e-6)]
                strictly = [p for p in range(P) if np.all(x > parts[p, :3] + 1e-5) and np.all(x < parts[p, 3:] - 1e-5)]
                assert part[r, k] in inside
                assert strictly in ([], [part[r, k]])
    return cnt


def test_tiling_invariants_2x2():
    cfg = di.config("c3_2x2")
    cnt = _tiling_checks(cfg, 600, seed=0)
    assert cnt.max() <= 3                    # a line crosses at most Gx+Gy-1 cells of a 2x2 tiling
    assert np.mean(cnt >= 2) >= 0.4          # workload recipe: at least 40 % of rays cross two or more boxes


def test_tiling_invariants_2x4():
    cfg = di.config("c5_share")
    cnt = _tiling_checks(cfg, 600, seed=1)
    assert cnt.max() <= 5 and cnt.min() >= 1


def test_brute_force_membership_along_ray():
    # dense point sampling along the ray recovers the same ordered list of boxes
    cfg = di.config("c3_2x2")
    parts = cfg["parts"].astype(np.float64)
    o, d = di.make_rays(cfg, seed=5, R=60)
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, 4)
    for r in range(60):
        ts = np.linspace(0.0, 30.0, 60001)
        x = o[r].astype(np.float64)[None] + ts[:, None] * d[r].astype(np.float64)[None]
        label = np.full(ts.size, -1)
        for p in range(4):
            inside = np.all((x >= parts[p, :3]) & (x < parts[p, 3:]), axis=1)
            label[inside] = p
        order = [int(label[i]) for i in range(ts.size) if label[i] >= 0 and (i == 0 or label[i] != label[i - 1])]
        # drop slivers thinner than the sampling step (the oracle keeps them; brute force may not see them)
        mine = [int(part[r, k]) for k in range(cnt[r]) if seg_t[r, k, 1] - seg_t[r, k, 0] > 2e-3]
        brute = [p for p in order]
        assert [p for p in brute if p in mine] == mine


def test_k_max_overflow_keeps_front_segments():
    cfg = di.config("c5_share")
    o, d = di.make_rays(cfg, seed=2, R=400)
    full_cnt, full_t, full_part, st = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, 6)
    assert st == 0 and full_cnt.max() >= 3
    cnt, seg_t, part, st = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, 2)
    assert st == 1
    np.testing.assert_array_equal(cnt, np.minimum(full_cnt, 2))
    for r in range(400):
        np.testing.assert_array_equal(seg_t[r, :cnt[r]], full_t[r, :cnt[r]])
        np.testing.assert_array_equal(part[r, :cnt[r]], full_part[r, :cnt[r]])


def test_bucket_is_stable_counting_sort():
    cfg = di.config("c3_2x2")
    o, d = di.make_rays(cfg, seed=3, R=500)
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, 4)
    off, seg_ray, seg_slot = oracle.bucket_segments(cnt, part, 4)
    rays, slots = np.nonzero(np.arange(4)[None, :] < cnt[:, None])
    keys = part[rays, slots]
    order = np.argsort(keys, kind="stable")                       # library routine as the reference
    np.testing.assert_array_equal(seg_ray, rays[order])
    np.testing.assert_array_equal(seg_slot, slots[order])
    np.testing.assert_array_equal(off, np.concatenate([[0], np.cumsum(np.bincount(keys, minlength=4))]))


def test_jitter_generator():
    # published splitmix64 vector: seed 0, first output 0xE220A8397B1DCDAF -> top 24 bits / 2^24
    assert oracle.jitter(0, 0, 0, 0) == 0xE220A8 / 2.0 ** 24
    xs = np.array([oracle.jitter(7, r, k, s) for r in range(40) for k in range(3) for s in range(32)])
    assert xs.min() >= 0.0 and xs.max() < 1.0
    assert abs(xs.mean() - 0.5) < 0.02 and abs(xs.var() - 1 / 12) < 0.01
    assert len(np.unique(xs)) > 0.99 * xs.size
    assert oracle.jitter(7, 1, 2, 3) != oracle.jitter(8, 1, 2, 3)


def test_stratified_samples_pave_the_segment():
    cfg = di.config("c3_2x2")
    parts = cfg["parts"]
    o, d = di.make_rays(cfg, seed=4, R=200)
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, parts, 0.0, 4)
    off, seg_ray, seg_slot = oracle.bucket_segments(cnt, part, 4)
    S = 16
    for p in range(4):
        b, e = int(off[p]), int(off[p + 1])
        u, delta = oracle.sample_segments(o, d, seg_t, seg_ray, seg_slot, b, e, parts[p], S, seed=11)
        u = u.reshape(e - b, S, 3); delta = delta.reshape(e - b, S)
        assert u.min() > -1e-5 and u.max() < 1 + 1e-5          # samples of a segment lie in its own box
        for j in range(e - b):
            r, k = seg_ray[b + j], seg_slot[b + j]
            t_in, t_out = (float(v) for v in seg_t[r, k])
            np.testing.assert_allclose(delta[j].astype(np.float64).sum(), t_out - t_in, rtol=1e-6)
            # recover t from u along the ray's dominant axis and check its stratum
            x = parts[p, :3] + u[j].astype(np.float64) * (parts[p, 3:] - parts[p, :3]).astype(np.float64)
            a = int(np.argmax(np.abs(d[r])))
            t = (x[:, a] - o[r, a]) / d[r, a]
            s_idx = (t - t_in) / float(delta[j, 0])
            assert np.all(s_idx > np.arange(S) - 1e-3) and np.all(s_idx < np.arange(S) + 1 + 1e-3)
    # explicit jitter array: xi = 0.5 puts every sample at its stratum centre
    b, e = int(off[0]), int(off[1])
    u, delta = oracle.sample_segments(o, d, seg_t, seg_ray, seg_slot, b, e, parts[0], S,
                                      jitter_arr=np.full((e - b) * S, 0.5, np.float32))
    r, k = seg_ray[b], seg_slot[b]
    t_mid = seg_t[r, k, 0] + (np.arange(S) + 0.5) * delta[0]
    x = o[r][None] + t_mid[:, None] * d[r][None]
    np.testing.assert_allclose(u[:S], (x - parts[0, :3]) / (parts[0, 3:] - parts[0, :3]), atol=2e-6)


def test_spherical_harmonics():
    # constants and axis values
    out = oracle.sh(np.array([[0, 0, 1], [1, 0, 0], [0, 1, 0]], np.float32), 4)
    assert abs(out[0, 0] - 0.5 / np.sqrt(np.pi)) < 1e-15
    assert abs(out[0, 2] - np.sqrt(3 / (4 * np.pi))) < 1e-15          # Y_1^0 = sqrt(3/4pi) z
    assert abs(out[0, 6] - np.sqrt(5 / (16 * np.pi)) * 2) < 1e-15      # Y_2^0 = sqrt(5/16pi)(3z^2-1)
    assert abs(abs(out[1, 3]) - np.sqrt(3 / (4 * np.pi))) < 1e-15      # |Y_1^1| on the x axis
    assert abs(abs(out[2, 1]) - np.sqrt(3 / (4 * np.pi))) < 1e-15      # |Y_1^-1| on the y axis
    # orthonormality by Gauss-Legendre x uniform-azimuth quadrature (exact for these polynomials)
    xs, ws = np.polynomial.legendre.leggauss(12)
    phis = 2 * np.pi * (np.arange(24) + 0.5) / 24
    ct, ph = np.meshgrid(xs, phis, indexing="ij")
    st = np.sqrt(1 - ct ** 2)
    dirs = np.stack([st * np.cos(ph), st * np.sin(ph), ct], -1).reshape(-1, 3)
    w = (ws[:, None] * np.full((1, 24), 2 * np.pi / 24)).reshape(-1)
    Y = oracle.sh(dirs.astype(np.float64).astype(np.float32), 4)
    # float32 directions are not exactly unit length; the oracle normalises, so the Gram matrix is still I
    gram = (Y * w[:, None]).T @ Y
    np.testing.assert_allclose(gram, np.eye(16), atol=2e-6)
    # addition theorem: sum_m Y_lm^2 = (2l+1)/4pi for every direction
    rnd = np.random.default_rng(0).standard_normal((100, 3)).astype(np.float32)
    Y = oracle.sh(rnd, 4)
    for l in range(4):
        np.testing.assert_allclose((Y[:, l * l:(l + 1) ** 2] ** 2).sum(1), (2 * l + 1) / (4 * np.pi), rtol=1e-12)
    # degree 2 is the prefix of degree 4
    np.testing.assert_array_equal(oracle.sh(rnd, 2), Y[:, :4])


# ---------------------------------------------------------------------------- partitions with a hole (Sec. 4.2.2)
def _cascade():
    cfg = di.config("c6_cascade")
    return cfg, cfg["parts"], cfg["holes"]


def test_cascade_segments_pave_the_outer_box():
    cfg, parts, holes = _cascade()
    R = 500
    o, d = di.make_rays(cfg, seed=2, R=R)
    cnt, seg_t, part, status = oracle.ray_aabb_segments(o, d, parts, 0.0, 10, holes=holes)
    assert status == 0
    scene = np.concatenate([parts[:, :3].min(0), parts[:, 3:].max(0)])[None]
    wcnt, wt, _, _ = oracle.ray_aabb_segments(o, d, scene, 0.0, 1)
    seen_two = 0
    for r in range(R):
        K = cnt[r]
        assert (K > 0) == (wcnt[r] > 0)
        if K == 0:
            continue
        t = seg_t[r, :K]
        assert np.all(t[:, 1] > t[:, 0])
        np.testing.assert_array_equal(t[1:, 0], t[:-1, 1])          # fine and coarse pieces share bit-identical boundaries
        assert abs(t[0, 0] - wt[r, 0, 0]) <= 1e-5 * max(1.0, abs(wt[r, 0, 0]))
        assert abs(t[-1, 1] - wt[r, 0, 1]) <= 1e-5 * max(1.0, abs(wt[r, 0, 1]))
        ids = list(part[r, :K])
        seen_two += any(ids.count(p) == 2 for p in ids)
        assert all(ids.count(p) <= (2 if p >= 4 else 1) for p in ids)     # only a region with a hole is met twice
        for k in range(K):
            p = part[r, k]
            for frac in (0.02, 0.5, 0.98):
                x = o[r].astype(np.float64) + (t[k, 0] + frac * (float(t[k, 1]) - float(t[k, 0]))) * d[r].astype(np.float64)
                assert np.all(x >= parts[p, :3] - 1e-5) and np.all(x <= parts[p, 3:] + 1e-5)
                if p >= 4:      # not strictly inside the hole
                    assert not (np.all(x > holes[p, :3] + 1e-5) and np.all(x < holes[p, 3:] - 1e-5))
    assert seen_two > 20        # the recipe does produce rays that enter a coarse region twice


def test_cascade_brute_force_labels():
    cfg, parts, holes = _cascade()
    o, d = di.make_rays(cfg, seed=7, R=40)
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, parts, 0.0, 10, holes=holes)
    P64, H64 = parts.astype(np.float64), holes.astype(np.float64)
    for r in range(40):
        ts = np.linspace(0.0, 30.0, 120001)
        x = o[r].astype(np.float64)[None] + ts[:, None] * d[r].astype(np.float64)[None]
        label = np.full(ts.size, -1)
        for p in range(8):
            inside = np.all((x >= P64[p, :3]) & (x < P64[p, 3:]), axis=1)
            if p >= 4:
                inside &= ~np.all((x >= H64[p, :3]) & (x < H64[p, 3:]), axis=1)
            label[inside] = p
        order = [int(label[i]) for i in range(ts.size) if label[i] >= 0 and (i == 0 or label[i] != label[i - 1])]
        mine = [int(part[r, k]) for k in range(cnt[r]) if seg_t[r, k, 1] - seg_t[r, k, 0] > 2e-3]
        kept, it = [], iter(order)
        assert all(any(q == p for q in it) for p in mine), (r, order, mine)       # `mine` is a subsequence of the brute-force order


def test_hole_without_volume_or_out_of_reach_changes_nothing():
    cfg, parts, holes = _cascade()
    o, d = di.make_rays(cfg, seed=3, R=300)
    ref = oracle.ray_aabb_segments(o, d, parts, 0.0, 10)
    flat = np.zeros_like(holes)
    flat[:, 3:5] = 1.0                                  # zero height: no volume
    got = oracle.ray_aabb_segments(o, d, parts, 0.0, 10, holes=flat)
    for a, b in zip(ref[:3], got[:3]):
        np.testing.assert_array_equal(a, b)
    far = np.tile(np.array([50, 50, 50, 51, 51, 51], np.float32), (8, 1))    # a hole no ray reaches
    got = oracle.ray_aabb_segments(o, d, parts, 0.0, 10, holes=far)
    for a, b in zip(ref[:3], got[:3]):
        np.testing.assert_array_equal(a, b)


def test_single_box_with_a_centred_hole():
    # textbook case: unit cube with a cube hole in the middle, ray along x through the centre
    box = np.array([[0, 0, 0, 4, 4, 4]], np.float32)
    hole = np.array([[1, 1, 1, 3, 3, 3]], np.float32)
    o = np.array([[-1, 2, 2], [-1, 0.5, 2], [2, 2, 2]], np.float32)
    d = np.array([[1, 0, 0], [1, 0, 0], [1, 0, 0]], np.float32)
    cnt, t, part, _ = oracle.ray_aabb_segments(o, d, box, 0.0, 4, holes=hole)
    assert list(cnt) == [2, 1, 1]
    np.testing.assert_array_equal(t[0, :2], [[1, 2], [4, 5]])
    np.testing.assert_array_equal(t[1, 0], [1, 5])                        # passes beside the hole
    np.testing.assert_array_equal(t[2, 0], [1, 2])                        # starts inside the hole (t_min = 0): only the far piece


def test_hole_that_overhangs_its_box_is_cut_to_the_box():
    """Sec. 4.2.2 reading: a coarse partition covers its outer box minus the inner box.  Given the WHOLE inner box as the
    hole of every outer partition, the hole reaches beyond each partition: the pieces must stay inside the partition's own
    interval on the ray.  Checked by brute force: points along the ray, labelled by box membership minus hole membership."""
    outer = np.array([[-3, -3, 0, 0, 0, 0.5], [0, -3, 0, 3, 0, 0.5], [-3, 0, 0, 0, 3, 0.5], [0, 0, 0, 3, 3, 0.5]], np.float32)
    inner = np.tile(np.array([-1, -1, 0, 1, 1, 0.25], np.float32), (4, 1))           # overhangs every outer box
    rng = np.random.default_rng(5)
    R = 400
    o = np.stack([rng.uniform(-3, 3, R), rng.uniform(-3, 3, R), np.full(R, 1.5)], 1).astype(np.float32)
    tgt = np.stack([rng.uniform(-3, 3, R), rng.uniform(-3, 3, R), np.zeros(R)], 1)
    d = (tgt - o); d = (d / np.linalg.norm(d, axis=1, keepdims=True)).astype(np.float32)
    cnt, seg_t, part, status = oracle.ray_aabb_segments(o, d, outer, 0.0, 8, holes=inner)
    assert status == 0
    seen_cut = 0
    for r in range(R):
        K = cnt[r]
        t = seg_t[r, :K].astype(np.float64)
        assert np.all(t[:, 1] > t[:, 0]) and np.all(t[1:, 0] >= t[:-1, 1])          # ordered, never overlapping
        # brute force: total length per partition of {points in box p and outside the hole}
        ts = np.linspace(0.0, 10.0, 100001)
        x = o[r].astype(np.float64)[None] + ts[:, None] * d[r].astype(np.float64)[None]
        in_hole = np.all((x >= inner[0, :3]) & (x < inner[0, 3:]), axis=1)
        for p in range(4):
            inside = np.all((x >= outer[p, :3]) & (x < outer[p, 3:]), axis=1) & ~in_hole
            want = inside.sum() * (ts[1] - ts[0])
            got = sum(t[k, 1] - t[k, 0] for k in range(K) if part[r, k] == p)
            assert abs(got - want) <= 5e-4, (r, p, got, want)
        # every piece lies inside its own box (this is what fails without the cut)
        for k in range(K):
            mid = o[r].astype(np.float64) + 0.5 * (t[k, 0] + t[k, 1]) * d[r].astype(np.float64)
            p = part[r, k]
            assert np.all(mid >= outer[p, :3] - 1e-6) and np.all(mid <= outer[p, 3:] + 1e-6)
        seen_cut += int(in_hole.any() and K >= 2)
    assert seen_cut > 20
