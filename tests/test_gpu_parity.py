"""GPU parity: every entry point of libdistgrid against the CPU oracle on the same seeded inputs.

Bar: bit-exact for segment bookkeeping, bucket lists, sample coordinates and corner indices;
relative error <= 1e-5 for the fp32 encode, composite and merge; <= 2e-3 for the fp16-input MLPs
and for gradients accumulated with atomics.  Sizes span several tiles and a ragged tail.
"""
import sys

import numpy as np
import pytest
import torch

import dg_inputs as di
import oracle
import oracle.step as ostep
from paper_2405_04416_amd import binding as B

from gpu_util import (DEV, TOL_F16, TOL_F32, dev, from_planes, gpu_grid, gpu_mlp, gpu_models, have_gpu, host, make_step,
                      rel_err, to_planes)

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not have_gpu(), reason="needs a GPU")]


def say(msg):
    print("[case]", msg)
    sys.stdout.flush()


def ora_grid(cfg, part=0):
    g = cfg["grid"]
    b = g.get("growth") or oracle.growth_factor(g["n_min"], g["n_max"], g["L"])
    return oracle.grid_init(g["L"], g["F"], g["log2_T"], g["n_min"], b, di.box_extent(cfg["parts"][part]))


# ---------------------------------------------------------------------------- segments
def _run_segments(o, d, parts, k_max, t_min=0.0, holes=None):
    R, P = o.shape[0], parts.shape[0]
    i32 = torch.int32
    cnt = torch.zeros(max(R, 1), dtype=i32, device=DEV)
    seg_t = torch.zeros(max(R, 1), k_max, 2, device=DEV)
    part = torch.zeros(max(R, 1), k_max, dtype=i32, device=DEV)
    off = torch.zeros(P + 1, dtype=i32, device=DEV)
    ray = torch.zeros(max(R * k_max, 1), dtype=i32, device=DEV)
    slot = torch.zeros(max(R * k_max, 1), dtype=i32, device=DEV)
    status = torch.zeros(1, dtype=i32, device=DEV)
    ws = torch.zeros(max(B.dg_segments_workspace_bytes(R, P) // 4, 1), dtype=i32, device=DEV)
    od, dd = (dev(o), dev(d)) if R else (torch.zeros(1, 3, device=DEV), torch.zeros(1, 3, device=DEV))
    B.dg_ray_aabb_segments(od[:R], dd[:R], dev(parts), t_min, k_max, cnt, seg_t, part, status, off, ray, slot, ws,
                           holes=None if holes is None else dev(holes))
    torch.cuda.synchronize()
    return host(cnt)[:R], host(seg_t)[:R], host(part)[:R], int(host(status)[0]), host(off), host(ray), host(slot)


@pytest.mark.parametrize("name,R,k_max", [("c3_2x2", 5000, 4), ("c5_share", 3001, 6), ("c2_ngp", 1000, 1),
                                          ("c1_tiny", 1024, 1), ("c5_share", 2000, 2), ("c6_cascade", 6001, 10),
                                          ("c6_cascade", 2500, 3), ("c6_cascade", 999, 12)])
def test_segments_bit_exact(name, R, k_max):
    say("segments %s R=%d k_max=%d" % (name, R, k_max))
    cfg = di.config(name)
    o, d = di.make_rays(cfg, seed=7, R=R)
    # a few hand-placed rays: inside a shared face, parallel to an axis, missing everything
    o[:3] = [[0.0, -3.0, 0.1], [0.5, 0.5, 5.0], [50.0, 50.0, 50.0]]
    d[:3] = [[0.0, 1.0, 0.0], [0.0, 0.0, -1.0], [0.0, 0.0, 1.0]]
    P = cfg["parts"].shape[0]
    cnt, seg_t, part, status, off, ray, slot = _run_segments(o, d, cfg["parts"], k_max, holes=cfg.get("holes"))
    rc, rt, rp, rs = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, k_max, holes=cfg.get("holes"))
    np.testing.assert_array_equal(cnt, rc)
    np.testing.assert_array_equal(seg_t.view(np.uint32), rt.view(np.uint32))      # bit for bit
    np.testing.assert_array_equal(part, rp)
    assert status == rs
    roff, rray, rslot = oracle.bucket_segments(rc, rp, P)
    np.testing.assert_array_equal(off, roff)
    n = int(roff[-1])
    np.testing.assert_array_equal(ray[:n], rray)
    np.testing.assert_array_equal(slot[:n], rslot)


def test_segments_hole_that_overhangs_its_box():
    """The whole inner box given as the hole of every outer partition (Sec. 4.2.2 read as outer box minus inner box):
    the pieces are cut to each partition's own interval; bit for bit against the oracle."""
    say("segments with overhanging holes")
    cfg = di.config("c6_cascade")
    parts = cfg["parts"][4:]
    holes = np.tile(np.array([-1, -1, 0, 1, 1, 0.25], np.float32), (4, 1))
    o, d = di.make_rays(cfg, seed=12, R=4001)
    cnt, seg_t, part, status, off, ray, slot = _run_segments(o, d, parts, 8, holes=holes)
    rc, rt, rp, rs = oracle.ray_aabb_segments(o, d, parts, 0.0, 8, holes=holes)
    np.testing.assert_array_equal(cnt, rc)
    np.testing.assert_array_equal(seg_t.view(np.uint32), rt.view(np.uint32))
    np.testing.assert_array_equal(part, rp)
    assert status == rs and rc.max() >= 3


def test_segments_empty_batch():
    cfg = di.config("c3_2x2")
    cnt, seg_t, part, status, off, ray, slot = _run_segments(np.zeros((0, 3), np.float32), np.zeros((0, 3), np.float32),
                                                            cfg["parts"], 4)
    assert list(off) == [0] * 5 and status == 0


@pytest.mark.parametrize("use_array", [True, False])
def test_sampling_bit_exact(use_array):
    say("sampling array=%s" % use_array)
    cfg = di.config("c3_2x2")
    parts, S, k_max, R = cfg["parts"], 24, 4, 3000
    o, d = di.make_rays(cfg, seed=8, R=R)
    rc, rt, rp, _ = oracle.ray_aabb_segments(o, d, parts, 0.0, k_max)
    off, ray, slot = oracle.bucket_segments(rc, rp, 4)
    od, dd, td = dev(o), dev(d), dev(rt)
    rayd, slotd = dev(ray.astype(np.int32)), dev(slot.astype(np.int32))
    for p in range(4):
        b, e = int(off[p]), int(off[p + 1])
        n = (e - b) * S
        jit = di.make_jitter(n, seed=p) if use_array else None
        u = torch.zeros(n, 3, device=DEV); delta = torch.zeros(n, device=DEV); t = torch.zeros(n, device=DEV)
        B.dg_sample_segments(od, dd, td, rayd[b:e], slotd[b:e], e - b, k_max, parts[p], S, 99,
                             None if jit is None else dev(jit), u, delta, t if p % 2 == 0 else None)
        ru, rdelta, rt_s = oracle.sample_segments(o, d, rt, ray, slot, b, e, parts[p], S, seed=99, jitter_arr=jit, want_t=True)
        np.testing.assert_array_equal(host(u).view(np.uint32), ru.view(np.uint32))
        np.testing.assert_array_equal(host(delta).view(np.uint32), rdelta.view(np.uint32))
        if p % 2 == 0:
            np.testing.assert_array_equal(host(t).view(np.uint32), rt_s.view(np.uint32))      # sample distances, bit for bit


@pytest.mark.parametrize("degree", [1, 2, 3, 4])
def test_dir_encode(degree):
    d = np.random.default_rng(3).standard_normal((1000, 3)).astype(np.float32)
    d[0] = [0, 0, 1]; d[1] = [0, 0, 0]
    idx = np.random.default_rng(4).integers(0, 1000, 777).astype(np.int32)
    out = torch.zeros(777, degree * degree, dtype=torch.float16, device=DEV)
    B.dg_dir_encode(dev(d), dev(idx), 777, degree, out)
    ref = oracle.sh(d[idx], degree)
    ref[idx == 1] = oracle.sh(np.array([[0, 0, 1]], np.float32), degree)      # zero vector: library uses +z
    assert np.max(np.abs(host(out).astype(np.float64) - ref)) <= 1e-3          # fp16 rounding of values <= 1.1
    out2 = torch.zeros(1000, degree * degree, dtype=torch.float16, device=DEV)
    B.dg_dir_encode(dev(d), None, 1000, degree, out2)
    np.testing.assert_array_equal(host(out2)[idx], host(out))


# ---------------------------------------------------------------------------- encode
GRIDS = {
    "c1": lambda: (di.config("c1_tiny"), None),
    "c2": lambda: (di.config("c2_ngp"), None),
    "mixed_small": lambda: (None, dict(L=6, F=2, log2_T=10, n_min=4, growth=1.7, extent=[1.0, 2.0, 0.5])),
    "one_level_dense": lambda: (None, dict(L=1, F=2, log2_T=12, n_min=15, growth=1.0, extent=[1.0, 1.0, 1.0])),
    # 37^3 vertices in one dense level: 7 bins of 8192 entries, odd row length, so x-pairs straddle bin boundaries
    "dense_odd": lambda: (None, dict(L=1, F=2, log2_T=16, n_min=36, growth=1.0, extent=[1.0, 1.0, 1.0])),
    # two dense levels of 18^3 = 5832 entries: the first fits the LDS prefix, the second is binned and is a single bin
    "one_bin": lambda: (None, dict(L=2, F=2, log2_T=16, n_min=17, growth=1.0, extent=[1.0, 1.0, 1.0])),
    # T = 2^21: a dense level of 34 bins and hashed levels of 256 bins (more than one wavefront's worth)
    "wide": lambda: (None, dict(L=4, F=2, log2_T=21, n_min=64, growth=2.0, extent=[1.0, 1.0, 1.0])),
    # T = 2^24, three hashed levels: 6144 (level, bin) pairs, too many for the counters to sit in LDS
    "huge": lambda: (None, dict(L=3, F=2, log2_T=24, n_min=512, growth=2.0, extent=[1.0, 1.0, 1.0])),
}


def _coords(N, flavour, seed):
    """independent points, or stretches of 64 consecutive samples along short segments (as a ray gives them)"""
    if flavour == "points":
        return di.make_unit_coords(N, seed=seed)
    rng = np.random.default_rng(seed)
    n_seg = -(-N // 64)
    a = rng.random((n_seg, 1, 3))
    step = rng.standard_normal((n_seg, 1, 3)) * rng.choice([1e-4, 2e-3, 1e-2], size=(n_seg, 1, 1))
    u = a + step * np.arange(64).reshape(1, 64, 1)
    return np.clip(u, 0.0, 1.0).reshape(-1, 3)[:N].astype(np.float32)


def _both_grids(key):
    cfg, spec = GRIDS[key]()
    if cfg is not None:
        return gpu_grid(cfg), ora_grid(cfg), cfg["table_range"]
    g = B.dg_grid_desc_init(spec["L"], spec["F"], spec["log2_T"], spec["n_min"], spec["growth"], spec["extent"])
    r = oracle.grid_init(spec["L"], spec["F"], spec["log2_T"], spec["n_min"], spec["growth"], spec["extent"])
    return g, r, 1.0


@pytest.mark.parametrize("key,N", [("c1", 32768), ("c2", 10007), ("mixed_small", 3333), ("one_level_dense", 257),
                                   ("c2", 1), ("c2", 0), ("dense_odd", 4099), ("wide", 5003), ("huge", 5003)])
def test_encode_fwd_and_indices(key, N):
    say("encode fwd %s N=%d" % (key, N))
    g, r, rng_range = _both_grids(key)
    L = g.n_levels
    table = di.make_table(r.n_entries, 2, rng_range, seed=1)
    u = di.make_unit_coords(max(N, 1), seed=2)[:N]
    if N > 16:
        u[:6] = [[0, 0, 0], [1, 1, 1], [-0.3, 0.5, 2.0], [1, 0, 0.5], [0.999999, 0.999999, 0.999999], [0.5, 0.5, 0.5]]
    td, ud = dev(table), dev(u) if N else torch.zeros(1, 3, device=DEV)[:0]
    idx = torch.zeros(max(N, 1), L, 8, dtype=torch.int32, device=DEV)
    feat = torch.zeros(L, max(N, 1), 2, device=DEV)[:, :N].contiguous()            # level-major planes
    feat16 = torch.zeros(L, max(N, 1), 2, dtype=torch.float16, device=DEV)[:, :N].contiguous()
    B.dg_hashgrid_corner_indices(g, ud, N, idx)
    B.dg_hashgrid_encode_fwd(g, td, ud, N, feat)
    B.dg_hashgrid_encode_fwd(g, td, ud, N, feat16)
    torch.cuda.synchronize()
    if N == 0:
        return
    ref, ridx = oracle.encode_fwd(r, table, u, want_idx=True)
    np.testing.assert_array_equal(host(idx).view(np.uint32), ridx)                 # bit-exact indices
    bound = oracle.encode_fwd(r, table, u, abs_terms=True)                          # sum |w||theta| per output
    err = np.abs(from_planes(feat, N, 2 * L).astype(np.float64) - ref)
    assert np.all(err <= TOL_F32 * bound + 1e-30), float(np.max(err / (bound + 1e-30)))
    # fp16 output: the fp32 value rounded once
    err16 = np.abs(from_planes(feat16, N, 2 * L).astype(np.float64) - ref)
    assert np.all(err16 <= 2.0 ** -11 * np.abs(ref) + TOL_F32 * bound + 6e-8)


@pytest.mark.parametrize("mode", ["atomic", "binned", "binned_batched"])
@pytest.mark.parametrize("key,N,flavour", [("c1", 32768, "points"), ("c2", 10007, "points"), ("mixed_small", 3333, "points"),
                                           ("one_level_dense", 700, "points"), ("c2", 20011, "rays"),
                                           ("dense_odd", 150001, "points"), ("dense_odd", 30000, "rays"),
                                           ("wide", 20011, "points"), ("wide", 9000, "rays"), ("huge", 20011, "points"),
                                           ("c2", 1, "points"), ("c2", 7, "rays"), ("c2", 513, "rays"), ("c2", 2048 * 3 + 5, "rays"),
                                           ("one_bin", 60011, "rays"), ("one_bin", 3001, "points"),
                                           # the sweep for many bins with one tile, one and a bit, two and a bit (a workgroup takes two per step)
                                           ("huge", 1, "points"), ("wide", 513, "rays"), ("huge", 1025, "rays"), ("wide", 512 * 257 + 3, "rays")])
def test_encode_bwd(key, N, flavour, mode):
    say("encode bwd %s N=%d %s %s" % (key, N, flavour, mode))
    g, r, _ = _both_grids(key)
    L = g.n_levels
    u = _coords(N, flavour, seed=5)
    dfeat = (np.random.default_rng(6).standard_normal((N, 2 * L)) * 1e-3).astype(np.float32)
    dfeat[::7] = 0.0
    dtable = torch.zeros(r.n_entries, 2, device=DEV)
    ws = None
    if mode != "atomic":
        need = B.dg_hashgrid_encode_bwd_workspace_bytes(g, N)
        if mode == "binned_batched":                                   # room for a few tiles only: several batches
            need = B.dg_hashgrid_encode_bwd_workspace_bytes(g, 2048)
        ws = torch.zeros(need // 4 + 64, device=DEV)
    B.dg_hashgrid_encode_bwd(g, dev(u), dev(to_planes(dfeat)), N, dtable, ws)
    B.dg_hashgrid_encode_bwd(g, dev(u), dev(to_planes(dfeat)), N, dtable, ws)   # "+=": twice gives twice
    ref = 2.0 * oracle.encode_bwd(r, u, dfeat.astype(np.float64))
    got = host(dtable).astype(np.float64)
    for l in range(L):                                                # judged level by level
        sl = slice(r.first[l], r.first[l + 1])
        assert rel_err(got[sl], ref[sl]) <= TOL_F16, l
    assert np.all(got[ref == 0] == 0)                                 # untouched entries stay untouched


# The binned pass runs 768 persistent workgroups over tiles of 512 samples.  The cases above give a workgroup one tile per
# level at most; these give it several, element by element against the oracle: records that wait for a full granule
# from one step to the next and the two halves of the waiting slots (narrow sweep, c2), queue cursors that advance step
# after step (sweep for many bins: wide, huge), bins whose records are split over several accumulating workgroups
# (one_bin: 3.2 M records in one bin), and a capped workspace that makes two batches of two tiles per workgroup each.
STEADY = 2 * 768 * 512


@pytest.mark.parametrize("key,N,capped", [("c2", STEADY + 12345, False), ("c2", 2 * STEADY, True), ("wide", STEADY + 777, False),
                                          ("huge", STEADY + 777, False), ("one_bin", STEADY + 13579, False)])
def test_encode_bwd_several_tiles_per_workgroup(key, N, capped):
    say("encode bwd steady state %s N=%d capped=%s" % (key, N, capped))
    g, r, _ = _both_grids(key)
    L = g.n_levels
    u = _coords(N, "rays", seed=25)
    dfeat = (np.random.default_rng(26).standard_normal((N, 2 * L)) * 1e-3).astype(np.float32)
    dfeat[::11] = 0.0
    dtable = torch.zeros(r.n_entries, 2, device=DEV)
    need = B.dg_hashgrid_encode_bwd_workspace_bytes(g, N // 2 + 512 if capped else N)
    assert not capped or need < B.dg_hashgrid_encode_bwd_workspace_bytes(g, N)
    ws = torch.zeros(need // 4 + 64, device=DEV)
    B.dg_hashgrid_encode_bwd(g, dev(u), dev(to_planes(dfeat)), N, dtable, ws)
    torch.cuda.synchronize()
    ref = oracle.encode_bwd(r, u, dfeat.astype(np.float64))
    got = host(dtable).astype(np.float64)
    for l in range(L):
        sl = slice(r.first[l], r.first[l + 1])
        assert rel_err(got[sl], ref[sl]) <= TOL_F16, l
    assert np.all(got[ref == 0] == 0)


@pytest.mark.parametrize("key,N", [("c2", 40011), ("huge", 30011), ("c1", 5000)])
def test_encode_bwd_counted_ahead(key, N):
    """The binned pass in two parts (queue sizes counted early, on another stream; the rest later) gives what the one call gives,
    and the oracle's result."""
    say("encode bwd counted ahead %s N=%d" % (key, N))
    g, r, _ = _both_grids(key)
    L = g.n_levels
    u = _coords(N, "rays", seed=45)
    dfeat = (np.random.default_rng(46).standard_normal((N, 2 * L)) * 1e-3).astype(np.float32)
    ud, dd = dev(u), dev(to_planes(dfeat))
    ws = torch.zeros(B.dg_hashgrid_encode_bwd_workspace_bytes(g, N) // 4 + 64, device=DEV)
    whole = torch.zeros(r.n_entries, 2, device=DEV)
    B.dg_hashgrid_encode_bwd(g, ud, dd, N, whole, ws)
    torch.cuda.synchronize()
    ws.fill_(float("nan"))                                   # nothing of the first call may be left to lean on
    parts = torch.zeros(r.n_entries, 2, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.dg_hashgrid_encode_bwd_count(g, ud, N, ws)
        done = torch.cuda.Event()
        done.record()
    torch.cuda.current_stream().wait_event(done)
    B.dg_hashgrid_encode_bwd_counted(g, ud, dd, N, parts, ws)
    torch.cuda.synchronize()
    ref = oracle.encode_bwd(r, u, dfeat.astype(np.float64))
    a, b = host(whole).astype(np.float64), host(parts).astype(np.float64)
    for l in range(L):
        sl = slice(r.first[l], r.first[l + 1])
        assert rel_err(b[sl], a[sl]) <= 1e-6 and rel_err(b[sl], ref[sl]) <= TOL_F16, l
    # a workspace that cannot hold all samples in one batch is refused by both parts
    small = torch.zeros(B.dg_hashgrid_encode_bwd_workspace_bytes(g, max(N // 4, 512)) // 4, device=DEV)
    if small.numel() * 4 < B.dg_hashgrid_encode_bwd_workspace_bytes(g, N) and key != "c1":
        with pytest.raises(B.DistGridError):
            B.dg_hashgrid_encode_bwd_count(g, ud, N, small)
        with pytest.raises(B.DistGridError):
            B.dg_hashgrid_encode_bwd_counted(g, ud, dd, N, parts, small)


@pytest.mark.parametrize("bad", [np.inf, np.nan])
def test_encode_bwd_binned_marks_non_finite_gradients(bad):
    """A feature gradient that is infinite or NaN (an fp16 delta that overflowed under the loss scale) must not turn into
    finite numbers: the binned pass marks the table gradient with NaN."""
    say("encode bwd non-finite input %s" % bad)
    g, r, _ = _both_grids("c2")
    N = 5003
    u = _coords(N, "rays", seed=35)
    dfeat = (np.random.default_rng(36).standard_normal((N, 2 * g.n_levels)) * 1e-3).astype(np.float32)
    dfeat[1234, 20] = bad
    dtable = torch.zeros(r.n_entries, 2, device=DEV)
    ws = torch.zeros(B.dg_hashgrid_encode_bwd_workspace_bytes(g, N) // 4 + 64, device=DEV)
    B.dg_hashgrid_encode_bwd(g, dev(u), dev(to_planes(dfeat)), N, dtable, ws)
    torch.cuda.synchronize()
    assert not bool(torch.isfinite(dtable).all())


@pytest.mark.parametrize("with_ws", [False, True])
def test_encode_bwd_empty_batch(with_ws):
    """N = 0 adds nothing, with and without a workspace."""
    say("encode bwd empty batch ws=%s" % with_ws)
    g, r, _ = _both_grids("c2")
    dtable = torch.full((r.n_entries, 2), 3.0, device=DEV)
    ws = torch.zeros(B.dg_hashgrid_encode_bwd_workspace_bytes(g, 0) // 4 + 64, device=DEV) if with_ws else None
    empty = torch.zeros(1, 3, device=DEV)[:0]
    B.dg_hashgrid_encode_bwd(g, empty, torch.zeros(g.n_levels, 0, 2, device=DEV), 0, dtable, ws)
    torch.cuda.synchronize()
    assert bool((dtable == 3.0).all())


@pytest.mark.parametrize("key,N,flavour", [("c2", 30011, "rays"), ("wide", 20011, "points")])
def test_encode_bwd_binned_value_range(key, N, flavour):
    """The binned pass rounds a contribution to 18 mantissa bits and sums in fixed point scaled to the batch's largest
    magnitude: per entry the error stays within 2^-19 of the sum of |contributions| plus 2^-20 of that largest
    magnitude, for gradients that span 18 decades and sit right below powers of two (where rounding carries into the
    exponent)."""
    say("encode bwd value range %s N=%d %s" % (key, N, flavour))
    g, r, _ = _both_grids(key)
    L = g.n_levels
    u = _coords(N, flavour, seed=15)
    rng = np.random.default_rng(16)
    dfeat = (10.0 ** rng.uniform(-12, 6, (N, 2 * L)) * rng.choice([-1.0, 1.0], (N, 2 * L))).astype(np.float32)
    edge = np.nextafter(np.float32(2.0) ** rng.integers(-8, 8, (N // 5, 2 * L)).astype(np.float32), np.float32(0))
    dfeat[::5][:edge.shape[0]] = edge
    dtable = torch.zeros(r.n_entries, 2, device=DEV)
    ws = torch.zeros(B.dg_hashgrid_encode_bwd_workspace_bytes(g, N) // 4 + 64, device=DEV)
    B.dg_hashgrid_encode_bwd(g, dev(u), dev(to_planes(dfeat)), N, dtable, ws)
    ref = oracle.encode_bwd(r, u, dfeat.astype(np.float64))
    mass = oracle.encode_bwd(r, u, np.abs(dfeat).astype(np.float64))      # sum of |contributions| per entry
    got = host(dtable).astype(np.float64)
    largest = float(np.abs(dfeat).max())
    err = np.abs(got - ref)
    assert np.all(err <= 2.0 ** -19 * mass + 2.0 ** -20 * largest), float(np.max(err / (2.0 ** -19 * mass + 2.0 ** -20 * largest)))
    assert np.all(got[mass == 0] == 0)


@pytest.mark.parametrize("S,n_seg,k_max", [(64, 501, 4), (32, 77, 1), (100, 33, 3), (7, 1000, 12)])
def test_depth_channel(S, n_seg, k_max):
    """Evaluation depth (Sec. 4.4.2): per-segment expected distance and its merge, against the oracle."""
    say("depth S=%d n_seg=%d k_max=%d" % (S, n_seg, k_max))
    rng = np.random.default_rng(S * 1000 + n_seg)
    R = n_seg                                   # R * k_max >= n_seg distinct (ray, slot) pairs exist
    pairs = rng.permutation(R * k_max)[:n_seg]
    assert pairs.size == n_seg
    ray, slot = (pairs // k_max).astype(np.int32), (pairs % k_max).astype(np.int32)
    sigma = (rng.random(n_seg * S) * 40.0).astype(np.float32)
    sigma[rng.random(n_seg * S) < 0.3] = 0.0
    delta = (rng.random(n_seg * S) * 0.05).astype(np.float32)
    t = np.sort(rng.random((n_seg, S)) * 6.0, axis=1).reshape(-1).astype(np.float32)
    Dk = torch.zeros(R, k_max, device=DEV)
    B.dg_composite_segment_depth(dev(sigma), dev(delta), dev(t), n_seg, S, dev(ray), dev(slot), k_max, Dk)
    ref = oracle.composite_depth(sigma, delta, t, S)
    got = host(Dk)[ray, slot]
    assert np.all(np.abs(got - ref) <= TOL_F32 * np.maximum(np.abs(ref), 1e-3))
    # merge over random partials
    cnt = rng.integers(0, k_max + 1, R).astype(np.int32)
    Dk_h = (rng.random((R, k_max)) * 5.0).astype(np.float32)
    Tk_h = rng.random((R, k_max)).astype(np.float32)
    D = torch.full((R,), -1.0, device=DEV)
    B.dg_merge_depth(dev(Dk_h), dev(Tk_h), dev(cnt), R, k_max, D)
    refD = oracle.merge_depth(Dk_h, Tk_h, cnt.astype(np.uint32))
    assert np.all(np.abs(host(D) - refD) <= TOL_F32 * np.maximum(np.abs(refD), 1e-3))
    assert np.all(host(D)[cnt == 0] == 0.0)


# ---------------------------------------------------------------------------- MLPs
def _mlp_inputs(cfg, n, S, seed, scale=1.0):
    m = cfg["mlp"]
    n_feat = cfg["grid"]["L"] * cfg["grid"]["F"]
    w = di.make_mlp_weights(n_feat, m, seed=seed)
    rng = np.random.default_rng(seed + 1)
    feat = (rng.standard_normal((n, n_feat)) * scale).astype(np.float16)
    dirs = rng.standard_normal((-(-n // S), 3)).astype(np.float32)
    dir_enc = oracle.sh(dirs, m["sh_degree"]).astype(np.float16)
    odesc = oracle.mlp_desc(n_feat, m["n_hidden_d"], m["n_geo"], m["sh_degree"] ** 2, m["n_hidden_c"], m["n_layers_c"], 1, 1)
    return w, feat, dir_enc, odesc


@pytest.mark.parametrize("name,n,S", [("c2_ngp", 5000, 64), ("c1_tiny", 3001, 32), ("c2_ngp", 130, 7)])
def test_mlp_fwd(name, n, S):
    say("mlp fwd %s n=%d" % (name, n))
    cfg = di.config(name)
    w, feat, dir_enc, odesc = _mlp_inputs(cfg, n, S, seed=11)
    sigma = torch.zeros(n, device=DEV); rgb = torch.zeros(n, 3, device=DEV)
    B.dg_mlp_fwd(gpu_mlp(cfg), dev(w), dev(to_planes(feat)), dev(dir_enc), S, n, sigma, rgb)
    rs, rr = oracle.mlp_fwd(odesc, w.astype(np.float64), feat.astype(np.float64), dir_enc.astype(np.float64), S)
    assert rel_err(host(sigma), rs) <= TOL_F16
    assert rel_err(host(rgb), rr) <= TOL_F16


@pytest.mark.parametrize("name,n,S", [("c2_ngp", 5000, 64), ("c1_tiny", 3001, 32)])
def test_mlp_bwd(name, n, S):
    say("mlp bwd %s n=%d" % (name, n))
    cfg = di.config(name)
    w, feat, dir_enc, odesc = _mlp_inputs(cfg, n, S, seed=12)
    rng = np.random.default_rng(13)
    dsigma = (rng.standard_normal(n) * 1e-6).astype(np.float32)
    drgb = (rng.standard_normal((n, 3)) * 1e-6).astype(np.float32)
    scale = 2.0 ** 18
    mdesc = gpu_mlp(cfg)
    dfeat = torch.zeros(n, feat.shape[1], device=DEV)
    dW = torch.zeros(w.size, device=DEV)
    ws = torch.zeros(B.dg_mlp_bwd_workspace_bytes(mdesc, n) // 4 + 64, device=DEV)
    B.dg_mlp_bwd(mdesc, dev(w), dev(to_planes(feat)), dev(dir_enc), S, n, dev(dsigma), dev(drgb), scale, dfeat, dW, ws)
    rdf, rdw = oracle.mlp_bwd(odesc, w.astype(np.float64), feat.astype(np.float64), dir_enc.astype(np.float64), S,
                              dsigma.astype(np.float64), drgb.astype(np.float64), scale)
    assert rel_err(from_planes(dfeat, n, feat.shape[1]), rdf) <= TOL_F16
    pos = 0
    for (no, ni) in di.mlp_layer_shapes(feat.shape[1], cfg["mlp"]):       # judged matrix by matrix
        assert rel_err(host(dW)[pos:pos + no * ni], rdw[pos:pos + no * ni]) <= TOL_F16
        pos += no * ni


def test_mlp_bwd_several_tiles_per_wavefront():
    """The backward kernels keep the weight gradient in registers over all 32-sample tiles a persistent wavefront takes
    (2048 wavefronts): here every wavefront folds four or five tiles, judged matrix by matrix, and the feature gradient
    element by element."""
    n, S = 2 ** 18 + 4321, 64
    say("mlp bwd c2_ngp n=%d" % n)
    cfg = di.config("c2_ngp")
    w, feat, dir_enc, odesc = _mlp_inputs(cfg, n, S, seed=21)
    rng = np.random.default_rng(22)
    dsigma = (rng.standard_normal(n) * 1e-6).astype(np.float32)
    drgb = (rng.standard_normal((n, 3)) * 1e-6).astype(np.float32)
    scale = 2.0 ** 18
    mdesc = gpu_mlp(cfg)
    dfeat = torch.zeros(n, feat.shape[1], device=DEV)
    dW = torch.zeros(w.size, device=DEV)
    ws = torch.zeros(B.dg_mlp_bwd_workspace_bytes(mdesc, n) // 4 + 64, device=DEV)
    B.dg_mlp_bwd(mdesc, dev(w), dev(to_planes(feat)), dev(dir_enc), S, n, dev(dsigma), dev(drgb), scale, dfeat, dW, ws)
    torch.cuda.synchronize()
    rdf, rdw = oracle.mlp_bwd(odesc, w.astype(np.float64), feat.astype(np.float64), dir_enc.astype(np.float64), S,
                              dsigma.astype(np.float64), drgb.astype(np.float64), scale)
    # 8.5 M feature gradients: the largest deviation grows with the number of elements looked at, because now and then
    # a back-propagated delta sits on an fp16 rounding boundary and falls to the other side (fp32 against double
    # accumulation).  Measured on MI355X: 12 elements (6 samples) between 2e-3 and 4.6e-3, relative L2 error 1.4e-5.
    # The bar: at most one element in 10^5 beyond 2e-3, none beyond 1e-2, L2 error within 1e-4.
    got = from_planes(dfeat, n, feat.shape[1]).astype(np.float64)
    floor = float(np.mean(np.abs(rdf)))
    rel = np.abs(got - rdf) / np.maximum(np.abs(rdf), floor)
    assert int(np.sum(rel > TOL_F16)) <= rel.size // 100000 and float(rel.max()) <= 1e-2
    assert np.linalg.norm(got - rdf) <= 1e-4 * np.linalg.norm(rdf)
    pos = 0
    for (no, ni) in di.mlp_layer_shapes(feat.shape[1], cfg["mlp"]):
        assert rel_err(host(dW)[pos:pos + no * ni], rdw[pos:pos + no * ni]) <= TOL_F16
        pos += no * ni


@pytest.mark.parametrize("S,n_seg,n_app", [(64, 1201, 0), (48, 700, 0), (20, 333, 0), (1, 50, 0), (33, 257, 48)])
def test_mlp_composite_fused_forward(S, n_seg, n_app):
    """Evaluation rendering (Sec. 4.4.2) with networks and local rendering in one kernel: partial colour, transmittance
    and depth of every segment against the oracle's networks + quadrature, and against the separate entry points."""
    say("fused networks + rendering S=%d n_seg=%d n_app=%d" % (S, n_seg, n_app))
    cfg = di.config("c8_app" if n_app else "c2_ngp")
    n = n_seg * S
    w, feat, dir_enc, odesc = _mlp_inputs(cfg, n, S, seed=31, scale=0.5)
    rng = np.random.default_rng(32)
    n_feat = feat.shape[1]
    if n_app:
        app = rng.standard_normal((n_seg, n_app)).astype(np.float16)
        odesc = oracle.mlp_desc(n_feat, 64, 16, 16 + n_app, 64, 2, 1, 1)
        rows = np.concatenate([dir_enc, app], axis=1)
        from gpu_util import split_appearance_weights
        w_gpu = split_appearance_weights(w, n_feat, cfg["mlp"])
    else:
        app, rows, w_gpu = None, dir_enc, w
    delta = (rng.random(n) * 0.02 + 1e-3).astype(np.float32)
    t = np.sort(rng.random((n_seg, S)) * 4.0, axis=1).reshape(-1).astype(np.float32)
    R, k_max = n_seg + 3, 3
    seg_ray = rng.permutation(R)[:n_seg].astype(np.int32)
    seg_slot = rng.integers(0, k_max, n_seg).astype(np.int32)
    mdesc = gpu_mlp(cfg)
    fd, dd, ad = dev(to_planes(feat)), dev(dir_enc), None if app is None else dev(app)
    Ck = torch.zeros(R, k_max, 3, device=DEV); Tk = torch.ones(R, k_max, device=DEV); Dk = torch.zeros(R, k_max, device=DEV)
    B.dg_mlp_composite_fwd(mdesc, dev(w_gpu), fd, dd, ad, S, n_seg, dev(delta), dev(t), dev(seg_ray), dev(seg_slot), k_max, Ck, Tk, Dk)
    # the separate entry points on the same inputs
    sigma = torch.zeros(n, device=DEV); rgb = torch.zeros(n, 3, device=DEV)
    Ck2 = torch.zeros_like(Ck); Tk2 = torch.ones_like(Tk); Dk2 = torch.zeros_like(Dk)
    B.dg_mlp_fwd_app(mdesc, dev(w_gpu), fd, dd, ad, S, n, sigma, rgb)
    B.dg_composite_segment_fwd(sigma, rgb, dev(delta), n_seg, S, dev(seg_ray), dev(seg_slot), k_max, Ck2, Tk2)
    B.dg_composite_segment_depth(sigma, dev(delta), dev(t), n_seg, S, dev(seg_ray), dev(seg_slot), k_max, Dk2)
    torch.cuda.synchronize()
    for a, b in ((Ck, Ck2), (Tk, Tk2), (Dk, Dk2)):
        assert rel_err(host(a)[seg_ray, seg_slot], host(b)[seg_ray, seg_slot]) <= 1e-5
    rs, rr = oracle.mlp_fwd(odesc, w.astype(np.float64), feat.astype(np.float64), rows.astype(np.float64), S)
    rC, rT = oracle.composite_fwd(rs, rr, delta.astype(np.float64), S)
    rD = oracle.composite_depth(rs, delta.astype(np.float64), t.astype(np.float64), S)
    assert rel_err(host(Ck)[seg_ray, seg_slot], rC) <= TOL_F16
    assert rel_err(host(Tk)[seg_ray, seg_slot], rT) <= TOL_F16
    assert rel_err(host(Dk)[seg_ray, seg_slot], rD) <= TOL_F16
    untouched = np.ones((R, k_max), bool); untouched[seg_ray, seg_slot] = False
    assert np.all(host(Tk)[untouched] == 1) and np.all(host(Dk)[untouched] == 0)


# ---------------------------------------------------------------------------- rendering
@pytest.mark.parametrize("S,n_seg", [(64, 3000), (32, 1025), (48, 700), (7, 300), (150, 41), (1, 100)])
def test_composite_fwd_bwd(S, n_seg):
    say("composite S=%d n_seg=%d" % (S, n_seg))
    rng = np.random.default_rng(S)
    n = n_seg * S
    sigma = np.exp(rng.standard_normal(n) * 2.0).astype(np.float32)
    rgb = rng.random((n, 3), dtype=np.float32)
    delta = (rng.random(n, dtype=np.float32) * 0.05 + 0.001).astype(np.float32)
    R, k_max = n_seg + 5, 3
    seg_ray = rng.permutation(R)[:n_seg].astype(np.int32)
    seg_slot = rng.integers(0, k_max, n_seg).astype(np.int32)
    Ck = torch.zeros(R, k_max, 3, device=DEV); Tk = torch.ones(R, k_max, device=DEV)
    sd, rd, dd, rayd, slotd = dev(sigma), dev(rgb), dev(delta), dev(seg_ray), dev(seg_slot)
    B.dg_composite_segment_fwd(sd, rd, dd, n_seg, S, rayd, slotd, k_max, Ck, Tk)
    rC, rT = oracle.composite_fwd(sigma, rgb, delta, S)
    assert rel_err(host(Ck)[seg_ray, seg_slot], rC, floor=1e-30) <= TOL_F32       # all terms positive: plain relative
    assert rel_err(host(Tk)[seg_ray, seg_slot], rT, floor=1e-20) <= TOL_F32       # below 1e-20: judged absolutely
    gCk = rng.standard_normal((R, k_max, 3)).astype(np.float32)
    gTk = rng.standard_normal((R, k_max)).astype(np.float32)
    dsigma = torch.zeros(n, device=DEV); drgb = torch.zeros(n, 3, device=DEV)
    B.dg_composite_segment_bwd(sd, rd, dd, n_seg, S, rayd, slotd, k_max, dev(gCk), dev(gTk), dsigma, drgb)
    rds, rdc = oracle.composite_bwd(sigma, rgb, delta, S, gCk[seg_ray, seg_slot], gTk[seg_ray, seg_slot])
    assert rel_err(host(drgb), rdc, floor=1e-30) <= TOL_F32
    # d sigma mixes signs: judged against the magnitude of its own positive and negative parts
    mag = oracle.composite_bwd(sigma, rgb, delta, S, np.abs(gCk[seg_ray, seg_slot]), -np.abs(gTk[seg_ray, seg_slot]))[0]
    mag = np.abs(mag) + np.abs(rds)
    assert np.all(np.abs(host(dsigma) - rds) <= 20 * TOL_F32 * np.maximum(mag, np.mean(mag)))


@pytest.mark.parametrize("k_max", [1, 4, 8])
def test_merge_fwd_bwd(k_max):
    rng = np.random.default_rng(k_max)
    R = 5003
    Ck = rng.random((R, k_max, 3), dtype=np.float32)
    Tk = rng.random((R, k_max), dtype=np.float32)
    Tk[rng.random((R, k_max)) < 0.1] = 0.0
    cnt = rng.integers(0, k_max + 1, R).astype(np.int32)
    gC = rng.standard_normal((R, 3)).astype(np.float32)
    gT = rng.standard_normal(R).astype(np.float32)
    C = torch.zeros(R, 3, device=DEV); T = torch.zeros(R, device=DEV)
    B.dg_merge_segments(dev(Ck), dev(Tk), dev(cnt), R, k_max, C, T)
    rC, rT = oracle.merge_fwd(Ck, Tk, cnt)
    assert rel_err(host(C), rC, floor=1e-30) <= TOL_F32 and rel_err(host(T), rT, floor=1e-30) <= TOL_F32
    assert np.all(host(C)[cnt == 0] == 0) and np.all(host(T)[cnt == 0] == 1)
    gCk = torch.full((R, k_max, 3), 7.0, device=DEV); gTk = torch.full((R, k_max), 7.0, device=DEV)
    B.dg_merge_segments_bwd(dev(Ck), dev(Tk), dev(cnt), R, k_max, dev(gC), dev(gT), gCk, gTk)
    rgCk, rgTk = oracle.merge_bwd(Ck, Tk, cnt, gC, gT)
    assert rel_err(host(gCk), rgCk, floor=1e-30) <= TOL_F32
    mag = oracle.merge_bwd(Ck, Tk, cnt, np.abs(gC), np.abs(gT))[1]
    assert np.all(np.abs(host(gTk) - rgTk) <= 4 * TOL_F32 * np.maximum(mag, 1e-30))
    for r in range(0, R, 97):
        assert np.all(host(gCk)[r, cnt[r]:] == 0) and np.all(host(gTk)[r, cnt[r]:] == 0)


def test_loss_seed():
    rng = np.random.default_rng(0)
    R = 4099
    C, Cgt = rng.random((R, 3), dtype=np.float32), rng.random((R, 3), dtype=np.float32)
    T = rng.random(R, dtype=np.float32); T[:50] = 1.0
    for lam in (0.0, 1e-3):
        gC = torch.zeros(R, 3, device=DEV); gT = torch.zeros(R, device=DEV); loss = torch.zeros(1, device=DEV)
        B.dg_loss_seed(dev(C), dev(T), dev(Cgt), R, lam, gC, gT, loss)
        rl, rgC, rgT = oracle.loss(C, T, Cgt, lam)
        assert abs(float(loss.item()) - rl) <= 1e-5 * abs(rl)
        scale = np.mean(np.abs(rgC))
        assert np.all(np.abs(host(gC) - rgC) <= 1e-6 * scale + TOL_F32 * np.abs(rgC))
        assert rel_err(host(gT), rgT, floor=1e-30) <= TOL_F32 if lam else np.all(host(gT) == 0)
