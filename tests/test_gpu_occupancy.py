"""GPU parity of the occupancy grid and of occupancy-guided sampling against the CPU oracle.

Bar: bit-exact for cells, candidate points, densities after decay / maximum, bits, sample offsets, sample
coordinates, widths, distances and ray indices (fp32 bookkeeping with one rounding per operation on both sides);
relative error <= 1e-5 for the fp32 compositing of segments of different lengths.
"""
import sys

import numpy as np
import pytest
import torch

import dg_inputs as di
import oracle
from paper_2405_04416_amd import binding as B

from gpu_util import DEV, TOL_F32, dev, have_gpu, host, rel_err

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not have_gpu(), reason="needs a GPU")]

i32 = torch.int32


def say(msg):
    print("[case]", msg)
    sys.stdout.flush()


def _bits_dev(bits):
    return dev(bits.view(np.int32))


@pytest.mark.parametrize("N,ext", [(12, (1.0, 0.8, 0.3)), (40, (2.0, 2.0, 0.25)), (7, (0.3, 0.9, 0.9))])
def test_candidates_bit_exact(N, ext):
    say("occ candidates N=%d" % N)
    g_ref, g = oracle.occ_init(N, ext), B.dg_occ_desc_init(N, ext)
    n = g.n_cells
    rng = np.random.default_rng(N)
    occupied = rng.random(n) < 0.3
    bits = np.packbits(np.concatenate([occupied, np.zeros(-n % 32, bool)]), bitorder="little").view(np.uint32)
    for warmup, M, n_uniform, tries, it in [(True, n, 0, 32, 16), (False, 5001, 2500, 32, 4112), (False, 777, 0, 3, 9999),
                                            (False, 300, 300, 1, 20000)]:
        cell, u = torch.zeros(M, dtype=i32, device=DEV), torch.zeros(M, 3, device=DEV)
        B.dg_occ_candidates(g, _bits_dev(bits), M, n_uniform, warmup, 77, it, tries, cell, u)
        rc, ru = oracle.occ_candidates(g_ref, bits, M, n_uniform, warmup, 77, it, tries)
        np.testing.assert_array_equal(host(cell).view(np.uint32), rc)
        np.testing.assert_array_equal(host(u), ru)
        i0, m = M // 3, M - M // 3 - 1                                       # a piece of the same refresh
        B.dg_occ_candidates(g, _bits_dev(bits), m, n_uniform, warmup, 77, it, tries, cell, u, i0=i0)
        np.testing.assert_array_equal(host(cell).view(np.uint32)[:m], rc[i0:i0 + m])
        np.testing.assert_array_equal(host(u)[:m], ru[i0:i0 + m])


@pytest.mark.parametrize("n", [1, 63, 64, 1000, 100003])
def test_decay_update_bits_bit_exact(n):
    say("occ refresh n=%d" % n)
    rng = np.random.default_rng(n)
    dens_h = (rng.random(n) * 100).astype(np.float32)
    dens_h[rng.random(n) < 0.2] = 0.0
    dens = dev(dens_h)
    ref = dens_h.copy()
    for _ in range(3):
        B.dg_occ_decay(dens, 0.99)
        oracle.occ_decay(ref, np.float32(0.99))
    np.testing.assert_array_equal(host(dens), ref)
    M = 5 * n + 3
    cell = rng.integers(0, n, M).astype(np.uint32)
    sigma = (rng.random(M) * 150).astype(np.float32)
    sigma[rng.random(M) < 0.1] = 0.0
    B.dg_occ_update(dens, dev(cell.view(np.int32)), dev(sigma), M)
    oracle.occ_update(ref, cell, sigma)
    np.testing.assert_array_equal(host(dens), ref)
    for thr in (0.6, 60.0):
        bits = torch.full(((n + 31) // 32,), -1, dtype=i32, device=DEV)
        n_set = torch.zeros(1, dtype=i32, device=DEV)
        B.dg_occ_bits(dens, thr, bits, n_set)
        rb, rn = oracle.occ_bits(ref, thr)
        np.testing.assert_array_equal(host(bits).view(np.uint32), rb)
        assert int(host(n_set)[0]) == rn


def _segments(cfg, R, seed):
    o, d = di.make_rays(cfg, seed=seed, R=R)
    k_max = cfg["k_max"]
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, k_max, holes=cfg.get("holes"))
    off, seg_ray, seg_slot = oracle.bucket_segments(cnt, part, cfg["parts"].shape[0])
    return o, d, seg_t, off, seg_ray, seg_slot


def _march_gpu(o, d, seg_t, seg_ray, seg_slot, begin, end, box, g, bits, dt, max_steps, seed, capacity):
    n_seg = end - begin
    k_max = seg_t.shape[1]
    first = torch.full((n_seg + 1,), -1, dtype=i32, device=DEV)
    u, delta, t = torch.zeros(max(capacity, 1), 3, device=DEV), torch.zeros(max(capacity, 1), device=DEV), torch.zeros(max(capacity, 1), device=DEV)
    ray = torch.zeros(max(capacity, 1), dtype=i32, device=DEV)
    status = torch.zeros(1, dtype=i32, device=DEV)
    ws = torch.zeros(B.dg_march_workspace_bytes(n_seg) // 4, dtype=i32, device=DEV)
    sr = dev(seg_ray.view(np.int32))[begin:] if seg_ray.size > begin else torch.zeros(1, dtype=i32, device=DEV)
    ss = dev(seg_slot.view(np.int32))[begin:] if seg_slot.size > begin else torch.zeros(1, dtype=i32, device=DEV)
    B.dg_march_segments(dev(o), dev(d), dev(seg_t), sr, ss, n_seg, k_max, box, g, _bits_dev(bits), float(dt), max_steps, seed,
                        capacity, first, u, delta, t, ray, status, ws)
    torch.cuda.synchronize()
    return host(first).view(np.uint32), host(u), host(delta), host(t), host(ray).view(np.uint32), int(host(status)[0])


@pytest.mark.parametrize("name,R,N,max_steps,fill", [("c2_ngp", 3000, 64, 4096, "scene"), ("c2_ngp", 700, 512, 4096, "scene"),
                                                      ("c3_2x2", 2001, 48, 4096, "scene"), ("c2_ngp", 500, 64, 4096, "full"),
                                                      ("c2_ngp", 500, 64, 4096, "empty"), ("c2_ngp", 900, 64, 37, "scene"),
                                                      ("c6_cascade", 1500, 32, 4096, "scene")])
def test_march_bit_exact(name, R, N, max_steps, fill):
    say("march %s R=%d N=%d max_steps=%d %s" % (name, R, N, max_steps, fill))
    cfg = di.config(name)
    o, d, seg_t, off, seg_ray, seg_slot = _segments(cfg, R, seed=5)
    for p in range(cfg["parts"].shape[0]):
        box = cfg["parts"][p]
        ext = di.box_extent(box)
        g_ref, g = oracle.occ_init(N, ext), B.dg_occ_desc_init(N, ext)
        if fill == "scene":
            bits, _ = oracle.occ_bits(di.make_cell_densities(list(g_ref.shape), seed=p), 0.6)
        else:
            bits = np.full((g_ref.n_cells + 31) // 32, 0xFFFFFFFF if fill == "full" else 0, np.uint32)
        dt = np.float32(float(ext.max()) * np.sqrt(3.0) / 1024)
        begin, end = int(off[p]), int(off[p + 1])
        rf, ru, rd, rt, rr = oracle.march_segments(o, d, seg_t, seg_ray, seg_slot, begin, end, box, g_ref, bits, dt, max_steps, seed=21)
        n = int(rf[-1])
        first, u, delta, t, ray, status = _march_gpu(o, d, seg_t, seg_ray, seg_slot, begin, end, box, g, bits, dt, max_steps, 21, n + 5)
        assert status == 0
        np.testing.assert_array_equal(first, rf)
        np.testing.assert_array_equal(u[:n], ru)
        np.testing.assert_array_equal(delta[:n], rd)
        np.testing.assert_array_equal(t[:n], rt)
        np.testing.assert_array_equal(ray[:n], rr)
        if fill == "scene" and p == 0 and n > 10:
            # too little room: what fits is written, the rest is dropped and reported, offsets stay whole
            cap = n // 2
            first, u, delta, t, ray, status = _march_gpu(o, d, seg_t, seg_ray, seg_slot, begin, end, box, g, bits, dt, max_steps, 21, cap)
            assert status == 2
            np.testing.assert_array_equal(first, rf)
            np.testing.assert_array_equal(u[:cap], ru[:cap])
            np.testing.assert_array_equal(ray[:cap], rr[:cap])


def test_march_of_no_segments():
    say("march n_seg=0")
    cfg = di.config("c2_ngp")
    box = cfg["parts"][0]
    g = B.dg_occ_desc_init(16, di.box_extent(box))
    bits = np.zeros((g.n_cells + 31) // 32, np.uint32)
    o, d = di.make_rays(cfg, seed=1, R=4)
    first, *_ , status = _march_gpu(o, d, np.zeros((4, 1, 2), np.float32), np.zeros(0, np.uint32), np.zeros(0, np.uint32), 0, 0, box, g,
                                    bits, 0.01, 100, 0, 0)
    assert list(first) == [0] and status == 0


@pytest.mark.parametrize("n_seg,k_max,longest", [(501, 4, 150), (77, 1, 64), (33, 3, 400), (1000, 12, 9)])
def test_ragged_composite(n_seg, k_max, longest):
    say("ragged composite n_seg=%d k_max=%d longest=%d" % (n_seg, k_max, longest))
    rng = np.random.default_rng(n_seg)
    counts = rng.integers(0, longest + 1, n_seg)
    counts[rng.random(n_seg) < 0.15] = 0                                     # segments that see nothing
    counts[0] = longest
    first = np.concatenate([[0], np.cumsum(counts)]).astype(np.uint32)
    n = int(first[-1])
    R = n_seg
    pairs = rng.permutation(R * k_max)[:n_seg]
    ray, slot = (pairs // k_max).astype(np.int32), (pairs % k_max).astype(np.int32)
    sigma = (rng.random(n) * 40.0).astype(np.float32)
    sigma[rng.random(n) < 0.3] = 0.0
    delta = (rng.random(n) * 0.05).astype(np.float32)
    rgb = rng.random((n, 3)).astype(np.float32)
    t = (rng.random(n) * 6.0).astype(np.float32)
    args = (n_seg, dev(first.view(np.int32)), dev(ray), dev(slot), k_max)
    Ck, Tk, Dk = torch.full((R, k_max, 3), -1.0, device=DEV), torch.full((R, k_max), -1.0, device=DEV), torch.full((R, k_max), -1.0, device=DEV)
    B.dg_composite_ragged_fwd(dev(sigma), dev(rgb), dev(delta), *args, Ck, Tk)
    B.dg_composite_ragged_depth(dev(sigma), dev(delta), dev(t), *args, Dk)
    rC, rT = oracle.composite_fwd_ragged(sigma, rgb, delta, first)
    rD = oracle.composite_depth_ragged(sigma, delta, t, first)
    assert rel_err(host(Ck)[ray, slot], rC) <= TOL_F32
    assert np.all(np.abs(host(Tk)[ray, slot] - rT) <= TOL_F32 * np.maximum(rT, 1e-3))
    assert np.all(np.abs(host(Dk)[ray, slot] - rD) <= TOL_F32 * np.maximum(np.abs(rD), 1e-3))
    empty = counts == 0
    assert np.all(host(Ck)[ray, slot][empty] == 0) and np.all(host(Tk)[ray, slot][empty] == 1) and np.all(host(Dk)[ray, slot][empty] == 0)
    untouched = np.ones((R, k_max), bool)
    untouched[ray, slot] = False
    assert np.all(host(Tk)[untouched] == -1.0)
    # backward
    gCk, gTk = rng.standard_normal((R, k_max, 3)).astype(np.float32), rng.standard_normal((R, k_max)).astype(np.float32)
    dsigma, drgb = torch.zeros(max(n, 1), device=DEV), torch.zeros(max(n, 1), 3, device=DEV)
    B.dg_composite_ragged_bwd(dev(sigma), dev(rgb), dev(delta), *args, dev(gCk), dev(gTk), dsigma, drgb)
    rs, rc = oracle.composite_bwd_ragged(sigma, rgb, delta, first, gCk[ray, slot], gTk[ray, slot])
    assert rel_err(host(drgb)[:n], rc, floor=1e-30) <= TOL_F32
    # d sigma mixes signs: judged against the magnitude of its own positive and negative parts
    mag = oracle.composite_bwd_ragged(sigma, rgb, delta, first, np.abs(gCk[ray, slot]), -np.abs(gTk[ray, slot]))[0]
    mag = np.abs(mag) + np.abs(rs)
    assert np.all(np.abs(host(dsigma)[:n] - rs) <= 20 * TOL_F32 * np.maximum(mag, np.mean(mag)))
