"""GPU parity of the whole forward + backward pass with occupancy-guided sampling (Sec. 3.2, Sec. 5.1), and of the
occupancy refresh, against the oracle.  Sample bookkeeping is bit-exact; values follow the bars of the fixed-sample
step (fp16 MLP, atomically accumulated gradients: 2e-3)."""
import sys

import numpy as np
import pytest
import torch

import dg_inputs as di
import oracle
import oracle.step as ostep

from gpu_util import (DEV, TOL_F16, TOL_F32, assert_close_robust, dev, from_planes, gpu_models, gpu_occupancy, have_gpu, host,
                      make_step, rel_err, split_appearance_weights)

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not have_gpu(), reason="needs a GPU")]


def say(msg):
    print("[case]", msg)
    sys.stdout.flush()


def _compare(cfg, R, seed, lambda1, loss_scale, table_gain, max_samples):
    cfg = dict(cfg)
    cfg["table_range"] = cfg["table_range"] * table_gain
    o, d = di.make_rays(cfg, seed=seed, R=R)
    Cgt = di.make_targets(R, seed=seed)
    hm = ostep.make_models(cfg, seed=seed)
    ho = ostep.make_occupancy(cfg, seed=seed)
    gm = gpu_models(cfg, hm)
    app_h = app_d = None
    if cfg["mlp"].get("n_app"):
        table, image = di.make_appearance(cfg["n_images"], cfg["mlp"]["n_app"], R, seed=seed)
        app_h, app_d = (table, image), (dev(table), dev(image.view(np.int32)))
    step = make_step(cfg, gm, R, loss_scale=loss_scale, lambda1=lambda1, seed=seed, occupancy=gpu_occupancy(cfg, ho),
                     max_samples=max_samples, appearance=app_d)
    step.step(dev(o), dev(d), dev(Cgt))
    D = step.depth()
    torch.cuda.synchronize()
    ref = ostep.run_step(cfg, hm, o, d, Cgt, seed=seed, lambda1=lambda1, loss_scale=loss_scale, occ=ho, appearance=app_h)
    assert int(host(step.status)[0]) == 0
    np.testing.assert_array_equal(host(step.seg_count), ref["seg_count"])
    np.testing.assert_array_equal(host(step.part_offset), ref["part_offset"])
    for p, q in ref["per"].items():
        b, e = q["b"], q["e"]
        s0, N = step.samples[p]
        assert N == q["u"].shape[0]
        np.testing.assert_array_equal(host(step.first[b + p:e + p + 1]).view(np.uint32), q["first"])
        sl = slice(s0, s0 + N)
        np.testing.assert_array_equal(host(step.u[sl]).view(np.uint32), q["u"].view(np.uint32))
        np.testing.assert_array_equal(host(step.delta[sl]).view(np.uint32), q["delta"].view(np.uint32))
        assert rel_err(from_planes(step.feat[sl], N, q["feat"].shape[1]).astype(np.float64), q["feat"]) <= 1e-3
        assert_close_robust(host(step.sigma[sl]), q["sigma"], TOL_F16, "sigma")
        assert_close_robust(host(step.rgb[sl]), q["rgb"], TOL_F16, "rgb")
    cnt = ref["seg_count"]
    used = np.arange(cfg["k_max"])[None, :] < cnt[:, None]
    assert rel_err(host(step.Ck)[used], ref["Ck"][used]) <= TOL_F16
    assert rel_err(host(step.Tk)[used], ref["Tk"][used]) <= TOL_F16
    assert rel_err(host(step.C), ref["C"]) <= TOL_F16
    assert rel_err(host(step.T), ref["T"]) <= TOL_F16
    assert abs(float(step.loss.item()) - ref["loss"]) <= TOL_F16 * abs(ref["loss"])
    assert rel_err(host(step.gCk)[used], ref["gCk"][used]) <= TOL_F16
    for p, q in ref["per"].items():
        s0, N = step.samples[p]
        sl = slice(s0, s0 + N)
        assert_close_robust(host(step.dsigma[sl]), q["dsigma"], TOL_F16, "dsigma")
        assert_close_robust(host(step.drgb[sl]), q["drgb"], TOL_F16, "drgb")
        assert_close_robust(from_planes(step.dfeat[sl], N, q["dfeat"].shape[1]), q["dfeat"], TOL_F16, "dfeat")
        assert_close_robust(host(gm[p].dW), split_appearance_weights(q["dW"], q["feat"].shape[1], cfg["mlp"]), TOL_F16, "dW")
        grid = hm[p]["grid"]
        got = host(gm[p].dtable).astype(np.float64)
        for l in range(grid.L):
            s2 = slice(grid.first[l], grid.first[l + 1])
            assert_close_robust(got[s2], q["dtable"][s2], TOL_F16, "dtable level %d of part %d" % (l, p), min_outliers=32)
    # depth of the same samples: merged expected distance (Sec. 4.4.2)
    Dk = np.zeros((R, cfg["k_max"]))
    for p, q in ref["per"].items():
        b, e = q["b"], q["e"]
        first, u, delta, t, ray = oracle.march_segments(o, d, ref["seg_t"], ref["seg_ray"], ref["seg_slot"], b, e, cfg["parts"][p],
                                                        ho[p]["grid"], ho[p]["bits"], ho[p]["dt"], ho[p]["max_steps"], seed=seed)
        Dk[ref["seg_ray"][b:e], ref["seg_slot"][b:e]] = oracle.composite_depth_ragged(q["sigma"], delta, t, first)
    refD = oracle.merge_depth(Dk, ref["Tk"], cnt)
    assert rel_err(host(D), refD) <= TOL_F16
    return step, ref


def test_step_occupancy_single_box():
    say("step c7_occ: 1200 rays, occupancy grid of resolution 64, marching step of Instant-NGP")
    cfg = di.config("c7_occ")
    cfg["occ"] = dict(cfg["occ"], res=64)
    step, ref = _compare(cfg, 1200, seed=1, lambda1=1e-3, loss_scale=2.0 ** 14, table_gain=3000.0, max_samples=60000)
    counts = np.diff(ref["per"][0]["first"].astype(np.int64))
    assert counts.max() > 10 and np.any(counts == 0) and 3 < counts.mean() < 60


def test_step_occupancy_four_boxes():
    say("step c3_2x2 with occupancy grids of resolution 48, 900 rays, T = 2^16")
    cfg = di.config("c3_2x2")
    cfg["grid"] = dict(cfg["grid"], log2_T=16)
    cfg["occ"] = dict(res=48, max_steps=512)
    step, ref = _compare(cfg, 900, seed=2, lambda1=1e-3, loss_scale=2.0 ** 14, table_gain=3000.0, max_samples=200000)
    assert len(ref["per"]) == 4


def test_step_occupancy_with_appearance_features():
    say("step c8_app with an occupancy grid of resolution 64: one appearance row per sample, 16 appearance inputs")
    cfg = di.config("c8_app")
    cfg["mlp"] = dict(cfg["mlp"], n_app=16)
    cfg["occ"] = dict(res=64, max_steps=1024)
    _compare(cfg, 1000, seed=4, lambda1=1e-3, loss_scale=2.0 ** 14, table_gain=3000.0, max_samples=60000)


def test_sample_capacity_is_enforced():
    say("step c7_occ: too little room for the samples raises")
    cfg = di.config("c7_occ")
    cfg["occ"] = dict(cfg["occ"], res=64)
    R = 500
    o, d = di.make_rays(cfg, seed=1, R=R)
    hm = ostep.make_models(cfg, seed=1)
    ho = ostep.make_occupancy(cfg, seed=1)
    step = make_step(cfg, gpu_models(cfg, hm), R, occupancy=gpu_occupancy(cfg, ho), max_samples=100)
    from paper_2405_04416_amd.binding import DistGridError
    with pytest.raises(DistGridError):
        step.forward(dev(o), dev(d), dev(di.make_targets(R, seed=1)))
    torch.cuda.synchronize()
    assert int(host(step.status)[0]) == 2


@pytest.mark.parametrize("iteration", [0, 16, 4112, 10000, 7])
def test_occupancy_refresh(iteration):
    say("occupancy refresh at iteration %d" % iteration)
    cfg = di.config("c7_occ")
    cfg["occ"] = dict(cfg["occ"], res=40)
    cfg["table_range"] = 5.0                                        # the field's densities spread over 0.2 .. 20
    hm = ostep.make_models(cfg, seed=3)
    ho = ostep.make_occupancy(cfg, seed=3)
    for q in ho.values():                                          # stand-in densities on the scale of this field's
        q["density"] = (q["density"] * 0.02).astype(np.float32)
    step = make_step(cfg, gpu_models(cfg, hm), 64, occupancy=gpu_occupancy(cfg, ho), max_samples=3000)   # several pieces
    before = host(step.occ[0].density).copy()
    did = step.refresh_occupancy(iteration)
    torch.cuda.synchronize()
    assert did == ostep.refresh_occupancy(hm, ho, iteration, seed=0)
    assert did == (iteration % 16 == 0)
    if not did:
        np.testing.assert_array_equal(host(step.occ[0].density), before)
        return
    q = ho[0]
    got = host(step.occ[0].density)
    assert_close_robust(got, q["density"], TOL_F16, "density")
    thr = oracle.occ_schedule(iteration)[3]
    clear = np.abs(q["density"] - thr) > 4 * TOL_F16 * thr          # cells whose bit the fp16 field cannot flip
    gb = np.unpackbits(host(step.occ[0].bits).view(np.uint8), bitorder="little")[:got.size].astype(bool)
    rb = np.unpackbits(q["bits"].view(np.uint8), bitorder="little")[:got.size].astype(bool)
    np.testing.assert_array_equal(gb[clear], rb[clear])
    np.testing.assert_array_equal(gb, got > np.float32(thr))        # the bits belong to the library's own densities
    assert int(host(step.occ[0].n_set)[0]) == int(gb.sum())
    assert 0 < q["last_sigma"].min() and np.unique(q["last_cell"]).size > 0.3 * q["last_cell"].size
