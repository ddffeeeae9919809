"""GPU parity of the field MLPs with appearance features as further colour-net inputs (Sec. 4.4.3) against the oracle's
plain wide network.  Bar: 2e-3 (fp16 operands, atomically accumulated gradients)."""
import sys

import numpy as np
import pytest
import torch

import dg_inputs as di
import oracle
from paper_2405_04416_amd import binding as B

from gpu_util import (DEV, TOL_F16, assert_close_robust, dev, from_planes, have_gpu, host, rel_err, split_appearance_weights,
                      to_planes)

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not have_gpu(), reason="needs a GPU")]


def say(msg):
    print("[case]", msg)
    sys.stdout.flush()


def _case(n_app, n, S, seed):
    cfg = di.config("c8_app")
    m = dict(cfg["mlp"], n_app=n_app)
    n_feat = cfg["grid"]["L"] * cfg["grid"]["F"]
    w = di.make_mlp_weights(n_feat, m, seed=seed)                      # the oracle's packing: one wide first colour layer
    rng = np.random.default_rng(seed + 1)
    feat = rng.standard_normal((n, n_feat)).astype(np.float16)
    rows = -(-n // S)
    dirs = rng.standard_normal((rows, 3)).astype(np.float32)
    sh = oracle.sh(dirs, m["sh_degree"]).astype(np.float16)
    table, image = di.make_appearance(37, n_app, rows, seed=seed)
    wide = np.concatenate([sh, table[image]], axis=1)
    odesc = oracle.mlp_desc(n_feat, m["n_hidden_d"], m["n_geo"], wide.shape[1], m["n_hidden_c"], m["n_layers_c"], 1, 1)
    gdesc = B.dg_mlp_desc(n_feat, m["n_hidden_d"], m["n_geo"], m["sh_degree"] ** 2, m["n_hidden_c"], m["n_layers_c"], 1, n_app)
    return m, n_feat, w, feat, sh, table, image, wide, odesc, gdesc


@pytest.mark.parametrize("n_app,n,S", [(48, 5000, 64), (16, 3001, 64), (48, 777, 7), (16, 1000, 1), (48, 4100, 100)])
def test_mlp_with_appearance_inputs(n_app, n, S):
    say("mlp with %d appearance inputs, n=%d S=%d" % (n_app, n, S))
    m, n_feat, w, feat, sh, table, image, wide, odesc, gdesc = _case(n_app, n, S, seed=21)
    rows = -(-n // S)
    assert B.dg_mlp_weight_count(gdesc) == w.size
    # appearance rows through the library's gather
    app = torch.zeros(rows, n_app, dtype=torch.float16, device=DEV)
    B.dg_appearance_rows(dev(table), dev(image.view(np.int32)), None, rows, app)
    np.testing.assert_array_equal(host(app), table[image])
    idx = np.random.default_rng(1).integers(0, rows, 50).astype(np.int32)
    app2 = torch.zeros(50, n_app, dtype=torch.float16, device=DEV)
    B.dg_appearance_rows(dev(table), dev(image.view(np.int32)), dev(idx), 50, app2)
    np.testing.assert_array_equal(host(app2), table[image[idx]])
    # forward
    wg = split_appearance_weights(w, n_feat, m)
    sigma, rgb = torch.zeros(n, device=DEV), torch.zeros(n, 3, device=DEV)
    B.dg_mlp_fwd_app(gdesc, dev(wg), dev(to_planes(feat)), dev(sh), app, S, n, sigma, rgb)
    rs, rr = oracle.mlp_fwd(odesc, w.astype(np.float64), feat.astype(np.float64), wide.astype(np.float64), S)
    assert rel_err(host(sigma), rs) <= TOL_F16
    assert rel_err(host(rgb), rr) <= TOL_F16
    # the appearance inputs matter
    rs0, rr0 = oracle.mlp_fwd(odesc, w.astype(np.float64), feat.astype(np.float64),
                              np.concatenate([sh, np.zeros_like(table[image])], 1).astype(np.float64), S)
    assert np.abs(rr0 - rr).max() > 0.01
    # backward
    rng = np.random.default_rng(13)
    dsigma = (rng.standard_normal(n) * 1e-6).astype(np.float32)
    drgb = (rng.standard_normal((n, 3)) * 1e-6).astype(np.float32)
    scale = 2.0 ** 18
    dfeat = torch.zeros(n, n_feat, device=DEV)
    dW = torch.zeros(w.size, device=DEV)
    ws = torch.zeros(B.dg_mlp_bwd_app_workspace_bytes(gdesc, n, S) // 4 + 64, device=DEV)
    for _ in range(2):                                                     # the second call must not see the first one's row sums
        dW.zero_()
        B.dg_mlp_bwd_app(gdesc, dev(wg), dev(to_planes(feat)), dev(sh), app, S, n, dev(dsigma), dev(drgb), scale, dfeat, dW, ws)
    rdf, rdw = oracle.mlp_bwd(odesc, w.astype(np.float64), feat.astype(np.float64), wide.astype(np.float64), S,
                              dsigma.astype(np.float64), drgb.astype(np.float64), scale)
    assert_close_robust(from_planes(dfeat, n, n_feat), rdf, TOL_F16, "dfeat")     # a delta on an fp16 rounding boundary may flip
    got = host(dW).astype(np.float64)
    ref = split_appearance_weights(rdw, n_feat, m)
    pos = 0
    shapes = di.mlp_layer_shapes(n_feat, dict(m, n_app=0)) + [(m["n_hidden_c"], n_app)]
    for (no, ni) in shapes:                                                # judged matrix by matrix; the last one is Wapp
        assert rel_err(got[pos:pos + no * ni], ref[pos:pos + no * ni]) <= TOL_F16, (no, ni)
        pos += no * ni
    assert pos == w.size


def test_entry_points_without_appearance_are_unchanged():
    say("dg_mlp_fwd_app with n_app = 0 equals dg_mlp_fwd")
    cfg = di.config("c2_ngp")
    m = cfg["mlp"]
    n, S, n_feat = 3000, 64, 32
    w = di.make_mlp_weights(n_feat, m, seed=3)
    rng = np.random.default_rng(4)
    feat = rng.standard_normal((n, n_feat)).astype(np.float16)
    sh = oracle.sh(rng.standard_normal((-(-n // S), 3)).astype(np.float32), 4).astype(np.float16)
    desc = B.dg_mlp_desc(n_feat, 64, 16, 16, 64, 2, 1)
    out = []
    for call in (lambda s, r: B.dg_mlp_fwd(desc, dev(w), dev(to_planes(feat)), dev(sh), S, n, s, r),
                 lambda s, r: B.dg_mlp_fwd_app(desc, dev(w), dev(to_planes(feat)), dev(sh), None, S, n, s, r)):
        s, r = torch.zeros(n, device=DEV), torch.zeros(n, 3, device=DEV)
        call(s, r)
        out.append((host(s), host(r)))
    np.testing.assert_array_equal(out[0][0], out[1][0])
    np.testing.assert_array_equal(out[0][1], out[1][1])
    with pytest.raises(B.DistGridError):
        B.dg_mlp_fwd(B.dg_mlp_desc(n_feat, 64, 16, 16, 64, 2, 1, 48), dev(w), dev(to_planes(feat)), dev(sh), S, n, s, r)
    with pytest.raises(B.DistGridError):
        B.dg_mlp_fwd_app(B.dg_mlp_desc(n_feat, 64, 16, 16, 64, 2, 1, 32), dev(w), dev(to_planes(feat)), dev(sh),
                         torch.zeros(-(-n // S), 32, dtype=torch.float16, device=DEV), S, n, s, r)      # 32 is not a supported width
