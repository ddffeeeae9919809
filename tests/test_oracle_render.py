"""Pins for the oracle's MLPs, segment compositing, merge and loss (CPU only).

Sources: DistGrid Eq. 3 (segment rendering; closed form for a homogeneous
medium), Eq. 4-6 (merge; splitting a ray into K segments and merging must equal
unsegmented rendering), Eq. 7-8 (merge backward, checked by finite
differences), Eq. 9-10 (losses), Sec. 5.1 (sigmoid hidden activation in the
colour net, outputs clipped to [-15, 15] before the output activations);
numpy's float16 and matmul as library references for the fp16 rounding points.
"""
import numpy as np
import pytest

import dg_inputs as di
import oracle


# ------------------------------------------------------------------ fp16 rounding
def test_round_f16_matches_numpy_float16():
    rng = np.random.default_rng(0)
    xs = np.concatenate([
        rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 5, 4000),
        [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
         2.0 ** -14, 2.0 ** -14 - 2.0 ** -26, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 1e-9,
         0.1, 1 / 3, 2049.0, 2051.0]])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).astype(np.float64)
    got = np.array([oracle.round_f16(x) for x in xs])
    np.testing.assert_array_equal(got, ref)


# ------------------------------------------------------------------ MLPs
def _mlp_case(name, n, seed, S=4, round_f16=1, gain=1.0):
    cfg = di.config(name)
    m = cfg["mlp"]
    n_feat = cfg["grid"]["L"] * cfg["grid"]["F"]
    n_dir = m["sh_degree"] ** 2 + m.get("n_app", 0)       # appearance features (Sec. 4.4.3) follow the direction encoding
    desc = oracle.mlp_desc(n_feat, m["n_hidden_d"], m["n_geo"], n_dir, m["n_hidden_c"], m["n_layers_c"], 1, round_f16)
    w = di.make_mlp_weights(n_feat, m, seed=seed, gain=gain).astype(np.float64)
    rng = np.random.default_rng(seed + 100)
    feat = rng.standard_normal((n, n_feat)).astype(np.float16).astype(np.float64)
    dirs = rng.standard_normal((-(-n // S), 3)).astype(np.float32)
    dir_enc = oracle.sh(dirs, m["sh_degree"])
    if m.get("n_app"):
        table, image = di.make_appearance(7, m["n_app"], dirs.shape[0], seed=seed)
        dir_enc = np.concatenate([dir_enc, table[image].astype(np.float64)], axis=1)
    return cfg, desc, w, feat, dir_enc, S


def _numpy_mlp(cfg, w, feat, dir_enc, S, half):
    """Same network from numpy matmuls; `half` rounds through numpy's float16 at the stated points."""
    m = cfg["mlp"]
    n_feat = feat.shape[1]
    r = (lambda a: a.astype(np.float16).astype(np.float64)) if half else (lambda a: a)
    mats, pos = [], 0
    for (no, ni) in di.mlp_layer_shapes(n_feat, m):
        mats.append(w[pos:pos + no * ni].reshape(no, ni)); pos += no * ni
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    h1 = r(np.maximum(r(feat) @ mats[0].T, 0.0))
    geo = h1 @ mats[1].T
    sigma = np.exp(np.clip(geo[:, 0], -15, 15))
    xc = np.concatenate([r(geo), r(np.repeat(dir_enc, S, axis=0)[:feat.shape[0]])], axis=1)
    c = r(sig(xc @ mats[2].T))
    if m["n_layers_c"] == 2:
        c = r(sig(c @ mats[3].T))
    rgb = sig(np.clip(c @ mats[-1].T, -15, 15))
    return sigma, rgb


@pytest.mark.parametrize("name", ["c1_tiny", "c2_ngp", "c8_app"])
@pytest.mark.parametrize("half", [0, 1])
def test_mlp_fwd_against_numpy(name, half):
    cfg, desc, w, feat, dir_enc, S = _mlp_case(name, 300, seed=1, round_f16=half)
    sigma, rgb = oracle.mlp_fwd(desc, w, feat, dir_enc, S)
    ref_sigma, ref_rgb = _numpy_mlp(cfg, w, feat, dir_enc, S, half)
    # summation order differs (BLAS vs plain loop); a rounding flip at an fp16 point is possible but rare
    bad = np.abs(sigma - ref_sigma) > 1e-9 * np.abs(ref_sigma)
    assert bad.mean() <= (0.02 if half else 0.0)
    np.testing.assert_allclose(sigma, ref_sigma, rtol=5e-3 if half else 1e-12)
    np.testing.assert_allclose(rgb, ref_rgb, atol=2e-3 if half else 1e-12)


def test_mlp_output_clip():
    # large weights push raw outputs beyond +-15: sigma saturates at exp(+-15), gradients vanish there
    cfg, desc, w, feat, dir_enc, S = _mlp_case("c1_tiny", 200, seed=2, round_f16=0, gain=40.0)
    sigma, rgb = oracle.mlp_fwd(desc, w, feat, dir_enc, S)
    assert sigma.max() == np.exp(15.0) and sigma.min() >= np.exp(-15.0)
    assert rgb.max() <= 1 / (1 + np.exp(-15.0)) and rgb.min() >= 1 / (1 + np.exp(15.0))
    sat = sigma == np.exp(15.0)
    assert sat.any()
    dsig = np.ones(200); drgb = np.zeros((200, 3))
    dfeat, dw = oracle.mlp_bwd(desc, w, feat, dir_enc, S, dsig * sat, drgb)
    assert np.all(dfeat == 0) and np.all(dw == 0)


def test_appearance_inputs_with_zero_weights_change_nothing():
    # Sec. 4.4.3: appearance features are further inputs of the colour net; with their weight columns at zero the
    # network is the one without them, and the density never depends on them
    cfg, desc, w, feat, dir_enc, S = _mlp_case("c8_app", 100, seed=9)
    m = cfg["mlp"]
    shapes = di.mlp_layer_shapes(feat.shape[1], m)
    pos = sum(no * ni for no, ni in shapes[:2])
    no, ni = shapes[2]
    Wc1 = w[pos:pos + no * ni].reshape(no, ni).copy()
    n_narrow = ni - m["n_app"]
    sigma_full, rgb_full = oracle.mlp_fwd(desc, w, feat, dir_enc, S)
    Wc1[:, n_narrow:] = 0.0
    w0 = w.copy(); w0[pos:pos + no * ni] = Wc1.ravel()
    sigma0, rgb0 = oracle.mlp_fwd(desc, w0, feat, dir_enc, S)
    narrow = oracle.mlp_desc(desc.n_feat, desc.n_hidden_d, desc.n_geo, n_narrow - desc.n_geo, desc.n_hidden_c, desc.n_layers_c, 1, 1)
    w_narrow = np.concatenate([w[:pos], Wc1[:, :n_narrow].ravel(), w[pos + no * ni:]])
    sigma_n, rgb_n = oracle.mlp_fwd(narrow, w_narrow, feat, dir_enc[:, :n_narrow - desc.n_geo], S)
    np.testing.assert_array_equal(sigma0, sigma_n)
    np.testing.assert_array_equal(rgb0, rgb_n)
    np.testing.assert_array_equal(sigma_full, sigma_n)
    assert np.abs(rgb_full - rgb_n).max() > 1e-3
    # and their weight columns receive gradient, the others' gradient is that of the narrow net when they are zero
    gs, gr = np.zeros(100), np.ones((100, 3))
    _, dw0 = oracle.mlp_bwd(desc, w0, feat, dir_enc, S, gs, gr)
    _, dwn = oracle.mlp_bwd(narrow, w_narrow, feat, dir_enc[:, :n_narrow - desc.n_geo], S, gs, gr)
    g = dw0[pos:pos + no * ni].reshape(no, ni)
    np.testing.assert_allclose(g[:, :n_narrow].ravel(), dwn[pos:pos + no * n_narrow], rtol=1e-12, atol=1e-18)
    assert np.abs(g[:, n_narrow:]).max() > 0


@pytest.mark.parametrize("name", ["c1_tiny", "c2_ngp", "c8_app"])
def test_mlp_bwd_finite_differences(name):
    cfg, desc, w, feat, dir_enc, S = _mlp_case(name, 24, seed=3, round_f16=0)
    rng = np.random.default_rng(5)
    gs, gr = rng.standard_normal(24), rng.standard_normal((24, 3))

    def objective(w_, feat_):
        s, c = oracle.mlp_fwd(desc, w_, feat_, dir_enc, S)
        return np.sum(gs * s) + np.sum(gr * c)

    dfeat, dw = oracle.mlp_bwd(desc, w, feat, dir_enc, S, gs, gr)
    dfeat2, dw2 = oracle.mlp_bwd(desc, w, feat, dir_enc, S, gs, gr, loss_scale=1024.0)
    np.testing.assert_allclose(dfeat2, dfeat, rtol=1e-12, atol=1e-14)     # loss scale cancels exactly
    np.testing.assert_allclose(dw2, dw, rtol=1e-12, atol=1e-14)
    eps = 1e-6
    for k in rng.choice(w.size, 40, replace=False):
        wp, wm = w.copy(), w.copy(); wp[k] += eps; wm[k] -= eps
        fd = (objective(wp, feat) - objective(wm, feat)) / (2 * eps)
        assert abs(fd - dw[k]) <= 1e-6 * max(1.0, abs(fd)), (k, fd, dw[k])
    for _ in range(40):
        i, k = rng.integers(24), rng.integers(feat.shape[1])
        fp, fm = feat.copy(), feat.copy(); fp[i, k] += eps; fm[i, k] -= eps
        fd = (objective(w, fp) - objective(w, fm)) / (2 * eps)
        assert abs(fd - dfeat[i, k]) <= 1e-6 * max(1.0, abs(fd))


def test_mlp_bwd_rounded_stays_close_to_exact():
    cfg, desc, w, feat, dir_enc, S = _mlp_case("c2_ngp", 256, seed=4, round_f16=1)
    exact = oracle.mlp_desc(*[getattr(desc, f) for f, _ in desc._fields_][:7], 0)
    rng = np.random.default_rng(6)
    gs, gr = rng.standard_normal(256) * 1e-8, rng.standard_normal((256, 3)) * 1e-8    # loss-mean sized seeds
    dfe, dwe = oracle.mlp_bwd(exact, w, feat, dir_enc, S, gs, gr)
    dfr, dwr = oracle.mlp_bwd(desc, w, feat, dir_enc, S, gs, gr, loss_scale=2.0 ** 22)
    assert np.abs(dfr - dfe).max() <= 0.02 * np.abs(dfe).max()
    assert np.abs(dwr - dwe).max() <= 0.02 * np.abs(dwe).max()
    # without loss scaling the fp16 deltas underflow and the gradient collapses
    dfu, _ = oracle.mlp_bwd(desc, w, feat, dir_enc, S, gs, gr, loss_scale=1.0)
    assert np.abs(dfu - dfe).max() > 0.1 * np.abs(dfe).max()


# ------------------------------------------------------------------ composite
def test_composite_homogeneous_closed_form():
    # constant sigma and colour on [t_in, t_out]: T = exp(-sigma*len), C = c (1 - T), for any sample count
    for S in (1, 7, 64):
        for sig, length in ((0.0, 1.0), (0.3, 2.0), (5.0, 0.7), (200.0, 1.0)):
            rng = np.random.default_rng(S)
            widths = rng.random(S) + 0.1
            widths *= length / widths.sum()
            c = np.array([0.2, 0.5, 0.9])
            Cc, T = oracle.composite_fwd(np.full(S, sig), np.tile(c, (S, 1)), widths, S)
            assert abs(T[0] - np.exp(-sig * length)) <= 1e-14
            np.testing.assert_allclose(Cc[0], c * (1 - np.exp(-sig * length)), rtol=1e-13, atol=1e-16)


def test_composite_transmittance_is_exp_of_optical_depth():
    # Eq. 3: T = exp(-int sigma); in the quadrature T_k = exp(-sum sigma_i delta_i), also where single
    # samples are nearly opaque (sigma*delta up to ~100) and 1 - alpha would cancel in double
    rng = np.random.default_rng(0)
    S = 16
    sigma = np.exp(rng.standard_normal(40 * S) * 2.5)
    delta = rng.random(40 * S) * 0.05 + 0.001
    _, T = oracle.composite_fwd(sigma, rng.random((40 * S, 3)), delta, S)
    depth = (sigma * delta).reshape(40, S).sum(1)
    assert depth.max() > 60
    np.testing.assert_allclose(T, np.exp(-depth), rtol=1e-12)


def _random_samples(n_seg, S, seed):
    rng = np.random.default_rng(seed)
    sigma = np.exp(rng.standard_normal(n_seg * S) * 1.5)
    rgb = rng.random((n_seg * S, 3))
    delta = rng.random(n_seg * S) * 0.1 + 0.01
    return sigma, rgb, delta


def test_segmented_equals_unsegmented():
    # one long list of samples vs the same list cut into K contiguous groups, composited then merged
    S_total = 48
    sigma, rgb, delta = _random_samples(20, S_total, seed=1)
    whole_C, whole_T = oracle.composite_fwd(sigma, rgb, delta, S_total)
    for K in (1, 2, 3, 4):
        S = S_total // K
        Ck, Tk = oracle.composite_fwd(sigma, rgb, delta, S)
        Cc, T = oracle.merge_fwd(Ck.reshape(20, K, 3), Tk.reshape(20, K), np.full(20, K, np.uint32))
        np.testing.assert_allclose(Cc, whole_C, rtol=1e-13)
        np.testing.assert_allclose(T, whole_T, rtol=1e-13)


def test_composite_bwd_finite_differences():
    S = 9
    sigma, rgb, delta = _random_samples(5, S, seed=2)
    rng = np.random.default_rng(3)
    gC, gT = rng.standard_normal((5, 3)), rng.standard_normal(5)

    def objective(s_, c_):
        Cc, T = oracle.composite_fwd(s_, c_, delta, S)
        return np.sum(gC * Cc) + np.sum(gT * T)

    dsigma, drgb = oracle.composite_bwd(sigma, rgb, delta, S, gC, gT)
    eps = 1e-6
    for n in range(sigma.size):
        sp, sm = sigma.copy(), sigma.copy(); sp[n] += eps; sm[n] -= eps
        fd = (objective(sp, rgb) - objective(sm, rgb)) / (2 * eps)
        assert abs(fd - dsigma[n]) <= 1e-7 * max(1.0, abs(fd))
        for c in range(3):
            cp, cm = rgb.copy(), rgb.copy(); cp[n, c] += eps; cm[n, c] -= eps
            fd = (objective(sigma, cp) - objective(sigma, cm)) / (2 * eps)
            assert abs(fd - drgb[n, c]) <= 1e-7 * max(1.0, abs(fd))
    # homogeneous medium, analytic derivative: d/dsigma of sum_s over the whole segment
    sig, length, S2 = 0.8, 1.5, 6
    d = np.full(S2, length / S2)
    ds, _ = oracle.composite_bwd(np.full(S2, sig), np.tile([0.3, 0.6, 0.9], (S2, 1)), d, S2,
                                 np.array([[1.0, 0, 0]]), np.array([0.0]))
    assert abs(ds.sum() - 0.3 * length * np.exp(-sig * length)) <= 1e-13     # d/dsigma c(1-e^{-sigma L})


# ------------------------------------------------------------------ merge
def _random_partials(R, k_max, seed, zero_T=False):
    rng = np.random.default_rng(seed)
    Ck, Tk = rng.random((R, k_max, 3)), rng.random((R, k_max))
    if zero_T:
        Tk[rng.random((R, k_max)) < 0.3] = 0.0
    cnt = rng.integers(0, k_max + 1, R).astype(np.uint32)
    return Ck, Tk, cnt


def test_merge_is_an_associative_monoid():
    # (C1,T1) o (C2,T2) = (C1 + T1 C2, T1 T2), identity (0, 1): any bracketing of Eq. 5/6 agrees
    Ck, Tk, _ = _random_partials(50, 4, seed=1)
    full = np.full(50, 4, np.uint32)
    Cc, T = oracle.merge_fwd(Ck, Tk, full)
    op = lambda a, b: (a[0] + a[1][:, None] * b[0], a[1] * b[1])
    parts = [(Ck[:, k], Tk[:, k]) for k in range(4)]
    left = op(op(op(parts[0], parts[1]), parts[2]), parts[3])
    right = op(parts[0], op(parts[1], op(parts[2], parts[3])))
    for got in (left, right):
        np.testing.assert_allclose(Cc, got[0], rtol=1e-14)
        np.testing.assert_allclose(T, got[1], rtol=1e-14)
    # K = 1 returns the partial, K = 0 the identity
    Cc, T = oracle.merge_fwd(Ck, Tk, np.ones(50, np.uint32))
    np.testing.assert_array_equal(Cc, Ck[:, 0]); np.testing.assert_array_equal(T, Tk[:, 0])
    Cc, T = oracle.merge_fwd(Ck, Tk, np.zeros(50, np.uint32))
    assert np.all(Cc == 0) and np.all(T == 1)


@pytest.mark.parametrize("zero_T", [False, True])
def test_merge_bwd_finite_differences(zero_T):
    R, k_max = 30, 4
    Ck, Tk, cnt = _random_partials(R, k_max, seed=2, zero_T=zero_T)
    rng = np.random.default_rng(4)
    gC, gT = rng.standard_normal((R, 3)), rng.standard_normal(R)

    def objective(c_, t_):
        Cc, T = oracle.merge_fwd(c_, t_, cnt)
        return np.sum(gC * Cc) + np.sum(gT * T)

    gCk, gTk = oracle.merge_bwd(Ck, Tk, cnt, gC, gT)
    eps = 1e-6
    for r in range(R):
        for k in range(k_max):
            tp, tm = Tk.copy(), Tk.copy(); tp[r, k] += eps; tm[r, k] -= eps
            fd = (objective(Ck, tp) - objective(Ck, tm)) / (2 * eps)
            assert abs(fd - gTk[r, k]) <= 1e-8 * max(1.0, abs(fd))
            cp, cm = Ck.copy(), Ck.copy(); cp[r, k, 1] += eps; cm[r, k, 1] -= eps
            fd = (objective(cp, Tk) - objective(cm, Tk)) / (2 * eps)
            assert abs(fd - gCk[r, k, 1]) <= 1e-8 * max(1.0, abs(fd))
    # slots beyond the count receive no gradient; K = 1 passes the seeds through
    for r in range(R):
        assert np.all(gCk[r, cnt[r]:] == 0) and np.all(gTk[r, cnt[r]:] == 0)
        if cnt[r] == 1:
            np.testing.assert_array_equal(gCk[r, 0], gC[r]); assert gTk[r, 0] == gT[r]


# ------------------------------------------------------------------ loss
def test_loss_and_seeds():
    rng = np.random.default_rng(0)
    R = 40
    Cc, Cgt, T = rng.random((R, 3)), rng.random((R, 3)), rng.random(R) * 0.9
    val, gC, gT = oracle.loss(Cc, T, Cgt, lambda1=1e-3)
    expect = np.sum((Cc - Cgt) ** 2) / R - 1e-3 * np.sum(np.log(1 - T)) / R       # Eq. 9 (as a mean) + Eq. 10
    assert abs(val - expect) <= 1e-14
    np.testing.assert_allclose(gC, 2 * (Cc - Cgt) / R, rtol=1e-14)
    np.testing.assert_allclose(gT, 1e-3 / (R * (1 - T)), rtol=1e-14)
    val0, gC0, gT0 = oracle.loss(Cc, T, Cgt, lambda1=0.0)
    assert abs(val0 - np.sum((Cc - Cgt) ** 2) / R) <= 1e-15 and np.all(gT0 == 0)
    # fully transparent rays (T = 1) sit on the clamp: finite loss, zero gradient
    val1, _, gT1 = oracle.loss(Cc, np.ones(R), Cgt, lambda1=1e-3)
    assert np.isfinite(val1) and np.all(gT1 == 0)


# ---------------------------------------------------------------------------- depth (evaluation rendering, Sec. 4.4.2)
def test_depth_is_the_colour_rule_applied_to_distances():
    # D_k = sum T_i alpha_i t_i is the composite of a "colour" whose value is the distance: the pinned colour routine
    # must give the same number in each channel
    rng = np.random.default_rng(31)
    S, n_seg = 24, 17
    sigma = rng.random(n_seg * S) * 30.0
    delta = rng.random(n_seg * S) * 0.05
    t = np.sort(rng.random((n_seg, S)) * 5.0, axis=1).reshape(-1)
    D = oracle.composite_depth(sigma, delta, t, S)
    C, _ = oracle.composite_fwd(sigma, np.repeat(t[:, None], 3, axis=1), delta, S)
    np.testing.assert_allclose(D, C[:, 0], rtol=1e-13)


def test_depth_closed_forms():
    S = 32
    delta = np.full(S, 0.01)
    t = 1.0 + (np.arange(S) + 0.5) * 0.01
    # all the distances equal c: D = c (1 - T)
    sigma = np.random.default_rng(32).random(S) * 50.0
    D = oracle.composite_depth(sigma, delta, np.full(S, 2.5), S)
    _, T = oracle.composite_fwd(sigma, np.zeros((S, 3)), delta, S)
    assert D[0] == pytest.approx(2.5 * (1.0 - T[0]), rel=1e-13)
    # an opaque sheet at sample 9 behind empty space: the depth is that sample's distance
    sigma = np.zeros(S)
    sigma[9] = 1e9
    assert oracle.composite_depth(sigma, delta, t, S)[0] == pytest.approx(t[9], rel=1e-13)
    # uniform medium: geometric weights T_i alpha_i = q^i (1 - q), q = exp(-sigma delta)
    sigma = np.full(S, 7.0)
    q = np.exp(-0.07)
    assert oracle.composite_depth(sigma, delta, t, S)[0] == pytest.approx(np.sum(q ** np.arange(S) * (1 - q) * t), rel=1e-12)


def test_depth_of_merged_segments_equals_depth_of_the_whole_ray():
    # the property that makes Eq. 5 exact for the discrete sums holds for the depth channel too
    rng = np.random.default_rng(33)
    S, K, R = 16, 4, 9
    sigma = rng.random((R, K * S)) * 20.0
    delta = rng.random((R, K * S)) * 0.05
    t = np.sort(rng.random((R, K * S)) * 4.0, axis=1)
    whole = oracle.composite_depth(sigma.reshape(-1), delta.reshape(-1), t.reshape(-1), K * S)
    Dk = oracle.composite_depth(sigma.reshape(-1), delta.reshape(-1), t.reshape(-1), S).reshape(R, K)
    _, Tk = oracle.composite_fwd(sigma.reshape(-1), np.zeros((R * K * S, 3)), delta.reshape(-1), S)
    merged = oracle.merge_depth(Dk, Tk.reshape(R, K), np.full(R, K, np.uint32))
    np.testing.assert_allclose(merged, whole, rtol=1e-12)
    # fewer segments than slots: unused slots are ignored
    merged2 = oracle.merge_depth(Dk, Tk.reshape(R, K), np.full(R, 2, np.uint32))
    np.testing.assert_allclose(merged2, Dk[:, 0] + Tk.reshape(R, K)[:, 0] * Dk[:, 1], rtol=1e-13)


def test_sample_distances_match_the_positions():
    cfg = di.config("c3_2x2")
    o, d = di.make_rays(cfg, seed=4, R=50)
    cnt, seg_t, part, _ = oracle.ray_aabb_segments(o, d, cfg["parts"], 0.0, 4)
    off, ray, slot = oracle.bucket_segments(cnt, part, 4)
    p = 0
    u, delta, t = oracle.sample_segments(o, d, seg_t, ray, slot, int(off[p]), int(off[p + 1]), cfg["parts"][p], 8, seed=3, want_t=True)
    lo, ext = cfg["parts"][p][:3].astype(np.float64), di.box_extent(cfg["parts"][p])
    x = lo + u.astype(np.float64) * ext
    rr = np.repeat(ray[int(off[p]):int(off[p + 1])], 8)
    expect = o[rr].astype(np.float64) + t[:, None].astype(np.float64) * d[rr].astype(np.float64)
    np.testing.assert_allclose(x, expect, atol=2e-6)
    tt = t.reshape(-1, 8)
    assert np.all(np.diff(tt, axis=1) > 0)
