"""Pins for the oracle's grid geometry, hash, dense map and encode (CPU only).

Each test ties the oracle to something other than itself: the hash primes
printed by Instant-NGP (Eq. 4), the shape rule of DistGrid Sec. 4.1, the dense
rule of Sec. 4.1, exact reproduction of affine fields by trilinear
interpolation, brute force over every vertex of a small level, and the
transpose identity between encode and its backward.
"""
import os

import numpy as np
import pytest

import dg_inputs as di
import oracle


def _grid(name):
    cfg = di.config(name)
    g = cfg["grid"]
    b = g.get("growth") or oracle.growth_factor(g["n_min"], g["n_max"], g["L"])
    return oracle.grid_init(g["L"], g["F"], g["log2_T"], g["n_min"], b, di.box_extent(cfg["parts"][0]))


def test_hash_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "hash_kat.txt")) if not l.startswith("#")]
    assert len(rows) >= 10
    for x, y, z, k, expect in rows:
        assert oracle.hash3(int(x), int(y), int(z), int(k)) == int(expect)


def test_hash_structure():
    # first prime is 1: the hash of (x,0,0) is x mod T; xor of the three one-axis hashes gives the whole
    rng = np.random.default_rng(1)
    for k in (12, 19, 24):
        for x, y, z in rng.integers(0, 9000, size=(50, 3)):
            assert oracle.hash3(x, 0, 0, k) == x % (1 << k)
            assert oracle.hash3(x, y, z, k) == (oracle.hash3(x, 0, 0, k) ^ oracle.hash3(0, y, 0, k)
                                                ^ oracle.hash3(0, 0, z, k))
            assert oracle.hash3(x, y, z, k) == oracle.hash3(x, y, z, 28) % (1 << k)


def test_level_resolutions():
    g = _grid("c1_tiny")                       # growth 1.5 given directly
    assert list(g.N)[:4] == [16, 24, 36, 54]
    for name, n_max in (("c2_ngp", 2048), ("c4_big", 8192)):
        g = _grid(name)
        N = list(g.N)[:16]
        assert N[0] == 16 and N[-1] == n_max   # end points of the geometric progression
        ratios = [N[i + 1] / N[i] for i in range(15)]
        b = (n_max / 16) ** (1 / 15)
        assert all(abs(r - b) < 0.08 for r in ratios)
        assert all(N[i] == int(np.floor(16 * b ** i + 1e-6)) for i in range(16))


def test_deformable_shape_rule():
    # Sec. 4.1: shape = ceil(a/s * N_l) per axis, s = longest side; box 2 x 2 x 0.25
    g = _grid("c2_ngp")
    expect = {0: (16, 16, 2), 1: (22, 22, 3), 2: (30, 30, 4), 3: (42, 42, 6), 15: (2048, 2048, 256)}
    for l, shp in expect.items():
        assert tuple(g.shape[l]) == shp
    # a cube reduces to (N, N, N)
    g = _grid("c1_tiny")
    for l in range(4):
        assert tuple(g.shape[l]) == (g.N[l],) * 3
    # longest axis need not be x
    g = oracle.grid_init(2, 2, 14, 8, 2.0, [0.5, 4.0, 1.0])
    assert tuple(g.shape[0]) == (1, 8, 2) and tuple(g.shape[1]) == (2, 16, 4)


def test_dense_rule_and_storage():
    # one-to-one map iff the level's vertex count fits the table (for a cube: (N+1)^3 <= T)
    for name in di.CONFIGS:
        g = _grid(name)
        T = 1 << g.log2_T
        total = 0
        for l in range(g.L):
            verts = int(np.prod([s + 1 for s in g.shape[l]]))
            assert bool(g.is_dense[l]) == (verts <= T)
            assert g.first[l] == total
            length = -(-verts // 8) * 8 if verts <= T else T
            total += length
        assert g.first[g.L] == total
        assert oracle.grid_param_count(g) == total * g.F <= g.L * T * g.F      # Sec. 3.2 bound
    g = _grid("c1_tiny")
    assert not any(g.is_dense[l] for l in range(4))          # 17^3 > 4096
    g = oracle.grid_init(3, 2, 12, 8, 1.5, [1, 1, 1])        # 9^3, 13^3 dense; 19^3 hashed
    assert [int(g.is_dense[l]) for l in range(3)] == [1, 1, 0]
    g = oracle.grid_init(1, 2, 12, 15, 1.0, [1, 1, 1])       # 16^3 == 4096: "<=" means dense
    assert g.is_dense[0] == 1


def test_dense_map_is_bijection_brute_force():
    g = oracle.grid_init(3, 2, 14, 6, 1.6, [2.0, 1.0, 0.5])
    for l in range(3):
        assert g.is_dense[l]
        nx, ny, nz = (s + 1 for s in g.shape[l])
        seen = {oracle.vertex_entry(g, l, x, y, z) for x in range(nx) for y in range(ny) for z in range(nz)}
        assert seen == set(range(nx * ny * nz))
    # hashed levels stay inside the table
    g = _grid("c1_tiny")
    rng = np.random.default_rng(0)
    for x, y, z in rng.integers(0, 55, size=(200, 3)):
        assert oracle.vertex_entry(g, 3, x, y, z) < 4096


def _vertex_positions(g, l):
    nx, ny, nz = (s + 1 for s in g.shape[l])
    X, Y, Z = np.meshgrid(np.arange(nx), np.arange(ny), np.arange(nz), indexing="ij")
    return X, Y, Z


def test_trilinear_reproduces_affine_fields():
    # dense levels of a flat box; table holds an anisotropic affine function of the vertex position
    g = oracle.grid_init(3, 2, 16, 5, 1.7, [2.0, 1.0, 0.25])
    coef = np.array([[0.3, -1.1, 2.7, 0.5], [-0.9, 0.4, 0.05, -2.0]])      # per feature: ax+by+cz+d
    table = np.zeros((g.n_entries, 2), np.float32)
    for l in range(3):
        X, Y, Z = _vertex_positions(g, l)
        nx, ny = g.shape[l][0] + 1, g.shape[l][1] + 1
        e = g.first[l] + X + nx * (Y + ny * Z)
        for f in range(2):
            # integer-valued coefficients times integer vertices stay exact in fp32
            table[e, f] = (np.round(coef[f, 0] * 16) * X + np.round(coef[f, 1] * 16) * Y
                           + np.round(coef[f, 2] * 16) * Z + np.round(coef[f, 3] * 16))
    u = di.make_unit_coords(500, seed=3)
    u[:8] = [[0, 0, 0], [1, 1, 1], [1, 0, 0], [0, 1, 0], [0, 0, 1], [0.5, 0.5, 0.5], [1, 1, 0], [0, 1, 1]]
    feat = oracle.encode_fwd(g, table, u)
    for l in range(3):
        gain = np.array(g.gain[l], np.float64)
        pos = (u * np.array(g.gain[l], np.float32)).astype(np.float64)     # fp32 product, as the method fixes
        assert np.all(pos <= np.array(g.shape[l])) and np.allclose(pos, u.astype(np.float64) * gain, rtol=1e-6)
        for f in range(2):
            c = np.round(coef[f] * 16)
            expect = c[0] * pos[:, 0] + c[1] * pos[:, 1] + c[2] * pos[:, 2] + c[3]
            np.testing.assert_allclose(feat[:, l * 2 + f], expect, rtol=0, atol=1e-9)


def test_encode_at_vertices_and_partition_of_unity():
    # hashed levels: a sample that sits on a vertex returns that vertex's (hashed) entry
    g = _grid("c1_tiny")
    table = di.make_table(g.n_entries, 2, 0.1, seed=5)
    rng = np.random.default_rng(2)
    for l in range(4):
        N = g.N[l]
        v = rng.integers(0, N + 1, size=(64, 3))
        u = (v / N).astype(np.float32)
        # only use vertices whose fp32 product lands exactly on the integer
        ok = np.all((u * np.float32(N)) == v, axis=1)
        assert ok.sum() > 20
        feat, idx = oracle.encode_fwd(g, table, u[ok], want_idx=True)
        for i, (x, y, z) in enumerate(v[ok]):
            e = g.first[l] + oracle.hash3(x, y, z, 12)
            np.testing.assert_allclose(feat[i, 2 * l:2 * l + 2], table[e].astype(np.float64), atol=1e-12)
    ones = np.ones((g.n_entries, 2), np.float32)
    u = di.make_unit_coords(300, seed=1)
    np.testing.assert_allclose(oracle.encode_fwd(g, ones, u), 1.0, atol=1e-12)


def test_encode_corner_indices_brute_force():
    # all eight corner indices of random samples against an independent floor/offset computation
    g = _grid("c2_ngp")
    u = di.make_unit_coords(200, seed=9)
    table = np.zeros((g.n_entries, 2), np.float32)
    _, idx = oracle.encode_fwd(g, table, u, want_idx=True)
    for l in (0, 5, 7, 8, 15):
        gain = np.array(g.gain[l], np.float32)
        cell = np.minimum(np.floor(u * gain).astype(np.int64), np.array(g.shape[l]) - 1)
        for c in range(8):
            off = np.array([c & 1, (c >> 1) & 1, (c >> 2) & 1])
            v = cell + off
            if g.is_dense[l]:
                nx, ny = g.shape[l][0] + 1, g.shape[l][1] + 1
                e = v[:, 0] + nx * (v[:, 1] + ny * v[:, 2])
                assert e.max() < g.first[l + 1] - g.first[l]
            else:
                e = (v[:, 0] ^ (v[:, 1] * 2654435761 % 2 ** 32) ^ (v[:, 2] * 805459861 % 2 ** 32)) % (1 << 19)
            np.testing.assert_array_equal(idx[:, l, c], g.first[l] + e)


def test_encode_bwd_is_transpose():
    g = oracle.grid_init(5, 2, 10, 4, 1.6, [1.0, 2.0, 0.5])       # mixes dense and hashed levels
    assert 0 < sum(g.is_dense[l] for l in range(5)) < 5
    table = di.make_table(g.n_entries, 2, 1.0, seed=2)
    u = di.make_unit_coords(400, seed=4)
    G = np.random.default_rng(3).standard_normal((400, 10))
    lhs = np.sum(G * oracle.encode_fwd(g, table, u))
    dtable = oracle.encode_bwd(g, u, G)
    rhs = np.sum(dtable * table.astype(np.float64))
    assert abs(lhs - rhs) <= 1e-10 * abs(lhs)
    # gradient of a single output w.r.t. one entry by finite differences (encode is linear: exact)
    e, f = int(np.argmax(np.abs(dtable[:, 0]))), 0
    t2 = table.copy(); t2[e, f] += 0.5
    fd = np.sum(G * (oracle.encode_fwd(g, t2, u) - oracle.encode_fwd(g, table, u))) / (float(t2[e, f]) - float(table[e, f]))
    assert abs(fd - dtable[e, f]) <= 1e-9 * abs(fd)


def test_clamping_outside_unit_cube():
    g = _grid("c1_tiny")
    table = di.make_table(g.n_entries, 2, 0.1, seed=5)
    a = oracle.encode_fwd(g, table, np.array([[-0.5, 2.0, 0.25]], np.float32))
    b = oracle.encode_fwd(g, table, np.array([[0.0, 1.0, 0.25]], np.float32))
    np.testing.assert_array_equal(a, b)


def test_param_count_brute_force():
    # The parameter count is what the levels need to be stored: found here without the dense/hashed rule, by visiting
    # every vertex of every level of small grids and looking at which table entries are reached.  A level's storage is
    # the span of entries it reaches, rounded up to the 8-entry granule of the layout; the count is F times their sum.
    for args in ((4, 2, 6, 3, 2.7, [1.0, 1.0, 1.0]),           # 4^3 vertices against T = 64: dense; 9^3, 22^3, 60^3: hashed
                 (3, 2, 5, 4, 3.0, [2.0, 1.0, 0.25]),          # a flat box, T = 32
                 (3, 4, 6, 3, 5.0, [1.0, 3.0, 1.0])):          # F = 4, longest axis y
        g = oracle.grid_init(*args)
        spans, kinds = [], []
        for l in range(g.L):
            nx, ny, nz = (s + 1 for s in g.shape[l])
            reached = {oracle.vertex_entry(g, l, x, y, z) for x in range(nx) for y in range(ny) for z in range(nz)}
            assert min(reached) == 0
            spans.append(-(-(max(reached) + 1) // 8) * 8)
            kinds.append(len(reached) == nx * ny * nz)           # one entry per vertex, or shared entries
            if not kinds[-1]:
                assert nx * ny * nz > 8 * (1 << g.log2_T)        # chosen so that a hashed level reaches its whole table
        assert any(kinds) and not all(kinds)
        assert oracle.grid_param_count(g) == g.F * sum(spans)
        assert [g.first[l + 1] - g.first[l] for l in range(g.L)] == spans


def test_param_count_against_the_papers_bound_and_totals():
    # Sec. 3.2: the count is bounded by L * T * F; Sec. 5.3 prints 334.1 M parameters for T = 2^24 x 1 and 264.6 M for
    # T = 2^21 x 4, both below that bound, as the counts of the configurations here are.  (The printed totals themselves
    # cannot be reproduced: the scenes' extents and base resolution are not given.)
    assert 334.1e6 < 16 * 2 ** 24 * 2 and 264.6e6 < 4 * 16 * 2 ** 21 * 2
    for name in ("c4_big", "c5_share", "c3_2x2"):
        g = _grid(name)
        assert oracle.grid_param_count(g) < g.L * (1 << g.log2_T) * g.F
