"""CPU oracle for the DistGrid training hot path -- TEST INFRASTRUCTURE ONLY.

A ctypes front end over ``dgo.c`` (plain C, double precision, single thread).
Nothing in the product package may import this module; it exists so that the
tests, the smoke check and the benchmark's cpu-baseline leg can compare the HIP
library with an independent statement of the method (DistGrid, arXiv
2405.04416: Sec. 3.2 and 4.1 for the grid, Sec. 4.2.1 for ray/box segments,
Eq. 3 and Eq. 5-10 for rendering, merge and losses).
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dgo.c")
_LIB = os.path.join(_HERE, "libdgo.so")
MAX_LEVELS = 16


def build(force=False):
    """Compile dgo.c with the host C compiler (no GPU code involved)."""
    stale = (not os.path.exists(_LIB)) or any(
        os.path.getmtime(os.path.join(_HERE, f)) > os.path.getmtime(_LIB) for f in ("dgo.c", "dgo.h"))
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Grid(C.Structure):
    _fields_ = [("L", C.c_uint32), ("F", C.c_uint32), ("log2_T", C.c_uint32),
                ("N", C.c_uint32 * MAX_LEVELS),
                ("shape", (C.c_uint32 * 3) * MAX_LEVELS),
                ("is_dense", C.c_uint32 * MAX_LEVELS),
                ("first", C.c_uint64 * (MAX_LEVELS + 1)),
                ("gain", (C.c_float * 3) * MAX_LEVELS)]

    @property
    def n_entries(self):
        return int(self.first[self.L])


class Mlp(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_feat", "n_hidden_d", "n_geo", "n_dir", "n_hidden_c",
                                          "n_layers_c", "act_c", "round_f16")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.dgo_growth_factor.restype = C.c_double
        _lib.dgo_growth_factor.argtypes = [C.c_uint32] * 3
        _lib.dgo_grid_init.restype = C.c_int
        _lib.dgo_grid_init.argtypes = [C.POINTER(Grid), C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                       C.c_double, C.POINTER(C.c_double)]
        _lib.dgo_grid_param_count.restype = C.c_uint64
        _lib.dgo_grid_param_count.argtypes = [C.POINTER(Grid)]
        _lib.dgo_hash.restype = C.c_uint32
        _lib.dgo_hash.argtypes = [C.c_uint32] * 4
        _lib.dgo_vertex_entry.restype = C.c_uint32
        _lib.dgo_vertex_entry.argtypes = [C.POINTER(Grid)] + [C.c_uint32] * 4
        _lib.dgo_jitter.restype = C.c_float
        _lib.dgo_jitter.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        _lib.dgo_round_f16.restype = C.c_double
        _lib.dgo_round_f16.argtypes = [C.c_double]
        _lib.dgo_mlp_weight_count.restype = C.c_uint64
        _lib.dgo_mlp_weight_count.argtypes = [C.POINTER(Mlp)]
        _lib.dgo_loss.restype = C.c_double
        _lib.dgo_adam_step.restype = None
        _lib.dgo_cosine_lr.restype = C.c_double
        _lib.dgo_cosine_lr.argtypes = [C.c_double, C.c_double, C.c_uint64, C.c_uint64]
        for name in ("dgo_encode_fwd", "dgo_encode_bwd", "dgo_ray_aabb_segments", "dgo_bucket_segments",
                     "dgo_sample_segments", "dgo_sh", "dgo_mlp_fwd", "dgo_mlp_bwd", "dgo_composite_fwd",
                     "dgo_composite_bwd", "dgo_merge_fwd", "dgo_merge_bwd", "dgo_composite_depth", "dgo_merge_depth"):
            getattr(_lib, name).restype = None
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


# ---------------------------------------------------------------- grid
def growth_factor(n_min, n_max, L):
    return lib().dgo_growth_factor(n_min, n_max, L)


def grid_init(L, F, log2_T, n_min, growth, extent):
    g = Grid()
    ext = (C.c_double * 3)(*[float(e) for e in extent])
    rc = lib().dgo_grid_init(C.byref(g), L, F, log2_T, n_min, float(growth), ext)
    if rc != 0:
        raise ValueError("dgo_grid_init rejected its arguments")
    return g


def grid_param_count(g):
    return int(lib().dgo_grid_param_count(C.byref(g)))


def hash3(x, y, z, log2_T):
    return int(lib().dgo_hash(int(x), int(y), int(z), int(log2_T)))


def vertex_entry(g, level, x, y, z):
    return int(lib().dgo_vertex_entry(C.byref(g), level, x, y, z))


def encode_fwd(g, table, u, want_idx=False, abs_terms=False):
    table = _arr(table, np.float32)
    u = _arr(u, np.float32).reshape(-1, 3)
    n = u.shape[0]
    feat = np.zeros((n, g.L * g.F), np.float64)
    idx = np.zeros((n, g.L, 8), np.uint32) if want_idx else None
    lib().dgo_encode_fwd(C.byref(g), _p(table), _p(u), C.c_uint64(n), _p(feat), _p(idx), C.c_int(int(abs_terms)))
    return (feat, idx) if want_idx else feat


def encode_bwd(g, u, dfeat):
    u = _arr(u, np.float32).reshape(-1, 3)
    dfeat = _arr(dfeat, np.float64)
    dtable = np.zeros((g.n_entries, g.F), np.float64)
    lib().dgo_encode_bwd(C.byref(g), _p(u), _p(dfeat), C.c_uint64(u.shape[0]), _p(dtable))
    return dtable


# ---------------------------------------------------------------- rays and segments
def ray_aabb_segments(o, d, aabb, t_min, k_max, holes=None):
    o = _arr(o, np.float32).reshape(-1, 3)
    d = _arr(d, np.float32).reshape(-1, 3)
    aabb = _arr(aabb, np.float32).reshape(-1, 6)
    R, P = o.shape[0], aabb.shape[0]
    if holes is not None:
        holes = _arr(holes, np.float32).reshape(-1, 6)
        assert holes.shape[0] == P
    cnt = np.zeros(R, np.uint32)
    seg_t = np.zeros((R, k_max, 2), np.float32)
    seg_part = np.zeros((R, k_max), np.int32)
    status = np.zeros(1, np.uint32)
    lib().dgo_ray_aabb_segments(_p(o), _p(d), C.c_uint32(R), _p(aabb), _p(holes), C.c_uint32(P), C.c_float(t_min),
                                C.c_uint32(k_max), _p(cnt), _p(seg_t), _p(seg_part), _p(status))
    return cnt, seg_t, seg_part, int(status[0])


def bucket_segments(seg_count, seg_part, P):
    seg_count = _arr(seg_count, np.uint32)
    seg_part = _arr(seg_part, np.int32)
    R, k_max = seg_part.shape
    n = int(seg_count.sum())
    off = np.zeros(P + 1, np.uint32)
    seg_ray = np.zeros(max(n, 1), np.uint32)
    seg_slot = np.zeros(max(n, 1), np.uint32)
    lib().dgo_bucket_segments(_p(seg_count), _p(seg_part), C.c_uint32(R), C.c_uint32(k_max), C.c_uint32(P),
                              _p(off), _p(seg_ray), _p(seg_slot))
    return off, seg_ray[:n], seg_slot[:n]


def jitter(seed, ray, slot, s):
    return float(lib().dgo_jitter(C.c_uint64(seed), ray, slot, s))


def sample_segments(o, d, seg_t, seg_ray, seg_slot, seg_begin, seg_end, aabb6, S, seed=0, jitter_arr=None, want_t=False):
    o = _arr(o, np.float32)
    d = _arr(d, np.float32)
    seg_t = _arr(seg_t, np.float32)
    k_max = seg_t.shape[1]
    seg_ray = _arr(seg_ray, np.uint32)
    seg_slot = _arr(seg_slot, np.uint32)
    aabb6 = _arr(aabb6, np.float32)
    n = (seg_end - seg_begin) * S
    u = np.zeros((n, 3), np.float32)
    delta = np.zeros(n, np.float32)
    t = np.zeros(n, np.float32) if want_t else None
    if jitter_arr is not None:
        jitter_arr = _arr(jitter_arr, np.float32)
        assert jitter_arr.size >= n
    lib().dgo_sample_segments(_p(o), _p(d), _p(seg_t), _p(seg_ray), _p(seg_slot), C.c_uint32(seg_begin),
                              C.c_uint32(seg_end), C.c_uint32(k_max), _p(aabb6), C.c_uint32(S),
                              C.c_uint64(seed), _p(jitter_arr), _p(u), _p(delta), _p(t))
    return (u, delta, t) if want_t else (u, delta)


def sh(d, degree):
    d = _arr(d, np.float32).reshape(-1, 3)
    out = np.zeros((d.shape[0], degree * degree), np.float64)
    lib().dgo_sh(_p(d), C.c_uint64(d.shape[0]), C.c_uint32(degree), _p(out))
    return out


# ---------------------------------------------------------------- MLPs
def round_f16(x):
    return float(lib().dgo_round_f16(float(x)))


def mlp_desc(n_feat, n_hidden_d, n_geo, n_dir, n_hidden_c, n_layers_c, act_c=1, round_f16=1):
    return Mlp(n_feat, n_hidden_d, n_geo, n_dir, n_hidden_c, n_layers_c, act_c, round_f16)


def mlp_weight_count(m):
    return int(lib().dgo_mlp_weight_count(C.byref(m)))


def mlp_fwd(m, w, feat, dir_enc, S):
    w = _arr(w, np.float64)
    feat = _arr(feat, np.float64).reshape(-1, m.n_feat)
    dir_enc = _arr(dir_enc, np.float64).reshape(-1, m.n_dir)
    n = feat.shape[0]
    assert w.size == mlp_weight_count(m) and dir_enc.shape[0] * S >= n
    sigma = np.zeros(n, np.float64)
    rgb = np.zeros((n, 3), np.float64)
    lib().dgo_mlp_fwd(C.byref(m), _p(w), _p(feat), _p(dir_enc), C.c_uint32(S), C.c_uint64(n), _p(sigma), _p(rgb))
    return sigma, rgb


def mlp_bwd(m, w, feat, dir_enc, S, dsigma, drgb, loss_scale=1.0):
    w = _arr(w, np.float64)
    feat = _arr(feat, np.float64).reshape(-1, m.n_feat)
    dir_enc = _arr(dir_enc, np.float64).reshape(-1, m.n_dir)
    dsigma = _arr(dsigma, np.float64)
    drgb = _arr(drgb, np.float64)
    n = feat.shape[0]
    dfeat = np.zeros((n, m.n_feat), np.float64)
    dw = np.zeros(w.size, np.float64)
    lib().dgo_mlp_bwd(C.byref(m), _p(w), _p(feat), _p(dir_enc), C.c_uint32(S), C.c_uint64(n), _p(dsigma),
                      _p(drgb), C.c_double(loss_scale), _p(dfeat), _p(dw))
    return dfeat, dw


# ---------------------------------------------------------------- rendering
def composite_fwd(sigma, rgb, delta, S):
    sigma = _arr(sigma, np.float64)
    rgb = _arr(rgb, np.float64)
    delta = _arr(delta, np.float64)
    n_seg = sigma.size // S
    Cc = np.zeros((n_seg, 3), np.float64)
    T = np.zeros(n_seg, np.float64)
    lib().dgo_composite_fwd(_p(sigma), _p(rgb), _p(delta), C.c_uint32(n_seg), C.c_uint32(S), _p(Cc), _p(T))
    return Cc, T


def composite_bwd(sigma, rgb, delta, S, gC, gT):
    sigma = _arr(sigma, np.float64)
    rgb = _arr(rgb, np.float64)
    delta = _arr(delta, np.float64)
    gC = _arr(gC, np.float64)
    gT = _arr(gT, np.float64)
    n_seg = sigma.size // S
    dsigma = np.zeros(sigma.size, np.float64)
    drgb = np.zeros((sigma.size, 3), np.float64)
    lib().dgo_composite_bwd(_p(sigma), _p(rgb), _p(delta), C.c_uint32(n_seg), C.c_uint32(S), _p(gC), _p(gT),
                            _p(dsigma), _p(drgb))
    return dsigma, drgb


def composite_depth(sigma, delta, t, S):
    """Per-segment expected distance sum_i T_i alpha_i t_i (evaluation rendering, Sec. 4.4.2)."""
    sigma, delta, t = _arr(sigma, np.float64), _arr(delta, np.float64), _arr(t, np.float64)
    n_seg = sigma.size // S
    D = np.zeros(n_seg, np.float64)
    lib().dgo_composite_depth(_p(sigma), _p(delta), _p(t), C.c_uint32(n_seg), C.c_uint32(S), _p(D))
    return D


def merge_depth(Dk, Tk, seg_count):
    Dk, Tk = _arr(Dk, np.float64), _arr(Tk, np.float64)
    seg_count = _arr(seg_count, np.uint32)
    R, k_max = Tk.shape
    D = np.zeros(R, np.float64)
    lib().dgo_merge_depth(_p(Dk), _p(Tk), _p(seg_count), C.c_uint32(R), C.c_uint32(k_max), _p(D))
    return D


def merge_fwd(Ck, Tk, seg_count):
    Ck = _arr(Ck, np.float64)
    Tk = _arr(Tk, np.float64)
    seg_count = _arr(seg_count, np.uint32)
    R, k_max = Tk.shape
    Cc = np.zeros((R, 3), np.float64)
    T = np.zeros(R, np.float64)
    lib().dgo_merge_fwd(_p(Ck), _p(Tk), _p(seg_count), C.c_uint32(R), C.c_uint32(k_max), _p(Cc), _p(T))
    return Cc, T


def merge_bwd(Ck, Tk, seg_count, gC, gT):
    Ck = _arr(Ck, np.float64)
    Tk = _arr(Tk, np.float64)
    seg_count = _arr(seg_count, np.uint32)
    gC = _arr(gC, np.float64)
    gT = _arr(gT, np.float64)
    R, k_max = Tk.shape
    gCk = np.zeros((R, k_max, 3), np.float64)
    gTk = np.zeros((R, k_max), np.float64)
    lib().dgo_merge_bwd(_p(Ck), _p(Tk), _p(seg_count), C.c_uint32(R), C.c_uint32(k_max), _p(gC), _p(gT),
                        _p(gCk), _p(gTk))
    return gCk, gTk


def loss(Cc, T, Cgt, lambda1=0.0, want_grad=True):
    Cc = _arr(Cc, np.float64)
    T = _arr(T, np.float64)
    Cgt = _arr(Cgt, np.float64)
    R = T.size
    gC = np.zeros((R, 3), np.float64) if want_grad else None
    gT = np.zeros(R, np.float64) if want_grad else None
    val = lib().dgo_loss(_p(Cc), _p(T), _p(Cgt), C.c_uint32(R), C.c_double(lambda1), _p(gC), _p(gT))
    return (val, gC, gT) if want_grad else val


# ---------------------------------------------------------------- optimiser
def adam_step(theta, grad, m, v, lr, step, beta1=0.9, beta2=0.99, eps=1e-15, l2=0.0, skip_zero=False):
    """In place on float64 arrays theta, m, v (Sec. 5.1: Adam); returns them."""
    for a in (theta, m, v):
        assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    g = _arr(grad, np.float64)
    lib().dgo_adam_step(_p(theta), _p(g), _p(m), _p(v), C.c_uint64(theta.size), C.c_double(lr), C.c_double(beta1),
                        C.c_double(beta2), C.c_double(eps), C.c_uint32(step), C.c_double(l2), C.c_int(1 if skip_zero else 0))
    return theta, m, v


def cosine_lr(lr0, lr1, iteration, total):
    return lib().dgo_cosine_lr(lr0, lr1, iteration, total)


# ---------------------------------------------------------------- occupancy grid and marching
class Occ(C.Structure):
    """Deformable occupancy grid geometry (Sec. 4.1, Sec. 5.1)."""
    _fields_ = [("shape", C.c_uint32 * 3), ("n_cells", C.c_uint32), ("gain", C.c_float * 3)]


def occ_init(N, extent):
    g = Occ()
    ext = (C.c_double * 3)(*[float(e) for e in extent])
    rc = lib().dgo_occ_init(C.byref(g), C.c_uint32(N), ext)
    if rc != 0:
        raise ValueError("dgo_occ_init failed")
    return g


def occ_cell(g, u):
    u = _arr(u, np.float32).reshape(-1, 3)
    f = lib().dgo_occ_cell
    f.restype = C.c_uint32
    return np.array([f(C.byref(g), _p(u[i])) for i in range(u.shape[0])], np.uint32)


def occ_schedule(iteration):
    """(update_now, warmup, decay, threshold) at a training iteration (Sec. 5.1)."""
    a, b, c, d = C.c_int(), C.c_int(), C.c_float(), C.c_float()
    lib().dgo_occ_schedule(C.c_uint64(iteration), C.byref(a), C.byref(b), C.byref(c), C.byref(d))
    return bool(a.value), bool(b.value), c.value, d.value


def rand64(seed, counter):
    f = lib().dgo_rand64
    f.restype = C.c_uint64
    return int(f(C.c_uint64(seed), C.c_uint64(counter)))


def occ_candidates(g, bits, M, n_uniform, warmup, seed, iteration, tries=32, i0=0):
    bits = _arr(bits, np.uint32)
    cell = np.zeros(M, np.uint32)
    u = np.zeros((M, 3), np.float32)
    lib().dgo_occ_candidates(C.byref(g), _p(bits), C.c_uint32(i0), C.c_uint32(M), C.c_uint32(n_uniform), C.c_int(1 if warmup else 0),
                             C.c_uint64(seed), C.c_uint32(iteration), C.c_uint32(tries), _p(cell), _p(u))
    return cell, u


def occ_decay(density, factor):
    assert density.dtype == np.float32 and density.flags["C_CONTIGUOUS"]
    lib().dgo_occ_decay(_p(density), C.c_uint32(density.size), C.c_float(factor))
    return density


def occ_update(density, cell, sigma):
    assert density.dtype == np.float32 and density.flags["C_CONTIGUOUS"]
    cell, sigma = _arr(cell, np.uint32), _arr(sigma, np.float32)
    lib().dgo_occ_update(_p(density), _p(cell), _p(sigma), C.c_uint32(cell.size))
    return density


def occ_bits(density, threshold):
    density = _arr(density, np.float32)
    bits = np.zeros((density.size + 31) // 32, np.uint32)
    f = lib().dgo_occ_bits
    f.restype = C.c_uint32
    n_set = f(_p(density), C.c_uint32(density.size), C.c_float(threshold), _p(bits))
    return bits, int(n_set)


def march_segments(o, d, seg_t, seg_ray, seg_slot, seg_begin, seg_end, aabb6, g, bits, dt, max_steps=4096, seed=0):
    """Occupancy-guided samples of one box's segments: (first [n_seg+1], u, delta, t, sample_ray)."""
    o, d, seg_t = _arr(o, np.float32), _arr(d, np.float32), _arr(seg_t, np.float32)
    k_max = seg_t.shape[1]
    seg_ray, seg_slot = _arr(seg_ray, np.uint32), _arr(seg_slot, np.uint32)
    aabb6, bits = _arr(aabb6, np.float32), _arr(bits, np.uint32)
    first = np.zeros(seg_end - seg_begin + 1, np.uint32)
    f = lib().dgo_march_segments
    f.restype = C.c_uint32

    def call(u, delta, t, ray):
        return f(_p(o), _p(d), _p(seg_t), _p(seg_ray), _p(seg_slot), C.c_uint32(seg_begin), C.c_uint32(seg_end),
                 C.c_uint32(k_max), _p(aabb6), C.byref(g), _p(bits), C.c_float(dt), C.c_uint32(max_steps),
                 C.c_uint64(seed), _p(first), _p(u), _p(delta), _p(t), _p(ray))

    n = call(None, None, None, None)
    u, delta, t = np.zeros((n, 3), np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32)
    ray = np.zeros(n, np.uint32)
    assert call(u, delta, t, ray) == n
    return first, u, delta, t, ray


def composite_fwd_ragged(sigma, rgb, delta, first):
    sigma, rgb, delta = _arr(sigma, np.float64), _arr(rgb, np.float64), _arr(delta, np.float64)
    first = _arr(first, np.uint32)
    n_seg = first.size - 1
    Cc, T = np.zeros((n_seg, 3), np.float64), np.zeros(n_seg, np.float64)
    lib().dgo_composite_fwd_ragged(_p(sigma), _p(rgb), _p(delta), C.c_uint32(n_seg), _p(first), _p(Cc), _p(T))
    return Cc, T


def composite_bwd_ragged(sigma, rgb, delta, first, gC, gT):
    sigma, rgb, delta = _arr(sigma, np.float64), _arr(rgb, np.float64), _arr(delta, np.float64)
    gC, gT, first = _arr(gC, np.float64), _arr(gT, np.float64), _arr(first, np.uint32)
    n_seg = first.size - 1
    dsigma, drgb = np.zeros(sigma.size, np.float64), np.zeros((sigma.size, 3), np.float64)
    lib().dgo_composite_bwd_ragged(_p(sigma), _p(rgb), _p(delta), C.c_uint32(n_seg), _p(first), _p(gC), _p(gT),
                                   _p(dsigma), _p(drgb))
    return dsigma, drgb


def composite_depth_ragged(sigma, delta, t, first):
    sigma, delta, t = _arr(sigma, np.float64), _arr(delta, np.float64), _arr(t, np.float64)
    first = _arr(first, np.uint32)
    D = np.zeros(first.size - 1, np.float64)
    lib().dgo_composite_depth_ragged(_p(sigma), _p(delta), _p(t), C.c_uint32(first.size - 1), _p(first), _p(D))
    return D
