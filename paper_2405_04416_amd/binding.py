"""Thin ctypes binding over libdistgrid.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/distgrid.h) and does
nothing but check tensor dtype / device / contiguity, pass raw pointers and the current HIP
stream, and raise on a non-zero return code.  PyTorch supplies device memory and streams; all
arithmetic of the hot path runs in the library's kernels.  There is no fallback: if the shared
library is missing the import of this module's `lib()` raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdistgrid.so")

DG_F32, DG_F16 = 0, 1
MAX_LEVELS = 16


class GridDesc(C.Structure):
    _fields_ = [("n_levels", C.c_uint32), ("n_features", C.c_uint32), ("log2_T", C.c_uint32),
                ("n_entries", C.c_uint32),
                ("n_voxels", C.c_uint32 * MAX_LEVELS),
                ("res", (C.c_uint32 * 3) * MAX_LEVELS),
                ("dense", C.c_uint32 * MAX_LEVELS),
                ("offset", C.c_uint32 * (MAX_LEVELS + 1)),
                ("scale", (C.c_float * 3) * MAX_LEVELS)]


class MlpDesc(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_feat", "n_hidden_d", "n_geo", "n_dir", "n_hidden_c", "n_layers_c",
                                          "act_c", "n_app")]


class OccDesc(C.Structure):
    _fields_ = [("res", C.c_uint32 * 3), ("n_cells", C.c_uint32), ("scale", C.c_float * 3)]


class DistGridError(RuntimeError):
    pass


_lib = None

_SIGNATURES = {
    "dg_last_error": (C.c_char_p, []),
    "dg_growth_factor": (C.c_double, [C.c_uint32] * 3),
    "dg_grid_desc_init": (C.c_int, [C.POINTER(GridDesc), C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_double,
                                    C.POINTER(C.c_double)]),
    "dg_segments_workspace_bytes": (C.c_size_t, [C.c_uint32, C.c_uint32]),
    "dg_ray_aabb_segments": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32, C.c_float, C.c_uint32,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_size_t, C.c_void_p]),
    "dg_ray_aabb_segments_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32, C.c_float, C.c_uint32,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p]),
    "dg_sample_segments": (C.c_int, [C.c_void_p] * 5 + [C.c_uint32, C.c_uint32, C.POINTER(C.c_float), C.c_uint32,
                                                        C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dg_dir_encode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p]),
    "dg_hashgrid_encode_fwd": (C.c_int, [C.POINTER(GridDesc), C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32,
                                         C.c_void_p]),
    "dg_hashgrid_encode_bwd_workspace_bytes": (C.c_size_t, [C.POINTER(GridDesc), C.c_uint64]),
    "dg_hashgrid_encode_bwd": (C.c_int, [C.POINTER(GridDesc), C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p,
                                         C.c_size_t, C.c_void_p]),
    "dg_hashgrid_encode_bwd_count": (C.c_int, [C.POINTER(GridDesc), C.c_void_p, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dg_hashgrid_encode_bwd_counted": (C.c_int, [C.POINTER(GridDesc), C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p,
                                                 C.c_size_t, C.c_void_p]),
    "dg_hashgrid_corner_indices": (C.c_int, [C.POINTER(GridDesc), C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]),
    "dg_mlp_weight_count": (C.c_size_t, [C.POINTER(MlpDesc)]),
    "dg_mlp_fwd": (C.c_int, [C.POINTER(MlpDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p,
                             C.c_void_p, C.c_void_p]),
    "dg_mlp_bwd_workspace_bytes": (C.c_size_t, [C.POINTER(MlpDesc), C.c_uint64]),
    "dg_mlp_bwd": (C.c_int, [C.POINTER(MlpDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p,
                             C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dg_mlp_fwd_app": (C.c_int, [C.POINTER(MlpDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64,
                                 C.c_void_p, C.c_void_p, C.c_void_p]),
    "dg_mlp_bwd_app_workspace_bytes": (C.c_size_t, [C.POINTER(MlpDesc), C.c_uint64, C.c_uint32]),
    "dg_mlp_bwd_app": (C.c_int, [C.POINTER(MlpDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64,
                                 C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dg_mlp_composite_fwd": (C.c_int, [C.POINTER(MlpDesc)] + [C.c_void_p] * 4 + [C.c_uint32, C.c_uint32] + [C.c_void_p] * 4 + [C.c_uint32]
                             + [C.c_void_p] * 4),
    "dg_appearance_rows": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p]),
    "dg_composite_segment_fwd": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32,
                                                              C.c_void_p, C.c_void_p, C.c_void_p]),
    "dg_composite_segment_bwd": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32]
                                 + [C.c_void_p] * 5),
    "dg_merge_segments": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_uint32] + [C.c_void_p] * 3),
    "dg_merge_segments_bwd": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_uint32] + [C.c_void_p] * 5),
    "dg_loss_seed": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_float] + [C.c_void_p] * 4),
    "dg_composite_segment_depth": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]),
    "dg_merge_depth": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]),
    "dg_adam_step": (C.c_int, [C.c_void_p] * 4 + [C.c_uint64] + [C.c_float] * 4 + [C.c_uint32, C.c_float, C.c_uint32] + [C.c_void_p] * 2),
    "dg_cosine_lr": (C.c_float, [C.c_float, C.c_float, C.c_uint64, C.c_uint64]),
    "dg_occ_desc_init": (C.c_int, [C.POINTER(OccDesc), C.c_uint32, C.POINTER(C.c_double)]),
    "dg_occ_schedule": (None, [C.c_uint64, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_float), C.POINTER(C.c_float)]),
    "dg_occ_candidates": (C.c_int, [C.POINTER(OccDesc), C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32,
                                    C.c_void_p, C.c_void_p, C.c_void_p]),
    "dg_occ_decay": (C.c_int, [C.c_void_p, C.c_uint32, C.c_float, C.c_void_p]),
    "dg_occ_update": (C.c_int, [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]),
    "dg_occ_bits": (C.c_int, [C.c_void_p, C.c_uint32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dg_march_workspace_bytes": (C.c_size_t, [C.c_uint32]),
    "dg_march_segments": (C.c_int, [C.c_void_p] * 5 + [C.c_uint32, C.c_uint32, C.POINTER(C.c_float), C.POINTER(OccDesc), C.c_void_p, C.c_float,
                                                       C.c_uint32, C.c_uint64, C.c_uint32] + [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p]),
    "dg_composite_ragged_fwd": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                                             C.c_void_p, C.c_void_p, C.c_void_p]),
    "dg_composite_ragged_depth": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                                               C.c_void_p, C.c_void_p]),
    "dg_composite_ragged_bwd": (C.c_int, [C.c_void_p] * 3 + [C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32]
                                + [C.c_void_p] * 5),
}

EXPORTS = tuple(_SIGNATURES)


def lib():
    """Loads the HIP library; raises if it has not been built (there is no CPU fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise DistGridError("libdistgrid.so is not built: run `python -m paper_2405_04416_amd.build`")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(rc):
    if rc != 0:
        raise DistGridError("libdistgrid error %d: %s" % (rc, lib().dg_last_error().decode()))


def _ptr(t, dtype=None, optional=False):
    if t is None:
        if optional:
            return None
        raise DistGridError("missing tensor argument")
    if not t.is_cuda:
        raise DistGridError("tensor must live on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise DistGridError("expected %s, got %s" % (dtype, t.dtype))
    if not t.is_contiguous():
        raise DistGridError("tensor must be contiguous")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


# ------------------------------------------------------------------ host helpers
def dg_growth_factor(n_min, n_max, L):
    return lib().dg_growth_factor(n_min, n_max, L)


def dg_grid_desc_init(L, F, log2_T, n_min, growth, extent):
    desc = GridDesc()
    ext = (C.c_double * 3)(*[float(e) for e in extent])
    _check(lib().dg_grid_desc_init(C.byref(desc), L, F, log2_T, n_min, float(growth), ext))
    return desc


def dg_mlp_desc(n_feat, n_hidden_d, n_geo, n_dir, n_hidden_c, n_layers_c, act_c=1, n_app=0):
    return MlpDesc(n_feat, n_hidden_d, n_geo, n_dir, n_hidden_c, n_layers_c, act_c, n_app)


def dg_mlp_weight_count(desc):
    return int(lib().dg_mlp_weight_count(C.byref(desc)))


def dg_segments_workspace_bytes(R, P):
    return int(lib().dg_segments_workspace_bytes(R, P))


def dg_mlp_bwd_workspace_bytes(desc, N):
    return int(lib().dg_mlp_bwd_workspace_bytes(C.byref(desc), N))


def dg_mlp_bwd_app_workspace_bytes(desc, N, S):
    return int(lib().dg_mlp_bwd_app_workspace_bytes(C.byref(desc), N, S))


# ------------------------------------------------------------------ device entry points
def dg_ray_aabb_segments(o, d, parts, t_min, k_max, seg_count, seg_t, seg_part, status, part_offset=None, seg_ray=None,
                         seg_slot=None, ws=None, holes=None):
    R, P = o.shape[0], parts.shape[0]
    assert holes is None or tuple(holes.shape) == tuple(parts.shape)
    _check(lib().dg_ray_aabb_segments(
        _ptr(o, torch.float32), _ptr(d, torch.float32), R, _ptr(parts, torch.float32), _ptr(holes, torch.float32, True), P, t_min, k_max,
        _ptr(seg_count, torch.int32), _ptr(seg_t, torch.float32), _ptr(seg_part, torch.int32),
        _ptr(part_offset, torch.int32, True), _ptr(seg_ray, torch.int32, True), _ptr(seg_slot, torch.int32, True),
        _ptr(status, torch.int32), _ptr(ws, None, True), 0 if ws is None else ws.numel() * ws.element_size(), _stream()))


SEGMENTS_STATIC_COUNTERS = 1 << 18


def dg_ray_aabb_segments_static(o, d, parts, t_min, k_max, seg_count, seg_t, seg_part, status, part_offset=None, seg_ray=None,
                                seg_slot=None, holes=None):
    R, P = o.shape[0], parts.shape[0]
    assert holes is None or tuple(holes.shape) == tuple(parts.shape)
    _check(lib().dg_ray_aabb_segments_static(
        _ptr(o, torch.float32), _ptr(d, torch.float32), R, _ptr(parts, torch.float32), _ptr(holes, torch.float32, True), P, t_min, k_max,
        _ptr(seg_count, torch.int32), _ptr(seg_t, torch.float32), _ptr(seg_part, torch.int32),
        _ptr(part_offset, torch.int32, True), _ptr(seg_ray, torch.int32, True), _ptr(seg_slot, torch.int32, True),
        _ptr(status, torch.int32), _stream()))


def dg_sample_segments(o, d, seg_t, seg_ray, seg_slot, n_seg, k_max, box, S, seed, jitter, u, delta, t=None):
    box_c = (C.c_float * 6)(*[float(b) for b in box])
    _check(lib().dg_sample_segments(
        _ptr(o, torch.float32), _ptr(d, torch.float32), _ptr(seg_t, torch.float32), _ptr(seg_ray, torch.int32),
        _ptr(seg_slot, torch.int32), n_seg, k_max, box_c, S, seed, _ptr(jitter, torch.float32, True),
        _ptr(u, torch.float32), _ptr(delta, torch.float32), _ptr(t, torch.float32, True), _stream()))


def dg_dir_encode(d, index, n, degree, out):
    _check(lib().dg_dir_encode(_ptr(d, torch.float32), _ptr(index, torch.int32, True), n, degree,
                               _ptr(out, torch.float16), _stream()))


def dg_hashgrid_encode_fwd(desc, table, u, N, feat):
    dt = DG_F16 if feat.dtype == torch.float16 else DG_F32
    _check(lib().dg_hashgrid_encode_fwd(C.byref(desc), _ptr(table, torch.float32), _ptr(u, torch.float32), N,
                                        _ptr(feat, torch.float16 if dt else torch.float32), dt, _stream()))


def dg_hashgrid_encode_bwd_workspace_bytes(desc, N):
    return int(lib().dg_hashgrid_encode_bwd_workspace_bytes(C.byref(desc), N))


def dg_hashgrid_encode_bwd(desc, u, dfeat, N, dtable, ws=None):
    _check(lib().dg_hashgrid_encode_bwd(C.byref(desc), _ptr(u, torch.float32), _ptr(dfeat, torch.float32), N,
                                        _ptr(dtable, torch.float32), _ptr(ws, None, True),
                                        0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def dg_hashgrid_encode_bwd_count(desc, u, N, ws):
    _check(lib().dg_hashgrid_encode_bwd_count(C.byref(desc), _ptr(u, torch.float32), N, _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def dg_hashgrid_encode_bwd_counted(desc, u, dfeat, N, dtable, ws):
    _check(lib().dg_hashgrid_encode_bwd_counted(C.byref(desc), _ptr(u, torch.float32), _ptr(dfeat, torch.float32), N,
                                                _ptr(dtable, torch.float32), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def dg_hashgrid_corner_indices(desc, u, N, idx):
    _check(lib().dg_hashgrid_corner_indices(C.byref(desc), _ptr(u, torch.float32), N, _ptr(idx, torch.int32), _stream()))


def dg_mlp_fwd(desc, weights, feat, dir_enc, S, N, sigma, rgb):
    _check(lib().dg_mlp_fwd(C.byref(desc), _ptr(weights, torch.float16), _ptr(feat, torch.float16),
                            _ptr(dir_enc, torch.float16), S, N, _ptr(sigma, torch.float32), _ptr(rgb, torch.float32),
                            _stream()))


def dg_mlp_bwd(desc, weights, feat, dir_enc, S, N, dsigma, drgb, loss_scale, dfeat, dW, ws):
    _check(lib().dg_mlp_bwd(C.byref(desc), _ptr(weights, torch.float16), _ptr(feat, torch.float16),
                            _ptr(dir_enc, torch.float16), S, N, _ptr(dsigma, torch.float32), _ptr(drgb, torch.float32),
                            loss_scale, _ptr(dfeat, torch.float32), _ptr(dW, torch.float32), _ptr(ws),
                            ws.numel() * ws.element_size(), _stream()))


def dg_composite_segment_fwd(sigma, rgb, delta, n_seg, S, seg_ray, seg_slot, k_max, Ck, Tk):
    _check(lib().dg_composite_segment_fwd(
        _ptr(sigma, torch.float32), _ptr(rgb, torch.float32), _ptr(delta, torch.float32), n_seg, S,
        _ptr(seg_ray, torch.int32), _ptr(seg_slot, torch.int32), k_max, _ptr(Ck, torch.float32), _ptr(Tk, torch.float32),
        _stream()))


def dg_composite_segment_bwd(sigma, rgb, delta, n_seg, S, seg_ray, seg_slot, k_max, gCk, gTk, dsigma, drgb):
    _check(lib().dg_composite_segment_bwd(
        _ptr(sigma, torch.float32), _ptr(rgb, torch.float32), _ptr(delta, torch.float32), n_seg, S,
        _ptr(seg_ray, torch.int32), _ptr(seg_slot, torch.int32), k_max, _ptr(gCk, torch.float32), _ptr(gTk, torch.float32),
        _ptr(dsigma, torch.float32), _ptr(drgb, torch.float32), _stream()))


def dg_merge_segments(Ck, Tk, seg_count, R, k_max, Cout, Tout):
    _check(lib().dg_merge_segments(_ptr(Ck, torch.float32), _ptr(Tk, torch.float32), _ptr(seg_count, torch.int32), R, k_max,
                                   _ptr(Cout, torch.float32), _ptr(Tout, torch.float32), _stream()))


def dg_merge_segments_bwd(Ck, Tk, seg_count, R, k_max, gC, gT, gCk, gTk):
    _check(lib().dg_merge_segments_bwd(_ptr(Ck, torch.float32), _ptr(Tk, torch.float32), _ptr(seg_count, torch.int32), R,
                                       k_max, _ptr(gC, torch.float32), _ptr(gT, torch.float32), _ptr(gCk, torch.float32),
                                       _ptr(gTk, torch.float32), _stream()))


def dg_loss_seed(Cin, Tin, Cgt, R, lambda1, gC, gT, loss=None):
    _check(lib().dg_loss_seed(_ptr(Cin, torch.float32), _ptr(Tin, torch.float32), _ptr(Cgt, torch.float32), R, lambda1,
                              _ptr(gC, torch.float32), _ptr(gT, torch.float32), _ptr(loss, torch.float32, True), _stream()))


def dg_adam_step(param, grad, m, v, lr, step, beta1=0.9, beta2=0.99, eps=1e-15, l2=0.0, skip_zero_grad=False, param_half=None):
    n = param.numel()
    assert grad.numel() == n and m.numel() == n and v.numel() == n and (param_half is None or param_half.numel() == n)
    _check(lib().dg_adam_step(_ptr(param, torch.float32), _ptr(grad, torch.float32), _ptr(m, torch.float32), _ptr(v, torch.float32),
                              n, lr, beta1, beta2, eps, step, l2, 1 if skip_zero_grad else 0,
                              _ptr(param_half, torch.float16, True), _stream()))


def dg_cosine_lr(lr0, lr1, iteration, total):
    return float(lib().dg_cosine_lr(lr0, lr1, iteration, total))


def dg_composite_segment_depth(sigma, delta, t, n_seg, S, seg_ray, seg_slot, k_max, Dk):
    assert min(sigma.numel(), delta.numel(), t.numel()) >= n_seg * S and min(seg_ray.numel(), seg_slot.numel()) >= n_seg
    _check(lib().dg_composite_segment_depth(_ptr(sigma, torch.float32), _ptr(delta, torch.float32), _ptr(t, torch.float32), n_seg, S,
                                            _ptr(seg_ray, torch.int32), _ptr(seg_slot, torch.int32), k_max, _ptr(Dk, torch.float32),
                                            _stream()))


def dg_merge_depth(Dk, Tk, seg_count, R, k_max, D):
    assert min(Dk.numel(), Tk.numel()) >= R * k_max and min(seg_count.numel(), D.numel()) >= R
    _check(lib().dg_merge_depth(_ptr(Dk, torch.float32), _ptr(Tk, torch.float32), _ptr(seg_count, torch.int32), R, k_max,
                                _ptr(D, torch.float32), _stream()))


# ------------------------------------------------------------------ occupancy grid and occupancy-guided sampling
def dg_occ_desc_init(N, extent):
    desc = OccDesc()
    ext = (C.c_double * 3)(*[float(e) for e in extent])
    _check(lib().dg_occ_desc_init(C.byref(desc), N, ext))
    return desc


def dg_occ_schedule(iteration):
    """(update_now, warmup, decay, threshold) at a training iteration."""
    a, b, c, d = C.c_int(), C.c_int(), C.c_float(), C.c_float()
    lib().dg_occ_schedule(iteration, C.byref(a), C.byref(b), C.byref(c), C.byref(d))
    return bool(a.value), bool(b.value), c.value, d.value


def dg_occ_candidates(desc, bits, M, n_uniform, warmup, seed, iteration, tries, cell, u, i0=0):
    assert cell.numel() >= M and u.numel() >= 3 * M and (bits is None or bits.numel() >= (desc.n_cells + 31) // 32)
    _check(lib().dg_occ_candidates(C.byref(desc), _ptr(bits, torch.int32, True), i0, M, n_uniform, 1 if warmup else 0, seed, iteration,
                                   tries, _ptr(cell, torch.int32), _ptr(u, torch.float32), _stream()))


def dg_occ_decay(density, factor):
    _check(lib().dg_occ_decay(_ptr(density, torch.float32), density.numel(), factor, _stream()))


def dg_occ_update(density, cell, sigma, M):
    assert cell.numel() >= M and sigma.numel() >= M
    _check(lib().dg_occ_update(_ptr(density, torch.float32), density.numel(), _ptr(cell, torch.int32), _ptr(sigma, torch.float32), M,
                               _stream()))


def dg_occ_bits(density, threshold, bits, n_set=None):
    assert bits.numel() >= (density.numel() + 31) // 32
    _check(lib().dg_occ_bits(_ptr(density, torch.float32), density.numel(), threshold, _ptr(bits, torch.int32),
                             _ptr(n_set, torch.int32, True), _stream()))


def dg_march_workspace_bytes(n_seg):
    return int(lib().dg_march_workspace_bytes(n_seg))


def dg_march_segments(o, d, seg_t, seg_ray, seg_slot, n_seg, k_max, box, occ, bits, dt, max_steps, seed, capacity, first, u, delta, t,
                      sample_ray, status, ws):
    assert first.numel() >= n_seg + 1 and bits.numel() >= (occ.n_cells + 31) // 32
    assert min(seg_ray.numel(), seg_slot.numel()) >= n_seg
    assert u.numel() >= 3 * capacity and min(delta.numel(), t.numel(), sample_ray.numel()) >= capacity
    box_c = (C.c_float * 6)(*[float(b) for b in box])
    _check(lib().dg_march_segments(
        _ptr(o, torch.float32), _ptr(d, torch.float32), _ptr(seg_t, torch.float32), _ptr(seg_ray, torch.int32),
        _ptr(seg_slot, torch.int32), n_seg, k_max, box_c, C.byref(occ), _ptr(bits, torch.int32), dt, max_steps, seed, capacity,
        _ptr(first, torch.int32), _ptr(u, torch.float32), _ptr(delta, torch.float32), _ptr(t, torch.float32),
        _ptr(sample_ray, torch.int32), _ptr(status, torch.int32), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def dg_composite_ragged_fwd(sigma, rgb, delta, n_seg, first, seg_ray, seg_slot, k_max, Ck, Tk):
    assert first.numel() >= n_seg + 1 and min(seg_ray.numel(), seg_slot.numel()) >= n_seg
    _check(lib().dg_composite_ragged_fwd(
        _ptr(sigma, torch.float32), _ptr(rgb, torch.float32), _ptr(delta, torch.float32), n_seg, _ptr(first, torch.int32),
        _ptr(seg_ray, torch.int32), _ptr(seg_slot, torch.int32), k_max, _ptr(Ck, torch.float32), _ptr(Tk, torch.float32), _stream()))


def dg_composite_ragged_depth(sigma, delta, t, n_seg, first, seg_ray, seg_slot, k_max, Dk):
    assert first.numel() >= n_seg + 1 and min(seg_ray.numel(), seg_slot.numel()) >= n_seg
    _check(lib().dg_composite_ragged_depth(
        _ptr(sigma, torch.float32), _ptr(delta, torch.float32), _ptr(t, torch.float32), n_seg, _ptr(first, torch.int32),
        _ptr(seg_ray, torch.int32), _ptr(seg_slot, torch.int32), k_max, _ptr(Dk, torch.float32), _stream()))


def dg_composite_ragged_bwd(sigma, rgb, delta, n_seg, first, seg_ray, seg_slot, k_max, gCk, gTk, dsigma, drgb):
    assert first.numel() >= n_seg + 1 and min(seg_ray.numel(), seg_slot.numel()) >= n_seg
    _check(lib().dg_composite_ragged_bwd(
        _ptr(sigma, torch.float32), _ptr(rgb, torch.float32), _ptr(delta, torch.float32), n_seg, _ptr(first, torch.int32),
        _ptr(seg_ray, torch.int32), _ptr(seg_slot, torch.int32), k_max, _ptr(gCk, torch.float32), _ptr(gTk, torch.float32),
        _ptr(dsigma, torch.float32), _ptr(drgb, torch.float32), _stream()))


# ------------------------------------------------------------------ appearance features as colour-net inputs
def dg_appearance_rows(table, image_of_ray, index, n, out):
    n_app = table.shape[-1]
    assert out.numel() >= n * n_app and (index is None or index.numel() >= n)
    _check(lib().dg_appearance_rows(_ptr(table, torch.float16), _ptr(image_of_ray, torch.int32), _ptr(index, torch.int32, True), n,
                                    n_app, _ptr(out, torch.float16), _stream()))


def dg_mlp_fwd_app(desc, weights, feat, dir_enc, app, S, N, sigma, rgb):
    rows = -(-N // S)
    assert dir_enc.numel() >= rows * desc.n_dir and (app is None or app.numel() >= rows * desc.n_app)
    _check(lib().dg_mlp_fwd_app(C.byref(desc), _ptr(weights, torch.float16), _ptr(feat, torch.float16), _ptr(dir_enc, torch.float16),
                                _ptr(app, torch.float16, True), S, N, _ptr(sigma, torch.float32), _ptr(rgb, torch.float32), _stream()))


def dg_mlp_composite_fwd(desc, weights, feat, dir_enc, app, S, n_seg, delta, t, seg_ray, seg_slot, k_max, Ck, Tk, Dk):
    N = n_seg * S
    assert dir_enc.numel() >= n_seg * desc.n_dir and (app is None or app.numel() >= n_seg * desc.n_app)
    assert feat.numel() >= N * desc.n_feat and delta.numel() >= N and (t is None or t.numel() >= N)
    assert min(seg_ray.numel(), seg_slot.numel()) >= n_seg
    _check(lib().dg_mlp_composite_fwd(C.byref(desc), _ptr(weights, torch.float16), _ptr(feat, torch.float16), _ptr(dir_enc, torch.float16),
                                      _ptr(app, torch.float16, True), S, n_seg, _ptr(delta, torch.float32), _ptr(t, torch.float32, True),
                                      _ptr(seg_ray, torch.int32), _ptr(seg_slot, torch.int32), k_max, _ptr(Ck, torch.float32),
                                      _ptr(Tk, torch.float32), _ptr(Dk, torch.float32, True), _stream()))


def dg_mlp_bwd_app(desc, weights, feat, dir_enc, app, S, N, dsigma, drgb, loss_scale, dfeat, dW, ws):
    rows = -(-N // S)
    assert dir_enc.numel() >= rows * desc.n_dir and (app is None or app.numel() >= rows * desc.n_app)
    assert dW.numel() >= dg_mlp_weight_count(desc)
    _check(lib().dg_mlp_bwd_app(C.byref(desc), _ptr(weights, torch.float16), _ptr(feat, torch.float16), _ptr(dir_enc, torch.float16),
                                _ptr(app, torch.float16, True), S, N, _ptr(dsigma, torch.float32), _ptr(drgb, torch.float32),
                                loss_scale, _ptr(dfeat, torch.float32), _ptr(dW, torch.float32), _ptr(ws),
                                ws.numel() * ws.element_size(), _stream()))
