"""The entry point for callers that cannot allocate: dg_ray_aabb_segments_static keeps the counter table of the
distribution step in a fixed device array of the library.  Called through the raw C ABI and compared, bit for bit,
with dg_ray_aabb_segments on the same inputs: two calls in a row, the second on a smaller input (the array keeps the
first call's contents), then the limit's error path."""
import ctypes as C

import numpy as np
import pytest
import torch

import dg_inputs as di
from paper_2405_04416_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _buffers(R, P, k_max):
    z = lambda *s, dt=torch.int32: torch.full(s, -7, dtype=dt, device=DEV)
    return dict(seg_count=z(R), seg_t=z(R, k_max, 2, dt=torch.float32), seg_part=z(R, k_max), part_offset=z(P + 1),
                seg_ray=z(R * k_max), seg_slot=z(R * k_max), status=torch.zeros(1, dtype=torch.int32, device=DEV))


def _call(static, o, d, parts, holes, k_max, out, ws=None):
    lib = B.lib()
    R, P = o.shape[0], parts.shape[0]
    p = lambda t: C.c_void_p(t.data_ptr()) if t is not None else None
    head = (p(o), p(d), R, p(parts), p(holes), P, C.c_float(0.0), k_max, p(out["seg_count"]), p(out["seg_t"]), p(out["seg_part"]),
            p(out["part_offset"]), p(out["seg_ray"]), p(out["seg_slot"]), p(out["status"]))
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if static:
        return lib.dg_ray_aabb_segments_static(*head, stream)
    return lib.dg_ray_aabb_segments(*head, p(ws), ws.numel() * 4, stream)


@pytest.mark.skipif(not torch.cuda.is_available(), reason="needs a GPU")
def test_static_scratch_entry_point_matches_workspace_entry_point():
    for name, R in (("c6_cascade", 100003), ("c3_2x2", 5001)):       # the second call is smaller and has fewer boxes
        cfg = di.config(name)
        o, d = di.make_rays(cfg, seed=3, R=R)
        to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
        od, dd, parts = to(o), to(d), to(cfg["parts"])
        holes = to(cfg["holes"]) if "holes" in cfg else None
        P, k_max = parts.shape[0], cfg["k_max"]
        ref, got = _buffers(R, P, k_max), _buffers(R, P, k_max)
        ws = torch.zeros(max(B.dg_segments_workspace_bytes(R, P) // 4, 1), dtype=torch.int32, device=DEV)
        print("case", name, "R", R, "P", P, flush=True)
        assert _call(False, od, dd, parts, holes, k_max, ref, ws) == 0, B.lib().dg_last_error()
        assert _call(True, od, dd, parts, holes, k_max, got) == 0, B.lib().dg_last_error()
        torch.cuda.synchronize()
        n = int(ref["part_offset"][-1].item())
        assert n > R // 2
        for key in ref:
            a, b = ref[key].cpu().numpy(), got[key].cpu().numpy()
            if key in ("seg_ray", "seg_slot"):
                a, b = a[:n], b[:n]
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (name, key)


@pytest.mark.skipif(not torch.cuda.is_available(), reason="needs a GPU")
def test_static_scratch_entry_point_rejects_sizes_beyond_its_table():
    # ceil(R/256) * P counters must fit the fixed table: checked on the host before anything is enqueued or read
    R, P = (B.SEGMENTS_STATIC_COUNTERS // 64 + 1) * 256, 64
    o = torch.zeros(8, 3, device=DEV)                   # never touched: the call fails on its size check
    out = _buffers(8, P, 1)
    lib = B.lib()
    p = lambda t: C.c_void_p(t.data_ptr())
    rc = lib.dg_ray_aabb_segments_static(p(o), p(o), R, p(o), None, P, C.c_float(0.0), 1, p(out["seg_count"]), p(out["seg_t"]),
                                         p(out["seg_part"]), p(out["part_offset"]), p(out["seg_ray"]), p(out["seg_slot"]),
                                         p(out["status"]), None)
    assert rc == -3 and b"exceed" in lib.dg_last_error()
    torch.cuda.synchronize()
