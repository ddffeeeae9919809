"""Measured peaks of the GPU for the hot path's access patterns (libdgpeaks.so, csrc/peaks.hip): stream copy, random
8- and 16-byte gathers, random fp32 atomic adds, a loop of fp16 matrix instructions.  `measure()` times each with
events on the current stream and returns the rates; the benchmark reports every kernel against them next to the
datasheet peaks.  Argument marshalling and timing only."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdgpeaks.so")
EXPORTS = ("pk_stream_copy", "pk_stream_read", "pk_random_gather", "pk_random_atomic_add", "pk_mfma_loop")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdgpeaks.so is not built: run `python -m paper_2405_04416_amd.build`")
        h = C.CDLL(LIB_PATH)
        h.pk_stream_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        h.pk_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        h.pk_random_gather.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        h.pk_random_atomic_add.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        h.pk_mfma_loop.argtypes = [C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        for n in EXPORTS:
            getattr(h, n).restype = C.c_int
        _lib = h
    return _lib


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _time_ms(fn, reps=3):
    """Best of `reps` timed runs after one untimed one (events on the stream the kernels are launched on)."""
    fn()
    best = None
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        b.synchronize()
        ms = a.elapsed_time(b)
        best = ms if best is None else min(best, ms)
    return best


def stream_copy(src, dst):
    rc = lib().pk_stream_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream())
    assert rc == 0, rc


def stream_read(src, sink):
    assert sink.numel() >= 256 * 8192
    rc = lib().pk_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream())
    assert rc == 0, rc


def random_gather(table, log2_entries, entry_bytes, n_lanes, per_lane, seed, sink):
    assert table.numel() * table.element_size() >= (entry_bytes << log2_entries) and sink.numel() >= n_lanes
    rc = lib().pk_random_gather(table.data_ptr(), log2_entries, entry_bytes, n_lanes, per_lane, seed, sink.data_ptr(), _stream())
    assert rc == 0, rc


def random_atomic_add(table, log2_entries, n_lanes, per_lane, seed):
    assert table.dtype == torch.float32 and table.numel() >= (1 << log2_entries)
    rc = lib().pk_random_atomic_add(table.data_ptr(), log2_entries, n_lanes, per_lane, seed, _stream())
    assert rc == 0, rc


def mfma_loop(n_waves, iters, sink):
    assert sink.dtype == torch.float32 and sink.numel() >= 64 * n_waves
    rc = lib().pk_mfma_loop(n_waves, iters, sink.data_ptr(), _stream())
    assert rc == 0, rc


def measure(device="cuda:0"):
    """{name: rate} of the yardstick kernels on `device`; about a second of GPU time, 2.1 GiB of device memory."""
    out = {}
    gib = 1 << 30
    buf = torch.empty(2 * gib // 4, dtype=torch.int32, device=device)
    buf.random_(0, 1 << 20)
    src, dst = buf[:gib // 4], buf[gib // 4:]
    ms = _time_ms(lambda: stream_copy(src, dst))
    out["stream_copy_GBps"] = round(2 * gib / ms / 1e6, 1)                       # read + written
    n_lanes, per_lane = 256 * 2048, 64
    sink = torch.empty(256 * 8192, dtype=torch.int32, device=device)
    ms = _time_ms(lambda: stream_read(buf, sink))
    out["stream_read_GBps"] = round(2 * gib / ms / 1e6, 1)
    gathers = n_lanes * per_lane
    for entry_bytes in (16, 8):
        for mib in (128, 1024):
            log2_entries = (mib << 20).bit_length() - 1 - (4 if entry_bytes == 16 else 3)
            ms = _time_ms(lambda: random_gather(buf, log2_entries, entry_bytes, n_lanes, per_lane, 1, sink))
            out["random_gather_%dB_%dMiB_Gps" % (entry_bytes, mib)] = round(gathers / ms / 1e6, 2)
    for mib in (128, 1024):
        tab = buf[:(mib << 20) // 4].view(torch.float32)
        tab.zero_()
        ms = _time_ms(lambda: random_atomic_add(tab, (mib << 20).bit_length() - 3, n_lanes, 64, 1))
        out["random_atomic_add_f32_%dMiB_Gps" % mib] = round(n_lanes * 64 / ms / 1e6, 2)
    n_waves, iters = 256 * 4 * 4, 4096
    fsink = torch.empty(64 * n_waves, dtype=torch.float32, device=device)
    ms = _time_ms(lambda: mfma_loop(n_waves, iters, fsink))
    out["mfma_f16_32x32x16_TFLOPs"] = round(n_waves * iters * 4 * 32768 / ms / 1e9, 1)
    return out
