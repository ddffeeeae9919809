"""The yardstick kernels of the benchmark (libdgpeaks.so) do what their rates are computed from: the copy copies, every
gather reads the entry it is meant to read, every atomic add lands, the matrix loop multiplies."""
import numpy as np
import pytest
import torch

from paper_2405_04416_amd import peaks as P

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not torch.cuda.is_available(), reason="needs a GPU")]
DEV = "cuda:0"


def _mix32(x):
    x = np.asarray(x, np.uint64)
    m = np.uint64(0xffffffff)
    x ^= x >> np.uint64(16); x = (x * np.uint64(0x7feb352d)) & m
    x ^= x >> np.uint64(15); x = (x * np.uint64(0x846ca68b)) & m
    x ^= x >> np.uint64(16)
    return x


def test_stream_copy_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    P.stream_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_stream_read_reads_everything():
    src = torch.randint(0, 2 ** 31 - 1, (1 << 20,), dtype=torch.int32, device=DEV)
    sink = torch.zeros(256 * 8192, dtype=torch.int32, device=DEV)
    P.stream_read(src, sink)
    torch.cuda.synchronize()
    want = np.bitwise_xor.reduce(src.cpu().numpy().view(np.uint32))
    assert np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)) == want


@pytest.mark.parametrize("entry_bytes", [8, 16])
def test_random_gather_reads_the_entries_of_its_counter_sequence(entry_bytes):
    log2_entries, n_lanes, per_lane, seed = 12, 512, 16, 5
    words = entry_bytes // 4
    table = np.random.default_rng(0).integers(0, 2 ** 31, (1 << log2_entries, words)).astype(np.int32)
    sink = torch.zeros(n_lanes, dtype=torch.int32, device=DEV)
    P.random_gather(torch.from_numpy(table).to(DEV), log2_entries, entry_bytes, n_lanes, per_lane, seed, sink)
    torch.cuda.synchronize()
    t = np.arange(n_lanes, dtype=np.uint64)[:, None]
    ctr = (t * np.uint64(per_lane) + np.uint64(seed) + np.arange(per_lane, dtype=np.uint64)[None, :]) & np.uint64(0xffffffff)
    idx = (_mix32(ctr) & np.uint64((1 << log2_entries) - 1)).astype(np.int64)
    picked = table.view(np.uint32)[idx]                      # [lanes, per_lane, words]
    want = np.bitwise_xor.reduce(picked[:, :, 0] ^ picked[:, :, 1], axis=1)
    assert np.array_equal(sink.cpu().numpy().view(np.uint32), want)


def test_random_atomic_add_lands_every_add():
    log2_entries, n_lanes, per_lane = 10, 1024, 8
    tab = torch.zeros(1 << log2_entries, dtype=torch.float32, device=DEV)
    P.random_atomic_add(tab, log2_entries, n_lanes, per_lane, 3)
    torch.cuda.synchronize()
    ctr = (np.arange(n_lanes * per_lane, dtype=np.uint64) + np.uint64(3)) & np.uint64(0xffffffff)
    want = np.bincount((_mix32(ctr) & np.uint64((1 << log2_entries) - 1)).astype(np.int64), minlength=1 << log2_entries)
    assert np.array_equal(tab.cpu().numpy(), want.astype(np.float32))


def test_mfma_loop_multiplies():
    # one accumulator element after `iters` rounds is iters * sum_k a[i,k] b[k,j]; the sink holds, per lane, the sum of the
    # lane's 16 elements of all four accumulators, so the sum over a wavefront is 4 * iters * sum_ij (A B)_ij
    iters = 3
    sink = torch.zeros(64 * 4, dtype=torch.float32, device=DEV)
    P.mfma_loop(4, iters, sink)
    torch.cuda.synchronize()
    lane = np.arange(64)
    a = np.stack([(0.001 * ((lane + j) % 7)).astype(np.float32).astype(np.float16) for j in range(8)], 1).astype(np.float64)   # [lane, j]
    b = np.stack([(0.002 * ((lane * 3 + j) % 5)).astype(np.float32).astype(np.float16) for j in range(8)], 1).astype(np.float64)
    # lane = 32 h + i holds A[i, 8h + j] and B[8h + j, i]
    A = np.zeros((32, 16)); Bm = np.zeros((16, 32))
    for h in range(2):
        A[:, 8 * h:8 * h + 8] = a[32 * h:32 * h + 32]
        Bm[8 * h:8 * h + 8, :] = b[32 * h:32 * h + 32].T
    want = 4 * iters * float((A @ Bm).sum())
    got = sink.cpu().numpy().astype(np.float64).reshape(4, 64).sum(1)
    assert np.allclose(got, want, rtol=1e-4)
