"""Host-only checks of the C ABI: the library loads, exports every declared symbol, validates
arguments, and its grid descriptor agrees with the oracle's geometry (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import dg_inputs as di
import oracle
from paper_2405_04416_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "distgrid.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dg_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 18
    handle = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), n
    assert set(B.EXPORTS) == set(names)


def test_peaks_library_exports_its_symbols():
    from paper_2405_04416_amd import peaks
    handle = C.CDLL(peaks.LIB_PATH)
    for n in peaks.EXPORTS:
        assert hasattr(handle, n), n


def test_no_oracle_in_product_path():
    pkg = os.path.join(ROOT, "paper_2405_04416_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "dgo_" not in src, f


@pytest.mark.parametrize("name", list(di.CONFIGS))
def test_grid_descriptor_matches_oracle_geometry(name):
    cfg = di.config(name)
    g = cfg["grid"]
    ext = di.box_extent(cfg["parts"][0])
    b_lib = g.get("growth") or B.dg_growth_factor(g["n_min"], g["n_max"], g["L"])
    b_ora = g.get("growth") or oracle.growth_factor(g["n_min"], g["n_max"], g["L"])
    desc = B.dg_grid_desc_init(g["L"], g["F"], g["log2_T"], g["n_min"], b_lib, ext)
    ref = oracle.grid_init(g["L"], g["F"], g["log2_T"], g["n_min"], b_ora, ext)
    assert desc.n_levels == ref.L and desc.n_entries == ref.n_entries
    for l in range(ref.L):
        assert desc.n_voxels[l] == ref.N[l]
        assert tuple(desc.res[l]) == tuple(ref.shape[l])
        assert desc.dense[l] == ref.is_dense[l]
        assert desc.offset[l] == ref.first[l]
        assert tuple(desc.scale[l]) == tuple(ref.gain[l])          # bit-identical fp32
    assert desc.offset[ref.L] == ref.first[ref.L]


def test_argument_validation_on_host():
    with pytest.raises(B.DistGridError):
        B.dg_grid_desc_init(17, 2, 19, 16, 1.3, [1, 1, 1])
    with pytest.raises(B.DistGridError):
        B.dg_grid_desc_init(4, 4, 19, 16, 1.3, [1, 1, 1])
    with pytest.raises(B.DistGridError):
        B.dg_grid_desc_init(4, 2, 19, 16, 1.3, [1, 0, 1])
    assert b"extent" in B.lib().dg_last_error()
    m = B.dg_mlp_desc(32, 64, 16, 16, 64, 2)
    assert B.dg_mlp_weight_count(m) == 64 * 32 + 16 * 64 + 64 * 32 + 64 * 64 + 3 * 64
    assert B.dg_mlp_weight_count(m) == oracle.mlp_weight_count(oracle.mlp_desc(32, 64, 16, 16, 64, 2))
    assert B.dg_segments_workspace_bytes(1000, 4) >= 4 * 4 * 4
    # null pointers with N = 0 are accepted, unsupported shapes are refused before any launch
    desc = B.dg_grid_desc_init(4, 2, 12, 16, 1.5, [1, 1, 1])
    assert B.lib().dg_hashgrid_encode_fwd(C.byref(desc), None, None, 0, None, 0, None) == 0
    assert B.lib().dg_hashgrid_encode_fwd(C.byref(desc), None, None, 5, None, 0, None) == -1
    bad = B.dg_mlp_desc(24, 64, 16, 16, 64, 2)
    assert B.lib().dg_mlp_fwd(C.byref(bad), None, None, None, 4, 0, None, None, None) == -2


def test_occupancy_host_side():
    for N, ext in [(512, (2.0, 2.0, 0.25)), (8, (4.0, 2.0, 1.0)), (10, (1.0, 1.0, 0.25)), (33, (0.7, 3.1, 1.9))]:
        desc, ref = B.dg_occ_desc_init(N, ext), oracle.occ_init(N, ext)
        assert tuple(desc.res) == tuple(ref.shape) and desc.n_cells == ref.n_cells
        assert tuple(desc.scale) == tuple(ref.gain)                     # bit-identical fp32
    for it in list(range(0, 40)) + [4095, 4096, 9999, 10000, 10016, 299999]:
        assert B.dg_occ_schedule(it) == oracle.occ_schedule(it)
    with pytest.raises(B.DistGridError):
        B.dg_occ_desc_init(0, [1, 1, 1])
    with pytest.raises(B.DistGridError):
        B.dg_occ_desc_init(8, [1, -1, 1])
    with pytest.raises(B.DistGridError):
        B.dg_occ_desc_init(2048, [1, 1, 1])                             # 2^33 cells
    desc = B.dg_occ_desc_init(8, [1, 1, 1])
    lib = B.lib()
    assert lib.dg_occ_candidates(C.byref(desc), None, 0, 0, 0, 0, 0, 0, 32, None, None, None) == 0
    assert lib.dg_occ_candidates(C.byref(desc), None, 510, 5, 0, 1, 0, 0, 32, None, None, None) == -1    # warm-up: candidate i is cell i
    assert lib.dg_occ_candidates(C.byref(desc), None, 0, 5, 0, 0, 0, 0, 65, None, None, None) == -1
    assert lib.dg_march_workspace_bytes(0) >= 4 and lib.dg_march_workspace_bytes(1 << 20) >= 4 * 513
    box = (C.c_float * 6)(0, 0, 0, 1, 1, 1)
    assert lib.dg_march_segments(None, None, None, None, None, 0, 1, box, C.byref(desc), None, 0.0, 10, 0, 0, None, None, None, None,
                                 None, None, None, 0, None) == -1          # dt must be positive
    assert lib.dg_march_segments(None, None, None, None, None, 0, 1, box, C.byref(desc), None, 0.1, 70000, 0, 0, None, None, None,
                                 None, None, None, None, 0, None) == -1    # the jitter counter has 16 bits for the stratum
    assert lib.dg_composite_ragged_fwd(None, None, None, 0, None, None, None, 1, None, None, None) == 0
    assert lib.dg_composite_ragged_fwd(None, None, None, 3, None, None, None, 1, None, None, None) == -1


def test_optimiser_host_side():
    # the schedule is a host function: same values as the oracle's (fp32 result of a double computation)
    for it in (0, 1, 1234, 150000, 299999, 300000, 10 ** 6):
        assert B.dg_cosine_lr(0.05, 0.005, it, 300000) == pytest.approx(oracle.cosine_lr(0.05, 0.005, it, 300000), rel=2e-7)
    L = B.lib()
    f = C.c_float
    args = lambda n, step, b1=0.9, eps=1e-15: (None, None, None, None, C.c_uint64(n), f(0.01), f(b1), f(0.99), f(eps), step, f(0.0), 1, None, None)
    assert L.dg_adam_step(*args(0, 1)) == 0                 # nothing to do
    assert L.dg_adam_step(*args(8, 1)) == -1                # null pointers
    assert b"null" in L.dg_last_error()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "ONE GPU" in res.stderr
