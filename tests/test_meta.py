"""Host logic of libpsattn (no GPU): the metadata builder against the oracle's
brute-force block mask, bit for bit; error codes; exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2410_20305_amd as ps
import psattn_workloads as W
from oracle import psattn_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def oracle_meta(w, tq, tk, btq, btk):
    Ic, Ir, D = orc.index_arrays(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    fwd = orc.csr_q_major(orc.classify_tiles(Ic, Ir, D, tq, tk))
    bwd = orc.csr_k_major(orc.classify_tiles(Ic, Ir, D, btq, btk))
    return fwd, bwd, orc.token_descriptors(Ic, Ir, D), (Ic, Ir, D)


def assert_meta_equal(w, tq, tk, btq, btk):
    m = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens,
                             tq, tk, btq, btk, host_only=True)
    fwd, bwd, desc, (Ic, Ir, D) = oracle_meta(w, tq, tk, btq, btk)
    for grid, ref in ((ps.GRID_FWD, fwd), (ps.GRID_BWD, bwd)):
        rp, idx, cls = m.csr(grid)
        assert rp.dtype == np.int32 and idx.dtype == np.int32 and cls.dtype == np.uint8
        assert rp.tobytes() == ref[0].tobytes()
        assert idx.tobytes() == ref[1].tobytes()
        assert cls.tobytes() == ref[2].tobytes()
    assert m.tok_desc().tobytes() == desc.tobytes()
    t = m.tiles(ps.GRID_FWD)
    assert (t["tile_q"], t["tile_k"]) == (tq, tk)
    assert t["n_q_tiles"] == -(-w.total_tokens // tq) and t["n_k_tiles"] == -(-w.total_tokens // tk)
    return m, (Ic, Ir, D)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_meta_matches_oracle_on_configs(name):
    """Default grids (the ones the bf16 kernels run on), all five configurations."""
    w = W.make_workload(name)
    m, _ = assert_meta_equal(w, 128, 64, 64, 128)
    p, c, r = (x.astype(np.int64) for x in (w.prefix_len, w.chosen_len, w.rejected_len))
    tri = lambda n: n * (n + 1) // 2
    assert m.allowed_pairs() == int((tri(p) + c * p + tri(c) + r * p + tri(r)).sum())
    d = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens,
                             host_only=True)
    assert d.tiles(ps.GRID_FWD)["tile_q"] == 128 and d.tiles(ps.GRID_FWD)["tile_k"] == 64
    assert d.tiles(ps.GRID_BWD)["tile_q"] == 64 and d.tiles(ps.GRID_BWD)["tile_k"] == 128
    assert d.csr(ps.GRID_FWD)[1].tobytes() == m.csr(ps.GRID_FWD)[1].tobytes()


def test_meta_128_grid_counts_config3():
    w = W.make_workload("cfg3")
    m, _ = assert_meta_equal(w, 128, 128, 128, 128)
    cls = m.csr(ps.GRID_FWD)[2]
    assert int((cls == ps.TILE_FULL).sum()) == 1897 and int((cls == ps.TILE_PARTIAL).sum()) == 756


@pytest.mark.parametrize("seed", range(12))
def test_meta_random_small(seed):
    rng = np.random.default_rng(seed)
    tiles = [1, 2, 3, 4, 8]
    tq, tk, btq, btk = (int(rng.choice(tiles)) for _ in range(4))
    ns = int(rng.integers(0, 5))
    samples, offs, cur = [], [], int(rng.integers(0, 4))
    for _ in range(ns):
        s = tuple(int(x) for x in rng.integers(0, 10, 3))
        if sum(s) == 0:
            s = (0, 1, 0)
        samples.append(s)
        offs.append(cur)
        cur += sum(s) + int(rng.integers(0, 4)) * int(rng.integers(0, 2))
    T = cur + int(rng.integers(0, 5))
    w = W.custom_workload(samples, offsets=offs, total_tokens=T)
    m, (Ic, Ir, D) = assert_meta_equal(w, tq, tk, btq, btk)
    # key-side descriptors: the queries that read key j are exactly [j, key_hi[j])
    mask = orc.dense_mask(Ic, Ir, D) if T else np.zeros((0, 0), bool)
    kh = m.key_desc()
    for j in range(T):
        qs = np.nonzero(mask[:, j])[0]
        want = list(range(j, int(kh[j]))) if kh[j] > j else []
        assert qs.tolist() == want
    assert m.allowed_pairs() == int(mask.sum())


def test_meta_edge_cases():
    # everything is padding
    m = ps.psattn_build_meta([], [], [], [], 10, 4, 4, 4, 4, host_only=True)
    rp, idx, cls = m.csr(ps.GRID_FWD)
    assert rp.tolist() == [0, 0, 0, 0] and len(idx) == 0
    assert np.all(m.tok_desc()[:, 0] == np.iinfo(np.int32).max)
    # empty buffer
    m = ps.psattn_build_meta([], [], [], [], 0, host_only=True)
    assert m.tiles()["n_q_tiles"] == 0 and m.allowed_pairs() == 0
    # a tile that is exactly one full rectangle, and a clipped one that must not be FULL
    m = ps.psattn_build_meta([0], [12], [0], [0], 12, 4, 4, 4, 4, host_only=True)
    rp, idx, cls = m.csr(ps.GRID_FWD)
    assert idx.tolist() == [0, 0, 1, 0, 1, 2] and cls.tolist() == [1, 2, 1, 2, 2, 1]
    m = ps.psattn_build_meta([0], [10], [0], [0], 10, 4, 4, 4, 4, host_only=True)
    rp, idx, cls = m.csr(ps.GRID_FWD)
    assert cls.tolist() == [1, 2, 1, 1, 1, 1]  # last q-tile is clipped: never FULL


def test_meta_errors():
    def status(*a, **k):
        with pytest.raises(ps.PsattnError) as e:
            ps.psattn_build_meta(*a, host_only=True, **k)
        return e.value.status
    assert status([0], [-1], [1], [1], 8) == -1                 # negative length
    assert status([0], [0], [0], [0], 8) == -1                  # empty sample
    assert status([0], [1], [1], [1], 8, tile_q=-2) == -1       # bad tile
    assert status([4, 0], [2, 2], [0, 0], [0, 0], 8) == -2      # unsorted
    assert status([0, 2], [2, 2], [1, 0], [0, 0], 8) == -2      # overlap
    assert status([0], [4], [4], [4], 8) == -3                  # beyond the buffer
    # a grid whose tile index would not fit the 30 bits a list entry has for it: refused before anything is built
    assert status([0], [4], [2], [2], 1 << 29, tile_q=1, tile_k=1, bwd_tile_q=1, bwd_tile_k=1) == -6
    lib = ps.load_library()
    assert lib.psattn_build_meta_host(1, None, None, None, None, 4, 0, 0, 0, 0,
                                      ctypes.byref(ctypes.c_void_p())) == -1
    assert lib.psattn_free_meta(None) == 0
    # kernels refuse a host-only meta without touching any device
    m = ps.psattn_build_meta([0], [4], [2], [2], 8, host_only=True)
    assert lib.psattn_fwd(m.handle, 1, 4, 2, 128, 0.1, None, None, None, None, None, None) == -7
    assert lib.psattn_fwd(m.handle, 1, 3, 2, 128, 0.1, None, None, None, None, None, None) == -1
    assert lib.psattn_fwd(m.handle, 1, 4, 2, 96, 0.1, None, None, None, None, None, None) == -1
    assert lib.psattn_fwd(None, 1, 4, 2, 128, 0.1, None, None, None, None, None, None) == -1
    assert lib.psattn_strerror(-2).decode().startswith("samples")


def test_probe_entry_points_validate_before_touching_a_device():
    lib = ps.load_library()
    one = ctypes.c_void_p(8)  # never dereferenced: every call below is rejected on its arguments
    assert lib.psattn_probe_mfma_peak(0, 2, 0, one, None) == -1      # no workgroups
    assert lib.psattn_probe_mfma_peak(4, 3, 0, one, None) == -1      # odd round count
    assert lib.psattn_probe_mfma_peak(4, 2, 3, one, None) == -1      # unknown operand pattern
    assert lib.psattn_probe_mfma_peak(4, 2, 1, None, None) == -1     # no sink
    m = ps.psattn_build_meta([0], [4], [2], [2], 8, host_only=True)
    assert lib.psattn_probe_dq_atomics(m.handle, 4, 3, one, 0, None) == -1   # heads do not divide
    assert lib.psattn_probe_dq_atomics(m.handle, 4, 2, one, 0, None) == -7   # host-only meta


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "psattn.h")).read()
    declared = set(re.findall(r"\b(psattn_[a-z_]+)\s*\(", header))
    declared -= {"psattn_status", "psattn_dtype"}
    assert declared == set(ps.binding.EXPORTS)
    lib = ctypes.CDLL(ps.lib_path())
    for name in sorted(declared):
        assert hasattr(lib, name), name


def test_layer_library_exports_every_declared_symbol():
    """include/psattn_layer.h against libpsattn_layer.so (loads rocBLAS; no device call is made)."""
    from paper_2410_20305_amd.layer import load_layer_library
    header = open(os.path.join(ROOT, "include", "psattn_layer.h")).read()
    body = header[header.index("typedef struct psattn_layer"):]
    declared = set(re.findall(r"\b(psattn_layer_[a-z_]+)\s*\(", body))
    assert declared == {"psattn_layer_create", "psattn_layer_free", "psattn_layer_workspace_bytes", "psattn_layer_fwd",
                        "psattn_layer_bwd"}
    lib = load_layer_library()
    for name in sorted(declared):
        assert hasattr(lib, name), name
