"""psattn_build_meta_multi (any number of responses per prompt) against the oracle's
brute-force block mask and descriptors, bit for bit; equality with psattn_build_meta at two
responses; error codes.  CPU only."""
import numpy as np
import pytest

import paper_2410_20305_amd as ps
import psattn_workloads as W
from oracle import psattn_oracle as orc


def tri(n):
    return n * (n + 1) // 2


def random_table(rng, n_samples, max_len, max_resp):
    off, P, ptr, rl, cur = [], [], [0], [], int(rng.integers(0, 4))
    for _ in range(n_samples):
        k = int(rng.integers(0, max_resp + 1))
        p = int(rng.integers(0, max_len))
        lens = [int(x) for x in rng.integers(0, max_len, size=k)]
        if p + sum(lens) == 0:
            p = 1
        off.append(cur)
        P.append(p)
        rl += lens
        ptr.append(len(rl))
        cur += p + sum(lens) + int(rng.integers(0, 3))
    return off, P, ptr, rl, cur + int(rng.integers(0, 5))


def assert_equal_to_oracle(off, P, ptr, rl, T, tiles):
    tq, tk, btq, btk = tiles
    m = ps.psattn_build_meta_multi(off, P, ptr, rl, T, tq, tk, btq, btk, host_only=True)
    D, B = orc.branch_arrays(off, P, ptr, rl, T)
    mask = lambda *a: orc.dense_branch_mask(D, B, *a)
    fwd = orc.csr_q_major(orc.classify_tiles(None, None, D, tq, tk, mask=mask))
    bwd = orc.csr_k_major(orc.classify_tiles(None, None, D, btq, btk, mask=mask))
    for grid, ref in ((ps.GRID_FWD, fwd), (ps.GRID_BWD, bwd)):
        rp, idx, cls = m.csr(grid)
        assert rp.tobytes() == ref[0].tobytes() and idx.tobytes() == ref[1].tobytes() and cls.tobytes() == ref[2].tobytes()
    assert m.tok_desc().tobytes() == orc.branch_token_descriptors(D, B).tobytes()
    full = mask(0, T, 0, T)
    assert m.allowed_pairs() == int(full.sum())
    # key side: the queries that read key j are exactly [j, key_hi[j])
    kh = m.key_desc()
    for j in range(T):
        qs = np.nonzero(full[:, j])[0]
        if len(qs):
            assert qs[0] == j and qs[-1] == kh[j] - 1 and len(qs) == kh[j] - j
        else:
            assert kh[j] == 0
    return m


@pytest.mark.parametrize("seed", range(16))
def test_multi_meta_matches_oracle_random(seed):
    rng = np.random.default_rng(300 + seed)
    off, P, ptr, rl, T = random_table(rng, int(rng.integers(1, 5)), 12, 5)
    tiles = tuple(int(x) for x in rng.choice([1, 2, 3, 4, 8], size=4))
    assert_equal_to_oracle(off, P, ptr, rl, T, tiles)


def test_multi_meta_default_grids_four_responses():
    """Sizes that span several default tiles (128 x 64 and 64 x 128)."""
    off, P, ptr, rl = [3, 700], [150, 40], [0, 4, 7], [60, 33, 129, 70, 200, 5, 64]
    assert_equal_to_oracle(off, P, ptr, rl, 1100, (128, 64, 64, 128))


@pytest.mark.parametrize("name", ["cfg2", "cfg4"])
def test_two_responses_equal_the_paired_entry_point(name):
    w = W.make_workload(name)
    a = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens, host_only=True)
    ptr = 2 * np.arange(w.n_samples + 1)
    rl = np.stack([w.chosen_len, w.rejected_len], axis=1).reshape(-1)
    b = ps.psattn_build_meta_multi(w.offset, w.prefix_len, ptr, rl, w.total_tokens, host_only=True)
    for grid in (ps.GRID_FWD, ps.GRID_BWD):
        for x, y in zip(a.csr(grid), b.csr(grid)):
            assert x.tobytes() == y.tobytes()
    assert a.tok_desc().tobytes() == b.tok_desc().tobytes()
    assert a.key_desc().tobytes() == b.key_desc().tobytes()
    assert a.allowed_pairs() == b.allowed_pairs()


def test_multi_meta_errors():
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_build_meta_multi([0], [0], [0, 2], [0, 0], 4, host_only=True)       # empty sample
    assert e.value.status == -1
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_build_meta_multi([0], [2], [0, 2], [3, -1], 9, host_only=True)      # negative length
    assert e.value.status == -1
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_build_meta_multi([0], [2], [0, 3], [3, 3, 3], 10, host_only=True)   # 11 tokens in 10
    assert e.value.status == -3
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_build_meta_multi([0, 4], [2, 2], [0, 1, 2], [3, 3], 12, host_only=True)  # overlap
    assert e.value.status == -2
    lib = ps.load_library()
    import ctypes
    h = ctypes.c_void_p()
    bad_ptr = np.array([1, 2], dtype=np.int32)   # resp_ptr[0] must be 0
    one = np.array([1], dtype=np.int32)
    assert lib.psattn_build_meta_multi_host(1, one.ctypes.data, one.ctypes.data, bad_ptr.ctypes.data, one.ctypes.data,
                                            8, 0, 0, 0, 0, ctypes.byref(h)) == -1
    m = ps.psattn_build_meta_multi([0], [5], [0, 0], [], 5, host_only=True)           # no response: plain causal
    assert m.allowed_pairs() == tri(5)
