"""The library's host packer (psattn_pack_ffd) against the oracle's First-Fit-Decreasing loop,
bit for bit, on random sample tables and on the packed configurations; error codes.  CPU only."""
import numpy as np
import pytest

import paper_2410_20305_amd as ps
import psattn_workloads as W
from oracle import psattn_oracle as orc


def lib_vs_oracle(p, c, r, row_len, max_rows=0):
    got = ps.psattn_pack_ffd(p, c, r, row_len, max_rows)
    lengths = (np.asarray(p, np.int64) + c + r).tolist()
    off, n_rows = orc.ffd_pack(lengths, row_len, max_rows)
    assert got["offset"].dtype == np.int32 and got["offset"].tobytes() == off.tobytes()
    assert got["n_rows"] == n_rows
    placed = off >= 0
    assert got["padding_tokens"] == n_rows * row_len - int(np.asarray(lengths)[placed].sum())
    order = got["order"]
    assert sorted(order.tolist()) == list(range(len(lengths)))
    k = int(placed.sum())
    assert np.all(np.diff(off[order[:k]]) > 0) and np.all(off[order[k:]] == -1)
    return got


@pytest.mark.parametrize("seed", range(30))
def test_library_matches_oracle_random(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(0, 200))
    row_len = int(rng.integers(8, 400))
    p, c, r = (rng.integers(0, row_len // 3 + 1, size=n).astype(np.int32) for _ in range(3))
    p = np.maximum(p, 1).astype(np.int32)
    lib_vs_oracle(p, c, r, row_len, max_rows=int(rng.integers(0, 4)) * int(rng.integers(0, 2)))


@pytest.mark.parametrize("name", ["cfg4", "cfg5"])
def test_library_matches_oracle_on_packed_configs(name):
    """The samples of the packed configurations, re-packed: FFD never needs more rows than the
    in-order greedy rule, and the packed table is accepted by the block-mask builder."""
    w = W.make_workload(name)
    got = lib_vs_oracle(w.prefix_len, w.chosen_len, w.rejected_len, w.row_len)
    greedy_rows = w.total_tokens // w.row_len
    assert got["n_rows"] <= greedy_rows
    o = got["order"]
    m = ps.psattn_build_meta(got["offset"][o], w.prefix_len[o], w.chosen_len[o], w.rejected_len[o],
                             got["n_rows"] * w.row_len, host_only=True)
    p, c, r = (x.astype(np.int64) for x in (w.prefix_len, w.chosen_len, w.rejected_len))
    tri = lambda n: n * (n + 1) // 2
    assert m.allowed_pairs() == int((tri(p) + c * p + tri(c) + r * p + tri(r)).sum())


def test_library_errors():
    lib = ps.load_library()
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_pack_ffd([5], [3], [4], 10)            # 12 tokens in a row of 10
    assert e.value.status == -3
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_pack_ffd([0], [0], [0], 10)            # empty sample
    assert e.value.status == -1
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_pack_ffd([1], [1], [1], 0)
    assert e.value.status == -1
    assert lib.psattn_pack_ffd(1, None, None, None, 10, 0, None, None, None, None) == -1
    big = np.full(3, 2 ** 30, dtype=np.int32)
    z = np.zeros(3, dtype=np.int32)
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_pack_ffd(big, z, z, 2 ** 30)           # three rows of 2^30 tokens: offsets overflow int32
    assert e.value.status == -6
    empty = ps.psattn_pack_ffd([], [], [], 16)
    assert empty["n_rows"] == 0 and empty["padding_tokens"] == 0
