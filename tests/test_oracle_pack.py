"""Pins of the oracle's First-Fit-Decreasing loop (Section 4.3.2): a hand-worked example, the
first-fit property checked by replay on the result, the 11/9 OPT + 6/9 bound against a
brute-force optimum, the row limit.  CPU only; nothing here calls the library."""
import itertools
import os

import numpy as np
import pytest

from oracle import psattn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def check_first_fit_by_replay(lengths, row_len, offset, n_rows, max_rows=0):
    """The defining property, checked on the result instead of re-running the loop: going
    through the units from longest to shortest (ties by index), each placed unit sits in the
    lowest row that had room at that moment, directly behind that row's earlier units; a unit
    left out fits no row and the row limit is reached."""
    n = len(lengths)
    fill = [0] * n_rows
    opened = 0
    for i in sorted(range(n), key=lambda i: (-int(lengths[i]), i)):
        L = int(lengths[i])
        room = [r for r in range(opened) if fill[r] + L <= row_len]
        if offset[i] < 0:
            assert not room and max_rows > 0 and opened == max_rows
            continue
        r, pos = divmod(int(offset[i]), row_len)
        if room:
            assert r == room[0]
        else:
            assert r == opened
            opened += 1
        assert pos == fill[r]
        fill[r] += L
    assert opened == n_rows


def optimal_rows(lengths, row_len):
    """Fewest rows that hold all units, by exhaustive assignment (tiny inputs only)."""
    n = len(lengths)
    for k in range(1, n + 1):
        for assign in itertools.product(range(k), repeat=n):
            fill = [0] * k
            for L, r in zip(lengths, assign):
                fill[r] += L
            if max(fill) <= row_len:
                return k
    return n


def test_oracle_hand_worked_example():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "ffd_row10.txt")) if ln.strip() and not ln.startswith("#")]
    lengths = [int(r[1]) for r in rows]
    off, n_rows = orc.ffd_pack(lengths, 10)
    assert n_rows == 3
    for r in rows:
        u, row, pos, flat = int(r[0]), int(r[2]), int(r[3]), int(r[4])
        assert flat == row * 10 + pos
        assert off[u] == flat


def test_oracle_equal_lengths_keep_their_order():
    off, n_rows = orc.ffd_pack([3, 3, 3, 3], 6)
    assert n_rows == 2 and off.tolist() == [0, 3, 6, 9]


@pytest.mark.parametrize("seed", range(20))
def test_oracle_first_fit_property_and_bound(seed):
    rng = np.random.default_rng(seed)
    row_len = int(rng.integers(6, 15))
    lengths = [int(x) for x in rng.integers(1, row_len + 1, size=int(rng.integers(1, 8)))]
    off, n_rows = orc.ffd_pack(lengths, row_len)
    check_first_fit_by_replay(lengths, row_len, off, n_rows)
    opt = optimal_rows(lengths, row_len)
    assert opt <= n_rows <= (11 * opt + 6) // 9          # FFD <= 11/9 OPT + 6/9 (tight bound)
    # nothing overlaps, nothing crosses a row boundary, everything is placed
    used = np.zeros(n_rows * row_len, dtype=int)
    for L, o in zip(lengths, off):
        assert o >= 0 and o // row_len == (o + L - 1) // row_len
        used[o:o + L] += 1
    assert used.max() == 1 and used.sum() == sum(lengths)


def test_oracle_row_limit_leaves_units_out():
    lengths = [6, 6, 6, 3, 3, 1]
    off, n_rows = orc.ffd_pack(lengths, 10, max_rows=2)
    assert n_rows == 2
    check_first_fit_by_replay(lengths, 10, off, n_rows, max_rows=2)
    assert off.tolist() == [0, 10, -1, 6, 16, 9]


