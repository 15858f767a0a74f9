"""Pins for the oracle's masks and block classification (CPU only).

Nothing here calls the HIP path.  The mask functions are checked against the
explicit set description that follows from Algorithm 1 (a prompt or chosen
query sees every earlier token of its sample; a rejected query sees the prompt
and the earlier rejected tokens), against closed-form pair counts, and against
the paper's two ideal-speedup footnotes (Section 4.2).
"""
import itertools
import os

import numpy as np
import pytest

import psattn_workloads as W
from oracle import psattn_oracle as orc


def tri(n):
    return n * (n + 1) // 2


def explicit_allowed_set(o, p, c, r):
    """{(q, kv)} written out from the prose of Section 3.1, no boolean algebra."""
    C, R = o + p, o + p + c
    pairs = set()
    for q in range(o, o + p + c + r):
        if q < R:                       # prompt or chosen token: plain causal inside the sample
            keys = range(o, q + 1)
        else:                           # rejected token: prompt, then its own response
            keys = list(range(o, C)) + list(range(R, q + 1))
        for kv in keys:
            pairs.add((q, kv))
    return pairs


@pytest.mark.parametrize("p,c,r", list(itertools.product(range(5), repeat=3)))
def test_algorithm1_exhaustive(p, c, r):
    n = p + c + r
    if n == 0:
        return
    q = np.arange(n)[:, None]
    kv = np.arange(n)[None, :]
    m = orc.prefix_sharing_mask(q, kv, p, p + c)
    got = {(int(a), int(b)) for a, b in zip(*np.nonzero(m))}
    assert got == explicit_allowed_set(0, p, c, r)
    assert len(got) == tri(p) + c * p + tri(c) + r * p + tri(r)


@pytest.mark.parametrize("p,c,r", [(0, 0, 1), (3, 2, 2), (2, 0, 3), (0, 4, 1), (4, 1, 0), (1, 1, 1)])
def test_algorithm3_two_samples_and_padding(p, c, r):
    # [pad][sample A][pad pad][sample B = (2,3,1)][pad]
    samples = [(p, c, r), (2, 3, 1)]
    offs = [1, 1 + p + c + r + 2]
    T = offs[1] + 6 + 1
    Ic, Ir, D = orc.index_arrays(offs, [s[0] for s in samples], [s[1] for s in samples],
                                 [s[2] for s in samples], T)
    m = orc.dense_mask(Ic, Ir, D)
    got = {(int(a), int(b)) for a, b in zip(*np.nonzero(m))}
    want = set()
    for o, s in zip(offs, samples):
        want |= explicit_allowed_set(o, *s)
    assert got == want
    # padding rows and columns are empty
    pad = np.nonzero(D == orc.PAD_DOC)[0]
    assert not m[pad].any() and not m[:, pad].any()
    # inside one sample Algorithm 3 equals Algorithm 1 shifted by the offset
    o = offs[0]
    n = p + c + r
    q = np.arange(n)[:, None]
    kv = np.arange(n)[None, :]
    assert np.array_equal(m[o:o + n, o:o + n], orc.prefix_sharing_mask(q, kv, p, p + c))
    assert orc.count_allowed(Ic, Ir, D, stripe=3) == len(want)


def test_algorithm2_is_degenerate_case():
    """With chosen_len = rejected_len = 0 every document is one [prompt|response]
    unit and Algorithm 3 equals the response-id mask of Algorithm 2."""
    lens = [5, 3, 7, 1]
    offs = [0, 5, 9, 17]
    T = 20
    z = [0] * 4
    Ic, Ir, D = orc.index_arrays(offs, lens, z, z, T)
    R = orc.response_ids(offs, lens, z, z, T)
    q = np.arange(T)[:, None]
    kv = np.arange(T)[None, :]
    assert np.array_equal(orc.dense_mask(Ic, Ir, D), orc.response_id_mask(q, kv, R))


def test_config1_counts():
    w = W.make_workload("cfg1")
    Ic, Ir, D = orc.index_arrays(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    assert orc.count_allowed(Ic, Ir, D) == 11920
    pw, _, _ = W.paired_workload(w)
    Ic, Ir, D = orc.index_arrays(pw.offset, pw.prefix_len, pw.chosen_len, pw.rejected_len, pw.total_tokens)
    assert orc.count_allowed(Ic, Ir, D) == 16576 == tri(96 + 24) + tri(96 + 40)


@pytest.mark.parametrize("p,c", [(4096, 512), (2048, 2048), (8192, 256)])
def test_ideal_speedup_footnotes(p, c):
    """Section 4.2 footnotes: token ratio 2(p+c)/(p+2c) holds exactly at c = r;
    pair ratio tends to 2(p+c)^2 / (2(p+c)^2 - p^2) for long sequences."""
    r = c
    Ic, Ir, D = orc.index_arrays([0], [p], [c], [r], p + c + r)
    # count on a stripe sample would not be exact: use the full count (stripes keep memory small)
    shared = orc.count_allowed(Ic, Ir, D, stripe=512)
    assert shared == tri(p) + c * p + tri(c) + r * p + tri(r)
    paired = tri(p + c) + tri(p + r)
    ideal = 2 * (p + c) ** 2 / (2 * (p + c) ** 2 - p ** 2)
    assert abs(paired / shared - ideal) / ideal < 2e-3
    assert (2 * p + c + r) / (p + c + r) == pytest.approx(2 * (p + c) / (p + 2 * c), rel=1e-12)


def test_paired_mask_matches_shared_mask_through_src_map():
    """The paired format attends to exactly the same source tokens (Section 2.1):
    mapping paired tokens back to shared tokens reproduces the shared mask rows."""
    w = W.custom_workload([(5, 3, 4), (2, 0, 3), (0, 2, 2)], total_tokens=24)
    pw, src, dup = W.paired_workload(w)
    Ic, Ir, D = orc.index_arrays(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    pIc, pIr, pD = orc.index_arrays(pw.offset, pw.prefix_len, pw.chosen_len, pw.rejected_len, pw.total_tokens)
    ms = orc.dense_mask(Ic, Ir, D)
    mp = orc.dense_mask(pIc, pIr, pD)
    for t in range(pw.total_tokens):
        if src[t] < 0:
            assert not mp[t].any()
            continue
        keys_shared = set(np.nonzero(ms[src[t]])[0].tolist())
        keys_paired = set(src[np.nonzero(mp[t])[0]].tolist())
        assert keys_shared == keys_paired


# ---------------------------------------------------------------- block mask
def brute_tile_class(m, T, tq, tk, a, b):
    """Independent per-tile loop over the dense boolean matrix m."""
    q_lo, q_hi = a * tq, min(T, (a + 1) * tq)
    k_lo, k_hi = b * tk, min(T, (b + 1) * tk)
    n = 0
    for i in range(q_lo, q_hi):
        for j in range(k_lo, k_hi):
            n += bool(m[i, j])
    if n == 0:
        return orc.SKIPPED
    if (a + 1) * tq <= T and (b + 1) * tk <= T and n == tq * tk:
        return orc.FULL
    return orc.PARTIAL


@pytest.mark.parametrize("tile_q,tile_k", [(1, 1), (2, 3), (4, 4), (8, 4), (3, 8)])
def test_classify_small_grids(tile_q, tile_k):
    rng = np.random.default_rng(tile_q * 10 + tile_k)
    for _ in range(6):
        ns = int(rng.integers(1, 4))
        samples = [tuple(int(x) for x in rng.integers(0, 9, 3)) for _ in range(ns)]
        samples = [s if sum(s) else (1, 0, 0) for s in samples]
        offs, cur = [], int(rng.integers(0, 3))
        for s in samples:
            offs.append(cur)
            cur += sum(s) + int(rng.integers(0, 3))
        T = cur + int(rng.integers(0, 3))
        Ic, Ir, D = orc.index_arrays(offs, [s[0] for s in samples], [s[1] for s in samples],
                                     [s[2] for s in samples], T)
        m = orc.dense_mask(Ic, Ir, D)
        cls = orc.classify_tiles(Ic, Ir, D, tile_q, tile_k)
        for a in range(cls.shape[0]):
            for b in range(cls.shape[1]):
                assert cls[a, b] == brute_tile_class(m, T, tile_q, tile_k, a, b)
        row_ptr, idx, cl = orc.csr_q_major(cls)
        assert row_ptr[-1] == (cls != 0).sum() == len(idx) == len(cl)
        for a in range(cls.shape[0]):
            ks = idx[row_ptr[a]:row_ptr[a + 1]]
            assert np.all(np.diff(ks) > 0)
            assert np.array_equal(cl[row_ptr[a]:row_ptr[a + 1]], cls[a, ks])
        kp, qi, kc = orc.csr_k_major(cls)
        assert kp[-1] == row_ptr[-1]
        for b in range(cls.shape[1]):
            qs = qi[kp[b]:kp[b + 1]]
            assert np.array_equal(kc[kp[b]:kp[b + 1]], cls[qs, b])


def test_token_descriptors():
    offs, P, C, R = [1, 9], [3, 0], [2, 2], [2, 3]
    T = 15
    Ic, Ir, D = orc.index_arrays(offs, P, C, R, T)
    desc = orc.token_descriptors(Ic, Ir, D)
    m = orc.dense_mask(Ic, Ir, D)
    for i in range(T):
        s, lo, hi = (int(x) for x in desc[i])
        keys = {j for j in range(T) if j <= i and j >= s and not (lo <= j < hi)}
        assert keys == set(np.nonzero(m[i])[0].tolist())
    assert desc[0, 0] == orc.PAD_START and desc[8, 0] == orc.PAD_START
    assert tuple(desc[6]) == (1, 4, 6) and tuple(desc[3]) == (1, 0, 0)
    assert tuple(desc[11]) == (9, 9, 11)


def test_tile_counts_config2():
    """128 x 128 global grid on the second configuration: per-row allowed pair
    count from the tiles must add up to the closed-form total."""
    w = W.make_workload("cfg2")
    Ic, Ir, D = orc.index_arrays(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    cls = orc.classify_tiles(Ic, Ir, D, 128, 128)
    assert int((cls == orc.FULL).sum()) == 173 and int((cls == orc.PARTIAL).sum()) == 197
    p, c, r = (x.astype(np.int64) for x in (w.prefix_len, w.chosen_len, w.rejected_len))
    total = int((tri(p) + c * p + tri(c) + r * p + tri(r)).sum())
    assert total == 4263407
    T = w.total_tokens
    acc = 0
    for a, b in zip(*np.nonzero(cls)):
        acc += int(orc.dense_mask(Ic, Ir, D, a * 128, min(T, a * 128 + 128), b * 128, min(T, b * 128 + 128)).sum())
    assert acc == total


# ---- fixtures written out by hand / from the paper's printed formulas (tests/golden)
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _read_matrix(name):
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, name)) if ln.strip() and not ln.startswith("#")]
    return np.array(rows, dtype=np.int64).astype(bool)


def test_golden_mask_single_sequence():
    want = _read_matrix("mask_p3_c2_r2.txt")
    q = np.arange(7)[:, None]
    kv = np.arange(7)[None, :]
    assert np.array_equal(orc.prefix_sharing_mask(q, kv, 3, 5), want)
    Ic, Ir, D = orc.index_arrays([0], [3], [2], [2], 7)
    assert np.array_equal(orc.dense_mask(Ic, Ir, D), want)
    assert orc.count_allowed(Ic, Ir, D) == int(want.sum()) == 24  # 6 + 6 + 3 + 6 + 3


def test_golden_mask_packed_row_with_padding():
    want = _read_matrix("mask_packed_two_samples.txt")
    Ic, Ir, D = orc.index_arrays([0, 4], [2, 1], [1, 1], [1, 1], 8)
    assert np.array_equal(orc.dense_mask(Ic, Ir, D), want)
    assert orc.count_allowed(Ic, Ir, D) == int(want.sum())


def test_golden_ideal_speedups():
    for ln in open(os.path.join(GOLDEN, "ideal_speedups.txt")):
        if not ln.strip() or ln.startswith("#"):
            continue
        p, c, lin, quad = ln.split()
        p, c, lin, quad = int(p), int(c), float(lin), float(quad)
        # token counts: exact; pair counts: the formula is the limit for long sequences
        assert (2 * p + 2 * c) / (p + 2 * c) == pytest.approx(lin, rel=1e-9)
        shared = tri(p) + 2 * (c * p + tri(c))
        paired = 2 * tri(p + c)
        assert paired / shared == pytest.approx(quad, rel=4.0 / (p + c))
        if p + 2 * c <= 1536:  # the oracle's own count, where the dense mask is small
            Ic, Ir, D = orc.index_arrays([0], [p], [c], [c], p + 2 * c)
            assert orc.count_allowed(Ic, Ir, D) == shared
