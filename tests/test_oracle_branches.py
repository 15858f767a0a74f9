"""Pins for the oracle's mask with any number of responses per prompt (the tree-mask reading
of Section 2.2: prompt = trunk, responses = branches).  CPU only; nothing calls the library.

The mask is checked against an explicit set description, against the separately pinned
two-response mask, against plain causal attention (one response), and through the
no-contamination invariant: every response's outputs and gradients equal ordinary causal
attention on [prompt | that response] alone, the prompt's dK/dV being the sum over responses.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import psattn_oracle as orc


def tri(n):
    return n * (n + 1) // 2


def explicit_pairs(o, p, resps):
    """{(q, kv)} written out: a prompt token reads the prompt up to itself; a token of a
    response reads the whole prompt and its own response up to itself."""
    pairs = set()
    for q in range(o, o + p):
        pairs |= {(q, kv) for kv in range(o, q + 1)}
    start = o + p
    for n in resps:
        for q in range(start, start + n):
            pairs |= {(q, kv) for kv in range(o, o + p)} | {(q, kv) for kv in range(start, q + 1)}
        start += n
    return pairs


@pytest.mark.parametrize("p,resps", [(p, r) for p in range(3) for k in range(4)
                                     for r in itertools.product(range(3), repeat=k)])
def test_branch_mask_exhaustive(p, resps):
    n = p + sum(resps)
    if n == 0:
        return
    D, B = orc.branch_arrays([1], [p], [0, len(resps)], list(resps), n + 3)
    m = orc.dense_branch_mask(D, B)
    got = {(int(a), int(b)) for a, b in zip(*np.nonzero(m))}
    assert got == explicit_pairs(1, p, resps)
    assert len(got) == tri(p) + sum(r * p + tri(r) for r in resps)


@pytest.mark.parametrize("p,c,r", [(3, 2, 2), (0, 4, 1), (5, 0, 3), (4, 3, 0), (1, 1, 1)])
def test_two_branches_equal_the_two_response_mask(p, c, r):
    offs, T = [2, 2 + p + c + r + 1], 2 * (p + c + r) + 5
    Ic, Ir, D2 = orc.index_arrays(offs, [p, p], [c, c], [r, r], T)
    D, B = orc.branch_arrays(offs, [p, p], [0, 2, 4], [c, r, c, r], T)
    assert np.array_equal(D, D2)
    assert np.array_equal(orc.dense_branch_mask(D, B), orc.dense_mask(Ic, Ir, D2))
    assert np.array_equal(orc.branch_token_descriptors(D, B), orc.token_descriptors(Ic, Ir, D2))
    ref = orc.classify_tiles(Ic, Ir, D2, 4, 3)
    assert np.array_equal(orc.classify_tiles(None, None, D, 4, 3, mask=lambda *a: orc.dense_branch_mask(D, B, *a)), ref)


def test_one_branch_is_plain_causal():
    D, B = orc.branch_arrays([0, 9], [4, 0], [0, 1, 2], [5, 6], 16)
    m = orc.dense_branch_mask(D, B)
    q = np.arange(16)[:, None]
    kv = np.arange(16)[None, :]
    want = (kv <= q) & (D[q] == D[kv]) & (D[q] >= 0)
    assert np.array_equal(m, want)


def test_descriptors_reproduce_the_mask():
    """allowed(q, kv) == (s_q <= kv <= q and not hole_lo_q <= kv < hole_hi_q)."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        k = int(rng.integers(0, 5))
        p = int(rng.integers(0, 5))
        resps = [int(x) for x in rng.integers(0, 4, size=k)]
        if p + sum(resps) == 0:
            continue
        o = int(rng.integers(0, 3))
        T = o + p + sum(resps) + int(rng.integers(0, 3))
        D, B = orc.branch_arrays([o], [p], [0, k], resps, T)
        desc = orc.branch_token_descriptors(D, B).astype(np.int64)
        q = np.arange(T)[:, None]
        kv = np.arange(T)[None, :]
        from_desc = (kv >= desc[:, 0:1]) & (kv <= q) & ~((kv >= desc[:, 1:2]) & (kv < desc[:, 2:3]))
        assert np.array_equal(from_desc, orc.dense_branch_mask(D, B))


def test_no_contamination_with_four_responses():
    """Forward and backward over [prompt | r1 | r2 | r3 | r4] against torch's plain causal
    attention on each [prompt | r_j] alone; the prompt's dK/dV are the sums."""
    rng = np.random.default_rng(7)
    p, resps, d = 5, [3, 1, 4, 2], 8
    n = p + sum(resps)
    Q, K, V, dO = (rng.standard_normal((n, 1, d)) for _ in range(4))
    D, B = orc.branch_arrays([0], [p], [0, 4], resps, n)
    mask = lambda *a: orc.dense_branch_mask(D, B, *a)
    scale = 0.37
    got = orc.backward(Q, K, V, dO, scale, None, None, D, mask=mask)
    dK_prompt = np.zeros((p, d))
    dV_prompt = np.zeros((p, d))
    start = p
    for j, nr in enumerate(resps):
        idx = list(range(p)) + list(range(start, start + nr))
        t = lambda x: torch.tensor(x[idx, 0][None, None], dtype=torch.float64, requires_grad=True)
        q, k, v = t(Q), t(K), t(V)
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=scale)
        g = dO[idx, 0].copy()
        if j > 0:
            g[:p] = 0.0                      # the prompt's own output gradient is counted once
        o.backward(torch.tensor(g[None, None]))
        o = o.detach().numpy()[0, 0]
        rows = list(range(start, start + nr))
        assert np.abs(got["O"][rows, 0] - o[p:]).max() < 1e-12
        assert np.abs(got["dQ"][rows, 0] - q.grad.numpy()[0, 0][p:]).max() < 1e-12
        assert np.abs(got["dK"][rows, 0] - k.grad.numpy()[0, 0][p:]).max() < 1e-12
        assert np.abs(got["dV"][rows, 0] - v.grad.numpy()[0, 0][p:]).max() < 1e-12
        if j == 0:
            assert np.abs(got["O"][:p, 0] - o[:p]).max() < 1e-12
            assert np.abs(got["dQ"][:p, 0] - q.grad.numpy()[0, 0][:p]).max() < 1e-12
        dK_prompt += k.grad.numpy()[0, 0][:p]
        dV_prompt += v.grad.numpy()[0, 0][:p]
        start += nr
    assert np.abs(got["dK"][:p, 0] - dK_prompt).max() < 1e-12
    assert np.abs(got["dV"][:p, 0] - dV_prompt).max() < 1e-12
