"""Pins for the oracle's rotary embedding and position ids (Section 3.1: position ids are set
so that each response sits where it would in the paired format).  CPU only."""
import numpy as np
import pytest
import torch

from oracle import psattn_oracle as orc


def test_position_ids_restart_behind_the_prompt():
    # [pad][p=3 | 2 | 4 | 1][pad][p=0 | 2]
    D, B = orc.branch_arrays([1, 12], [3, 0], [0, 3, 4], [2, 4, 1, 2], 15)
    assert orc.position_ids(D, B).tolist() == [0, 0, 1, 2, 3, 4, 3, 4, 5, 6, 3, 0, 0, 1, 0]


def test_rotation_equals_explicit_2x2_matrices():
    """Every pair (i, i + d/2) of every token is multiplied by [[cos, -sin], [sin, cos]] of
    pos * theta^(-2i/d), written out element by element."""
    rng = np.random.default_rng(0)
    T, H, d, theta = 5, 2, 8, 100.0
    x = rng.standard_normal((T, H, d))
    pos = np.array([0, 1, 7, 3, 1000])
    got = orc.rope_rotate(x, pos, theta)
    for t in range(T):
        for h in range(H):
            for i in range(d // 2):
                a = float(pos[t]) * theta ** (-2.0 * i / d)
                R = np.array([[np.cos(a), -np.sin(a)], [np.sin(a), np.cos(a)]])
                want = R @ np.array([x[t, h, i], x[t, h, i + d // 2]])
                assert abs(got[t, h, i] - want[0]) < 1e-12 and abs(got[t, h, i + d // 2] - want[1]) < 1e-12
    assert np.array_equal(got[0], x[0])                                    # position 0: identity
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    assert np.allclose(orc.rope_rotate(got, pos, theta, inverse=True), x, atol=1e-12)


def test_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    base = None
    for shift in (0, 5, 123):
        s = float((orc.rope_rotate(q, [9 + shift], 10000.0) * orc.rope_rotate(k, [4 + shift], 10000.0)).sum())
        base = s if base is None else base
        assert abs(s - base) < 1e-10


def causal_reference(Qs, Ks, Vs, dOs, scale, theta):
    """Plain causal attention over one [prompt | response] sequence with ordinary positions
    0 .. n-1, via torch (complex-number rotary embedding, autograd)."""
    n, d = Qs.shape
    i = torch.arange(d // 2, dtype=torch.float64)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * theta ** (-2.0 * i / d)[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)

    def rope(x):  # pair (i, i + d/2) as one complex number
        z = torch.complex(x[:, :d // 2], x[:, d // 2:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)
    q, k, v = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (Qs, Ks, Vs))
    o = torch.nn.functional.scaled_dot_product_attention(rope(q)[None, None], rope(k)[None, None], v[None, None],
                                                         is_causal=True, scale=scale)[0, 0]
    o.backward(torch.tensor(dOs))
    return o.detach().numpy(), q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


@pytest.mark.parametrize("resps", [[3, 4], [2, 1, 5]])
def test_shared_prefix_with_reset_positions_equals_paired_format(resps):
    """Outputs and gradients of every response equal ordinary causal attention with ordinary
    rotary positions on [prompt | that response] alone; the prompt's dK (w.r.t. the unrotated
    K) and dV are the sums over the responses."""
    rng = np.random.default_rng(2)
    p, d, theta, scale = 4, 8, 50.0, 0.41
    n = p + sum(resps)
    Q, K, V, dO = (rng.standard_normal((n, 1, d)) for _ in range(4))
    D, B = orc.branch_arrays([0], [p], [0, len(resps)], resps, n)
    got = orc.backward_rope(Q, K, V, dO, scale, theta, D, B, lambda *a: orc.dense_branch_mask(D, B, *a))
    dKp, dVp = np.zeros((p, d)), np.zeros((p, d))
    start = p
    for j, nr in enumerate(resps):
        idx = list(range(p)) + list(range(start, start + nr))
        g = dO[idx, 0].copy()
        if j > 0:
            g[:p] = 0.0
        o, dq, dk, dv = causal_reference(Q[idx, 0], K[idx, 0], V[idx, 0], g, scale, theta)
        rows = list(range(start, start + nr))
        for name, ref in (("O", o), ("dQ", dq), ("dK", dk), ("dV", dv)):
            assert np.abs(got[name][rows, 0] - ref[p:]).max() < 1e-11, name
        if j == 0:
            assert np.abs(got["O"][:p, 0] - o[:p]).max() < 1e-11 and np.abs(got["dQ"][:p, 0] - dq[:p]).max() < 1e-11
        dKp += dk[:p]
        dVp += dv[:p]
        start += nr
    assert np.abs(got["dK"][:p, 0] - dKp).max() < 1e-11 and np.abs(got["dV"][:p, 0] - dVp).max() < 1e-11


def test_rope_gradients_by_finite_differences():
    rng = np.random.default_rng(3)
    p, resps, d, theta, scale = 2, [2, 3], 4, 20.0, 0.5
    n = p + sum(resps)
    Q, K, V, dO = (rng.standard_normal((n, 1, d)) for _ in range(4))
    D, B = orc.branch_arrays([0], [p], [0, 2], resps, n)
    mask = lambda *a: orc.dense_branch_mask(D, B, *a)
    got = orc.backward_rope(Q, K, V, dO, scale, theta, D, B, mask)

    def loss(Q_, K_):
        return float((orc.backward_rope(Q_, K_, V, dO, scale, theta, D, B, mask)["O"] * dO).sum())
    eps = 1e-6
    for name, X in (("dQ", Q), ("dK", K)):
        for t in range(n):
            for x in range(d):
                Xp, Xm = X.copy(), X.copy()
                Xp[t, 0, x] += eps
                Xm[t, 0, x] -= eps
                fd = (loss(Xp, K) - loss(Xm, K)) / (2 * eps) if name == "dQ" else (loss(Q, Xp) - loss(Q, Xm)) / (2 * eps)
                assert abs(fd - got[name][t, 0, x]) < 1e-6 * max(1.0, abs(fd))
