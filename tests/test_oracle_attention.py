"""Pins for the oracle's forward and backward arithmetic (CPU only, fp64).

None of these call the HIP path.  They pin the oracle to: a pure-Python
evaluation of the definition, a library attention routine (torch CPU fp64) in
the textbook causal special case and with an explicit boolean mask, torch
autograd and central finite differences for the gradients, and the claims the
paper makes about the method: the computation equals the normal paired format
(Sections 2.1, 3.1) and packed samples do not contaminate each other
(Section 3.2).
"""
import math

import numpy as np
import pytest
import torch

import psattn_workloads as W
from oracle import psattn_oracle as orc


def arrays(w):
    return orc.index_arrays(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)


def rand_tensors(w, seed):
    rng = np.random.default_rng(seed)
    T, d = w.total_tokens, w.head_dim
    return (rng.standard_normal((T, w.n_q_heads, d)), rng.standard_normal((T, w.n_kv_heads, d)),
            rng.standard_normal((T, w.n_kv_heads, d)), rng.standard_normal((T, w.n_q_heads, d)))


TINY = W.custom_workload([(3, 2, 2), (2, 1, 3)], offsets=[0, 8], total_tokens=15, hq=2, hkv=1, d=4)


def explicit_keys(w, i):
    """Allowed keys of query i from the prose of Section 3.1 (independent of the oracle's mask)."""
    for o, p, c, r in zip(w.offset, w.prefix_len, w.chosen_len, w.rejected_len):
        o, p, c, r = int(o), int(p), int(c), int(r)
        if o <= i < o + p + c + r:
            if i < o + p + c:
                return list(range(o, i + 1))
            return list(range(o, o + p)) + list(range(o + p + c, i + 1))
    return []


def brute_forward(w, Q, K, V, scale):
    T, Hq, d = Q.shape
    G = Hq // K.shape[1]
    O = [[[0.0] * d for _ in range(Hq)] for _ in range(T)]
    LSE = [[-math.inf] * T for _ in range(Hq)]
    for h in range(Hq):
        g = h // G
        for i in range(T):
            keys = explicit_keys(w, i)
            if not keys:
                continue
            s = []
            for j in keys:
                acc = 0.0
                for x in range(d):
                    acc += Q[i, h, x] * K[j, g, x]
                s.append(scale * acc)
            m = max(s)
            e = [math.exp(v - m) for v in s]
            l = sum(e)
            LSE[h][i] = m + math.log(l)
            for x in range(d):
                O[i][h][x] = sum(e[n] / l * V[j, g, x] for n, j in enumerate(keys))
    return np.array(O), np.array(LSE)


def test_forward_brute_force_tiny():
    w = TINY
    Q, K, V, _ = rand_tensors(w, 1)
    Ic, Ir, D = arrays(w)
    O, LSE = orc.forward(Q, K, V, 0.5, Ic, Ir, D)
    Ob, Lb = brute_forward(w, Q, K, V, 0.5)
    assert np.allclose(O, Ob, rtol=0, atol=1e-13)
    real = D != orc.PAD_DOC
    assert np.allclose(LSE[:, real], Lb[:, real], rtol=0, atol=1e-13)
    assert np.all(np.isneginf(LSE[:, ~real])) and np.all(O[~real] == 0)
    # per-document evaluation equals the single T x T evaluation
    O2, LSE2 = orc.forward(Q, K, V, 0.5, Ic, Ir, D, flat=True)
    assert np.allclose(O, O2, rtol=0, atol=1e-14) and np.array_equal(np.isneginf(LSE), np.isneginf(LSE2))
    assert np.allclose(LSE[:, real], LSE2[:, real], rtol=0, atol=1e-14)
    # single rows against all earlier keys
    Or, Lr = orc.forward_rows(Q, K, V, 0.5, Ic, Ir, D, 1, [0, 6, 14])
    assert np.allclose(Or, O[[0, 6, 14], 1], atol=1e-14) and np.allclose(Lr[:2], LSE[1, [0, 6]], atol=1e-14)


def torch_sdpa(Q, K, V, scale, mask=None, causal=False, dO=None):
    """Library routine, fp64, one head: returns O (and grads when dO is given)."""
    q = torch.tensor(Q, dtype=torch.float64, requires_grad=dO is not None)[None, None]
    k = torch.tensor(K, dtype=torch.float64, requires_grad=dO is not None)[None, None]
    v = torch.tensor(V, dtype=torch.float64, requires_grad=dO is not None)[None, None]
    q, k, v = (x.detach().requires_grad_(dO is not None) for x in (q, k, v))
    am = None if mask is None else torch.tensor(mask)[None, None]
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=am, is_causal=causal, scale=scale)
    if dO is None:
        return o[0, 0].numpy()
    o.backward(torch.tensor(dO, dtype=torch.float64)[None, None])
    return o[0, 0].detach().numpy(), q.grad[0, 0].numpy(), k.grad[0, 0].numpy(), v.grad[0, 0].numpy()


def test_causal_special_case_matches_library():
    """chosen_len = rejected_len = 0 is textbook causal softmax attention."""
    w = W.custom_workload([(37, 0, 0)], hq=1, hkv=1, d=16)
    Q, K, V, dO = rand_tensors(w, 2)
    Ic, Ir, D = arrays(w)
    res = orc.backward(Q, K, V, dO, 0.25, Ic, Ir, D)
    o, dq, dk, dv = torch_sdpa(Q[:, 0], K[:, 0], V[:, 0], 0.25, causal=True, dO=dO[:, 0])
    assert np.allclose(res["O"][:, 0], o, atol=1e-12)
    assert np.allclose(res["dQ"][:, 0], dq, atol=1e-12)
    assert np.allclose(res["dK"][:, 0], dk, atol=1e-12)
    assert np.allclose(res["dV"][:, 0], dv, atol=1e-12)


def test_general_mask_matches_library_and_autograd():
    w = W.custom_workload([(9, 5, 7), (4, 6, 0), (0, 3, 5)], hq=1, hkv=1, d=8)
    Q, K, V, dO = rand_tensors(w, 3)
    Ic, Ir, D = arrays(w)
    res = orc.backward(Q, K, V, dO, 0.3, Ic, Ir, D)
    # the library gets the mask from the explicit set description, not from the oracle
    T = w.total_tokens
    mask = np.zeros((T, T), dtype=bool)
    for i in range(T):
        mask[i, explicit_keys(w, i)] = True
    o, dq, dk, dv = torch_sdpa(Q[:, 0], K[:, 0], V[:, 0], 0.3, mask=mask, dO=dO[:, 0])
    for name, ref in (("O", o), ("dQ", dq), ("dK", dk), ("dV", dv)):
        assert np.allclose(res[name][:, 0], ref, atol=1e-12), name
    # LSE from a library logsumexp
    S = torch.tensor(0.3 * Q[:, 0] @ K[:, 0].T).masked_fill(~torch.tensor(mask), -math.inf)
    assert np.allclose(res["LSE"][0], torch.logsumexp(S, dim=1).numpy(), atol=1e-12)


def test_gradients_finite_differences():
    w = TINY
    Q, K, V, dO = rand_tensors(w, 4)
    Ic, Ir, D = arrays(w)
    scale = 0.7
    res = orc.backward(Q, K, V, dO, scale, Ic, Ir, D)

    def loss(q, k, v):
        o, _ = orc.forward(q, k, v, scale, Ic, Ir, D)
        return float((o * dO).sum())

    eps = 1e-6
    rng = np.random.default_rng(0)
    for name, X in (("dQ", Q), ("dK", K), ("dV", V)):
        idxs = [tuple(int(rng.integers(0, s)) for s in X.shape) for _ in range(25)]
        # include positions that must be exactly zero (padding) and prompt keys
        idxs += [(7, 0, 0), (0, 0, 1), (8, 0, 2)]
        for idx in idxs:
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            args_p = {"dQ": (Xp, K, V), "dK": (Q, Xp, V), "dV": (Q, K, Xp)}[name]
            args_m = {"dQ": (Xm, K, V), "dK": (Q, Xm, V), "dV": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - res[name][idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx)
    assert np.all(res["dQ"][7] == 0) and np.all(res["dK"][7] == 0) and np.all(res["dV"][7] == 0)


def test_row_sums():
    w = W.custom_workload([(6, 4, 5)], hq=1, hkv=1, d=8)
    Q, K, V, dO = rand_tensors(w, 5)
    Ic, Ir, D = arrays(w)
    allowed = orc.dense_mask(Ic, Ir, D)
    P, _ = orc._softmax_block(Q[:, 0], K[:, 0], allowed, 0.4)
    assert np.allclose(P.sum(1), 1.0, atol=1e-14) and np.all(P[~allowed] == 0)
    o = P @ V[:, 0]
    delta = (dO[:, 0] * o).sum(1)
    dS = P * (dO[:, 0] @ V[:, 0].T - delta[:, None])
    assert np.allclose(dS.sum(1), 0.0, atol=1e-13)


@pytest.mark.parametrize("p,c,r", [(7, 4, 6), (0, 5, 3), (5, 0, 4), (6, 3, 0), (1, 1, 1)])
def test_no_contamination_invariant(p, c, r):
    """Outputs and gradients equal plain causal attention on [prompt|chosen]
    and on [prompt|rejected] run separately; the prompt's dK, dV are the sum of both."""
    w = W.custom_workload([(p, c, r)], hq=2, hkv=1, d=8)
    Q, K, V, dO = rand_tensors(w, 6)
    scale = 0.35
    Ic, Ir, D = arrays(w)
    S = orc.backward(Q, K, V, dO, scale, Ic, Ir, D)
    ia = np.arange(0, p + c)
    ib = np.concatenate([np.arange(0, p), np.arange(p + c, p + c + r)])
    out = {}
    for tag, idx, zero_prefix in (("A", ia, False), ("B", ib, True)):
        n = len(idx)
        wa = W.custom_workload([(n, 0, 0)], hq=2, hkv=1, d=8)
        a = orc.index_arrays(wa.offset, wa.prefix_len, wa.chosen_len, wa.rejected_len, n) if n else None
        dOx = dO[idx].copy()
        if zero_prefix:
            dOx[:p] = 0
        if n == 0:
            continue
        out[tag] = orc.backward(Q[idx], K[idx], V[idx], dOx, scale, *a)
    if "A" in out:
        A = out["A"]
        assert np.allclose(S["O"][ia], A["O"], atol=1e-12) and np.allclose(S["LSE"][:, ia], A["LSE"], atol=1e-12)
        assert np.allclose(S["dQ"][ia], A["dQ"] + (0 if "B" not in out else
                           np.concatenate([out["B"]["dQ"][:p], np.zeros((c,) + A["dQ"].shape[1:])])), atol=1e-12)
        assert np.allclose(S["dK"][p:p + c], A["dK"][p:], atol=1e-12)
        assert np.allclose(S["dV"][p:p + c], A["dV"][p:], atol=1e-12)
    if "B" in out:
        B = out["B"]
        assert np.allclose(S["O"][ib], B["O"], atol=1e-12) and np.allclose(S["LSE"][:, ib], B["LSE"], atol=1e-12)
        assert np.allclose(S["dQ"][p + c:], B["dQ"][p:], atol=1e-12)
        assert np.allclose(S["dK"][p + c:], B["dK"][p:], atol=1e-12)
        assert np.allclose(S["dV"][p + c:], B["dV"][p:], atol=1e-12)
    if "A" in out and "B" in out and p:
        assert np.allclose(S["dK"][:p], out["A"]["dK"][:p] + out["B"]["dK"][:p], atol=1e-12)
        assert np.allclose(S["dV"][:p], out["A"]["dV"][:p] + out["B"]["dV"][:p], atol=1e-12)
        # B's prompt queries got zero dO, so their dQ is zero and the sum above is A's alone
        assert np.all(out["B"]["dQ"][:p] == 0)


def test_packing_independence_and_padding():
    samples = [(5, 3, 4), (2, 6, 1), (4, 0, 3)]
    packed = W.custom_workload(samples, offsets=[2, 14, 26], total_tokens=36, hq=4, hkv=2, d=8)
    Q, K, V, dO = rand_tensors(packed, 7)
    Ic, Ir, D = arrays(packed)
    R = orc.backward(Q, K, V, dO, 0.3, Ic, Ir, D)
    for o, s in zip([2, 14, 26], samples):
        n = sum(s)
        alone = W.custom_workload([s], hq=4, hkv=2, d=8)
        a = arrays(alone)
        A = orc.backward(Q[o:o + n], K[o:o + n], V[o:o + n], dO[o:o + n], 0.3, *a)
        for name in ("O", "dQ", "dK", "dV"):
            assert np.allclose(R[name][o:o + n], A[name], atol=1e-13), name
        assert np.allclose(R["LSE"][:, o:o + n], A["LSE"], atol=1e-13)
    pad = D == orc.PAD_DOC
    for name in ("O", "dQ", "dK", "dV"):
        assert np.all(R[name][pad] == 0)
    # values stored at padding positions never leak
    Q2, K2, V2, dO2 = (x.copy() for x in (Q, K, V, dO))
    for x in (Q2, K2, V2, dO2):
        x[pad] = 1e6
    R2 = orc.backward(Q2, K2, V2, dO2, 0.3, Ic, Ir, D)
    for name in ("O", "dQ", "dK", "dV"):
        assert np.array_equal(R[name], R2[name])
    # subset evaluation equals the full one on the requested part
    Rs = orc.backward(Q, K, V, dO, 0.3, Ic, Ir, D, heads=[2, 3], samples=[1])
    assert np.allclose(Rs["dQ"][14:23, 2:], R["dQ"][14:23, 2:], atol=0) and np.all(Rs["dQ"][:, :2] == 0)
    assert np.allclose(Rs["dK"][14:23, 1], R["dK"][14:23, 1], atol=1e-15) and np.all(Rs["dK"][:, 0] == 0)


def test_swap_responses_symmetry():
    """Chosen and rejected are independent given the prompt: exchanging the two
    segments permutes the results."""
    p, c, r = 6, 3, 5
    w1 = W.custom_workload([(p, c, r)], hq=1, hkv=1, d=8)
    w2 = W.custom_workload([(p, r, c)], hq=1, hkv=1, d=8)
    Q, K, V, dO = rand_tensors(w1, 8)
    perm = np.concatenate([np.arange(p), np.arange(p + c, p + c + r), np.arange(p, p + c)])
    R1 = orc.backward(Q, K, V, dO, 0.3, *arrays(w1))
    R2 = orc.backward(Q[perm], K[perm], V[perm], dO[perm], 0.3, *arrays(w2))
    for name in ("O", "dQ", "dK", "dV"):
        assert np.allclose(R1[name][perm], R2[name], atol=1e-13), name


def test_metamorphic_shift_and_scale():
    w = W.custom_workload([(5, 4, 3), (3, 2, 2)], hq=1, hkv=1, d=8)
    Q, K, V, _ = rand_tensors(w, 9)
    a = arrays(w)
    O, LSE = orc.forward(Q, K, V, 0.3, *a)
    # adding one vector u to every key of a document shifts each row's scores by a constant
    u = np.random.default_rng(1).standard_normal(8)
    K2 = K.copy()
    K2[:12, 0] += u
    O2, LSE2 = orc.forward(Q, K2, V, 0.3, *a)
    assert np.allclose(O, O2, atol=1e-12)
    assert np.allclose(LSE2[0, :12] - LSE[0, :12], 0.3 * Q[:12, 0] @ u, atol=1e-12)
    O3, _ = orc.forward(Q, K, 2.5 * V, 0.3, *a)
    assert np.allclose(O3, 2.5 * O, atol=1e-12)


def test_gqa_equals_repeated_kv():
    w = W.custom_workload([(5, 3, 4), (2, 2, 2)], hq=6, hkv=2, d=8)
    Q, K, V, dO = rand_tensors(w, 10)
    a = arrays(w)
    R = orc.backward(Q, K, V, dO, 0.3, *a)
    Kr, Vr = np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1)
    E = orc.backward(Q, Kr, Vr, dO, 0.3, *a)
    assert np.allclose(R["O"], E["O"], atol=1e-14) and np.allclose(R["dQ"], E["dQ"], atol=1e-14)
    T = w.total_tokens
    assert np.allclose(R["dK"], E["dK"].reshape(T, 2, 3, 8).sum(2), atol=1e-13)
    assert np.allclose(R["dV"], E["dV"].reshape(T, 2, 3, 8).sum(2), atol=1e-13)
