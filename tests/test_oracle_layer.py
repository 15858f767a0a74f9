"""Pin for the oracle's attention layer: the same layer built from torch operations in fp64
(linear, complex-number rotary embedding, scaled_dot_product_attention with an explicit boolean
mask written from the prose of Section 3.1) and differentiated by autograd.  CPU only."""
import numpy as np
import torch

from oracle import psattn_oracle as orc


def test_layer_matches_torch_autograd():
    rng = np.random.default_rng(0)
    hidden, Hq, Hkv, d, theta, scale = 12, 4, 2, 8, 30.0, 0.4
    off, P, ptr, rl, T = [1, 12], [3, 2], [0, 2, 5], [2, 4, 1, 2, 2], 20
    D, B = orc.branch_arrays(off, P, ptr, rl, T)
    X, dY = rng.standard_normal((T, hidden)), rng.standard_normal((T, hidden))
    Wq, Wo = rng.standard_normal((Hq * d, hidden)), rng.standard_normal((hidden, Hq * d))
    Wk, Wv = rng.standard_normal((Hkv * d, hidden)), rng.standard_normal((Hkv * d, hidden))
    got = orc.layer_backward(X, Wq, Wk, Wv, Wo, dY, scale, theta, D, B, lambda *a: orc.dense_branch_mask(D, B, *a), Hq, Hkv)

    # torch side: mask from the prose (own sample, not later, prompt or own response), ordinary tensors
    allowed = torch.zeros((T, T), dtype=torch.bool)
    pos = torch.zeros(T, dtype=torch.float64)
    for i, o in enumerate(off):
        p = P[i]
        branches = [(o, o + p)]
        t = o + p
        for n in rl[ptr[i]:ptr[i + 1]]:
            branches.append((t, t + n))
            t += n
        for bi, (lo, hi) in enumerate(branches):
            for q in range(lo, hi):
                pos[q] = q - lo if bi == 0 else p + (q - lo)
                allowed[q, o:o + p] = True if bi > 0 else False
                allowed[q, lo:q + 1] = True
    tt = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    x, wq, wk, wv, wo = tt(X), tt(Wq), tt(Wk), tt(Wv), tt(Wo)
    i = torch.arange(d // 2, dtype=torch.float64)
    rot = torch.polar(torch.ones(T, d // 2, dtype=torch.float64), pos[:, None] * theta ** (-2.0 * i / d)[None, :])

    def rope(z):  # [T, H, d]
        c = torch.complex(z[..., :d // 2], z[..., d // 2:]) * rot[:, None, :]
        return torch.cat([c.real, c.imag], dim=-1)
    q = rope((x @ wq.T).reshape(T, Hq, d)).permute(1, 0, 2)
    k = rope((x @ wk.T).reshape(T, Hkv, d)).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)
    v = (x @ wv.T).reshape(T, Hkv, d).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)
    real = torch.tensor(D >= 0)
    m = allowed.clone()
    m[~real] = True                         # padding rows: avoid an all-masked softmax, zeroed below
    o = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], attn_mask=m[None, None], scale=scale)[0]
    o = o.permute(1, 0, 2).reshape(T, Hq * d) * real[:, None]
    y = o @ wo.T
    y.backward(torch.tensor(dY))
    assert np.abs(got["Y"] - y.detach().numpy()).max() < 1e-10
    for name, t in (("dX", x), ("dWq", wq), ("dWk", wk), ("dWv", wv), ("dWo", wo)):
        assert np.abs(got[name] - t.grad.numpy()).max() < 1e-9, name
