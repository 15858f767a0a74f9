"""Pins for the oracle's per-response log-probabilities and DPO loss (Section 2.1, Eq. 1).
CPU only.  The log-probabilities in the prefix-shared sequence must equal what the paired
format gives: torch's cross entropy over [prompt | response] with next-token targets."""
import numpy as np
import pytest
import torch

from oracle import psattn_oracle as orc


def paired_logprob(logits_rows, ids):
    """Sum of next-token log-probabilities of ids[1:] given logits rows of ids[:-1] (torch)."""
    x = torch.tensor(logits_rows[:-1], dtype=torch.float64)
    y = torch.tensor(ids[1:], dtype=torch.long)
    return -float(torch.nn.functional.cross_entropy(x, y, reduction="none").sum())


def test_logprobs_equal_the_paired_format():
    rng = np.random.default_rng(0)
    V, p, resps = 11, 4, [3, 1, 5]
    n = p + sum(resps)
    off = 2
    T = off + n + 1
    logits = rng.standard_normal((T, V))
    ids = rng.integers(0, V, size=T)
    got = orc.response_logprobs(logits, ids, [off], [p], [0, len(resps)], resps)
    start = off + p
    for j, nr in enumerate(resps):
        rows = list(range(off, off + p)) + list(range(start, start + nr))
        full = paired_logprob(logits[rows], ids[rows])
        prompt_only = paired_logprob(logits[rows[:p]], ids[rows[:p]])
        assert abs(got[j] - (full - prompt_only)) < 1e-10      # log pi(y | x) = log pi(x, y) - log pi(x)
        start += nr


def test_uniform_logits_closed_form():
    V = 7
    logits = np.zeros((12, V))
    ids = np.arange(12) % V
    got = orc.response_logprobs(logits, ids, [0, 6], [2, 0], [0, 2, 3], [3, 1, 4])
    # every predicted token costs log V; the response behind an empty prompt loses its first token
    assert np.allclose(got, [-3 * np.log(V), -1 * np.log(V), -3 * np.log(V)])
    assert len(orc.prediction_items([0, 6], [2, 0], [0, 2, 3], [3, 1, 4])) == 3 + 1 + 3


def test_logprob_gradient_matches_autograd():
    rng = np.random.default_rng(1)
    V, off, p, resps = 9, 1, 3, [2, 4]
    T = off + p + sum(resps) + 2
    logits = rng.standard_normal((T, V))
    ids = rng.integers(0, V, size=T)
    d_logp = rng.standard_normal(2)
    g = orc.response_logprobs_grad(logits, ids, [off], [p], [0, 2], resps, d_logp)
    x = torch.tensor(logits, dtype=torch.float64, requires_grad=True)
    ls = torch.log_softmax(x, dim=-1)
    total = 0.0
    for j, row, tpos in orc.prediction_items([off], [p], [0, 2], resps):
        total = total + d_logp[j] * ls[row, int(ids[tpos])]
    total.backward()
    assert np.abs(g - x.grad.numpy()).max() < 1e-12
    # the last prompt row predicts the first token of both responses; rows that predict nothing are zero
    assert np.count_nonzero(np.abs(g).sum(axis=1)) == 1 + (2 - 1) + (4 - 1)


def test_dpo_loss_values_and_gradient():
    loss, d = orc.dpo_loss([-5.0, -7.0], [-5.0, -7.0], beta=0.1)
    assert abs(loss[0] - np.log(2.0)) < 1e-15                 # policy == reference: -log sigmoid(0)
    assert np.allclose(d, [-0.05, 0.05])
    rng = np.random.default_rng(2)
    lp, lr = rng.standard_normal(6) * 3, rng.standard_normal(6) * 3
    loss, d = orc.dpo_loss(lp, lr, beta=0.3)
    t = torch.tensor(lp, dtype=torch.float64, requires_grad=True)
    r = torch.tensor(lr, dtype=torch.float64)
    z = 0.3 * ((t[0::2] - r[0::2]) - (t[1::2] - r[1::2]))
    L = -torch.nn.functional.logsigmoid(z)
    L.sum().backward()
    assert np.abs(loss - L.detach().numpy()).max() < 1e-12 and np.abs(d - t.grad.numpy()).max() < 1e-12
