"""Per-response log-probabilities, their backward and the DPO loss on the GPU (through the C ABI)
against the oracle.  fp32 logits: log-probabilities within 1e-4 absolute of the fp64 oracle per
response (sums of up to a few hundred fp32 terms), gradients within 1e-6; bf16 logits: the same
forward bar (inputs are exact bf16 numbers, accumulation is fp32), gradient elements within half
a bf16 ulp + 1e-6."""
import numpy as np
import pytest

import paper_2410_20305_amd as ps
import psattn_workloads as W
from oracle import psattn_oracle as orc

pytestmark = pytest.mark.gpu

CASES = {
    # off, P, ptr, rl, T, V
    "two_responses_packed": ([3, 60], [20, 7], [0, 2, 4], [9, 14, 5, 11], 100, 1000),
    "multi_and_empty": ([0, 30, 50], [5, 0, 4], [0, 3, 5, 5], [4, 0, 6, 3, 2], 60, 257),   # vocab not a multiple of 8
    "single_token_responses": ([1], [2], [0, 2], [1, 1], 6, 64),
}


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", sorted(CASES))
def test_logprob_forward_backward(case, dtype):
    import torch
    off, P, ptr, rl, T, V = CASES[case]
    rng = np.random.default_rng(301)
    logits = (rng.standard_normal((T, V)) * 3).astype(np.float32)
    if dtype == "bf16":
        logits = W.bf16_round(logits)
    ids = rng.integers(0, V, size=T).astype(np.int32)
    ids[off[0] + P[0]:off[0] + P[0] + 1] = ids[off[0] + P[0] + rl[0]] if rl[0] and rl[1] else ids[off[0] + P[0]]  # two responses may start alike
    d_logp = rng.standard_normal(len(rl)).astype(np.float32)
    plan = ps.LogprobPlan(off, P, ptr, rl, T)
    items = orc.prediction_items(off, P, ptr, rl)
    assert plan.n_responses == len(rl) and plan.n_items == len(items)
    assert plan.n_rows == len({r for _, r, _ in items})
    dev = lambda x, dt=None: torch.from_numpy(x).to("cuda") if dt is None else torch.from_numpy(x).to("cuda").to(dt)
    lg = dev(logits, torch.bfloat16 if dtype == "bf16" else torch.float32)
    tid = dev(ids)
    row_lse, logp = ps.psattn_logprob_fwd(plan, lg, tid)
    dlog = torch.full_like(lg, float("nan"))
    ps.psattn_logprob_bwd(plan, lg, tid, row_lse, dev(d_logp), dlogits=dlog)
    torch.cuda.synchronize()
    ref = orc.response_logprobs(logits, ids, off, P, ptr, rl)
    assert np.abs(logp.cpu().numpy().astype(np.float64) - ref).max() <= 1e-4
    gref = orc.response_logprobs_grad(logits, ids, off, P, ptr, rl, d_logp.astype(np.float64))
    got = dlog.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    silent = np.abs(gref).sum(axis=1) == 0
    assert np.all(got[silent] == 0)                                   # rows that predict nothing: exact zeros
    tol = 1e-6 if dtype == "f32" else 2.0 ** -8 * np.abs(gref) + 1e-6   # half a bf16 ulp (8 significant bits)
    excess = float((np.abs(got - gref) - tol).max())
    assert excess <= 0, excess
    plan.free()


@pytest.mark.parametrize("sample", [0, 9])
def test_logprob_config5_vocab32000_sampled(sample):
    """Full size, the launch configuration bench.py times as `logprob_head`: config 5's sample table, bf16
    logits [65 536, 32 000] drawn on the device, both responses of one sample against the oracle.  A response's
    log-probability and the gradient rows of its sample depend on that sample's rows only, so the oracle runs
    on those rows (read back from the device) as a one-sample problem."""
    import torch
    w = W.make_workload("cfg5")
    T, V = w.total_tokens, 32000
    ptr = 2 * np.arange(w.n_samples + 1)
    rl = np.stack([w.chosen_len, w.rejected_len], axis=1).reshape(-1)
    plan = ps.LogprobPlan(w.offset, w.prefix_len, ptr, rl, T)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3050)
    lg = torch.empty((T, V), dtype=torch.bfloat16, device="cuda")
    for t0 in range(0, T, 8192):   # in pieces: the fp32 draw of the whole buffer would be 8 GB
        lg[t0:t0 + 8192] = (torch.randn((min(8192, T - t0), V), generator=gen, device="cuda") * 3).to(torch.bfloat16)
    tid = torch.randint(0, V, (T,), generator=gen, device="cuda", dtype=torch.int32)
    d_logp = torch.randn(len(rl), generator=gen, device="cuda")
    row_lse, logp = ps.psattn_logprob_fwd(plan, lg, tid)
    dlog = torch.full_like(lg, float("nan"))
    ps.psattn_logprob_bwd(plan, lg, tid, row_lse, d_logp, dlogits=dlog)
    torch.cuda.synchronize()
    o, p, c, r = (int(x[sample]) for x in (w.offset, w.prefix_len, w.chosen_len, w.rejected_len))
    n = p + c + r
    sub_logits = lg[o:o + n].float().cpu().numpy()
    sub_ids = tid[o:o + n].cpu().numpy()
    sub_d = d_logp[2 * sample:2 * sample + 2].cpu().numpy().astype(np.float64)
    ref = orc.response_logprobs(sub_logits, sub_ids, [0], [p], [0, 2], [c, r])
    got = logp[2 * sample:2 * sample + 2].cpu().numpy().astype(np.float64)
    # sums of up to a thousand fp32 terms of magnitude ~10: 1e-4 relative to the sum
    assert np.abs(got - ref).max() <= 1e-4 * max(1.0, float(np.abs(ref).max())), (got, ref)
    gref = orc.response_logprobs_grad(sub_logits, sub_ids, [0], [p], [0, 2], [c, r], sub_d)
    ggot = dlog[o:o + n].float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(ggot))
    silent = np.abs(gref).sum(axis=1) == 0
    assert np.all(ggot[silent] == 0)
    excess = float((np.abs(ggot - gref) - (2.0 ** -8 * np.abs(gref) + 1e-6)).max())
    assert excess <= 0, excess
    plan.free()


def test_dpo_loss_matches_oracle():
    import torch
    rng = np.random.default_rng(302)
    lp = (rng.standard_normal(10) * 20 - 100).astype(np.float32)
    lr = (lp + rng.standard_normal(10) * 5).astype(np.float32)
    loss, d = ps.psattn_dpo_loss(torch.from_numpy(lp).cuda(), torch.from_numpy(lr).cuda(), 0.1)
    ref_loss, ref_d = orc.dpo_loss(lp, lr, 0.1)
    assert np.abs(loss.cpu().numpy() - ref_loss).max() <= 1e-5
    assert np.abs(d.cpu().numpy() - ref_d).max() <= 1e-6
    same, _ = ps.psattn_dpo_loss(torch.from_numpy(lp).cuda(), torch.from_numpy(lp).cuda(), 0.7)
    assert np.abs(same.cpu().numpy() - np.log(2.0)).max() <= 1e-6   # policy == reference


def test_logprob_no_responses_and_no_samples():
    """Samples without responses predict nothing: every gradient row is zero; an empty table is accepted."""
    import torch
    plan = ps.LogprobPlan([0, 6], [4, 3], [0, 0, 0], [], 10)
    assert plan.n_responses == 0 and plan.n_rows == 0 and plan.n_items == 0
    lg = torch.randn((10, 32), device="cuda")
    tid = torch.zeros(10, dtype=torch.int32, device="cuda")
    row_lse, logp = ps.psattn_logprob_fwd(plan, lg, tid)
    g = torch.full_like(lg, float("nan"))
    ps.psattn_logprob_bwd(plan, lg, tid, row_lse, logp, dlogits=g)
    torch.cuda.synchronize()
    assert logp.numel() == 0 and float(g.abs().max()) == 0
    empty = ps.LogprobPlan([], [], [0], [], 4)
    assert empty.n_responses == 0


def test_logprob_errors():
    with pytest.raises(ps.PsattnError) as e:
        ps.LogprobPlan([0], [3], [0, 2], [2, 9], 8)                   # 14 tokens in a buffer of 8
    assert e.value.status == -3
    with pytest.raises(ps.PsattnError) as e:
        ps.LogprobPlan([0, 2], [3, 1], [0, 1, 2], [2, 2], 20)         # overlap
    assert e.value.status == -2
