"""Rotary embedding inside the attention op (psattn_fwd_rope / psattn_bwd_rope) against the
oracle: position ids, the rotated operands, forward outputs and the gradients with respect to
the UNROTATED Q and K.  The oracle rotates in fp64 and rounds the rotated Q, K to bfloat16 (the
format in which a bf16 model stores them), then runs its ordinary dense attention."""
import numpy as np
import pytest

import paper_2410_20305_amd as ps
import psattn_workloads as W
from oracle import psattn_oracle as orc


def two_response_tables(w):
    ptr = 2 * np.arange(w.n_samples + 1)
    rl = np.stack([w.chosen_len, w.rejected_len], axis=1).reshape(-1) if w.n_samples else np.zeros(0, np.int32)
    return ptr, rl


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4"])
def test_position_ids_match_oracle(name):
    """CPU: position ids derived from the block mask's descriptors == the oracle's definition."""
    w = W.make_workload(name)
    m = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens, host_only=True)
    ptr, rl = two_response_tables(w)
    D, B = orc.branch_arrays(w.offset, w.prefix_len, ptr, rl, w.total_tokens)
    pos, n_pos = m.positions()
    ref = orc.position_ids(D, B)
    assert np.array_equal(pos, ref)
    assert n_pos == int(ref.max()) + 1


def test_position_ids_multi_response():
    off, P, ptr, rl, T = [2, 40], [5, 0], [0, 3, 5], [4, 0, 6, 3, 2], 50
    m = ps.psattn_build_meta_multi(off, P, ptr, rl, T, host_only=True)
    D, B = orc.branch_arrays(off, P, ptr, rl, T)
    pos, n_pos = m.positions()
    assert np.array_equal(pos, orc.position_ids(D, B)) and n_pos == 11


def run_rope_case(off, P, ptr, rl, T, hq, hkv, theta, seed, max_positions=None):
    import torch
    from gpu_util import (BF16_LSE_TOL, check_grad, check_o, check_padding_zero, dq_delta_floor, to_dev, to_np)
    d = 128
    rng = np.random.default_rng(seed)
    tens = {n: W.bf16_round(rng.standard_normal((T, h, d), dtype=np.float32))
            for n, h in (("Q", hq), ("K", hkv), ("V", hkv), ("dO", hq))}
    scale = 1.0 / np.sqrt(d)
    meta = ps.psattn_build_meta_multi(off, P, ptr, rl, T)
    n_pos = meta.positions()[1]
    rope = ps.Rope(d, theta, max_positions or n_pos)
    Q, K, V, dO = (to_dev(tens[n], "bf16") for n in ("Q", "K", "V", "dO"))
    nan = lambda x: torch.full_like(x, float("nan"))
    O, Qr, Kr = nan(Q), nan(Q), nan(K)
    LSE = torch.full((hq, T), float("nan"), dtype=torch.float32, device="cuda")
    ps.psattn_fwd_rope(meta, rope, Q, K, V, scale, O=O, LSE=LSE, Qr=Qr, Kr=Kr)
    dQ, dK, dV = nan(Q), nan(K), nan(K)
    ps.psattn_bwd_rope(meta, rope, Qr, Kr, V, O, dO, LSE, scale, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    out = dict(O=to_np(O), LSE=to_np(LSE), dQ=to_np(dQ), dK=to_np(dK), dV=to_np(dV), Qr=to_np(Qr), Kr=to_np(Kr))
    D, B = orc.branch_arrays(off, P, ptr, rl, T)
    rnd = lambda x: W.bf16_round(x.astype(np.float32)).astype(np.float64)
    ref = orc.backward_rope(tens["Q"], tens["K"], tens["V"], tens["dO"], scale, theta, D, B,
                            lambda *a: orc.dense_branch_mask(D, B, *a), round_operands=rnd)
    real = D != orc.PAD_DOC
    # rotated operands: fp32 arithmetic on the GPU, fp64 in the oracle, both rounded to bf16 -> within one ulp
    exact = orc.rope_rotate(tens["Q"], ref["pos"], theta), orc.rope_rotate(tens["K"], ref["pos"], theta)
    for name, ex in zip(("Qr", "Kr"), exact):
        # half a bf16 ulp of the exact value, plus the fp32 rounding of the two products where they cancel
        excess = float((np.abs(out[name][real] - ex[real]) - 2.0 ** -8 * np.abs(ex[real])).max())
        assert excess <= 2e-6, (name, excess)
        assert np.mean(out[name][real] == ref[name][real]) > 0.99      # and almost always the same bf16 number
    check_padding_zero(out, D)
    check_o(out["O"], ref["O"], "rope")
    assert np.abs(out["LSE"][:, real] - ref["LSE"][:, real]).max() <= BF16_LSE_TOL
    check_grad(out["dQ"], ref["dQ"], "dQ", "rope", dq_delta_floor(tens["dO"], ref["O"], tens["K"], scale))
    for name in ("dK", "dV"):
        check_grad(out[name], ref[name], name, "rope")
    rope.free()
    meta.free()


@pytest.mark.gpu
def test_rope_two_responses_packed_with_padding():
    """The paper's format: several tiles, two packed samples, padding between and behind."""
    run_rope_case([5, 520], [200, 64], [0, 2, 4], [130, 170, 90, 33], 720, hq=4, hkv=2, theta=10000.0, seed=201)


@pytest.mark.gpu
def test_rope_multi_response_and_large_theta():
    run_rope_case([0, 400], [150, 20], [0, 3, 4], [60, 33, 129, 77], 500, hq=6, hkv=2, theta=500000.0, seed=202,
                  max_positions=4096)


@pytest.mark.gpu
@pytest.mark.parametrize("sample,kv_group", [(2, 0), (4, 7)])
def test_rope_config5_sampled(sample, kv_group):
    """Full size, the launch configuration bench.py times as `rope_fused` (config 5, theta 500 000): one
    sample x one kv-group (its 8 q-heads) against the oracle.  Position ids restart in every sample, so the
    sample taken alone at offset 0 is the same problem; the oracle runs on that slice."""
    import torch
    from gpu_util import BF16_LSE_TOL, check_grad, check_o, dq_delta_floor, to_dev
    w = W.make_workload("cfg5")
    tens = W.make_tensors(w)
    theta, d, T = 500000.0, w.head_dim, w.total_tokens
    G = w.n_q_heads // w.n_kv_heads
    meta = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, T)
    rope = ps.Rope(d, theta, meta.positions()[1])
    Q, K, V, dO = (to_dev(tens[n], "bf16") for n in ("Q", "K", "V", "dO"))
    nan = lambda x: torch.full_like(x, float("nan"))
    O, Qr, Kr = nan(Q), nan(Q), nan(K)
    LSE = torch.full((w.n_q_heads, T), float("nan"), dtype=torch.float32, device="cuda")
    ps.psattn_fwd_rope(meta, rope, Q, K, V, w.scale, O=O, LSE=LSE, Qr=Qr, Kr=Kr)
    dQ, dK, dV = nan(Q), nan(K), nan(K)
    ps.psattn_bwd_rope(meta, rope, Qr, Kr, V, O, dO, LSE, w.scale, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    o, p, c, r = (int(x[sample]) for x in (w.offset, w.prefix_len, w.chosen_len, w.rejected_len))
    n = p + c + r
    heads = slice(kv_group * G, (kv_group + 1) * G)
    np64 = lambda t: t.detach().to(torch.float32).cpu().numpy().astype(np.float64)
    out = dict(O=np64(O[o:o + n, heads]), LSE=np64(LSE[heads, o:o + n]), dQ=np64(dQ[o:o + n, heads]),
               dK=np64(dK[o:o + n, kv_group:kv_group + 1]), dV=np64(dV[o:o + n, kv_group:kv_group + 1]))
    for v in out.values():
        assert np.all(np.isfinite(v))
    sub = {"Q": tens["Q"][o:o + n, heads], "dO": tens["dO"][o:o + n, heads],
           "K": tens["K"][o:o + n, kv_group:kv_group + 1], "V": tens["V"][o:o + n, kv_group:kv_group + 1]}
    D, B = orc.branch_arrays([0], [p], [0, 2], [c, r], n)
    rnd = lambda x: W.bf16_round(x.astype(np.float32)).astype(np.float64)
    ref = orc.backward_rope(sub["Q"], sub["K"], sub["V"], sub["dO"], w.scale, theta, D, B,
                            lambda *a: orc.dense_branch_mask(D, B, *a), round_operands=rnd)
    what = "rope cfg5 sample %d kv-group %d" % (sample, kv_group)
    check_o(out["O"], ref["O"], what, tok0=o)
    assert np.abs(out["LSE"] - ref["LSE"]).max() <= BF16_LSE_TOL
    check_grad(out["dQ"], ref["dQ"], "dQ", what, dq_delta_floor(sub["dO"], ref["O"], sub["K"], w.scale))
    for name in ("dK", "dV"):
        check_grad(out[name], ref[name], name, what)
    rope.free()
    meta.free()


@pytest.mark.gpu
def test_rope_degenerate_buffers():
    """Nothing but padding, and a one-token sample: outputs are zeros / the token's own V row."""
    import torch
    rope = ps.Rope(128, 10000.0, 8)
    meta = ps.psattn_build_meta([], [], [], [], 70)
    q = torch.randn((70, 2, 128), device="cuda").to(torch.bfloat16)
    k = torch.randn((70, 1, 128), device="cuda").to(torch.bfloat16)
    O, LSE, Qr, Kr = ps.psattn_fwd_rope(meta, rope, q, k, k, 0.1)
    dQ, dK, dV = ps.psattn_bwd_rope(meta, rope, Qr, Kr, k, O, q, LSE, 0.1)
    torch.cuda.synchronize()
    assert float(O.float().abs().max()) == 0 and torch.isneginf(LSE).all()
    assert all(float(x.float().abs().max()) == 0 for x in (dQ, dK, dV))
    meta = ps.psattn_build_meta([3], [1], [0], [0], 5)
    q, k, v = q[:5].contiguous(), k[:5].contiguous(), torch.randn((5, 1, 128), device="cuda").to(torch.bfloat16)
    O, LSE, Qr, Kr = ps.psattn_fwd_rope(meta, rope, q, k, v, 0.1)
    torch.cuda.synchronize()
    assert torch.equal(O[3, 0], v[3, 0]) and torch.equal(O[3, 1], v[3, 0])     # one key: O is its V row
    assert torch.equal(Qr[3], q[3]) and torch.equal(Kr[3], k[3])               # position 0: unrotated
    assert float(O[[0, 1, 2, 4]].float().abs().max()) == 0


@pytest.mark.gpu
def test_rope_errors():
    import torch
    w = W.custom_workload([(100, 40, 30)], hq=2, hkv=1, d=128, dtype="bf16", seed=203)
    meta = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    small = ps.Rope(128, 10000.0, 100)           # the sample needs 140 positions
    q = torch.zeros((170, 2, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((170, 1, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ps.PsattnError) as e:
        ps.psattn_fwd_rope(meta, small, q, k, k, 0.1)
    assert e.value.status == -8
    with pytest.raises(ps.PsattnError) as e:
        ps.Rope(64, 10000.0, 16)
    assert e.value.status == -6
    with pytest.raises(ps.PsattnError) as e:
        ps.Rope(128, -1.0, 16)
    assert e.value.status == -1
