"""Helpers shared by the GPU parity tests: run the HIP path through the binding
and compare with the oracle.  (Not collected by pytest.)"""
import numpy as np
import torch

import paper_2410_20305_amd as ps
import psattn_workloads as W
from oracle import psattn_oracle as orc


def to_dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def run_gpu(w, tens, tiles=(0, 0, 0, 0), scale=None):
    """fwd + bwd on the GPU.  Returns dict of float64 numpy arrays and the Meta."""
    scale = w.scale if scale is None else scale
    meta = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens, *tiles)
    Q, K, V, dO = (to_dev(tens[n], w.dtype) for n in ("Q", "K", "V", "dO"))
    # poison the outputs: every element must be overwritten
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full((w.n_q_heads, w.total_tokens), float("nan"), dtype=torch.float32, device="cuda")
    ps.psattn_fwd(meta, Q, K, V, scale, O=O, LSE=LSE)
    dQ, dK, dV = torch.full_like(Q, float("nan")), torch.full_like(K, float("nan")), torch.full_like(V, float("nan"))
    ps.psattn_bwd(meta, Q, K, V, O, dO, LSE, scale, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    out = dict(O=to_np(O), LSE=to_np(LSE), dQ=to_np(dQ), dK=to_np(dK), dV=to_np(dV))
    return out, meta


def oracle_arrays(w):
    return orc.index_arrays(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)


def rel_l2(got, ref):
    den = np.sqrt((ref ** 2).sum())
    return float(np.sqrt(((got - ref) ** 2).sum()) / den) if den > 0 else float(np.abs(got).max())


def check_padding_zero(out, D):
    pad = D == orc.PAD_DOC
    for name in ("O", "dQ", "dK", "dV"):
        assert np.all(out[name][pad] == 0), name + " not zero at padding"
    assert np.all(np.isneginf(out["LSE"][:, pad]))
