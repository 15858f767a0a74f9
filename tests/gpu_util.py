"""Helpers shared by the GPU parity tests: run the HIP path through the binding
and compare with the oracle.  (Not collected by pytest.)"""
import json
import os

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


# ---------------------------------------------------------------- tolerances
F32_TOL = 1e-5
BF16_O_TOL, BF16_LSE_TOL, BF16_GRAD_TOL = 1e-2, 1e-3, 2e-2
BF16_ROW_FLOOR = 2e-2   # per-row gradient bar: 2e-2 of the row's own norm + this much of the tensor's RMS row norm

STATS = []              # one record per comparison, written out by conftest when PSATTN_PARITY_STATS is set


def bf16_half_ulp(x):
    """Half the spacing of bfloat16 numbers (8 significant bits) in the binade of |x|."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 8)


def bf16_o_tolerance(ref):
    """Bar on |O - ref| per element: max(1e-2, half a bf16 ulp of the reference + 5e-3).
    The oracle is fp64 and O is bf16, so an element in [2, 4) is up to 2^-7 = 0.0078 away by
    the rounding of the output alone and one in [4, 8) up to 0.0156; the 5e-3 on top covers
    the arithmetic (probabilities enter the second product rounded to bf16, 2^-9 relative,
    which on a row with two or three keys and |V| near 4 is another 0.004).  Below |ref| = 2
    the bar is exactly 1e-2.  Worst element seen: 0.01195 at |O| = 2.066, second token of a
    sample (two keys)."""
    return np.maximum(BF16_O_TOL, bf16_half_ulp(ref) + 5e-3)


def check_o(got, ref, what, tok0=0):
    """Elementwise O check against bf16_o_tolerance; records the worst element."""
    if got.size == 0:
        return
    err = np.abs(got - ref)
    tol = bf16_o_tolerance(ref)
    idx = np.unravel_index(np.argmax(err - tol), err.shape)
    idx2 = np.unravel_index(np.argmax(err), err.shape)
    STATS.append(dict(what=what, tensor="O", worst_err=float(err[idx2]), worst_ref=float(ref[idx2]),
                      worst_index=[int(i) for i in idx2], token0=int(tok0),
                      closest_to_bar_err=float(err[idx]), closest_to_bar_ref=float(ref[idx]),
                      closest_to_bar_tol=float(tol[idx]), closest_to_bar_index=[int(i) for i in idx],
                      max_abs_ref=float(np.abs(ref).max()), n_above_4=int((np.abs(ref) >= 4).sum())))
    assert np.all(err <= tol), (what, "O", float(err[idx]), float(ref[idx]), float(tol[idx]), idx)


def dq_delta_floor(dO, O_ref, K, scale):
    """Per (token, head) bound on the part of the dQ error that comes from delta: psattn_bwd
    computes delta = rowsum(dO o O) from the forward's bf16 O (as training does), the oracle
    from its own fp64 O.  Rounding O to bf16 moves every product by at most 2^-9 of itself, so
    |delta_gpu - delta| <= 2^-9 sum_d |dO_d O_d|; that shift enters dS_ij as p_ij times itself
    and dQ_i = scale sum_j dS_ij K_j by at most scale * max_j |K_j| times it (sum_j p_ij = 1).
    It does not shrink with the row's gradient, and it is largest on the first rows of a
    sample, where |O| is as large as |V|."""
    k_max = float(np.sqrt((np.asarray(K, dtype=np.float64) ** 2).sum(axis=-1)).max()) if K.size else 0.0
    return 2.0 ** -9 * np.abs(np.asarray(dO, dtype=np.float64) * O_ref).sum(axis=-1) * abs(scale) * k_max


def check_grad(got, ref, name, what, floor_rows=None):
    """Gradient tensor [tokens, heads, d]: the whole-tensor relative L2 bar, and a bar per
    (token, head) row so that a single wrong row cannot hide in the tensor norm: the row's
    error norm must stay within 2e-2 of the row's own norm plus BF16_ROW_FLOOR of the RMS row
    norm of the tensor, plus `floor_rows` where given (dQ: see dq_delta_floor)."""
    if got.size == 0:
        return
    e = rel_l2(got, ref)
    row_err = np.sqrt(((got - ref) ** 2).sum(axis=-1))
    row_ref = np.sqrt((ref ** 2).sum(axis=-1))
    rms = float(np.sqrt((row_ref ** 2).mean()))
    bar = BF16_GRAD_TOL * row_ref + BF16_ROW_FLOOR * rms + 1e-4   # 1e-4: tensors that are zero altogether (one-token samples)
    if floor_rows is not None:
        bar = bar + floor_rows
    worst = np.unravel_index(np.argmax(row_err / np.maximum(bar, 1e-300)), row_err.shape)
    STATS.append(dict(what=what, tensor=name, rel_l2=e, worst_row=[int(i) for i in worst],
                      worst_row_err=float(row_err[worst]), worst_row_ref=float(row_ref[worst]),
                      worst_row_bar=float(bar[worst]), rms_row_norm=rms,
                      max_row_rel=float((row_err / np.maximum(row_ref, 1e-300))[row_ref > 0.05 * rms].max())
                      if (row_ref > 0.05 * rms).any() else 0.0))
    assert e <= BF16_GRAD_TOL or float(np.abs(got - ref).max()) <= 1e-4, (what, name, "rel_l2", e)
    assert np.all(row_err <= bar), (what, name, "row", worst, float(row_err[worst]), float(bar[worst]))


def dump_stats():
    path = os.environ.get("PSATTN_PARITY_STATS")
    if path and STATS:
        os.makedirs(os.path.dirname(path) or ".", exist_ok=True)
        with open(path, "w") as f:
            json.dump(STATS, f, indent=1)
