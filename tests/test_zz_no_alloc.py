"""psattn_bwd_static (the entry point that allocates nothing) against psattn_bwd, through
the C ABI: two calls in a row on the shared static scratch, the second with a smaller
input, each bit-identical to the workspace variant (same kernels, same arithmetic order);
and the size limit."""
import numpy as np
import pytest
import torch

import paper_2410_20305_amd as ps
import psattn_workloads as W
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _both(w, seed_shift=0):
    tens = W.make_tensors(w)
    meta = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    Q, K, V, dO = (to_dev(tens[n], w.dtype) for n in ("Q", "K", "V", "dO"))
    O, LSE = ps.psattn_fwd(meta, Q, K, V, w.scale)
    ref = ps.psattn_bwd(meta, Q, K, V, O, dO, LSE, w.scale)
    got = tuple(torch.full_like(x, float("nan")) for x in ref)
    ps.psattn_bwd_static(meta, Q, K, V, O, dO, LSE, w.scale, *got)
    torch.cuda.synchronize()
    for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
        assert torch.isfinite(a.float()).all(), name
        assert torch.equal(a, b), name
    meta.free()


def test_static_backward_matches_workspace_backward_twice():
    big = W.custom_workload([(700, 150, 260), (300, 129, 65)], offsets=[3, 1200], total_tokens=1800, hq=8, hkv=2,
                            d=128, dtype="bf16", seed=101)
    small = W.custom_workload([(90, 40, 33)], offsets=[7], total_tokens=200, hq=4, hkv=2, d=128, dtype="bf16",
                              seed=102)
    _both(big)
    _both(small)   # smaller input on the scratch the first call left behind


def test_static_backward_fp32_generic_path():
    w = W.make_workload("cfg1")
    _both(w)


def test_static_backward_rejects_oversize():
    limit = ps.psattn_bwd_static_max_rows()
    T = 4096
    hq = limit // T + 1
    w = W.custom_workload([(T - 10, 4, 6)], hq=hq, hkv=1, d=64, dtype="bf16", seed=103)
    meta = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    lib = ps.load_library()
    one = torch.zeros(16, dtype=torch.bfloat16, device="cuda")  # never dereferenced: the call must refuse first
    p = one.data_ptr()
    st = lib.psattn_bwd_static(meta.handle, 1, hq, 1, 64, 0.1, p, p, p, p, p, p, p, p, p, None)
    assert st == -8
    meta.free()
