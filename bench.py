#!/usr/bin/env python3
"""Benchmark of the prefix-shared DPO attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--no-extras] [--no-cpu]
    python bench.py --sweep            # prefix x completion length grid (Section 4.2, Fig. 3)

One step = one pass of the whole hot path over one synthetic batch: block-mask
build (psattn_build_meta), forward (psattn_fwd), backward (psattn_bwd: delta, dQ,
dK/dV) and the stream-ordered release of the block mask.  Inputs are resident in
HBM before the timed region.  Prints ONE JSON line.  `value` is useful attention
TFLOP/s (14 * d * Hq * N_allowed FLOPs per step; masked pairs, padding and
recomputation earn nothing).  The default workload is the largest of the
configurations (cfg5).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0
SWEEP_BATCH = 4             # samples per point of the length sweeps (enough work to fill the chip at the short end)
LAYERS = 32                 # the block mask is built once per step and shared by every layer (Section 3.1)
PASSES = ["fwd", "delta", "dq", "dkdv"]
# algorithmic FLOPs per launch in units of d * Hq * N_allowed: forward 4 (S, PV); dQ pass 2 (dQ only: its
# recomputation of S and dP earns nothing); dK/dV pass 8 (S, dP, dV, dK)
ALG_UNITS = [4, 0, 2, 8]


def tri(n):
    return n * (n + 1) // 2


def allowed_pairs(w):
    p, c, r = (x.astype(np.int64) for x in (w.prefix_len, w.chosen_len, w.rejected_len))
    return int((tri(p) + c * p + tri(c) + r * p + tri(r)).sum())


def algorithmic_bytes(w, tokens):
    """Bytes the method itself must move per step, each tensor once (bf16: e = 2)."""
    e = 4 if w.dtype == "f32" else 2
    Hq, Hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    fwd = (Hq + 2 * Hkv) * d * e + Hq * d * e + 4 * Hq
    bwd = (3 * Hq + 2 * Hkv) * d * e + 8 * Hq + (Hq + 2 * Hkv) * d * e
    return tokens * (fwd + bwd)


class Runner:
    """Device tensors of one workload + the library calls of a step."""

    def __init__(self, w, tensors=None, seed=0):
        import torch
        import paper_2410_20305_amd as ps
        self.ps, self.torch, self.w = ps, torch, w
        dt = torch.float32 if w.dtype == "f32" else torch.bfloat16
        T, Hq, Hkv, d = w.total_tokens, w.n_q_heads, w.n_kv_heads, w.head_dim
        if tensors is not None:
            mk = lambda n: torch.from_numpy(tensors[n]).to("cuda").to(dt)
            self.Q, self.K, self.V, self.dO = mk("Q"), mk("K"), mk("V"), mk("dO")
        else:  # same distribution, drawn on the device
            g = torch.Generator(device="cuda")
            g.manual_seed(1000 + seed)
            mk = lambda h: torch.randn((T, h, d), generator=g, device="cuda", dtype=torch.float32).to(dt)
            self.Q, self.K, self.V, self.dO = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
        self.O = torch.empty_like(self.Q)
        self.LSE = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
        self.dQ, self.dK, self.dV = torch.empty_like(self.Q), torch.empty_like(self.K), torch.empty_like(self.V)
        meta = self.build_meta()
        self.mfma = meta.uses_mfma(ps.BF16 if w.dtype == "bf16" else ps.F32, d, w.scale, backward=True)
        self.ws = torch.empty(ps.psattn_bwd_workspace_bytes(meta, Hq, Hkv, d), dtype=torch.uint8, device="cuda")
        meta.free()
        self.flops = 14 * d * Hq * allowed_pairs(w)

    def build_meta(self):
        w = self.w
        return self.ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)

    def step(self):
        ps, w = self.ps, self.w
        meta = self.build_meta()
        if getattr(self, "rope", None) is not None:
            ps.psattn_fwd_rope(meta, self.rope, self.Q, self.K, self.V, w.scale, O=self.O, LSE=self.LSE, Qr=self.Qr,
                               Kr=self.Kr)
            ps.psattn_bwd_rope(meta, self.rope, self.Qr, self.Kr, self.V, self.O, self.dO, self.LSE, w.scale,
                               dQ=self.dQ, dK=self.dK, dV=self.dV, workspace=self.ws)
        else:
            ps.psattn_fwd(meta, self.Q, self.K, self.V, w.scale, O=self.O, LSE=self.LSE)
            ps.psattn_bwd(meta, self.Q, self.K, self.V, self.O, self.dO, self.LSE, w.scale, dQ=self.dQ,
                          dK=self.dK, dV=self.dV, workspace=self.ws)
        meta.free_async()

    def enable_rope(self, theta=500000.0):
        """Switch step() to the entry points that apply the rotary embedding inside the op."""
        meta = self.build_meta()
        self.rope = self.ps.Rope(self.w.head_dim, theta, meta.positions()[1])
        meta.free()
        self.Qr, self.Kr = self.torch.empty_like(self.Q), self.torch.empty_like(self.K)

    def build_meta_ms(self, n=20):
        """Host wall time of psattn_build_meta alone (sample table -> block mask -> upload enqueued)."""
        ts = []
        for _ in range(n):
            t0 = time.perf_counter()
            m = self.build_meta()
            ts.append((time.perf_counter() - t0) * 1e3)
            m.free_async()
        self.torch.cuda.synchronize()
        return float(np.median(ts)), float(np.min(ts))

    def timed(self, steps, warmup):
        """Wall time of `steps` whole steps, bracketed by synchronize; per-step device time
        from events on the launch stream; per-pass kernel time from HIP events recorded by
        the library on the same stream."""
        torch, ps = self.torch, self.ps
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ps.psattn_profile_enable(True)
        ps.psattn_profile_read()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            self.step()
            marks[i + 1].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms, cnt = ps.psattn_profile_read()
        ps.psattn_profile_enable(False)
        per_pass = [float(ms[i] / max(1, cnt[i])) for i in range(4)]
        per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
        return (t1 - t0) / steps * 1e3, per_pass, per_step


def kernel_algorithmic_bytes(w, i):
    """Bytes pass i (0 forward, 2 dQ, 3 dK/dV) must move per launch, each tensor once (bf16 tensors,
    fp32 statistics); per token, times the buffer's tokens."""
    Hq, Hkv, d, e = w.n_q_heads, w.n_kv_heads, w.head_dim, 2
    per_token = {0: (Hq + 2 * Hkv) * d * e + Hq * d * e + 4 * Hq,
                 2: (3 * Hq + 2 * Hkv) * d * e + 4 * Hq + Hq * d * e + 8 * Hq,
                 3: (2 * Hq + 2 * Hkv) * d * e + 8 * Hq + 2 * Hkv * d * e}[i]
    return w.total_tokens * per_token


def roofline_of(w, per_pass, ps, traffic_table, name):
    """Roofline object of the dominant kernel of one workload, against whichever of the two limits
    (bf16 MFMA peak for its algorithmic FLOPs, HBM bandwidth for its algorithmic bytes) binds it."""
    dom = max((0, 2, 3), key=lambda i: per_pass[i])
    n_allowed = allowed_pairs(w)
    flops = ALG_UNITS[dom] * w.head_dim * w.n_q_heads * n_allowed
    nbytes = kernel_algorithmic_bytes(w, dom)
    t = per_pass[dom] * 1e-3
    kernel = ps.psattn_kernel_name(1, dom)
    tr = traffic_table.get("%s/%s" % (name, kernel))
    common = dict(kernel=kernel, traffic=int(tr["read_bytes"] + tr["write_bytes"]) if tr else None,
                  traffic_source="rocprofv3 FETCH_SIZE/WRITE_SIZE summary committed under profiles/hbm_traffic.txt "
                                 "(not measured by this run)" if tr else None,
                  avg_launch_ms=round(per_pass[dom], 4), algorithmic_flops_per_launch=flops,
                  algorithmic_bytes_per_launch=nbytes)
    if nbytes / (PEAK_HBM_GBS * 1e9) > flops / (PEAK_BF16_TFLOPS * 1e12):
        ach = nbytes / t / 1e9
        return dict(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s", frac=round(ach / PEAK_HBM_GBS, 4),
                    **common)
    ach = flops / t / 1e12
    return dict(bound="mfma", achieved=round(ach, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                frac=round(ach / PEAK_BF16_TFLOPS, 4), **common)


def mfma_ceiling(ps, torch, reps=4):
    """What an MFMA-only kernel sustains right now on this device on operands whose sign and mantissa bits are
    random (the clock the device holds under matrix load depends on how much the data toggles): TFLOP/s, from the
    difference of two launch lengths so that launch overhead cancels."""
    lib = ps.load_library()
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    n_wg, t = 512, {}
    for iters in (4000, 12000):
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            st = lib.psattn_probe_mfma_peak(n_wg, iters, 1, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
            b.record()
            torch.cuda.synchronize()
            if st != 0:
                return None
            ts.append(a.elapsed_time(b))
        t[iters] = float(np.median(ts[1:]))
    return n_wg * 16 * 8000 * 32768 / ((t[12000] - t[4000]) * 1e-3) / 1e12


def summarize(w, ms_step, per_pass, per_step, flops):
    kern = sum(per_pass)
    t_mfma = flops / (PEAK_BF16_TFLOPS * 1e12) * 1e3
    t_hbm = algorithmic_bytes(w, w.total_tokens) / (PEAK_HBM_GBS * 1e9) * 1e3
    bound = max(t_mfma, t_hbm)
    return dict(ms_per_step=round(ms_step, 4), ms_per_step_median=round(float(np.median(per_step)), 4),
                ms_per_step_min=round(float(np.min(per_step)), 4), ms_kernels=round(kern, 4),
                ms_fwd=round(per_pass[0], 4), ms_delta=round(per_pass[1], 4), ms_dq=round(per_pass[2], 4),
                ms_dkdv=round(per_pass[3], 4),
                useful_tflops=round(flops / (ms_step * 1e-3) / 1e12, 2),
                useful_tflops_kernels_only=round(flops / (kern * 1e-3) / 1e12, 2) if kern > 0 else None,
                pct_mfma_peak=round(100 * flops / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                roofline_ms_mfma=round(t_mfma, 4), roofline_ms_hbm=round(t_hbm, 4),
                binding_roofline="hbm" if t_hbm > t_mfma else "mfma",
                frac_of_binding_roofline=round(bound / ms_step, 4))


def cpu_baseline(w, tens, budget_s=20.0):
    """The oracle as it stands, timed on this host on a bounded sample of the
    workload: whole (sample, kv-group) blocks, forward + backward, until the budget
    is used.  Reported in the metric's unit (useful TFLOP/s of the blocks done)."""
    from oracle import psattn_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    Ic, Ir, D = orc.index_arrays(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
    G = w.n_q_heads // w.n_kv_heads
    done_flops, done_token_heads, blocks = 0, 0, 0
    # shortest samples first, so that the budget buys several whole blocks even on the largest workload
    order = np.argsort(w.prefix_len.astype(np.int64) + w.chosen_len + w.rejected_len, kind="stable")
    t0 = time.perf_counter()
    for g in range(w.n_kv_heads):
        for s in order:
            s = int(s)
            heads = list(range(g * G, (g + 1) * G))
            orc.backward(tens["Q"], tens["K"], tens["V"], tens["dO"], w.scale, Ic, Ir, D, heads=heads, samples=[s])
            p, c, r = int(w.prefix_len[s]), int(w.chosen_len[s]), int(w.rejected_len[s])
            n_allowed = tri(p) + c * p + tri(c) + r * p + tri(r)
            done_flops += 14 * w.head_dim * G * n_allowed
            done_token_heads += (p + c + r) * G
            blocks += 1
            if time.perf_counter() - t0 > budget_s:
                break
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return dict(value=round(done_flops / dt / 1e12, 6), unit="TFLOP/s", cores=int(cores), kind="oracle",
                sample="%d of %d (sample, kv-group) blocks of %s (shortest samples first), each with its %d q-heads, "
                       "fwd+bwd, fp64 numpy, %.1f s; tokens_per_s scales the blocks done to all %d q-heads" %
                       (blocks, w.n_samples * w.n_kv_heads, w.name, G, dt, w.n_q_heads),
                tokens_per_s=round(done_token_heads / w.n_q_heads / dt, 1))


def length_sweep(W, steps, warmup):
    """Attention forward + backward time of a small batch, prefix-shared against paired, over a
    grid of prompt and completion lengths (Section 4.2's self-attention micro-benchmark:
    Mistral-7B-shaped heads, 32 q / 8 kv, d = 128; chosen and rejected of equal length)."""
    rows = []
    for p in (1024, 4096, 8192, 16384):
        for c in (128, 512, 2048, 4096):
            w = W.custom_workload([(p, c, c)] * SWEEP_BATCH, hq=32, hkv=8, d=128, dtype="bf16", seed=p + c, name="sweep")
            pw, _, _ = W.paired_workload(w)
            rs, rp = Runner(w, None, seed=1), Runner(pw, None, seed=1)
            ms_s, pp_s, _ = rs.timed(steps, warmup)
            ms_p, pp_p, _ = rp.timed(steps, warmup)
            rows.append(dict(prefix=p, completion=c, shared_ms=round(sum(pp_s), 4), paired_ms=round(sum(pp_p), 4),
                             speedup=round(sum(pp_p) / sum(pp_s), 3),
                             ideal=round(allowed_pairs(pw) / allowed_pairs(w), 3),
                             paper_ideal=round(2 * (p + c) ** 2 / (2 * (p + c) ** 2 - p ** 2), 3),
                             shared_pct_peak=round(100 * rs.flops / (sum(pp_s) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2)))
            del rs, rp
    return rows


def layer_sweep(W, steps, warmup):
    """Forward + backward time of one whole self-attention layer on a small batch, prefix-shared against
    paired (Section 4.2's attention-layer micro-benchmark: the projections are linear in the tokens,
    the attention quadratic)."""
    import torch
    import paper_2410_20305_amd as ps
    from paper_2410_20305_amd.layer import Layer
    hidden, Hq, Hkv, d = 4096, 32, 8, 128
    layer = Layer(hidden, Hq, Hkv, d)
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    rnd = lambda *shape, s=1.0: (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * s).to(torch.bfloat16)
    Wq, Wk, Wv = rnd(Hq * d, hidden, s=hidden ** -0.5), rnd(Hkv * d, hidden, s=hidden ** -0.5), rnd(Hkv * d, hidden, s=hidden ** -0.5)
    Wo = rnd(hidden, Hq * d, s=(Hq * d) ** -0.5)
    rope = ps.Rope(d, 10000.0, 32768)

    def time_layout(w):
        meta = ps.psattn_build_meta(w.offset, w.prefix_len, w.chosen_len, w.rejected_len, w.total_tokens)
        T = w.total_tokens
        X, dY = rnd(T, hidden), rnd(T, hidden)
        ws = torch.empty(layer.workspace_bytes(meta), dtype=torch.uint8, device="cuda")
        Y = torch.empty_like(X)
        grads = tuple(torch.empty_like(t) for t in (X, Wq, Wk, Wv, Wo))
        ts = []
        for it in range(warmup + steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            layer.forward(meta, rope, w.scale, X, Wq, Wk, Wv, Wo, ws, Y=Y)
            layer.backward(meta, rope, w.scale, X, Wq, Wk, Wv, Wo, dY, ws, grads=grads)
            b.record()
            torch.cuda.synchronize()
            if it >= warmup:
                ts.append(a.elapsed_time(b))
        meta.free()
        return float(np.median(ts))

    rows = []
    for p in (1024, 4096, 8192, 16384):
        for c in (128, 512, 2048):
            w = W.custom_workload([(p, c, c)] * SWEEP_BATCH, hq=Hq, hkv=Hkv, d=d, dtype="bf16", seed=p + c, name="layer")
            pw, _, _ = W.paired_workload(w)
            ms_s, ms_p = time_layout(w), time_layout(pw)
            rows.append(dict(prefix=p, completion=c, shared_ms=round(ms_s, 4), paired_ms=round(ms_p, 4),
                             speedup=round(ms_p / ms_s, 3), token_ratio=round((2 * p + 2 * c) / (p + 2 * c), 3),
                             attention_pair_ratio=round(allowed_pairs(pw) / allowed_pairs(w), 3)))
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--no-extras", action="store_true", help="skip the other configurations and the paired baseline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--sweep", action="store_true", help="prefix x completion length grid instead of the configurations")
    ap.add_argument("--layer", action="store_true",
                    help="whole attention layer (projections + RoPE + attention + output projection), prefix x completion grid")
    ap.add_argument("--mfma-probe", action="store_true", help="time an MFMA-only kernel: the matrix-core ceiling under load")
    ap.add_argument("--dq-atomics-probe", action="store_true",
                    help="time the fp32 atomic adds a one-pass backward would need for dQ, on every configuration")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run a plain 1 GiB device copy 5 times and exit (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path "
              "(samples and kv-head groups are independent, so N GPUs would each run this same kernel "
              "on their share with no exchange step).  Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2410_20305_amd as ps
    import psattn_workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the HIP library has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    ps.load_library()
    torch.cuda.set_device(0)
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel() * 4, "copy_probe_bytes_written": src.numel() * 4,
                          "launches": 5}))
        return
    if args.mfma_probe:
        # matrix-core ceiling of this device under load: MFMA-only kernel, 1, 2 and 4 waves per SIMD, on one constant
        # operand pair, on random operands and on constant values spread over eight register sets; then the attention kernels themselves on all-zero inputs (same instruction
        # stream, idle data paths), which separates what the clock costs from what the schedule costs
        lib = ps.load_library()
        sink = torch.zeros(1, dtype=torch.float32, device="cuda")
        res = {}
        for mode, operands in enumerate(("constant", "random", "constant_in_eight_registers")):
            for label, n_wg in (("one_wave_per_simd", 256), ("two_waves_per_simd", 512), ("four_waves_per_simd", 1024)):
                iters = 20000
                ts = []
                for _ in range(5):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    st = lib.psattn_probe_mfma_peak(n_wg, iters, mode, sink.data_ptr(),
                                                    torch.cuda.current_stream().cuda_stream)
                    b.record()
                    torch.cuda.synchronize()
                    assert st == 0
                    ts.append(a.elapsed_time(b))
                ms = float(np.median(ts[1:]))
                flops = n_wg * 4 * 4 * iters * 32768
                res[operands + "_operands_" + label] = dict(
                    workgroups=n_wg, mfma_per_wave=4 * iters, ms=round(ms, 4), tflops=round(flops / (ms * 1e-3) / 1e12, 1),
                    frac_of_published_peak=round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                    cycles_per_mfma_at_2p4GHz=round(ms * 1e-3 * 2.4e9 / (4 * iters * (n_wg // 256)), 2))
        w = W.make_workload(args.workload)
        r = Runner(w, None, seed=w.seed)
        kernels = {}
        for label in ("workload_inputs", "zero_inputs"):
            if label == "zero_inputs":
                for x in (r.Q, r.K, r.V, r.dO):
                    x.zero_()
            _, pp, _ = r.timed(10, 3)
            kernels[label] = dict(ms_fwd=round(pp[0], 4), ms_dq=round(pp[2], 4), ms_dkdv=round(pp[3], 4))
        print(json.dumps({"metric": "bf16 MFMA-only kernel (v_mfma_f32_32x32x16_bf16, register operands)", "unit": "TFLOP/s",
                          "published_peak": PEAK_BF16_TFLOPS, "runs": res,
                          "attention_kernels": dict(workload=w.name, **kernels)}))
        return
    if args.dq_atomics_probe:
        # the memory operations a one-pass backward would add for dQ, timed alone (see include/psattn.h)
        res = {}
        for name in ("cfg2", "cfg3", "cfg4", "cfg5"):
            wx = W.make_workload(name)
            meta = ps.psattn_build_meta(wx.offset, wx.prefix_len, wx.chosen_len, wx.rejected_len, wx.total_tokens)
            acc = torch.zeros((wx.total_tokens, wx.n_q_heads, 128), dtype=torch.float32, device="cuda")
            r = {}
            for mode, label in ((0, "atomic_add_ms"), (1, "plain_store_ms")):
                ts = []
                for _ in range(4):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    ps.psattn_probe_dq_atomics(meta, wx.n_q_heads, wx.n_kv_heads, acc, mode)
                    b.record()
                    torch.cuda.synchronize()
                    ts.append(a.elapsed_time(b))
                r[label] = round(min(ts[1:]), 4)
            n_visits = int(meta.tiles(ps.GRID_BWD)["n_entries"]) * wx.n_q_heads
            r["tile_visits"] = n_visits
            r["payload_GB"] = round(n_visits * 64 * 128 * 4 / 1e9, 3)
            res[name] = r
            meta.free()
            del acc
        print(json.dumps({"metric": "dQ accumulation traffic of a one-pass backward, alone", "unit": "ms", "configs": res}))
        return
    if args.layer:
        print(json.dumps({"metric": "attention layer fwd+bwd ms, prefix-shared vs paired, batch of %d equal samples" % SWEEP_BATCH, "unit": "ms",
                          "shape": "hidden 4096, 32q/8kv d128 bf16 (Mistral-7B attention layer), RoPE inside the op",
                          "grid": layer_sweep(W, min(args.steps, 10), 2)}))
        return
    if args.sweep:
        print(json.dumps({"metric": "attention fwd+bwd ms, prefix-shared vs paired, batch of %d equal samples" % SWEEP_BATCH, "unit": "ms",
                          "heads": "32q/8kv d128 bf16", "grid": length_sweep(W, min(args.steps, 10), 2)}))
        return

    traffic_table = {}
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")) as f:
            traffic_table = json.load(f)
    except (OSError, ValueError):
        pass

    w = W.make_workload(args.workload)
    tens = W.make_tensors(w)
    run = Runner(w, tens)
    assert run.mfma, "the benchmark configurations must run on the MFMA kernels"
    ms_step, per_pass, per_step = run.timed(args.steps, args.warmup)
    bm_med, bm_min = run.build_meta_ms()
    main_res = summarize(w, ms_step, per_pass, per_step, run.flops)
    value = run.flops / (ms_step * 1e-3) / 1e12
    n_allowed = allowed_pairs(w)

    out = {
        "metric": "useful attn TFLOP/s fwd+bwd", "value": round(value, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload, "n_samples": w.n_samples, "tokens": w.unique_tokens,
                   "buffer_tokens": w.total_tokens, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "allowed_pairs": n_allowed,
                   "step": "build_meta + fwd + bwd(delta, dQ, dK/dV) + free_meta_async"},
        "pct_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
        "tokens_per_s": round(w.unique_tokens / (ms_step * 1e-3), 1),
        "ms_per_step_median": main_res["ms_per_step_median"], "ms_per_step_min": main_res["ms_per_step_min"],
        "build_meta_ms": round(bm_med, 4), "build_meta_ms_min": round(bm_min, 4),
        "build_meta_ms_amortised_over_%d_layers" % LAYERS: round(bm_med / LAYERS, 5),
        "detail": main_res,
        "roofline": roofline_of(w, per_pass, ps, traffic_table, args.workload),
    }
    # the device's own matrix-core ceiling, measured in this run (MFMA-only kernel on operands with random sign and
    # mantissa bits), beside the published peak the roofline object is priced against
    ceil = mfma_ceiling(ps, torch)
    if ceil:
        executed = {0: 4, 2: 6, 3: 8}   # contraction units a pass executes (the dQ pass recomputes S and dP)
        units = w.head_dim * w.n_q_heads * n_allowed
        t_bound = sum(executed.values()) * units / (ceil * 1e12) * 1e3
        out["mfma_ceiling"] = {
            "what": "MFMA-only kernel (v_mfma_f32_32x32x16_bf16, register operands with random sign and mantissa bits), "
                    "measured in this run",
            "tflops": round(ceil, 1), "frac_of_published_peak": round(ceil / PEAK_BF16_TFLOPS, 4),
            "dominant_kernel_achieved_over_ceiling": round(out["roofline"]["achieved"] / ceil, 4)
            if out["roofline"]["bound"] == "mfma" else None,
            "ms_per_step_if_every_executed_mfma_ran_at_ceiling": round(t_bound, 4),
            "that_bound_over_step": round(t_bound / sum(per_pass), 4)}
    algb = algorithmic_bytes(w, w.total_tokens)
    out["hbm_algorithmic_GBs"] = round(algb / (sum(per_pass) * 1e-3) / 1e9, 1)

    if not args.no_extras:
        extras = {}
        for name in ("cfg2", "cfg3", "cfg4", "cfg5"):
            wx = W.make_workload(name)
            steps = max(5, min(args.steps, 20))
            rx = run if name == args.workload else Runner(wx, None, seed=wx.seed)
            ms_s, pp, pst = (ms_step, per_pass, per_step) if name == args.workload else rx.timed(steps, 3)
            res = summarize(wx, ms_s, pp, pst, rx.flops)
            res["tokens_per_s"] = round(wx.unique_tokens / (ms_s * 1e-3), 1)
            res["roofline"] = roofline_of(wx, pp, ps, traffic_table, name)
            bm, _ = rx.build_meta_ms(10)
            res["build_meta_ms"] = round(bm, 4)
            # unshared paired baseline on the same samples, same kernels
            pw, _, _ = W.paired_workload(wx)
            rp = Runner(pw, None, seed=wx.seed)
            ms_p, pp_p, _ = rp.timed(steps, 3)
            res["paired_ms_per_step"] = round(ms_p, 4)
            res["paired_tokens_per_s"] = round(wx.unique_tokens / (ms_p * 1e-3), 1)
            res["speedup_vs_paired"] = round(ms_p / ms_s, 3)
            res["speedup_vs_paired_kernels_only"] = round(sum(pp_p) / sum(pp), 3)
            res["ideal_attn_speedup"] = round(allowed_pairs(pw) / allowed_pairs(wx), 3)
            extras[name] = res
            del rp
            if rx is not run:
                del rx
            torch.cuda.empty_cache()
        out["all_configs"] = extras
        # First-Fit-Decreasing packing of the same samples (Section 4.3.2) against the in-order greedy rule
        ffd = {}
        for name in ("cfg4", "cfg5"):
            wx = W.make_workload(name)
            t0 = time.perf_counter()
            pk = ps.psattn_pack_ffd(wx.prefix_len, wx.chosen_len, wx.rejected_len, wx.row_len)
            pack_ms = (time.perf_counter() - t0) * 1e3
            wf = W.with_layout(wx, pk["offset"], pk["order"], pk["n_rows"] * wx.row_len, name=name + "-ffd")
            rf = Runner(wf, None, seed=wx.seed)
            ms_f, pp_f, pst_f = rf.timed(max(5, min(args.steps, 20)), 3)
            ffd[name] = dict(rows_greedy=wx.total_tokens // wx.row_len, rows_ffd=pk["n_rows"],
                             padding_fraction_greedy=round(1 - wx.unique_tokens / wx.total_tokens, 4),
                             padding_fraction_ffd=round(pk["padding_tokens"] / max(1, pk["n_rows"] * wx.row_len), 4),
                             pack_ms=round(pack_ms, 4), ms_per_step_ffd=round(ms_f, 4),
                             ms_per_step_greedy=extras[name]["ms_per_step"],
                             pct_mfma_peak_ffd=round(100 * rf.flops / (ms_f * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2))
            # a larger pool drawn from the same length distribution (host only): rows needed by either rule
            cfg = W.CONFIGS[name]
            rng = np.random.default_rng(cfg["seed"] + 77)
            n_pool = 512
            P, Cc, R = (rng.integers(cfg[k][0], cfg[k][1], size=n_pool, endpoint=True).astype(np.int32) for k in "pcr")
            lens = P.astype(np.int64) + Cc + R
            rows_g, fill = 1, 0
            for L in lens:                     # in-order greedy: close the row when the next sample does not fit
                if fill + L > wx.row_len:
                    rows_g, fill = rows_g + 1, 0
                fill += int(L)
            pkp = ps.psattn_pack_ffd(P, Cc, R, wx.row_len)
            ffd[name]["pool_%d_samples" % n_pool] = dict(
                rows_greedy=rows_g, rows_ffd=pkp["n_rows"],
                padding_fraction_greedy=round(1 - int(lens.sum()) / (rows_g * wx.row_len), 4),
                padding_fraction_ffd=round(1 - int(lens.sum()) / (pkp["n_rows"] * wx.row_len), 4))
            del rf
            torch.cuda.empty_cache()
        out["ffd_packing"] = ffd
        # rotary embedding with the position ids of the paired format applied inside the op (Section 3.1):
        # whole step with it against the step without it, next to what a separate elementwise RoPE pass
        # over Q and K (read + write, forward; the same again for dQ, dK in the backward) would move
        run.enable_rope()
        ms_r, pp_r, pst_r = run.timed(max(5, min(args.steps, 20)), 3)
        e = 2
        sep_bytes = 2 * 2 * w.total_tokens * (w.n_q_heads + w.n_kv_heads) * w.head_dim * e
        out["rope_fused"] = dict(workload=args.workload, ms_per_step=round(ms_r, 4), ms_per_step_without=round(ms_step, 4),
                                 overhead_ms=round(ms_r - ms_step, 4),
                                 ms_fwd=round(pp_r[0], 4), ms_dq=round(pp_r[2], 4), ms_dkdv=round(pp_r[3], 4),
                                 separate_pass_bytes=sep_bytes,
                                 separate_pass_ms_at_hbm_peak=round(sep_bytes / (PEAK_HBM_GBS * 1e9) * 1e3, 4))
        out["paper_context"] = "paper reports 1.1-1.5x (1.3-1.6x packed) end-to-end training speedup on 8xH100"

    if not args.no_extras:
        # per-response log-probabilities + DPO loss + backward to the logits (Section 2.1, Eq. 1) on the same
        # sample table, Mistral-7B vocabulary; all three passes stream logits rows: HBM roofline
        V = 32000
        ptr = 2 * np.arange(w.n_samples + 1, dtype=np.int32)
        rl = np.stack([w.chosen_len, w.rejected_len], axis=1).reshape(-1).astype(np.int32)
        plan = ps.LogprobPlan(w.offset, w.prefix_len, ptr, rl, w.total_tokens)
        g = torch.Generator(device="cuda")
        g.manual_seed(9)
        logits = torch.randn((w.total_tokens, V), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        ids = torch.randint(0, V, (w.total_tokens,), generator=g, device="cuda", dtype=torch.int32)
        row_lse = torch.zeros(w.total_tokens, dtype=torch.float32, device="cuda")
        logp = torch.empty(plan.n_responses, dtype=torch.float32, device="cuda")
        dlogits = torch.empty_like(logits)
        ref_lp = logp.clone()
        t_f, t_b = [], []
        for it in range(8):
            a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            a.record()
            ps.psattn_logprob_fwd(plan, logits, ids, row_lse, logp)
            b.record()
            _, dlp = ps.psattn_dpo_loss(logp, ref_lp if it else logp, 0.1)
            ps.psattn_logprob_bwd(plan, logits, ids, row_lse, dlp, dlogits)
            c.record()
            torch.cuda.synchronize()
            if it >= 2:
                t_f.append(a.elapsed_time(b))
                t_b.append(b.elapsed_time(c))
        fb = plan.n_rows * V * 2
        bb = plan.n_rows * V * 2 + w.total_tokens * V * 2
        out["logprob_head"] = dict(workload=args.workload, vocab=V, dtype="bf16", predicting_rows=plan.n_rows,
                                   buffer_rows=w.total_tokens, ms_fwd=round(float(np.median(t_f)), 4),
                                   ms_loss_bwd=round(float(np.median(t_b)), 4),
                                   fwd_GBs=round(fb / (float(np.median(t_f)) * 1e-3) / 1e9, 1),
                                   bwd_GBs=round(bb / (float(np.median(t_b)) * 1e-3) / 1e9, 1),
                                   roofline=dict(bound="hbm", kernel="psattn_lp_bwd", achieved=round(bb / (float(np.median(t_b)) * 1e-3) / 1e9, 1),
                                                 peak=PEAK_HBM_GBS, unit="GB/s",
                                                 frac=round(bb / (float(np.median(t_b)) * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                                 traffic=None, algorithmic_bytes_per_launch=bb))
        del logits, dlogits
        torch.cuda.empty_cache()

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, tens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
