"""Seeded synthetic inputs for prefix-shared DPO attention.

This module only draws lengths and tensors and lays samples out in a flat
token buffer.  It contains none of the method's arithmetic (no mask, no
softmax, no tile logic): the CPU oracle and the HIP path both receive what it
returns and nothing else is shared between them.

Layouts follow the paper's data formatting (Section 3.1: one sequence
[prompt | chosen | rejected] per sample; Section 3.2 / 4.3.2: several samples
packed into a fixed-length row, rows padded to the packing length).  The paper's
(b, q) coordinates map to the flat token index b * row_len + q.

The five configurations stand in for the paper's datasets (Table 1 / Table 2),
which are not available here: only the length statistics are imitated.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "Workload", "CONFIGS", "make_workload", "make_tensors", "paired_workload", "with_layout",
    "custom_workload", "bf16_round", "to_bf16_bits", "from_bf16_bits",
]


@dataclass
class Workload:
    """Sample table + head configuration of one synthetic batch."""
    name: str
    dtype: str                    # "f32" or "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    total_tokens: int             # T: buffer length including padding
    offset: np.ndarray            # int32 [n_samples] flat start token of every sample
    prefix_len: np.ndarray        # int32 [n_samples]
    chosen_len: np.ndarray        # int32 [n_samples]
    rejected_len: np.ndarray      # int32 [n_samples]
    seed: int = 0
    row_len: int = 0              # 0 = unpacked (samples back to back)
    scale: float = 0.0
    notes: dict = field(default_factory=dict)

    @property
    def n_samples(self) -> int:
        return int(self.offset.shape[0])

    @property
    def unique_tokens(self) -> int:
        return int((self.prefix_len.astype(np.int64) + self.chosen_len + self.rejected_len).sum())

    @property
    def paired_tokens(self) -> int:
        p = self.prefix_len.astype(np.int64)
        return int((2 * p + self.chosen_len + self.rejected_len).sum())


def _i32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _draw(rng, lo_hi):
    lo, hi = lo_hi
    return int(rng.integers(lo, hi, endpoint=True))


def _back_to_back(rng, n, pr, cr, rr):
    off, P, C, R = [], [], [], []
    cur = 0
    for _ in range(n):
        p = _draw(rng, pr)
        c = _draw(rng, cr)
        r = _draw(rng, rr)
        off.append(cur)
        P.append(p)
        C.append(c)
        R.append(r)
        cur += p + c + r
    return off, P, C, R, cur


def _greedy_rows(rng, n_rows, row_len, pr, cr, rr):
    """Draw samples in sequence; append to the current row if the sample fits,
    otherwise close the row (the remainder is padding) and start the next row
    with that sample.  Stops once n_rows rows are closed; the sample that
    overflowed the last row is dropped."""
    off, P, C, R = [], [], [], []
    row, fill = 0, 0
    while True:
        p = _draw(rng, pr)
        c = _draw(rng, cr)
        r = _draw(rng, rr)
        n = p + c + r
        if n > row_len:
            raise ValueError("sample longer than a packed row")
        if fill + n > row_len:
            row += 1
            fill = 0
            if row == n_rows:
                break
        off.append(row * row_len + fill)
        P.append(p)
        C.append(c)
        R.append(r)
        fill += n
    return off, P, C, R, n_rows * row_len


# name -> recipe.  Seeds: lengths use default_rng(seed); tensors default_rng(seed + 1000).
CONFIGS = {
    "cfg1": dict(dtype="f32", hq=1, hkv=1, d=64, seed=0, kind="fixed",
                 samples=[(96, 24, 40)]),
    "cfg2": dict(dtype="bf16", hq=32, hkv=8, d=128, seed=2, kind="b2b", n=8,
                 p=(256, 1024), c=(64, 384), r=(64, 384)),
    "cfg3": dict(dtype="bf16", hq=32, hkv=8, d=128, seed=3, kind="b2b", n=16,
                 p=(1024, 3072), c=(32, 192), r=(32, 192)),
    "cfg4": dict(dtype="bf16", hq=32, hkv=8, d=128, seed=4, kind="rows", rows=8, row_len=8192,
                 p=(32, 256), c=(32, 256), r=(32, 256)),
    "cfg5": dict(dtype="bf16", hq=64, hkv=8, d=128, seed=5, kind="rows", rows=4, row_len=16384,
                 p=(2048, 6144), c=(128, 1024), r=(128, 1024)),
}


def make_workload(name: str) -> Workload:
    """Build the sample table of one of the five named configurations."""
    cfg = CONFIGS[name]
    rng = np.random.default_rng(cfg["seed"])
    row_len = 0
    if cfg["kind"] == "fixed":
        off, P, C, R = [], [], [], []
        cur = 0
        for (p, c, r) in cfg["samples"]:
            off.append(cur)
            P.append(p)
            C.append(c)
            R.append(r)
            cur += p + c + r
        total = cur
    elif cfg["kind"] == "b2b":
        off, P, C, R, total = _back_to_back(rng, cfg["n"], cfg["p"], cfg["c"], cfg["r"])
    else:
        row_len = cfg["row_len"]
        off, P, C, R, total = _greedy_rows(rng, cfg["rows"], row_len, cfg["p"], cfg["c"], cfg["r"])
    d = cfg["d"]
    return Workload(name=name, dtype=cfg["dtype"], n_q_heads=cfg["hq"], n_kv_heads=cfg["hkv"],
                    head_dim=d, total_tokens=int(total), offset=_i32(off), prefix_len=_i32(P),
                    chosen_len=_i32(C), rejected_len=_i32(R), seed=cfg["seed"], row_len=row_len,
                    scale=float(1.0 / np.sqrt(d)))


def custom_workload(samples, *, offsets=None, total_tokens=None, hq=1, hkv=1, d=64, dtype="f32",
                    seed=0, name="custom", scale=None) -> Workload:
    """Hand-specified sample table, for tests.  samples = [(p, c, r), ...]."""
    P = [s[0] for s in samples]
    C = [s[1] for s in samples]
    R = [s[2] for s in samples]
    if offsets is None:
        offsets, cur = [], 0
        for (p, c, r) in samples:
            offsets.append(cur)
            cur += p + c + r
    end = max([o + p + c + r for o, (p, c, r) in zip(offsets, samples)], default=0)
    if total_tokens is None:
        total_tokens = end
    return Workload(name=name, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d,
                    total_tokens=int(total_tokens), offset=_i32(offsets), prefix_len=_i32(P),
                    chosen_len=_i32(C), rejected_len=_i32(R), seed=seed,
                    scale=float(1.0 / np.sqrt(d)) if scale is None else float(scale))


def with_layout(w: Workload, offset, order, total_tokens, name=None) -> Workload:
    """The same samples at other positions: `offset[i]` is the new flat start of sample i
    (negative = sample left out) and `order` lists the samples by increasing offset, as a
    packer returns them.  Only re-lays the table; the positions come from the caller."""
    offset = np.asarray(offset)
    order = np.asarray([i for i in np.asarray(order) if offset[i] >= 0], dtype=np.int64)
    return Workload(name=name or (w.name + "-relaid"), dtype=w.dtype, n_q_heads=w.n_q_heads,
                    n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, total_tokens=int(total_tokens),
                    offset=_i32(offset[order]), prefix_len=_i32(w.prefix_len[order]),
                    chosen_len=_i32(w.chosen_len[order]), rejected_len=_i32(w.rejected_len[order]),
                    seed=w.seed, row_len=w.row_len, scale=w.scale)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16, returned as float32."""
    return from_bf16_bits(to_bf16_bits(x))


def make_tensors(w: Workload, names=("Q", "K", "V", "dO")) -> dict:
    """N(0,1) float32 tensors in the order Q, K, V, dO from default_rng(seed + 1000).

    Shapes [T, H, d] with d fastest.  For bf16 workloads the values are rounded
    once here, so both consumers receive identical (bf16-representable) numbers.
    Padding positions are filled too: they must not influence any real token.
    """
    rng = np.random.default_rng(w.seed + 1000)
    out = {}
    for nm in ("Q", "K", "V", "dO"):
        h = w.n_q_heads if nm in ("Q", "dO") else w.n_kv_heads
        x = rng.standard_normal((w.total_tokens, h, w.head_dim), dtype=np.float32)
        if w.dtype == "bf16":
            x = bf16_round(x)
        if nm in names:
            out[nm] = x
    return out


def paired_workload(w: Workload):
    """The unshared 'normal paired' format of the same samples (Section 2.1):
    every sample becomes two plain-causal documents [prompt|chosen] and
    [prompt|rejected].  Packed workloads re-pack units of 2p+c+r tokens greedily
    into rows of the same length (more rows result).

    Returns (workload, src, dup) where src[t] is the shared-format token that
    paired token t copies (-1 for padding) and dup[t] is True for the second
    copy of a prompt token (its dO is zeroed so gradients stay comparable).
    """
    off, P = [], []
    src_chunks = []
    units = []
    for i in range(w.n_samples):
        o, p, c, r = int(w.offset[i]), int(w.prefix_len[i]), int(w.chosen_len[i]), int(w.rejected_len[i])
        units.append((o, p, c, r))
    cur = 0
    row_len = w.row_len
    total = 0
    src_list, dup_list = [], []
    if row_len:
        row, fill = 0, 0
        for (o, p, c, r) in units:
            n = 2 * p + c + r
            if n > row_len:
                raise ValueError("paired unit longer than a packed row")
            if fill + n > row_len:
                row += 1
                fill = 0
            base = row * row_len + fill
            off += [base, base + p + c]
            P += [p + c, p + r]
            src_list.append((base, o, p, c, r))
            fill += n
        total = (row + 1) * row_len
    else:
        for (o, p, c, r) in units:
            off += [cur, cur + p + c]
            P += [p + c, p + r]
            src_list.append((cur, o, p, c, r))
            cur += 2 * p + c + r
        total = cur
    src = np.full(total, -1, dtype=np.int64)
    dup = np.zeros(total, dtype=bool)
    for (base, o, p, c, r) in src_list:
        src[base:base + p + c] = np.arange(o, o + p + c)
        src[base + p + c:base + 2 * p + c] = np.arange(o, o + p)
        dup[base + p + c:base + 2 * p + c] = True
        src[base + 2 * p + c:base + 2 * p + c + r] = np.arange(o + p + c, o + p + c + r)
    z = np.zeros(len(off), dtype=np.int32)
    pw = Workload(name=w.name + "-paired", dtype=w.dtype, n_q_heads=w.n_q_heads,
                  n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, total_tokens=int(total),
                  offset=_i32(off), prefix_len=_i32(P), chosen_len=z.copy(), rejected_len=z.copy(),
                  seed=w.seed, row_len=row_len, scale=w.scale)
    return pw, src, dup
