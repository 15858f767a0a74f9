"""CPU oracle for prefix-shared DPO attention (forward, backward, block mask).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
the library computes.  Only the tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does.  It shares no
code with the HIP path and does not import it.

What it follows:
  * the prefix-sharing mask (Algorithm 1) and its packed form (Algorithm 3),
    stated through token roles (prompt / chosen / rejected) found from the
    materialised per-token arrays I_chosen, I_rejected (completion start indices)
    and D (document ids): a token reads the not-later tokens of its own sample,
    except that rejected tokens do not read chosen tokens (Section 3.1);
  * the baseline packing mask of Algorithm 2 (per-token response ids R);
  * ordinary softmax attention on the allowed pairs (Section 3.1 states that
    nothing else changes), with the textbook explicit backward;
  * the per-mini-batch block mask of Section 3.1 (blocks with no allowed pair are
    skipped), as a brute-force classification over the dense boolean mask;
  * First-Fit-Decreasing packing of whole samples into fixed-length rows
    (Section 4.3.2), as the textbook loop;
  * rotary position embedding with the position ids of Section 3.1 (every
    response restarts right behind the prompt, as in the paired format);
  * the total log-probability of every response and the DPO loss of Eq. 1
    (Section 2.1), with their gradients;
  * a whole self-attention layer (projections, rotary embedding, attention,
    output projection) with its explicit backward (Section 4.2's attention-layer
    micro-benchmark).

Readings where the paper is silent (all restated where they are used):
  - start indices are row-absolute positions (they are compared with q and kv);
  - padding tokens belong to no document: they are never keys, their query row
    is empty, and every output at a padding position is exactly zero
    (LSE = -inf);
  - grouped-query heads: q-heads [g*G, (g+1)*G) use kv-head g;
  - the softmax scale is a parameter; LSE is the natural log of the sum of
    exp(scaled scores).

Arithmetic is float64 throughout.  A matmul, max, exp, sum and log are the only
library steps; there is no tiling or fusion, each sample's block is dense.

Parity pins (see tests/test_oracle_*.py): explicit set description of the mask,
closed-form pair counts and the paper's two ideal-speedup footnotes, pure-Python
brute force, torch fp64 scaled_dot_product_attention (+autograd), finite
differences, the no-contamination invariant against plain causal attention on
[prompt|chosen] and [prompt|rejected], packing independence, response swap
symmetry, GQA expansion; for the packer a hand-worked example, the first-fit
property checked by replay, and the 11/9 OPT + 6/9 bound against a brute-force
optimum; for the rotary embedding explicit 2x2 rotation matrices, the
relative-position property, finite differences, and equality with plain causal
attention over [prompt | response] with ordinary positions; for the
log-probabilities torch's cross entropy over the paired format, a closed form
for uniform logits and autograd; for the layer the same layer built from torch
operations and differentiated by autograd.  No function here is unpinned.
"""
from __future__ import annotations

import numpy as np

SKIPPED, PARTIAL, FULL = 0, 1, 2
PAD_DOC = -1
PAD_START = np.iinfo(np.int32).max


# --------------------------------------------------------------------------
# per-token arrays (the inputs of Algorithm 3)
# --------------------------------------------------------------------------
def index_arrays(offset, prefix_len, chosen_len, rejected_len, total_tokens):
    """Materialise I_chosen, I_rejected, D for a flat buffer of total_tokens.

    Every token of document i stores that document's chosen start
    offset+prefix and rejected start offset+prefix+chosen (Algorithm 3 reads
    them at the query position).  Padding gets D = -1 and zero indices.
    """
    T = int(total_tokens)
    I_chosen = np.zeros(T, dtype=np.int64)
    I_rejected = np.zeros(T, dtype=np.int64)
    D = np.full(T, PAD_DOC, dtype=np.int64)
    for i in range(len(offset)):
        o, p, c, r = int(offset[i]), int(prefix_len[i]), int(chosen_len[i]), int(rejected_len[i])
        n = p + c + r
        if o < 0 or p < 0 or c < 0 or r < 0 or o + n > T:
            raise ValueError("sample %d out of range" % i)
        if np.any(D[o:o + n] != PAD_DOC):
            raise ValueError("sample %d overlaps another" % i)
        D[o:o + n] = i
        I_chosen[o:o + n] = o + p
        I_rejected[o:o + n] = o + p + c
    return I_chosen, I_rejected, D


def response_ids(offset, prefix_len, chosen_len, rejected_len, total_tokens):
    """Per-token response ids R of Algorithm 2 for the paired format, in which
    each document is one [prompt | response] unit (chosen_len = rejected_len = 0
    in this library's sample table)."""
    T = int(total_tokens)
    R = np.full(T, PAD_DOC, dtype=np.int64)
    for i in range(len(offset)):
        n = int(prefix_len[i]) + int(chosen_len[i]) + int(rejected_len[i])
        R[int(offset[i]):int(offset[i]) + n] = i
    return R


# --------------------------------------------------------------------------
# masks
# --------------------------------------------------------------------------
# Every token of a sample plays one of three roles.  Section 3.1 states who may read
# whom: a token reads earlier tokens of its own sample (and itself), and the only
# role pair that is forbidden on top of that is "a rejected-response token reading a
# chosen-response token".  The three masks below are that sentence; the per-token
# arrays of Algorithms 1-3 (completion start indices, document / response ids) are
# only used to find a token's role and sample.
PROMPT, CHOSEN, REJECTED = 0, 1, 2


def _role(t, chosen_start, rejected_start):
    """Role of position t in a sample whose chosen response starts at chosen_start and
    whose rejected response starts at rejected_start (chosen_start <= rejected_start)."""
    t = np.asarray(t)
    return np.where(t < chosen_start, PROMPT, np.where(t < rejected_start, CHOSEN, REJECTED))


def prefix_sharing_mask(q, kv, chosen_ind, rejected_ind):
    """Mask of Algorithm 1 for one sample (positions relative to the same origin as
    the two start indices): not-later tokens, minus rejected-reads-chosen."""
    q, kv = np.asarray(q), np.asarray(kv)
    forbidden_roles = (_role(q, chosen_ind, rejected_ind) == REJECTED) & \
                      (_role(kv, chosen_ind, rejected_ind) == CHOSEN)
    return (kv <= q) & ~forbidden_roles


def packed_prefix_sharing_mask(q, kv, I_chosen, I_rejected, D):
    """Mask of Algorithm 3 over the flat buffer.  q, kv: broadcastable integer arrays.
    Roles are taken relative to the query's sample (the start indices stored at the
    query position); a key of another sample, or padding on either side (which is in
    no sample, itself included), never matches."""
    q, kv = np.asarray(q), np.asarray(kv)
    same_sample = (D[q] == D[kv]) & (D[q] != PAD_DOC)
    q_role = _role(q, I_chosen[q], I_rejected[q])
    kv_role = _role(kv, I_chosen[q], I_rejected[q])
    return same_sample & (kv <= q) & ~((q_role == REJECTED) & (kv_role == CHOSEN))


def response_id_mask(q, kv, R):
    """Mask of Algorithm 2 (packing without prefix sharing): every [prompt | response]
    unit has its own id and a token reads the not-later tokens of its unit."""
    q, kv = np.asarray(q), np.asarray(kv)
    same_unit = (R[q] == R[kv]) & (R[q] != PAD_DOC)
    return same_unit & (kv <= q)


# ---- any number of responses per prompt
# Section 2.2 notes the kinship of the prefix-sharing mask with tree-structured attention
# masks: the prompt is the trunk, every response a branch.  A token reads the not-later
# tokens of its own sample that lie on its path to the root: the prompt, and its own
# branch.  With two branches this is exactly the mask above.
def branch_arrays(offset, prefix_len, resp_ptr, resp_len, total_tokens):
    """Per-token sample id D (-1 = padding) and branch id B (0 = prompt, j = j-th response,
    counted from 1) for samples [prompt | response 1 | ... | response k]; the responses of
    sample i are resp_len[resp_ptr[i] : resp_ptr[i + 1]]."""
    T = int(total_tokens)
    D = np.full(T, PAD_DOC, dtype=np.int64)
    B = np.zeros(T, dtype=np.int64)
    for i in range(len(offset)):
        t = int(offset[i])
        lens = [int(prefix_len[i])] + [int(x) for x in resp_len[int(resp_ptr[i]):int(resp_ptr[i + 1])]]
        if t < 0 or min(lens) < 0 or t + sum(lens) > T:
            raise ValueError("sample %d out of range" % i)
        if np.any(D[t:t + sum(lens)] != PAD_DOC):
            raise ValueError("sample %d overlaps another" % i)
        for j, n in enumerate(lens):
            D[t:t + n] = i
            B[t:t + n] = j
            t += n
    return D, B


def branch_mask(q, kv, D, B):
    """allowed(q, kv) for samples with any number of responses."""
    q, kv = np.asarray(q), np.asarray(kv)
    same_sample = (D[q] == D[kv]) & (D[q] != PAD_DOC)
    on_path = (B[kv] == 0) | (B[kv] == B[q])
    return same_sample & (kv <= q) & on_path


def dense_branch_mask(D, B, q_lo=0, q_hi=None, k_lo=0, k_hi=None):
    T = D.shape[0]
    q_hi = T if q_hi is None else q_hi
    k_hi = T if k_hi is None else k_hi
    q = np.arange(q_lo, q_hi, dtype=np.int64)[:, None]
    kv = np.arange(k_lo, k_hi, dtype=np.int64)[None, :]
    return branch_mask(q, kv, D, B)


def branch_token_descriptors(D, B):
    """Per-token (s, hole_lo, hole_hi) as int32 [T, 3] for any number of responses: s = first
    token of the sample; the keys in [s, q] that a token of response j >= 2 must not read are
    the earlier responses, one contiguous range [first token behind the prompt, first token
    of response j); (0, 0) for everything else; s = INT32_MAX for padding."""
    T = D.shape[0]
    desc = np.zeros((T, 3), dtype=np.int32)
    first_of_sample, first_of_branch = {}, {}
    for t in range(T):                      # first positions, in one sweep
        if D[t] != PAD_DOC:
            first_of_sample.setdefault(int(D[t]), t)
            first_of_branch.setdefault((int(D[t]), int(B[t])), t)
    for t in range(T):
        d, b = int(D[t]), int(B[t])
        if d == PAD_DOC:
            desc[t, 0] = PAD_START
            continue
        desc[t, 0] = first_of_sample[d]
        if b >= 2:
            # first token behind the prompt (if every earlier response is empty that is the
            # token's own response, and the range is empty)
            desc[t, 1] = min(first_of_branch[(d, j)] for j in range(1, b + 1) if (d, j) in first_of_branch)
            desc[t, 2] = first_of_branch[(d, b)]
    return desc


def dense_mask(I_chosen, I_rejected, D, q_lo=0, q_hi=None, k_lo=0, k_hi=None):
    """Boolean matrix allowed[q - q_lo, kv - k_lo] of Algorithm 3."""
    T = D.shape[0]
    q_hi = T if q_hi is None else q_hi
    k_hi = T if k_hi is None else k_hi
    q = np.arange(q_lo, q_hi, dtype=np.int64)[:, None]
    kv = np.arange(k_lo, k_hi, dtype=np.int64)[None, :]
    return packed_prefix_sharing_mask(q, kv, I_chosen, I_rejected, D)


def count_allowed(I_chosen, I_rejected, D, stripe=256):
    """Number of allowed (q, kv) pairs, counted on the dense mask stripe by stripe."""
    T = D.shape[0]
    total = 0
    for q_lo in range(0, T, stripe):
        q_hi = min(T, q_lo + stripe)
        total += int(dense_mask(I_chosen, I_rejected, D, q_lo, q_hi, 0, q_hi).sum())
    return total


# --------------------------------------------------------------------------
# block mask (Section 3.1: computed once per mini-batch, blocks with no allowed
# pair are skipped)
# --------------------------------------------------------------------------
def classify_tiles(I_chosen, I_rejected, D, tile_q, tile_k, mask=None):
    """Brute-force class of every (q-tile, k-tile) of the global grid.
    `mask(q_lo, q_hi, k_lo, k_hi)`, if given, replaces the two-response dense mask
    (see dense_branch_mask for samples with any number of responses).

    Tile t covers tokens [t*tile, min((t+1)*tile, T)).  SKIPPED: no allowed
    pair.  FULL: the unclipped tile_q x tile_k rectangle lies inside the buffer
    and every pair is allowed.  PARTIAL: anything else.  Returns a uint8 matrix
    [n_q_tiles, n_k_tiles].
    """
    T = D.shape[0]
    nq = (T + tile_q - 1) // tile_q
    nk = (T + tile_k - 1) // tile_k
    cls = np.zeros((nq, nk), dtype=np.uint8)
    for tq in range(nq):
        q_lo, q_hi = tq * tile_q, min(T, (tq + 1) * tile_q)
        # keys beyond the last query of the stripe fail the causal clause
        k_end = q_hi
        stripe = mask(q_lo, q_hi, 0, k_end) if mask else dense_mask(I_chosen, I_rejected, D, q_lo, q_hi, 0, k_end)
        for tk in range((k_end + tile_k - 1) // tile_k):
            k_lo, k_hi = tk * tile_k, min(T, (tk + 1) * tile_k)
            blk = stripe[:, k_lo:min(k_hi, k_end)]
            n_allowed = int(blk.sum())
            if n_allowed == 0:
                continue
            unclipped = (q_hi - q_lo == tile_q) and (k_hi - k_lo == tile_k)
            if unclipped and k_hi <= k_end and n_allowed == tile_q * tile_k:
                cls[tq, tk] = FULL
            else:
                cls[tq, tk] = PARTIAL
    return cls


def csr_q_major(cls):
    """q-major CSR of the non-skipped tiles: row_ptr[n_q+1], k-tile index
    (ascending inside a row) and class of every entry."""
    nq = cls.shape[0]
    row_ptr = np.zeros(nq + 1, dtype=np.int32)
    idx, cl = [], []
    for tq in range(nq):
        ks = np.nonzero(cls[tq])[0]
        idx.append(ks.astype(np.int32))
        cl.append(cls[tq, ks])
        row_ptr[tq + 1] = row_ptr[tq] + len(ks)
    idx = np.concatenate(idx) if idx else np.zeros(0, np.int32)
    cl = np.concatenate(cl) if cl else np.zeros(0, np.uint8)
    return row_ptr, idx.astype(np.int32), cl.astype(np.uint8)


def csr_k_major(cls):
    """k-major CSR (for dK/dV): row_ptr[n_k+1], q-tile index ascending, class."""
    return csr_q_major(np.ascontiguousarray(cls.T))


def token_descriptors(I_chosen, I_rejected, D):
    """Per-token (s, hole_lo, hole_hi) as int32 [T, 3]: s = first token of the
    token's document; (hole_lo, hole_hi) = (chosen start, rejected start) for
    tokens of the rejected response (the keys they must not see), else (0, 0);
    padding tokens get s = INT32_MAX."""
    T = D.shape[0]
    desc = np.zeros((T, 3), dtype=np.int32)
    first = {}
    for t in range(T):
        d = int(D[t])
        if d == PAD_DOC:
            desc[t, 0] = PAD_START
            continue
        if d not in first:
            first[d] = t
        desc[t, 0] = first[d]
        if I_rejected[t] <= t:
            desc[t, 1] = I_chosen[t]
            desc[t, 2] = I_rejected[t]
    return desc


# --------------------------------------------------------------------------
# attention on one dense block
# --------------------------------------------------------------------------
def _softmax_block(q, k, allowed, scale):
    """Scaled scores on allowed pairs, row softmax.  Returns P, LSE (fp64)."""
    S = scale * (q @ k.T)
    S = np.where(allowed, S, -np.inf)
    m = S.max(axis=1) if S.shape[1] else np.full(S.shape[0], -np.inf)
    m_fin = np.where(np.isfinite(m), m, 0.0)           # empty rows: avoid inf - inf
    E = np.exp(S - m_fin[:, None])                     # exp(-inf) = 0 at masked pairs
    l = E.sum(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = m_fin + np.log(l)                        # -inf for an empty row
        P = np.where(l[:, None] > 0, E / l[:, None], 0.0)
    return P, lse


def forward_block(q, k, v, allowed, scale):
    """O = softmax(scale q k^T on allowed) v for one head, dense.  fp64."""
    P, lse = _softmax_block(q, k, allowed, scale)
    return P @ v, lse, P


def backward_block(q, k, v, do, allowed, scale):
    """Explicit softmax-attention backward for one head, dense.  fp64.
    Returns dq, dk, dv, o, lse, delta."""
    P, lse = _softmax_block(q, k, allowed, scale)
    o = P @ v
    delta = (do * o).sum(axis=1)
    dv = P.T @ do
    dP = do @ v.T
    dS = P * (dP - delta[:, None])
    dq = scale * (dS @ k)
    dk = scale * (dS.T @ q)
    return dq, dk, dv, o, lse, delta


# --------------------------------------------------------------------------
# whole-buffer drivers
# --------------------------------------------------------------------------
def _as64(x):
    return np.asarray(x, dtype=np.float64)


def _blocks(D, samples):
    """Token ranges [lo, hi) of the documents to evaluate."""
    ids = np.unique(D[D != PAD_DOC]) if samples is None else np.asarray(samples)
    out = []
    for i in ids:
        t = np.nonzero(D == i)[0]
        if len(t):
            out.append((int(t[0]), int(t[-1]) + 1))
    return out


def forward(Q, K, V, scale, I_chosen, I_rejected, D, heads=None, samples=None, flat=False, mask=None):
    """Forward over the flat buffer.

    Q [T, Hq, d], K, V [T, Hkv, d] (any float dtype; used as float64).
    Returns O [T, Hq, d] and LSE [Hq, T].  Positions of padding tokens (and, when
    `heads` / `samples` restrict the work, everything not requested) hold
    O = 0 and LSE = -inf.  flat=True evaluates the whole T x T mask at once
    instead of one dense block per document (tiny inputs only); the document
    clause makes both forms identical.  `mask(q_lo, q_hi, k_lo, k_hi)`, if given,
    replaces the two-response dense mask (I_chosen, I_rejected are then unused).
    """
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    O = np.zeros((T, Hq, d))
    LSE = np.full((Hq, T), -np.inf)
    ranges = [(0, T)] if flat else _blocks(D, samples)
    for h in (range(Hq) if heads is None else heads):
        g = h // G
        for lo, hi in ranges:
            allowed = mask(lo, hi, lo, hi) if mask else dense_mask(I_chosen, I_rejected, D, lo, hi, lo, hi)
            o, lse, _ = forward_block(_as64(Q[lo:hi, h]), _as64(K[lo:hi, g]), _as64(V[lo:hi, g]),
                                      allowed, scale)
            O[lo:hi, h] = o
            LSE[h, lo:hi] = lse
    return O, LSE


def backward(Q, K, V, dO, scale, I_chosen, I_rejected, D, heads=None, samples=None, flat=False, mask=None):
    """Backward over the flat buffer from the oracle's own O and LSE.

    Returns dict with dQ [T, Hq, d], dK, dV [T, Hkv, d], O, LSE [Hq, T],
    delta [Hq, T].  dK and dV sum the contributions of the q-heads evaluated
    (all G heads of a group unless `heads` restricts them): the prompt's keys
    collect gradient from prompt, chosen and rejected queries alike.
    """
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = dict(dQ=np.zeros((T, Hq, d)), dK=np.zeros((T, Hkv, d)), dV=np.zeros((T, Hkv, d)),
               O=np.zeros((T, Hq, d)), LSE=np.full((Hq, T), -np.inf), delta=np.zeros((Hq, T)))
    ranges = [(0, T)] if flat else _blocks(D, samples)
    for h in (range(Hq) if heads is None else heads):
        g = h // G
        for lo, hi in ranges:
            allowed = mask(lo, hi, lo, hi) if mask else dense_mask(I_chosen, I_rejected, D, lo, hi, lo, hi)
            dq, dk, dv, o, lse, delta = backward_block(
                _as64(Q[lo:hi, h]), _as64(K[lo:hi, g]), _as64(V[lo:hi, g]), _as64(dO[lo:hi, h]),
                allowed, scale)
            out["dQ"][lo:hi, h] = dq
            out["dK"][lo:hi, g] += dk
            out["dV"][lo:hi, g] += dv
            out["O"][lo:hi, h] = o
            out["LSE"][h, lo:hi] = lse
            out["delta"][h, lo:hi] = delta
    return out


def forward_rows(Q, K, V, scale, I_chosen, I_rejected, D, h, rows):
    """O and LSE of individual query rows (one head), each computed from the
    definition against all keys up to the row.  For spot checks at sizes where
    the full problem is too large."""
    Hq, Hkv = Q.shape[1], K.shape[1]
    g = h // (Hq // Hkv)
    O = np.zeros((len(rows), Q.shape[2]))
    LSE = np.full(len(rows), -np.inf)
    for n, i in enumerate(rows):
        allowed = dense_mask(I_chosen, I_rejected, D, i, i + 1, 0, i + 1)
        o, lse, _ = forward_block(_as64(Q[i:i + 1, h]), _as64(K[:i + 1, g]), _as64(V[:i + 1, g]),
                                  allowed, scale)
        O[n] = o[0]
        LSE[n] = lse[0]
    return O, LSE


# --------------------------------------------------------------------------
# packing (Section 4.3.2: First-Fit-Decreasing sampler; the unit is a whole
# sample, Section 3.2)
# --------------------------------------------------------------------------
def ffd_pack(lengths, row_len, max_rows=0):
    """First-Fit-Decreasing, written out: take the units from the longest to the
    shortest (equal lengths in their original order); put each into the first row,
    in order of opening, that still has room, directly behind what the row already
    holds; open a new row when none has room (with max_rows > 0: leave the unit out
    when that many rows are open).  Returns (offset [n] with -1 for units left out,
    n_rows): offset = row * row_len + position in the row."""
    n = len(lengths)
    by_len = sorted(range(n), key=lambda i: -int(lengths[i]))   # Python's sort is stable
    fill = []                                                   # tokens used per open row
    offset = [-1] * n
    for i in by_len:
        need = int(lengths[i])
        if need <= 0 or need > row_len:
            raise ValueError("unit %d does not fit a row" % i)
        placed = False
        for r in range(len(fill)):
            if fill[r] + need <= row_len:
                offset[i] = r * row_len + fill[r]
                fill[r] += need
                placed = True
                break
        if not placed and (max_rows == 0 or len(fill) < max_rows):
            offset[i] = len(fill) * row_len
            fill.append(need)
    return np.asarray(offset, dtype=np.int32), len(fill)


# --------------------------------------------------------------------------
# rotary position embedding with the position ids of the paired format
# (Section 3.1: position ids are set so that each response sits where it would
# sit in the normal paired format, i.e. every response restarts right behind the
# prompt)
# --------------------------------------------------------------------------
def position_ids(D, B):
    """Position id of every token from its sample id D and branch id B (branch_arrays;
    for the paper's two responses B = 1 is chosen, B = 2 rejected): prompt tokens count
    from 0, the tokens of EVERY response count on from the prompt's length.  Padding: 0."""
    T = D.shape[0]
    pos = np.zeros(T, dtype=np.int64)
    prompt_len, seen = {}, {}
    for t in range(T):
        d, b = int(D[t]), int(B[t])
        if d == PAD_DOC:
            continue
        if b == 0:
            pos[t] = prompt_len.get(d, 0)
            prompt_len[d] = prompt_len.get(d, 0) + 1
        else:
            pos[t] = prompt_len.get(d, 0) + seen.get((d, b), 0)
            seen[(d, b)] = seen.get((d, b), 0) + 1
    return pos


def rope_angles(pos, head_dim, theta):
    """angle[t, i] = pos[t] * theta^(-2 i / head_dim), i = 0 .. head_dim/2 - 1."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.asarray(pos, dtype=np.float64)[:, None] * theta ** (-2.0 * i / head_dim)[None, :]


def rope_rotate(x, pos, theta, inverse=False):
    """Rotary embedding of x [T, H, d] (fp64): dimension i is paired with i + d/2 and the pair
    is turned by angle[t, i] (by -angle with inverse=True, which is also the map that takes a
    gradient w.r.t. the rotated tensor to the gradient w.r.t. the unrotated one)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    ang = rope_angles(pos, d, theta)
    if inverse:
        ang = -ang
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :d // 2], x[..., d // 2:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def backward_rope(Q, K, V, dO, scale, theta, D, B, mask, heads=None, samples=None, round_operands=None):
    """Attention with rotary embedding applied to Q and K first, forward and backward.
    `round_operands(x)`, if given, is applied to the rotated Q and K before the attention
    (a bf16 model stores the rotated activations in bf16).  dQ and dK are gradients w.r.t.
    the UNROTATED Q and K.  Also returns the rotated operands Qr, Kr."""
    pos = position_ids(D, B)
    Qr, Kr = rope_rotate(Q, pos, theta), rope_rotate(K, pos, theta)
    if round_operands is not None:
        Qr, Kr = round_operands(Qr), round_operands(Kr)
    out = backward(Qr, Kr, V, dO, scale, None, None, D, heads=heads, samples=samples, mask=mask)
    out["dQ"] = rope_rotate(out["dQ"], pos, theta, inverse=True)
    out["dK"] = rope_rotate(out["dK"], pos, theta, inverse=True)
    out["Qr"], out["Kr"], out["pos"] = Qr, Kr, pos
    return out


# --------------------------------------------------------------------------
# per-response log-probabilities and the DPO loss (Section 2.1, Eq. 1)
# --------------------------------------------------------------------------
# Eq. 1 needs log pi(y | x), the total log-probability of each completion.  In the
# prefix-shared sequence the logits row of token t predicts the next token of t's own
# branch: inside a response that is token t + 1; the LAST prompt token predicts the first
# token of every response.  (Eq. 1 is printed with a ratio of the two log-probabilities; it
# is read as DPO defines it, with the difference log pi_theta - log pi_ref, i.e. the log of
# the ratio.)
def prediction_items(offset, prefix_len, resp_ptr, resp_len):
    """[(response index, logits row, position of the target token)] in response order.  A
    response whose sample has an empty prompt has nothing to predict its first token from:
    that token contributes nothing."""
    items = []
    for i in range(len(offset)):
        o, p = int(offset[i]), int(prefix_len[i])
        start = o + p
        for j in range(int(resp_ptr[i]), int(resp_ptr[i + 1])):
            n = int(resp_len[j])
            for u in range(n):
                if u == 0:
                    if p > 0:
                        items.append((j, o + p - 1, start))
                else:
                    items.append((j, start + u - 1, start + u))
            start += n
    return items


def log_softmax_rows(logits):
    x = np.asarray(logits, dtype=np.float64)
    m = x.max(axis=-1, keepdims=True)
    return x - m - np.log(np.exp(x - m).sum(axis=-1, keepdims=True))


def response_logprobs(logits, token_ids, offset, prefix_len, resp_ptr, resp_len):
    """log pi(response j | prompt) for every response: the sum over its tokens of the
    log-softmax of the predicting row at that token's id.  logits [T, V], token_ids [T]."""
    n_resp = int(resp_ptr[-1]) if len(resp_ptr) else 0
    out = np.zeros(n_resp)
    items = prediction_items(offset, prefix_len, resp_ptr, resp_len)
    rows = sorted({r for _, r, _ in items})
    ls = dict(zip(rows, log_softmax_rows(np.asarray(logits)[rows]))) if rows else {}
    for j, row, tpos in items:
        out[j] += ls[row][int(token_ids[tpos])]
    return out


def response_logprobs_grad(logits, token_ids, offset, prefix_len, resp_ptr, resp_len, d_logp):
    """d(sum_j d_logp[j] * logp_j) / d logits, [T, V]: each item adds d_logp[j] * (onehot(target) -
    softmax(row)) to its row; rows that predict nothing stay zero."""
    x = np.asarray(logits, dtype=np.float64)
    g = np.zeros_like(x)
    for j, row, tpos in prediction_items(offset, prefix_len, resp_ptr, resp_len):
        p = np.exp(log_softmax_rows(x[row:row + 1])[0])
        g[row] -= d_logp[j] * p
        g[row, int(token_ids[tpos])] += d_logp[j]
    return g


def dpo_loss(logp_policy, logp_ref, beta):
    """Per-sample DPO loss for responses stored as (chosen, rejected) pairs:
    -log sigmoid(beta * ((pc - rc) - (pr - rr))), and its derivative w.r.t. the policy
    log-probabilities (same layout)."""
    lp, lr = np.asarray(logp_policy, dtype=np.float64), np.asarray(logp_ref, dtype=np.float64)
    z = beta * ((lp[0::2] - lr[0::2]) - (lp[1::2] - lr[1::2]))
    loss = np.logaddexp(0.0, -z)                 # -log sigmoid(z)
    dz = -1.0 / (1.0 + np.exp(z))                # d loss / d z = -sigmoid(-z)
    d = np.zeros_like(lp)
    d[0::2] = beta * dz
    d[1::2] = -beta * dz
    return loss, d


# --------------------------------------------------------------------------
# a whole self-attention layer (the "attention layer" micro-benchmark of Section 4.2)
# --------------------------------------------------------------------------
def layer_backward(X, Wq, Wk, Wv, Wo, dY, scale, theta, D, B, mask, n_q_heads, n_kv_heads, round_act=None):
    """y = attention(rope(x Wq^T), rope(x Wk^T), x Wv^T) Wo^T with its explicit backward.
    X, dY [T, hidden]; weights [out_features, in_features].  `round_act(x)`, if given, is
    applied wherever a bf16 model stores an activation (projections, rotated operands,
    attention output, the gradients handed between the stages).  Returns Y, dX, dWq, dWk, dWv,
    dWo (fp64)."""
    r = (lambda x: x) if round_act is None else round_act
    X, dY = np.asarray(X, dtype=np.float64), np.asarray(dY, dtype=np.float64)
    Wq, Wk, Wv, Wo = (np.asarray(w, dtype=np.float64) for w in (Wq, Wk, Wv, Wo))
    T = X.shape[0]
    d = Wq.shape[0] // n_q_heads
    Q = r(X @ Wq.T).reshape(T, n_q_heads, d)
    K = r(X @ Wk.T).reshape(T, n_kv_heads, d)
    V = r(X @ Wv.T).reshape(T, n_kv_heads, d)
    dO = r(dY @ Wo).reshape(T, n_q_heads, d)
    a = backward_rope(Q, K, V, dO, scale, theta, D, B, mask, round_operands=round_act)
    O = r(a["O"]).reshape(T, -1)
    dQ, dK, dV = (r(a[n]).reshape(T, -1) for n in ("dQ", "dK", "dV"))
    return dict(Y=O @ Wo.T, dWo=dY.T @ O, dWq=dQ.T @ X, dWk=dK.T @ X, dWv=dV.T @ X,
                dX=dQ @ Wq + dK @ Wk + dV @ Wv)
