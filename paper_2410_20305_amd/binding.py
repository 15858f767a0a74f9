"""ctypes marshalling for libpsattn.so.  Names mirror include/psattn.h."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

GRID_FWD, GRID_BWD = 0, 1
TILE_SKIPPED, TILE_PARTIAL, TILE_FULL = 0, 1, 2
F32, BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = [
    "psattn_build_meta", "psattn_build_meta_host", "psattn_free_meta", "psattn_meta_tiles",
    "psattn_meta_copy_csr", "psattn_meta_copy_tok_desc", "psattn_meta_copy_key_desc",
    "psattn_meta_allowed_pairs", "psattn_fwd", "psattn_bwd", "psattn_bwd_workspace_bytes",
    "psattn_kernel_name", "psattn_strerror", "psattn_profile_enable", "psattn_profile_read",
    "psattn_free_meta_async", "psattn_trim_pool", "psattn_uses_mfma",
    "psattn_bwd_static", "psattn_bwd_static_max_rows", "psattn_probe_dq_atomics", "psattn_probe_mfma_peak",
    "psattn_pack_ffd", "psattn_build_meta_multi", "psattn_build_meta_multi_host",
    "psattn_rope_create", "psattn_rope_free", "psattn_rope_k", "psattn_fwd_rope", "psattn_bwd_rope",
    "psattn_meta_copy_positions",
    "psattn_logprob_plan", "psattn_logprob_plan_free", "psattn_logprob_plan_info", "psattn_logprob_fwd",
    "psattn_logprob_bwd", "psattn_dpo_loss",
]


class PsattnError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, _strerror(status), status))


def lib_path() -> str:
    # PSATTN_LIB: another build of the same library, for A/B measurements of kernel variants
    return os.environ.get("PSATTN_LIB") or os.path.join(_HERE, "libpsattn.so")


def load_library():
    """Load libpsattn.so (built by paper_2410_20305_amd/build.py).  Raises if absent."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("libpsattn.so not built: run `python -m paper_2410_20305_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(path)
    i32, i64, vp, f32 = C.c_int32, C.c_int64, C.c_void_p, C.c_float
    pi32 = C.POINTER(C.c_int32)
    lib.psattn_build_meta.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, C.POINTER(vp)]
    lib.psattn_build_meta_host.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, C.POINTER(vp)]
    lib.psattn_build_meta_multi.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, C.POINTER(vp)]
    lib.psattn_build_meta_multi_host.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, C.POINTER(vp)]
    lib.psattn_rope_create.argtypes = [i32, f32, i32, vp, C.POINTER(vp)]
    lib.psattn_rope_free.argtypes = [vp]
    lib.psattn_rope_k.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    lib.psattn_fwd_rope.argtypes = [vp, vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.psattn_bwd_rope.argtypes = [vp, vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                    C.c_size_t, vp]
    lib.psattn_meta_copy_positions.argtypes = [vp, vp, pi32]
    lib.psattn_logprob_plan.argtypes = [i32, vp, vp, vp, vp, i32, vp, C.POINTER(vp)]
    lib.psattn_logprob_plan_free.argtypes = [vp]
    lib.psattn_logprob_plan_info.argtypes = [vp, pi32, pi32, C.POINTER(i64)]
    lib.psattn_logprob_fwd.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
    lib.psattn_logprob_bwd.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.psattn_dpo_loss.argtypes = [i32, f32, vp, vp, vp, vp, vp]
    lib.psattn_free_meta.argtypes = [vp]
    lib.psattn_free_meta_async.argtypes = [vp, vp]
    lib.psattn_trim_pool.argtypes = []
    lib.psattn_uses_mfma.argtypes = [vp, i32, i32, f32, i32]
    lib.psattn_meta_tiles.argtypes = [vp, i32, pi32, pi32, pi32, pi32, C.POINTER(i64)]
    lib.psattn_meta_copy_csr.argtypes = [vp, i32, vp, vp, vp]
    lib.psattn_meta_copy_tok_desc.argtypes = [vp, vp]
    lib.psattn_meta_copy_key_desc.argtypes = [vp, vp]
    lib.psattn_meta_allowed_pairs.argtypes = [vp, C.POINTER(i64)]
    lib.psattn_fwd.argtypes = [vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp]
    lib.psattn_bwd.argtypes = [vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                               C.c_size_t, vp]
    lib.psattn_bwd_static.argtypes = [vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.psattn_bwd_static_max_rows.argtypes = []
    lib.psattn_bwd_static_max_rows.restype = C.c_size_t
    lib.psattn_probe_dq_atomics.argtypes = [vp, i32, i32, vp, i32, vp]
    lib.psattn_probe_mfma_peak.argtypes = [i32, i32, i32, vp, vp]
    lib.psattn_pack_ffd.argtypes = [i32, vp, vp, vp, i32, i32, vp, vp, pi32, C.POINTER(i64)]
    lib.psattn_bwd_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.psattn_bwd_workspace_bytes.restype = C.c_size_t
    lib.psattn_kernel_name.argtypes = [i32, i32]
    lib.psattn_kernel_name.restype = C.c_char_p
    lib.psattn_profile_enable.argtypes = [i32]
    lib.psattn_profile_read.argtypes = [vp, vp]
    lib.psattn_strerror.argtypes = [C.c_int]
    lib.psattn_strerror.restype = C.c_char_p
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is C.c_int:
            fn.restype = C.c_int
    _LIB = lib
    return lib


def _strerror(status: int) -> str:
    try:
        return load_library().psattn_strerror(int(status)).decode()
    except Exception:
        return "status"


def _check(status, what):
    if status != 0:
        raise PsattnError(status, what)


def _i32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _stream_ptr(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


class Meta:
    """Owner of a psattn_meta handle."""

    def __init__(self, handle, total_tokens, on_device):
        self._h = handle
        self.total_tokens = int(total_tokens)
        self.on_device = on_device

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("meta already freed")
        return self._h

    def free(self):
        if self._h is not None:
            lib = load_library()
            _check(lib.psattn_free_meta(self._h), "psattn_free_meta")
            self._h = None

    def free_async(self, stream=None):
        """Stream-ordered release: the buffers are reused only after the work enqueued so
        far on `stream` (default: torch's current stream) has finished."""
        if self._h is not None:
            lib = load_library()
            _check(lib.psattn_free_meta_async(self._h, _stream_ptr(stream)), "psattn_free_meta_async")
            self._h = None

    def uses_mfma(self, dtype_code, head_dim, scale, backward=False) -> bool:
        st = load_library().psattn_uses_mfma(self.handle, int(dtype_code), int(head_dim), float(scale),
                                             1 if backward else 0)
        if st < 0:
            raise PsattnError(st, "psattn_uses_mfma")
        return bool(st)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def tiles(self, grid=GRID_FWD):
        lib = load_library()
        tq, tk, nq, nk, ne = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32(), C.c_int64()
        _check(lib.psattn_meta_tiles(self.handle, grid, C.byref(tq), C.byref(tk), C.byref(nq), C.byref(nk),
                                     C.byref(ne)), "psattn_meta_tiles")
        return dict(tile_q=tq.value, tile_k=tk.value, n_q_tiles=nq.value, n_k_tiles=nk.value,
                    n_entries=ne.value)

    def csr(self, grid=GRID_FWD):
        lib = load_library()
        t = self.tiles(grid)
        n_rows = t["n_q_tiles"] if grid == GRID_FWD else t["n_k_tiles"]
        row_ptr = np.zeros(n_rows + 1, dtype=np.int32)
        idx = np.zeros(max(1, t["n_entries"]), dtype=np.int32)
        cls = np.zeros(max(1, t["n_entries"]), dtype=np.uint8)
        _check(lib.psattn_meta_copy_csr(self.handle, grid, row_ptr.ctypes.data, idx.ctypes.data,
                                        cls.ctypes.data), "psattn_meta_copy_csr")
        return row_ptr, idx[:t["n_entries"]], cls[:t["n_entries"]]

    def tok_desc(self):
        lib = load_library()
        out = np.zeros((max(1, self.total_tokens), 3), dtype=np.int32)
        _check(lib.psattn_meta_copy_tok_desc(self.handle, out.ctypes.data), "psattn_meta_copy_tok_desc")
        return out[:self.total_tokens]

    def key_desc(self):
        lib = load_library()
        out = np.zeros(max(1, self.total_tokens), dtype=np.int32)
        _check(lib.psattn_meta_copy_key_desc(self.handle, out.ctypes.data), "psattn_meta_copy_key_desc")
        return out[:self.total_tokens]

    def positions(self):
        """(position id of every token, number of positions needed)."""
        lib = load_library()
        out = np.zeros(max(1, self.total_tokens), dtype=np.int32)
        n = C.c_int32()
        _check(lib.psattn_meta_copy_positions(self.handle, out.ctypes.data, C.byref(n)), "psattn_meta_copy_positions")
        return out[:self.total_tokens], n.value

    def allowed_pairs(self):
        lib = load_library()
        n = C.c_int64()
        _check(lib.psattn_meta_allowed_pairs(self.handle, C.byref(n)), "psattn_meta_allowed_pairs")
        return n.value


def psattn_build_meta(offset, prefix_len, chosen_len, rejected_len, total_tokens, tile_q=0, tile_k=0,
                      bwd_tile_q=0, bwd_tile_k=0, stream=None, host_only=False) -> Meta:
    lib = load_library()
    off, p, c, r = _i32(offset), _i32(prefix_len), _i32(chosen_len), _i32(rejected_len)
    n = off.shape[0]
    if not (p.shape[0] == c.shape[0] == r.shape[0] == n):
        raise ValueError("sample arrays differ in length")
    h = C.c_void_p()
    if host_only:
        st = lib.psattn_build_meta_host(n, off.ctypes.data, p.ctypes.data, c.ctypes.data, r.ctypes.data,
                                        int(total_tokens), tile_q, tile_k, bwd_tile_q, bwd_tile_k, C.byref(h))
        _check(st, "psattn_build_meta_host")
    else:
        st = lib.psattn_build_meta(n, off.ctypes.data, p.ctypes.data, c.ctypes.data, r.ctypes.data,
                                   int(total_tokens), tile_q, tile_k, bwd_tile_q, bwd_tile_k,
                                   _stream_ptr(stream), C.byref(h))
        _check(st, "psattn_build_meta")
    return Meta(h, total_tokens, not host_only)


def psattn_build_meta_multi(offset, prefix_len, resp_ptr, resp_len, total_tokens, tile_q=0, tile_k=0,
                            bwd_tile_q=0, bwd_tile_k=0, stream=None, host_only=False) -> Meta:
    """Block mask for samples with any number of responses per prompt (CSR-style resp_ptr / resp_len)."""
    lib = load_library()
    off, p, ptr, rl = _i32(offset), _i32(prefix_len), _i32(resp_ptr), _i32(resp_len)
    n = off.shape[0]
    if p.shape[0] != n or ptr.shape[0] != n + 1 or (n and rl.shape[0] != int(ptr[-1])):
        raise ValueError("sample arrays differ in length")
    rl_ptr = rl.ctypes.data if rl.shape[0] else None
    h = C.c_void_p()
    if host_only:
        st = lib.psattn_build_meta_multi_host(n, off.ctypes.data, p.ctypes.data, ptr.ctypes.data, rl_ptr,
                                              int(total_tokens), tile_q, tile_k, bwd_tile_q, bwd_tile_k, C.byref(h))
        _check(st, "psattn_build_meta_multi_host")
    else:
        st = lib.psattn_build_meta_multi(n, off.ctypes.data, p.ctypes.data, ptr.ctypes.data, rl_ptr,
                                         int(total_tokens), tile_q, tile_k, bwd_tile_q, bwd_tile_k,
                                         _stream_ptr(stream), C.byref(h))
        _check(st, "psattn_build_meta_multi")
    return Meta(h, total_tokens, not host_only)


def psattn_pack_ffd(prefix_len, chosen_len, rejected_len, row_len, max_rows=0):
    """First-Fit-Decreasing packing.  Returns dict(offset [n] (-1 = left out), order [n], n_rows,
    padding_tokens)."""
    lib = load_library()
    p, c, r = _i32(prefix_len), _i32(chosen_len), _i32(rejected_len)
    n = p.shape[0]
    if not (c.shape[0] == r.shape[0] == n):
        raise ValueError("sample arrays differ in length")
    offset = np.zeros(max(1, n), dtype=np.int32)
    order = np.zeros(max(1, n), dtype=np.int32)
    n_rows, pad = C.c_int32(), C.c_int64()
    st = lib.psattn_pack_ffd(n, p.ctypes.data, c.ctypes.data, r.ctypes.data, int(row_len), int(max_rows),
                             offset.ctypes.data, order.ctypes.data, C.byref(n_rows), C.byref(pad))
    _check(st, "psattn_pack_ffd")
    return dict(offset=offset[:n], order=order[:n], n_rows=n_rows.value, padding_tokens=pad.value)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("psattn supports float32 and bfloat16 tensors, got %s" % t.dtype)


def _check_tensor(t, name, shape, dtype):
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s has dtype %s, expected %s" % (name, t.dtype, dtype))


def psattn_fwd(meta: Meta, Q, K, V, scale, O=None, LSE=None, stream=None):
    """O, LSE = attention forward.  Q [T, Hq, d]; K, V [T, Hkv, d]; LSE [Hq, T] float32."""
    import torch
    lib = load_library()
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    _check_tensor(Q, "Q", (meta.total_tokens, Hq, d), None)
    _check_tensor(K, "K", (T, Hkv, d), Q.dtype)
    _check_tensor(V, "V", (T, Hkv, d), Q.dtype)
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((Hq, T), dtype=torch.float32, device=Q.device)
    _check_tensor(O, "O", Q.shape, Q.dtype)
    _check_tensor(LSE, "LSE", (Hq, T), torch.float32)
    st = lib.psattn_fwd(meta.handle, _dtype_code(Q), Hq, Hkv, d, float(scale), Q.data_ptr(), K.data_ptr(),
                        V.data_ptr(), O.data_ptr(), LSE.data_ptr(), _stream_ptr(stream))
    _check(st, "psattn_fwd")
    return O, LSE


def psattn_bwd_workspace_bytes(meta: Meta, n_q_heads, n_kv_heads, head_dim) -> int:
    return int(load_library().psattn_bwd_workspace_bytes(meta.handle, n_q_heads, n_kv_heads, head_dim))


def psattn_bwd(meta: Meta, Q, K, V, O, dO, LSE, scale, dQ=None, dK=None, dV=None, workspace=None,
               stream=None):
    """dQ, dK, dV = attention backward from the forward's O and LSE."""
    import torch
    lib = load_library()
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    _check_tensor(Q, "Q", (meta.total_tokens, Hq, d), None)
    _check_tensor(K, "K", (T, Hkv, d), Q.dtype)
    _check_tensor(V, "V", (T, Hkv, d), Q.dtype)
    _check_tensor(O, "O", Q.shape, Q.dtype)
    _check_tensor(dO, "dO", Q.shape, Q.dtype)
    _check_tensor(LSE, "LSE", (Hq, T), torch.float32)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    _check_tensor(dQ, "dQ", Q.shape, Q.dtype)
    _check_tensor(dK, "dK", K.shape, Q.dtype)
    _check_tensor(dV, "dV", V.shape, Q.dtype)
    need = psattn_bwd_workspace_bytes(meta, Hq, Hkv, d)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    ws_bytes = workspace.numel() * workspace.element_size()
    st = lib.psattn_bwd(meta.handle, _dtype_code(Q), Hq, Hkv, d, float(scale), Q.data_ptr(), K.data_ptr(),
                        V.data_ptr(), O.data_ptr(), dO.data_ptr(), LSE.data_ptr(), dQ.data_ptr(),
                        dK.data_ptr(), dV.data_ptr(), workspace.data_ptr(), ws_bytes, _stream_ptr(stream))
    _check(st, "psattn_bwd")
    return dQ, dK, dV


def psattn_bwd_static(meta: Meta, Q, K, V, O, dO, LSE, scale, dQ, dK, dV, stream=None):
    """psattn_bwd on the library's static scratch: allocates nothing, so the outputs must be given."""
    import torch
    lib = load_library()
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    _check_tensor(Q, "Q", (meta.total_tokens, Hq, d), None)
    for t, name, shape in ((K, "K", (T, Hkv, d)), (V, "V", (T, Hkv, d)), (O, "O", Q.shape), (dO, "dO", Q.shape),
                           (dQ, "dQ", Q.shape), (dK, "dK", K.shape), (dV, "dV", K.shape)):
        _check_tensor(t, name, shape, Q.dtype)
    _check_tensor(LSE, "LSE", (Hq, T), torch.float32)
    st = lib.psattn_bwd_static(meta.handle, _dtype_code(Q), Hq, Hkv, d, float(scale), Q.data_ptr(), K.data_ptr(),
                               V.data_ptr(), O.data_ptr(), dO.data_ptr(), LSE.data_ptr(), dQ.data_ptr(),
                               dK.data_ptr(), dV.data_ptr(), _stream_ptr(stream))
    _check(st, "psattn_bwd_static")
    return dQ, dK, dV


def psattn_bwd_static_max_rows() -> int:
    return int(load_library().psattn_bwd_static_max_rows())


class Rope:
    """Owner of a psattn_rope handle (cos/sin table on the current device)."""

    def __init__(self, head_dim, theta, max_positions, stream=None):
        lib = load_library()
        h = C.c_void_p()
        _check(lib.psattn_rope_create(int(head_dim), float(theta), int(max_positions), _stream_ptr(stream), C.byref(h)),
               "psattn_rope_create")
        self._h = h

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("rope table already freed")
        return self._h

    def free(self):
        if self._h is not None:
            _check(load_library().psattn_rope_free(self._h), "psattn_rope_free")
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def psattn_fwd_rope(meta: Meta, rope: Rope, Q, K, V, scale, O=None, LSE=None, Qr=None, Kr=None, stream=None):
    """O, LSE, Qr, Kr = forward with rotary embedding applied to the unrotated Q, K inside the op."""
    import torch
    lib = load_library()
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    _check_tensor(Q, "Q", (meta.total_tokens, Hq, d), None)
    _check_tensor(K, "K", (T, Hkv, d), Q.dtype)
    _check_tensor(V, "V", (T, Hkv, d), Q.dtype)
    O = torch.empty_like(Q) if O is None else O
    LSE = torch.empty((Hq, T), dtype=torch.float32, device=Q.device) if LSE is None else LSE
    Qr = torch.empty_like(Q) if Qr is None else Qr
    Kr = torch.empty_like(K) if Kr is None else Kr
    _check_tensor(O, "O", Q.shape, Q.dtype)
    _check_tensor(LSE, "LSE", (Hq, T), torch.float32)
    _check_tensor(Qr, "Qr", Q.shape, Q.dtype)
    _check_tensor(Kr, "Kr", K.shape, Q.dtype)
    st = lib.psattn_fwd_rope(meta.handle, rope.handle, _dtype_code(Q), Hq, Hkv, d, float(scale), Q.data_ptr(),
                             K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(), Qr.data_ptr(), Kr.data_ptr(),
                             _stream_ptr(stream))
    _check(st, "psattn_fwd_rope")
    return O, LSE, Qr, Kr


def psattn_bwd_rope(meta: Meta, rope: Rope, Qr, Kr, V, O, dO, LSE, scale, dQ=None, dK=None, dV=None, workspace=None,
                    stream=None):
    """dQ, dK, dV (w.r.t. the unrotated Q, K) from the forward's rotated Qr, Kr."""
    import torch
    lib = load_library()
    T, Hq, d = Qr.shape
    Hkv = Kr.shape[1]
    _check_tensor(Qr, "Qr", (meta.total_tokens, Hq, d), None)
    for t, name, shape in ((Kr, "Kr", (T, Hkv, d)), (V, "V", (T, Hkv, d)), (O, "O", Qr.shape), (dO, "dO", Qr.shape)):
        _check_tensor(t, name, shape, Qr.dtype)
    _check_tensor(LSE, "LSE", (Hq, T), torch.float32)
    dQ = torch.empty_like(Qr) if dQ is None else dQ
    dK = torch.empty_like(Kr) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    for t, name, shape in ((dQ, "dQ", Qr.shape), (dK, "dK", Kr.shape), (dV, "dV", Kr.shape)):
        _check_tensor(t, name, shape, Qr.dtype)
    need = psattn_bwd_workspace_bytes(meta, Hq, Hkv, d)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Qr.device)
    st = lib.psattn_bwd_rope(meta.handle, rope.handle, _dtype_code(Qr), Hq, Hkv, d, float(scale), Qr.data_ptr(),
                             Kr.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), LSE.data_ptr(), dQ.data_ptr(),
                             dK.data_ptr(), dV.data_ptr(), workspace.data_ptr(),
                             workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    _check(st, "psattn_bwd_rope")
    return dQ, dK, dV


class LogprobPlan:
    """Owner of a psattn_lp_plan handle."""

    def __init__(self, offset, prefix_len, resp_ptr, resp_len, total_tokens, stream=None):
        lib = load_library()
        off, p, ptr, rl = _i32(offset), _i32(prefix_len), _i32(resp_ptr), _i32(resp_len)
        h = C.c_void_p()
        _check(lib.psattn_logprob_plan(off.shape[0], off.ctypes.data, p.ctypes.data, ptr.ctypes.data,
                                       rl.ctypes.data if rl.shape[0] else None, int(total_tokens), _stream_ptr(stream),
                                       C.byref(h)), "psattn_logprob_plan")
        self._h = h
        self.total_tokens = int(total_tokens)
        a, b, c = C.c_int32(), C.c_int32(), C.c_int64()
        _check(lib.psattn_logprob_plan_info(h, C.byref(a), C.byref(b), C.byref(c)), "psattn_logprob_plan_info")
        self.n_responses, self.n_rows, self.n_items = a.value, b.value, c.value

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("plan already freed")
        return self._h

    def free(self):
        if self._h is not None:
            _check(load_library().psattn_logprob_plan_free(self._h), "psattn_logprob_plan_free")
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def psattn_logprob_fwd(plan: LogprobPlan, logits, token_ids, row_lse=None, resp_logp=None, stream=None):
    """row_lse [T], resp_logp [n_responses] from logits [T, vocab] and token_ids int32 [T]."""
    import torch
    T, V = logits.shape
    _check_tensor(logits, "logits", (plan.total_tokens, V), None)
    _check_tensor(token_ids, "token_ids", (T,), torch.int32)
    row_lse = torch.zeros(T, dtype=torch.float32, device=logits.device) if row_lse is None else row_lse
    resp_logp = torch.empty(plan.n_responses, dtype=torch.float32, device=logits.device) if resp_logp is None else resp_logp
    _check_tensor(row_lse, "row_lse", (T,), torch.float32)
    _check_tensor(resp_logp, "resp_logp", (plan.n_responses,), torch.float32)
    st = load_library().psattn_logprob_fwd(plan.handle, _dtype_code(logits), V, logits.data_ptr(), token_ids.data_ptr(),
                                           row_lse.data_ptr(), resp_logp.data_ptr(), _stream_ptr(stream))
    _check(st, "psattn_logprob_fwd")
    return row_lse, resp_logp


def psattn_logprob_bwd(plan: LogprobPlan, logits, token_ids, row_lse, d_resp_logp, dlogits=None, stream=None):
    import torch
    T, V = logits.shape
    _check_tensor(logits, "logits", (plan.total_tokens, V), None)
    _check_tensor(token_ids, "token_ids", (T,), torch.int32)
    _check_tensor(row_lse, "row_lse", (T,), torch.float32)
    _check_tensor(d_resp_logp, "d_resp_logp", (plan.n_responses,), torch.float32)
    dlogits = torch.empty_like(logits) if dlogits is None else dlogits
    _check_tensor(dlogits, "dlogits", logits.shape, logits.dtype)
    st = load_library().psattn_logprob_bwd(plan.handle, _dtype_code(logits), V, logits.data_ptr(), token_ids.data_ptr(),
                                           row_lse.data_ptr(), d_resp_logp.data_ptr(), dlogits.data_ptr(),
                                           _stream_ptr(stream))
    _check(st, "psattn_logprob_bwd")
    return dlogits


def psattn_dpo_loss(logp_policy, logp_ref, beta, stream=None):
    """loss [n_pairs], d_logp [2 n_pairs] for responses stored as (chosen, rejected) pairs."""
    import torch
    n = logp_policy.shape[0]
    if n % 2 or tuple(logp_ref.shape) != (n,):
        raise ValueError("log-probabilities must come in (chosen, rejected) pairs")
    _check_tensor(logp_policy, "logp_policy", (n,), torch.float32)
    _check_tensor(logp_ref, "logp_ref", (n,), torch.float32)
    loss = torch.empty(n // 2, dtype=torch.float32, device=logp_policy.device)
    d = torch.empty(n, dtype=torch.float32, device=logp_policy.device)
    st = load_library().psattn_dpo_loss(n // 2, float(beta), logp_policy.data_ptr(), logp_ref.data_ptr(), loss.data_ptr(),
                                        d.data_ptr(), _stream_ptr(stream))
    _check(st, "psattn_dpo_loss")
    return loss, d


def psattn_probe_dq_atomics(meta: Meta, n_q_heads, n_kv_heads, acc, mode, stream=None) -> None:
    """Measurement aid: the dQ memory operations of a one-pass backward (see include/psattn.h)."""
    if tuple(acc.shape) != (meta.total_tokens, n_q_heads, 128) or not acc.is_cuda or not acc.is_contiguous():
        raise ValueError("acc must be a contiguous float32 device tensor [T, n_q_heads, 128]")
    st = load_library().psattn_probe_dq_atomics(meta.handle, int(n_q_heads), int(n_kv_heads), acc.data_ptr(),
                                                int(mode), _stream_ptr(stream))
    _check(st, "psattn_probe_dq_atomics")


def psattn_trim_pool() -> None:
    _check(load_library().psattn_trim_pool(), "psattn_trim_pool")


def psattn_kernel_name(dt, kernel_pass) -> str:
    return load_library().psattn_kernel_name(int(dt), int(kernel_pass)).decode()


def psattn_profile_enable(on: bool) -> None:
    _check(load_library().psattn_profile_enable(1 if on else 0), "psattn_profile_enable")


def psattn_profile_read():
    """Returns (sum_ms[4], count[4]) per pass: 0 forward, 1 delta, 2 dQ, 3 dK/dV."""
    ms = np.zeros(4, dtype=np.float64)
    cnt = np.zeros(4, dtype=np.int64)
    _check(load_library().psattn_profile_read(ms.ctypes.data, cnt.ctypes.data), "psattn_profile_read")
    return ms, cnt
