"""ctypes marshalling for libpsattn_layer.so (include/psattn_layer.h): a whole self-attention
layer on prefix-shared sequences, projections through rocBLAS."""
from __future__ import annotations

import ctypes as C
import os

from . import binding as B

_LIB = None


def load_layer_library():
    global _LIB
    if _LIB is not None:
        return _LIB
    B.load_library()  # libpsattn.so first: the layer library resolves its symbols against it
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpsattn_layer.so")
    if not os.path.exists(path):
        raise ImportError("libpsattn_layer.so not built: run `python -m paper_2410_20305_amd.build`")
    lib = C.CDLL(path, mode=C.RTLD_GLOBAL)
    i32, vp, f32 = C.c_int32, C.c_void_p, C.c_float
    lib.psattn_layer_create.argtypes = [i32, i32, i32, i32, C.POINTER(vp)]
    lib.psattn_layer_free.argtypes = [vp]
    lib.psattn_layer_workspace_bytes.argtypes = [vp, vp, i32]
    lib.psattn_layer_workspace_bytes.restype = C.c_size_t
    lib.psattn_layer_fwd.argtypes = [vp, vp, vp, i32, f32] + [vp] * 7 + [C.c_size_t, vp]
    lib.psattn_layer_bwd.argtypes = [vp, vp, vp, i32, f32] + [vp] * 12 + [C.c_size_t, vp]
    _LIB = lib
    return lib


class Layer:
    """Owner of a psattn_layer handle."""

    def __init__(self, hidden, n_q_heads, n_kv_heads, head_dim=128):
        lib = load_layer_library()
        h = C.c_void_p()
        B._check(lib.psattn_layer_create(hidden, n_q_heads, n_kv_heads, head_dim, C.byref(h)), "psattn_layer_create")
        self._h, self.hidden, self.Hq, self.Hkv, self.d = h, hidden, n_q_heads, n_kv_heads, head_dim

    def free(self):
        if self._h is not None:
            B._check(load_layer_library().psattn_layer_free(self._h), "psattn_layer_free")
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def workspace_bytes(self, meta):
        return int(load_layer_library().psattn_layer_workspace_bytes(self._h, meta.handle, meta.total_tokens))

    def _check_shapes(self, T, X, Wq, Wk, Wv, Wo):
        import torch
        bf = torch.bfloat16
        B._check_tensor(X, "X", (T, self.hidden), bf)
        B._check_tensor(Wq, "Wq", (self.Hq * self.d, self.hidden), bf)
        B._check_tensor(Wk, "Wk", (self.Hkv * self.d, self.hidden), bf)
        B._check_tensor(Wv, "Wv", (self.Hkv * self.d, self.hidden), bf)
        B._check_tensor(Wo, "Wo", (self.hidden, self.Hq * self.d), bf)

    def forward(self, meta, rope, scale, X, Wq, Wk, Wv, Wo, workspace, Y=None, stream=None):
        import torch
        T = meta.total_tokens
        self._check_shapes(T, X, Wq, Wk, Wv, Wo)
        Y = torch.empty_like(X) if Y is None else Y
        B._check_tensor(Y, "Y", X.shape, X.dtype)
        st = load_layer_library().psattn_layer_fwd(self._h, meta.handle, rope.handle, T, float(scale), X.data_ptr(),
                                                   Wq.data_ptr(), Wk.data_ptr(), Wv.data_ptr(), Wo.data_ptr(), Y.data_ptr(),
                                                   workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                   B._stream_ptr(stream))
        B._check(st, "psattn_layer_fwd")
        return Y

    def backward(self, meta, rope, scale, X, Wq, Wk, Wv, Wo, dY, workspace, grads=None, stream=None):
        import torch
        T = meta.total_tokens
        self._check_shapes(T, X, Wq, Wk, Wv, Wo)
        B._check_tensor(dY, "dY", X.shape, X.dtype)
        if grads is None:
            grads = tuple(torch.empty_like(t) for t in (X, Wq, Wk, Wv, Wo))
        for g, t in zip(grads, (X, Wq, Wk, Wv, Wo)):
            B._check_tensor(g, "gradient", t.shape, t.dtype)
        st = load_layer_library().psattn_layer_bwd(self._h, meta.handle, rope.handle, T, float(scale), X.data_ptr(),
                                                   Wq.data_ptr(), Wk.data_ptr(), Wv.data_ptr(), Wo.data_ptr(), dY.data_ptr(),
                                                   *[g.data_ptr() for g in grads], workspace.data_ptr(),
                                                   workspace.numel() * workspace.element_size(), B._stream_ptr(stream))
        B._check(st, "psattn_layer_bwd")
        return grads
