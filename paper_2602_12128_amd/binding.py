"""ctypes binding of libhla.so: argument marshalling only.

Same names as the C ABI of include/hla.h (hla_create, hla_set_phi_weights, hla_forward,
hla_backward, hla_destroy, ...).  Every step of the method runs inside the library's HIP
kernels; torch is used for device memory and streams.  There is no CPU fallback: a missing
library raises at load time.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhla.so")

HLA_OK = 0
HLA_F32, HLA_BF16 = 0, 1
HLA_PHI_MLP, HLA_PHI_NONE = 0, 1
HLA_PATH_AUTO, HLA_PATH_GENERIC, HLA_PATH_MFMA = 0, 1, 2

EXPORTS = (
    "hla_create", "hla_set_phi_weights", "hla_forward", "hla_backward", "hla_destroy",
    "hla_status_string", "hla_active_path", "hla_profile_enable", "hla_profile_read",
    "hla_read_workspace", "hla_set_phi_weight_grads", "hla_forward_static",
    "hla_set_value_modulation", "hla_set_value_modulation_grads",
)
HLA_WS_FEATURES, HLA_WS_FEATURE_GRADS, HLA_WS_DENOMINATORS = 0, 1, 2


class hla_config(C.Structure):
    _fields_ = [
        ("head_dim", C.c_int32), ("feature_dim", C.c_int32), ("degree", C.c_int32),
        ("eps", C.c_float), ("io_dtype", C.c_int32), ("phi_mode", C.c_int32),
        ("kernel_path", C.c_int32), ("max_heads", C.c_int32), ("max_tokens", C.c_int64),
        ("max_seqs", C.c_int32), ("causal", C.c_int32), ("decay", C.c_float),
    ]


class hla_phi_weights(C.Structure):
    _fields_ = [
        ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
        ("head_stride_W1", C.c_int64), ("head_stride_b1", C.c_int64),
        ("head_stride_W2", C.c_int64), ("head_stride_b2", C.c_int64),
    ]


class hla_phi_weight_grads(C.Structure):
    _fields_ = [("dW1", C.c_void_p), ("db1", C.c_void_p), ("dW2", C.c_void_p), ("db2", C.c_void_p)]


class hla_vmod_weight_grads(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("dW1", "db1", "dW2", "db2", "dgamma", "dbeta")]


class hla_vmod_weights(C.Structure):
    _fields_ = [("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
                ("gamma", C.c_void_p), ("beta", C.c_void_p)]


class hla_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64),
                ("stride_n", C.c_int64)]


class HLAError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


_lib = None


def load_library() -> C.CDLL:
    """Load libhla.so (built in-tree by paper_2602_12128_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2602_12128_amd.build`")
    # torch first: its wheel carries a HIP runtime of its own, and the tensors this binding is handed
    # live in that runtime's context.  Loaded before torch, libhla.so would bring in the system's
    # runtime instead and every allocation of the library would fail (HLA_ERR_ALLOC at hla_create).
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    H = C.c_void_p
    lib.hla_create.argtypes = [C.POINTER(hla_config), C.POINTER(H)]
    lib.hla_create.restype = C.c_int
    lib.hla_set_phi_weights.argtypes = [H, C.POINTER(hla_phi_weights), C.c_int32, C.c_void_p]
    lib.hla_set_phi_weights.restype = C.c_int
    lib.hla_set_phi_weight_grads.argtypes = [H, C.POINTER(hla_phi_weight_grads), C.c_int32]
    lib.hla_set_phi_weight_grads.restype = C.c_int
    lib.hla_forward.argtypes = [H, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                C.c_int32, hla_tensor, hla_tensor, hla_tensor, hla_tensor,
                                C.c_void_p]
    lib.hla_forward.restype = C.c_int
    lib.hla_backward.argtypes = [H, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                 C.c_int32] + [hla_tensor] * 8 + [C.c_void_p]
    lib.hla_backward.restype = C.c_int
    lib.hla_set_value_modulation.argtypes = [H, C.POINTER(hla_vmod_weights), C.c_float, C.c_void_p]
    lib.hla_set_value_modulation_grads.argtypes = [H, C.POINTER(hla_vmod_weight_grads)]
    lib.hla_set_value_modulation_grads.restype = C.c_int
    lib.hla_set_value_modulation.restype = C.c_int
    lib.hla_forward_static.argtypes = [C.POINTER(hla_config), C.c_int32, C.c_int32, C.c_int32,
                                       hla_tensor, hla_tensor, hla_tensor, hla_tensor, C.c_void_p]
    lib.hla_forward_static.restype = C.c_int
    lib.hla_destroy.argtypes = [H]
    lib.hla_destroy.restype = C.c_int
    lib.hla_status_string.argtypes = [C.c_int]
    lib.hla_status_string.restype = C.c_char_p
    lib.hla_active_path.argtypes = [H]
    lib.hla_active_path.restype = C.c_int32
    lib.hla_profile_enable.argtypes = [H, C.c_int32]
    lib.hla_profile_enable.restype = C.c_int
    lib.hla_profile_read.argtypes = [H, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                     C.POINTER(C.c_int64)]
    lib.hla_profile_read.restype = C.c_int32
    lib.hla_read_workspace.argtypes = [H, C.c_int32, C.POINTER(C.c_float), C.c_int64, C.c_void_p]
    lib.hla_read_workspace.restype = C.c_int
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().hla_status_string(code).decode()


def _check(code: int, where: str):
    if code != HLA_OK:
        raise HLAError(code, where)


def _view(t) -> hla_tensor:
    """[B,H,N,w] torch tensor -> hla_tensor (strides in elements; innermost must be dense)."""
    if t.dim() != 4:
        raise ValueError("expected a 4-D [B,H,N,width] tensor")
    if t.shape[3] > 1 and t.stride(3) != 1:
        raise ValueError("innermost dimension must be contiguous")
    return hla_tensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def _stream_ptr(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


HLA_STATIC_SCRATCH_BYTES = 32 << 20


def hla_forward_static(Q, K, V, O, feature_dim: int = 6, degree: int = 3, eps: float = 1e-6,
                       io_dtype: int = HLA_BF16, kernel_path: int = HLA_PATH_AUTO, stream=None):
    """hla_forward_static of the C ABI: the forward on features (HLA_PHI_NONE), dense batch, no
    handle and no device allocation (the workspace is a static array inside the library)."""
    lib = load_library()
    B, H, N, d = V.shape
    cfg = hla_config(d, feature_dim, degree, eps, io_dtype, HLA_PHI_NONE, kernel_path, 1, 1, 1, 0)
    _check(lib.hla_forward_static(C.byref(cfg), B, H, N, _view(Q), _view(K), _view(V), _view(O),
                                  _stream_ptr(stream)), "hla_forward_static")


class HLA:
    """Owns one hla_handle.  Methods mirror the C entry points one to one."""

    def __init__(self, head_dim: int, feature_dim: int = 6, degree: int = 3, eps: float = 1e-6,
                 io_dtype: int = HLA_BF16, phi_mode: int = HLA_PHI_MLP,
                 kernel_path: int = HLA_PATH_AUTO, max_heads: int = 1, max_tokens: int = 1,
                 max_seqs: int = 1, causal: bool = False, decay: float = 1.0):
        self._lib = load_library()
        self.config = hla_config(head_dim, feature_dim, degree, eps, io_dtype, phi_mode,
                                 kernel_path, max_heads, max_tokens, max_seqs, int(causal), float(decay))
        self._h = C.c_void_p()
        _check(self._lib.hla_create(C.byref(self.config), C.byref(self._h)), "hla_create")
        self._keepalive = None
        self._keepalive_grads = None

    # -- hla_destroy
    def destroy(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.hla_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    @property
    def active_path(self) -> int:
        return self._lib.hla_active_path(self._h)

    # -- hla_set_phi_weights
    def set_phi_weights(self, maps: Sequence[dict], per_head: bool = False, stream=None):
        """maps: [phi_q, phi_k1, .., phi_kF], each {'W1','b1','W2','b2'} device tensors in the I/O
        dtype; with per_head=True each carries a leading head dimension."""
        arr = (hla_phi_weights * len(maps))()
        for i, m in enumerate(maps):
            for k in ("W1", "b1", "W2", "b2"):
                if not m[k].is_contiguous():
                    raise ValueError("weights must be contiguous")
            hs = (lambda t: t.stride(0)) if per_head else (lambda t: 0)
            arr[i] = hla_phi_weights(m["W1"].data_ptr(), m["b1"].data_ptr(), m["W2"].data_ptr(),
                                     m["b2"].data_ptr(), hs(m["W1"]), hs(m["b1"]), hs(m["W2"]),
                                     hs(m["b2"]))
        self._keepalive = list(maps)
        _check(self._lib.hla_set_phi_weights(self._h, arr, len(maps), _stream_ptr(stream)),
               "hla_set_phi_weights")

    # -- hla_set_phi_weight_grads
    def set_phi_weight_grads(self, maps: Optional[Sequence[dict]]):
        """maps: [phi_q, phi_k1, .., phi_kF], each {'dW1','db1','dW2','db2'} contiguous fp32 device
        tensors shaped like the weights (with the leading head dimension if the weights have
        one), overwritten by every following backward; None switches the outputs off."""
        import torch
        if maps is None:
            _check(self._lib.hla_set_phi_weight_grads(self._h, None, 0), "hla_set_phi_weight_grads")
            self._keepalive_grads = None
            return
        arr = (hla_phi_weight_grads * len(maps))()
        for i, m in enumerate(maps):
            for k in ("dW1", "db1", "dW2", "db2"):
                if m[k].dtype != torch.float32 or not m[k].is_contiguous():
                    raise ValueError("weight gradients must be contiguous fp32 tensors")
            arr[i] = hla_phi_weight_grads(m["dW1"].data_ptr(), m["db1"].data_ptr(),
                                          m["dW2"].data_ptr(), m["db2"].data_ptr())
        self._keepalive_grads = list(maps)
        _check(self._lib.hla_set_phi_weight_grads(self._h, arr, len(maps)),
               "hla_set_phi_weight_grads")

    # -- hla_set_value_modulation_grads
    def set_value_modulation_grads(self, maps: Optional[Sequence[dict]]):
        """maps: [phi_v1, phi_v2], each {'dW1','db1','dW2','db2','dgamma','dbeta'} contiguous fp32
        device tensors shaped like the weights, overwritten by every following backward; None
        switches the outputs off."""
        import torch
        if maps is None:
            _check(self._lib.hla_set_value_modulation_grads(self._h, None), "hla_set_value_modulation_grads")
            self._keepalive_vmod_grads = None
            return
        keys = ("dW1", "db1", "dW2", "db2", "dgamma", "dbeta")
        arr = (hla_vmod_weight_grads * 2)()
        for i, m in enumerate(maps):
            for k in keys:
                if m[k].dtype != torch.float32 or not m[k].is_contiguous():
                    raise ValueError("weight gradients must be contiguous fp32 tensors")
            arr[i] = hla_vmod_weight_grads(*(m[k].data_ptr() for k in keys))
        self._keepalive_vmod_grads = list(maps)
        _check(self._lib.hla_set_value_modulation_grads(self._h, arr), "hla_set_value_modulation_grads")

    # -- hla_set_value_modulation
    def set_value_modulation(self, maps: Optional[Sequence[dict]], ln_eps: float = 1e-5, stream=None):
        """maps: [phi_v1, phi_v2], each {'W1','b1','W2','b2','gamma','beta'} contiguous device
        tensors in the I/O dtype (W1, W2 [d, d]; the rest [d]); None switches the modulation off."""
        if maps is None:
            _check(self._lib.hla_set_value_modulation(self._h, None, 0.0, _stream_ptr(stream)),
                   "hla_set_value_modulation")
            self._keepalive_vmod = None
            return
        arr = (hla_vmod_weights * 2)()
        for i, m in enumerate(maps):
            for k in ("W1", "b1", "W2", "b2", "gamma", "beta"):
                if not m[k].is_contiguous():
                    raise ValueError("weights must be contiguous")
            arr[i] = hla_vmod_weights(*(m[k].data_ptr() for k in ("W1", "b1", "W2", "b2", "gamma", "beta")))
        self._keepalive_vmod = list(maps)
        _check(self._lib.hla_set_value_modulation(self._h, arr, ln_eps, _stream_ptr(stream)),
               "hla_set_value_modulation")

    @staticmethod
    def _cu(cu_seqlens: Optional[Sequence[int]]):
        if cu_seqlens is None:
            return None, 0
        arr = (C.c_int32 * len(cu_seqlens))(*cu_seqlens)
        return arr, len(cu_seqlens) - 1

    # -- hla_forward
    def forward(self, Q, K, V, O, cu_seqlens: Optional[Sequence[int]] = None, stream=None):
        B, H, N = V.shape[0], V.shape[1], V.shape[2]
        cu, ns = self._cu(cu_seqlens)
        _check(self._lib.hla_forward(self._h, B, H, N, cu, ns, _view(Q), _view(K), _view(V),
                                     _view(O), _stream_ptr(stream)), "hla_forward")

    # -- hla_backward
    def backward(self, Q, K, V, O, dO, dQ, dK, dV, cu_seqlens: Optional[Sequence[int]] = None,
                 stream=None):
        B, H, N = V.shape[0], V.shape[1], V.shape[2]
        cu, ns = self._cu(cu_seqlens)
        _check(self._lib.hla_backward(self._h, B, H, N, cu, ns, _view(Q), _view(K), _view(V),
                                      _view(O), _view(dO), _view(dQ), _view(dK), _view(dV),
                                      _stream_ptr(stream)), "hla_backward")

    # -- hla_read_workspace
    def read_workspace(self, kind: int, count: int, stream=None):
        """Returns a numpy float32 array of `count` values of the requested intermediate."""
        import numpy as np
        out = np.empty(count, dtype=np.float32)
        _check(self._lib.hla_read_workspace(self._h, kind, out.ctypes.data_as(C.POINTER(C.c_float)),
                                            count, _stream_ptr(stream)), "hla_read_workspace")
        return out

    # -- hla_profile_enable / hla_profile_read
    def profile_enable(self, on: bool):
        _check(self._lib.hla_profile_enable(self._h, int(on)), "hla_profile_enable")

    def profile_read(self) -> List[dict]:
        cap = 64
        names = (C.c_char_p * cap)()
        ms = (C.c_double * cap)()
        cnt = (C.c_int64 * cap)()
        n = self._lib.hla_profile_read(self._h, cap, names, ms, cnt)
        return [{"kernel": names[i].decode(), "total_ms": ms[i], "launches": cnt[i]}
                for i in range(min(n, cap))]
