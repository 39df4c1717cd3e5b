"""ctypes binding of librib_attn.so (the C ABI of include/rib_attn.h).

Argument marshalling only: every step of the operator runs in the HIP kernels.
Tensors are torch tensors on the GPU (used purely as device memory); their
data pointers, plus the current torch HIP stream, are what crosses the boundary.
If the shared library cannot be loaded the import of the symbols fails loudly;
there is no CPU fallback.
"""
import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librib_attn.so")

RIB_F32, RIB_BF16 = 0, 1
RIB_FLAG_FORCE_ROW_MAX = 1
RIB_FLAG_WIDE = 2
RIB_FLAG_VECTOR_ONLY = 4

RIB_OK = 0
STATUS_NAMES = {0: "RIB_OK", 1: "RIB_ERR_NULL", 2: "RIB_ERR_SHAPE", 3: "RIB_ERR_DTYPE",
                4: "RIB_ERR_UNSUPPORTED", 5: "RIB_ERR_WORKSPACE", 6: "RIB_ERR_LAUNCH"}

EXPORTS = ("rib_window_attn_fwd", "rib_window_attn_bwd", "rib_window_attn_bwd_workspace_bytes",
           "rib_status_string", "rib_window_attn_kernel_name",
           "rib_features_fwd", "rib_features_bwd", "rib_features_bwd_workspace_bytes",
           "rib_window_attn_gated_fwd", "rib_window_attn_gated_bwd", "rib_window_attn_gated_bwd_workspace_bytes",
           "rib_window_attn_bwd_static_scratch")
RIB_STATIC_SCRATCH_BYTES = 32 << 20


class RibParams(ctypes.Structure):
    """Mirror of `rib_params`."""
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("heads", ctypes.c_int32), ("d", ctypes.c_int32), ("r", ctypes.c_int32),
                ("window", ctypes.c_int32), ("shift", ctypes.c_int32),
                ("scale_c", ctypes.c_float), ("scale_p", ctypes.c_float),
                ("dtype", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("token_stride", ctypes.c_int64)]


class RibGenParams(ctypes.Structure):
    """Mirror of `rib_gen_params`."""
    _fields_ = [("window", ctypes.c_int32), ("heads", ctypes.c_int32), ("r", ctypes.c_int32),
                ("L", ctypes.c_int32), ("d_h", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class RibError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


_lib = None


def load() -> ctypes.CDLL:
    """Open the library (building it first only if no built copy exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build
        build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, fp = ctypes.c_void_p, ctypes.c_void_p
    pp = ctypes.POINTER(RibParams)
    lib.rib_window_attn_fwd.restype = ctypes.c_int
    lib.rib_window_attn_fwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, fp, vp]
    lib.rib_window_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.rib_window_attn_bwd_workspace_bytes.argtypes = [pp]
    lib.rib_window_attn_bwd.restype = ctypes.c_int
    lib.rib_window_attn_bwd.argtypes = [pp] + [vp] * 13 + [vp, ctypes.c_size_t, vp]
    lib.rib_window_attn_bwd_static_scratch.restype = ctypes.c_int
    lib.rib_window_attn_bwd_static_scratch.argtypes = [pp] + [vp] * 13 + [vp]
    lib.rib_status_string.restype = ctypes.c_char_p
    lib.rib_status_string.argtypes = [ctypes.c_int]
    lib.rib_window_attn_kernel_name.restype = ctypes.c_char_p
    lib.rib_window_attn_kernel_name.argtypes = [pp, ctypes.c_int]
    lib.rib_window_attn_gated_fwd.restype = ctypes.c_int
    lib.rib_window_attn_gated_fwd.argtypes = [pp] + [vp] * 9 + [vp]
    lib.rib_window_attn_gated_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.rib_window_attn_gated_bwd_workspace_bytes.argtypes = [pp]
    lib.rib_window_attn_gated_bwd.restype = ctypes.c_int
    lib.rib_window_attn_gated_bwd.argtypes = [pp] + [vp] * 15 + [vp, ctypes.c_size_t, vp]
    gp = ctypes.POINTER(RibGenParams)
    lib.rib_features_fwd.restype = ctypes.c_int
    lib.rib_features_fwd.argtypes = [gp] + [vp] * 6 + [vp]
    lib.rib_features_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.rib_features_bwd_workspace_bytes.argtypes = [gp]
    lib.rib_features_bwd.restype = ctypes.c_int
    lib.rib_features_bwd.argtypes = [gp] + [vp] * 10 + [vp, ctypes.c_size_t, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().rib_status_string(int(status)).decode()


def make_params(B, H, W, heads, d, r, window, shift, scale_c, scale_p, dtype, flags=0,
                token_stride=0) -> RibParams:
    if isinstance(dtype, str):
        dtype = {"f32": RIB_F32, "bf16": RIB_BF16}[dtype]
    return RibParams(B, H, W, heads, d, r, window, shift, scale_c, scale_p, dtype, flags, token_stride)


def params_of(wl, flags=0, token_stride=0) -> RibParams:
    """rib_params of a `workloads.Workload`."""
    return make_params(wl.B, wl.H, wl.W, wl.heads, wl.d, wl.r, wl.M, wl.s, wl.scale_c, wl.scale_p,
                       wl.dtype, flags, token_stride)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def kernel_name(p: RibParams, backward: bool = False) -> Optional[str]:
    s = load().rib_window_attn_kernel_name(ctypes.byref(p), int(backward))
    return s.decode() if s else None


def rib_window_attn_fwd_status(p, q, k, v, f_q, f_k, out, lse, stream=None) -> int:
    return load().rib_window_attn_fwd(ctypes.byref(p) if p is not None else None, _ptr(q), _ptr(k), _ptr(v),
                                      _ptr(f_q), _ptr(f_k), _ptr(out), _ptr(lse),
                                      _stream(stream) if stream != 0 else 0)


def rib_window_attn_fwd(p, q, k, v, f_q, f_k, out, lse=None, stream=None) -> None:
    st = rib_window_attn_fwd_status(p, q, k, v, f_q, f_k, out, lse, stream)
    if st != RIB_OK:
        raise RibError(st, "rib_window_attn_fwd")


def rib_window_attn_bwd_workspace_bytes(p) -> int:
    return int(load().rib_window_attn_bwd_workspace_bytes(ctypes.byref(p) if p is not None else None))


def rib_window_attn_bwd_status(p, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k,
                               workspace, workspace_bytes=None, stream=None) -> int:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else \
            workspace.numel() * workspace.element_size()
    return load().rib_window_attn_bwd(ctypes.byref(p) if p is not None else None, _ptr(q), _ptr(k), _ptr(v),
                                      _ptr(f_q), _ptr(f_k), _ptr(out), _ptr(d_out), _ptr(lse),
                                      _ptr(dq), _ptr(dk), _ptr(dv), _ptr(df_q), _ptr(df_k),
                                      _ptr(workspace), int(workspace_bytes),
                                      _stream(stream) if stream != 0 else 0)


def rib_window_attn_bwd(p, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k,
                        workspace, workspace_bytes=None, stream=None) -> None:
    st = rib_window_attn_bwd_status(p, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k,
                                    workspace, workspace_bytes, stream)
    if st != RIB_OK:
        raise RibError(st, "rib_window_attn_bwd")


def rib_window_attn_bwd_static_scratch_status(p, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k,
                                              stream=None) -> int:
    return load().rib_window_attn_bwd_static_scratch(ctypes.byref(p) if p is not None else None, _ptr(q), _ptr(k),
                                                     _ptr(v), _ptr(f_q), _ptr(f_k), _ptr(out), _ptr(d_out),
                                                     _ptr(lse), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(df_q), _ptr(df_k),
                                                     _stream(stream) if stream != 0 else 0)


def rib_window_attn_bwd_static_scratch(p, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k,
                                       stream=None) -> None:
    st = rib_window_attn_bwd_static_scratch_status(p, q, k, v, f_q, f_k, out, d_out, lse, dq, dk, dv, df_q, df_k,
                                                   stream)
    if st != RIB_OK:
        raise RibError(st, "rib_window_attn_bwd_static_scratch")


def rib_window_attn_gated_fwd_status(p, q, k, v, f_q, f_k, gate, out_gated, out_raw, lse, stream=None) -> int:
    return load().rib_window_attn_gated_fwd(ctypes.byref(p) if p is not None else None, _ptr(q), _ptr(k), _ptr(v),
                                            _ptr(f_q), _ptr(f_k), _ptr(gate), _ptr(out_gated), _ptr(out_raw),
                                            _ptr(lse), _stream(stream) if stream != 0 else 0)


def rib_window_attn_gated_fwd(p, q, k, v, f_q, f_k, gate, out_gated, out_raw=None, lse=None, stream=None) -> None:
    st = rib_window_attn_gated_fwd_status(p, q, k, v, f_q, f_k, gate, out_gated, out_raw, lse, stream)
    if st != RIB_OK:
        raise RibError(st, "rib_window_attn_gated_fwd")


def rib_window_attn_gated_bwd_workspace_bytes(p) -> int:
    return int(load().rib_window_attn_gated_bwd_workspace_bytes(ctypes.byref(p) if p is not None else None))


def rib_window_attn_gated_bwd_status(p, q, k, v, f_q, f_k, gate, out_raw, d_out_gated, lse, dq, dk, dv, dgate,
                                     df_q, df_k, workspace, workspace_bytes=None, stream=None) -> int:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else \
            workspace.numel() * workspace.element_size()
    return load().rib_window_attn_gated_bwd(ctypes.byref(p) if p is not None else None, _ptr(q), _ptr(k), _ptr(v),
                                            _ptr(f_q), _ptr(f_k), _ptr(gate), _ptr(out_raw), _ptr(d_out_gated),
                                            _ptr(lse), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dgate), _ptr(df_q),
                                            _ptr(df_k), _ptr(workspace), int(workspace_bytes),
                                            _stream(stream) if stream != 0 else 0)


def rib_window_attn_gated_bwd(p, q, k, v, f_q, f_k, gate, out_raw, d_out_gated, lse, dq, dk, dv, dgate, df_q, df_k,
                              workspace, workspace_bytes=None, stream=None) -> None:
    st = rib_window_attn_gated_bwd_status(p, q, k, v, f_q, f_k, gate, out_raw, d_out_gated, lse, dq, dk, dv, dgate,
                                          df_q, df_k, workspace, workspace_bytes, stream)
    if st != RIB_OK:
        raise RibError(st, "rib_window_attn_gated_bwd")


def make_gen_params(window, heads, r, L=10, d_h=32, dtype="f32") -> RibGenParams:
    if isinstance(dtype, str):
        dtype = {"f32": RIB_F32, "bf16": RIB_BF16}[dtype]
    return RibGenParams(window, heads, r, L, d_h, dtype)


def rib_features_fwd_status(p, W_h, b_h, W_pq, W_pk, f_q, f_k, stream=None) -> int:
    return load().rib_features_fwd(ctypes.byref(p) if p is not None else None, _ptr(W_h), _ptr(b_h), _ptr(W_pq),
                                   _ptr(W_pk), _ptr(f_q), _ptr(f_k), _stream(stream) if stream != 0 else 0)


def rib_features_fwd(p, W_h, b_h, W_pq, W_pk, f_q, f_k, stream=None) -> None:
    st = rib_features_fwd_status(p, W_h, b_h, W_pq, W_pk, f_q, f_k, stream)
    if st != RIB_OK:
        raise RibError(st, "rib_features_fwd")


def rib_features_bwd_workspace_bytes(p) -> int:
    return int(load().rib_features_bwd_workspace_bytes(ctypes.byref(p) if p is not None else None))


def rib_features_bwd_status(p, W_h, b_h, W_pq, W_pk, df_q, df_k, dW_h, db_h, dW_pq, dW_pk, workspace,
                            workspace_bytes=None, stream=None) -> int:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else \
            workspace.numel() * workspace.element_size()
    return load().rib_features_bwd(ctypes.byref(p) if p is not None else None, _ptr(W_h), _ptr(b_h), _ptr(W_pq),
                                   _ptr(W_pk), _ptr(df_q), _ptr(df_k), _ptr(dW_h), _ptr(db_h), _ptr(dW_pq),
                                   _ptr(dW_pk), _ptr(workspace), int(workspace_bytes),
                                   _stream(stream) if stream != 0 else 0)


def rib_features_bwd(p, W_h, b_h, W_pq, W_pk, df_q, df_k, dW_h, db_h, dW_pq, dW_pk, workspace,
                     workspace_bytes=None, stream=None) -> None:
    st = rib_features_bwd_status(p, W_h, b_h, W_pq, W_pk, df_q, df_k, dW_h, db_h, dW_pq, dW_pk, workspace,
                                 workspace_bytes, stream)
    if st != RIB_OK:
        raise RibError(st, "rib_features_bwd")


# ---- device-memory plumbing for tests, smoke and bench (no arithmetic) --------------------

def to_device(arr, dtype: str, device="cuda:0"):
    """float32 numpy array -> torch tensor of the workload's storage dtype on the GPU.
    For "bf16" the values must already be bf16-representable, so the cast is exact."""
    import torch
    t = torch.from_numpy(arr).to(device)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def alloc_workspace(p, device="cuda:0"):
    import torch
    n = rib_window_attn_bwd_workspace_bytes(p)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)
