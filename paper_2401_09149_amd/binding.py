"""ctypes binding of libie_attn.so (include/ie_attn.h).  Argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the path runs
in the HIP kernels behind the C ABI.  There is no fallback: if the library is missing or
a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("IE_ATTN_LIB") or os.path.join(_HERE, "libie_attn.so")  # override: for trying out a build

EXPORTS = ("ie_attn_fwd", "ie_attn_bwd_workspace_bytes", "ie_attn_bwd", "ie_attn_bwd_phases", "ie_attn_strerror",
           "ie_attn_last_hip_error")

_lib = None


class IeAttnError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"ie_attn error {code}: {text}")
        self.code = code


def load():
    """Load the shared library (built by paper_2401_09149_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.ie_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i64, i32, i32, i32, f32, i32, vp]
    lib.ie_attn_fwd.restype = ctypes.c_int
    lib.ie_attn_bwd_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32]
    lib.ie_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.ie_attn_bwd.argtypes = [vp] * 9 + [vp, i32, i64, i64, i32, i32, i32, f32, i32, vp, ctypes.c_size_t, vp]
    lib.ie_attn_bwd.restype = ctypes.c_int
    lib.ie_attn_bwd_phases.argtypes = [vp] * 9 + [vp, i32, i64, i64, i32, i32, i32, f32, i32, vp, ctypes.c_size_t, i32, vp]
    lib.ie_attn_bwd_phases.restype = ctypes.c_int
    lib.ie_attn_strerror.argtypes = [ctypes.c_int]
    lib.ie_attn_strerror.restype = ctypes.c_char_p
    lib.ie_attn_last_hip_error.argtypes = []
    lib.ie_attn_last_hip_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def ie_attn_strerror(code):
    return load().ie_attn_strerror(int(code)).decode()


def ie_attn_last_hip_error():
    return load().ie_attn_last_hip_error().decode()


def _raise(code):
    text = ie_attn_strerror(code)
    if code == -5:
        text += ": " + ie_attn_last_hip_error()
    raise IeAttnError(code, text)


def _ptr(t, dtype, what):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


def _stream(stream):
    return (stream if stream is not None else torch.cuda.current_stream()).cuda_stream


def _shape(q, k):
    B, S, Hq, D = q.shape
    if k.shape[0] != B or k.shape[1] != S or k.shape[3] != D:
        raise ValueError("q and k disagree on B, S or D")
    return B, S, Hq, k.shape[2], D


def _docs(cu_seqlens):
    if cu_seqlens is None:
        return None, 0
    return _ptr(cu_seqlens, torch.int32, "cu_seqlens"), cu_seqlens.numel() - 1


def ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, num_docs=0):
    return int(load().ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, num_docs))


def ie_attn_fwd(q, k, v, o, lse, cu_seqlens, scale, causal, stream=None):
    """o[B,S,Hq,D] bf16 and lse[B,Hq,S] fp32 are overwritten; all tensors live on the GPU."""
    B, S, Hq, Hkv, D = _shape(q, k)
    cu, nd = _docs(cu_seqlens)
    bf = torch.bfloat16
    rc = load().ie_attn_fwd(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"), _ptr(o, bf, "o"),
                            _ptr(lse, torch.float32, "lse"), cu, nd, B, S, Hq, Hkv, D, float(scale),
                            int(bool(causal)), _stream(stream))
    if rc != 0:
        _raise(rc)


BWD_DELTA, BWD_DQ, BWD_DKDV, BWD_ALL = 1, 2, 4, 7


def ie_attn_bwd(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace, stream=None):
    """dq, dk, dv are overwritten; `workspace` is a uint8 GPU tensor of ie_attn_bwd_workspace_bytes(...)."""
    ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace, BWD_ALL, stream)


def ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace, phases, stream=None):
    """Selected kernels of the backward pass (bit mask of BWD_DELTA, BWD_DQ, BWD_DKDV)."""
    B, S, Hq, Hkv, D = _shape(q, k)
    cu, nd = _docs(cu_seqlens)
    bf = torch.bfloat16
    ws = _ptr(workspace, torch.uint8, "workspace")
    rc = load().ie_attn_bwd_phases(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"), _ptr(o, bf, "o"),
                            _ptr(dout, bf, "dout"), _ptr(lse, torch.float32, "lse"), _ptr(dq, bf, "dq"),
                            _ptr(dk, bf, "dk"), _ptr(dv, bf, "dv"), cu, nd, B, S, Hq, Hkv, D, float(scale),
                            int(bool(causal)), ws, workspace.numel() if workspace is not None else 0,
                            int(phases), _stream(stream))
    if rc != 0:
        _raise(rc)


# -- conveniences that only allocate outputs (torch owns the memory) --------------------

def attn_fwd(q, k, v, scale, causal=True, cu_seqlens=None):
    B, S, Hq, Hkv, D = _shape(q, k)
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device=q.device)
    ie_attn_fwd(q, k, v, o, lse, cu_seqlens, scale, causal)
    return o, lse


def alloc_bwd_workspace(q, k, cu_seqlens=None):
    B, S, Hq, Hkv, D = _shape(q, k)
    nd = 0 if cu_seqlens is None else cu_seqlens.numel() - 1
    return torch.empty(ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, nd), dtype=torch.uint8, device=q.device)


def attn_bwd(q, k, v, o, dout, lse, scale, causal=True, cu_seqlens=None, workspace=None):
    if workspace is None:
        workspace = alloc_bwd_workspace(q, k, cu_seqlens)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ie_attn_bwd(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace)
    return dq, dk, dv
