"""ctypes binding of libie_attn.so (include/ie_attn.h, include/ie_sp.h, include/ie_linear.h).  Argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the path runs
in the HIP kernels behind the C ABI.  There is no fallback: if the library is missing or
a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("IE_ATTN_LIB") or os.path.join(_HERE, "libie_attn.so")  # override: for trying out a build

EXPORTS = ("ie_attn_fwd", "ie_attn_bwd_workspace_bytes", "ie_attn_bwd_fast_workspace_bytes", "ie_attn_bwd", "ie_attn_bwd_phases",
           "ie_attn_bwd_static", "ie_attn_fwd_sp", "ie_attn_bwd_sp", "ie_attn_set_tile_rows", "ie_attn_strerror",
           "ie_attn_last_hip_error",
           "ie_sp_pack_qkv", "ie_sp_unpack_qkv", "ie_sp_pack_o", "ie_sp_unpack_o",
           "ie_sp_pack_do", "ie_sp_unpack_do", "ie_sp_pack_dqkv", "ie_sp_unpack_dqkv",
           "ie_linear_fwd", "ie_linear_bwd_input", "ie_linear_bwd_weight")

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
    lib.ie_attn_bwd_fast_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32, i32]
    lib.ie_attn_bwd_fast_workspace_bytes.restype = ctypes.c_size_t
    lib.ie_attn_bwd.argtypes = [vp] * 9 + [vp, i32, i64, i64, i32, i32, i32, f32, i32, vp, ctypes.c_size_t, vp]
    lib.ie_attn_bwd.restype = ctypes.c_int
    lib.ie_attn_bwd_phases.argtypes = [vp] * 9 + [vp, i32, i64, i64, i32, i32, i32, f32, i32, vp, ctypes.c_size_t, i32, vp]
    lib.ie_attn_bwd_phases.restype = ctypes.c_int
    lib.ie_attn_bwd_static.argtypes = [vp] * 9 + [vp, i32, i64, i64, i32, i32, i32, f32, i32, vp]
    lib.ie_attn_bwd_static.restype = ctypes.c_int
    lib.ie_attn_fwd_sp.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, i32, f32, i32, vp]
    lib.ie_attn_fwd_sp.restype = ctypes.c_int
    lib.ie_attn_bwd_sp.argtypes = [vp] * 5 + [i64, i64, i32, i32, i32, i32, f32, i32, vp, ctypes.c_size_t, vp]
    lib.ie_attn_bwd_sp.restype = ctypes.c_int
    lib.ie_attn_set_tile_rows.argtypes = [i32]
    lib.ie_attn_strerror.argtypes = [ctypes.c_int]
    lib.ie_attn_strerror.restype = ctypes.c_char_p
    lib.ie_attn_last_hip_error.argtypes = []
    lib.ie_attn_last_hip_error.restype = ctypes.c_char_p
    shape_qkv, shape_o = [i64, i64, i32, i32, i32, i32, vp], [i64, i64, i32, i32, i32, vp]
    for name, args in (("ie_sp_pack_qkv", [vp, vp] + shape_qkv), ("ie_sp_unpack_qkv", [vp] * 4 + shape_qkv),
                       ("ie_sp_pack_o", [vp, vp] + shape_o), ("ie_sp_unpack_o", [vp, vp] + shape_o),
                       ("ie_sp_pack_do", [vp, vp] + shape_o), ("ie_sp_unpack_do", [vp, vp] + shape_o),
                       ("ie_sp_pack_dqkv", [vp] * 4 + shape_qkv), ("ie_sp_unpack_dqkv", [vp, vp] + shape_qkv)):
        getattr(lib, name).argtypes = args
        getattr(lib, name).restype = ctypes.c_int
    for name in ("ie_linear_fwd", "ie_linear_bwd_input", "ie_linear_bwd_weight"):
        getattr(lib, name).argtypes = [vp, vp, vp, i64, i64, i64, vp]
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def ie_attn_set_tile_rows(rows):
    """Query rows per work item at head dimension 128 (0 = chosen per call, 128, 256); returns the previous setting."""
    prev = load().ie_attn_set_tile_rows(int(rows))
    if prev < 0:
        _raise(prev)
    return prev


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


def _shape(q, k, **others):
    """B, S, Hq, Hkv, D of the call; `others`: further tensors by role (v, o, dout, dq like q; dk, dv like k; lse).
    The C ABI sees pointers only, so every shape is checked here: a kernel handed a smaller buffer would read or
    write past its end."""
    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("q and k must be [B, S, heads, D]")
    B, S, Hq, D = q.shape
    if k.shape[0] != B or k.shape[1] != S or k.shape[3] != D:
        raise ValueError("q and k disagree on B, S or D")
    for name, t in others.items():
        if t is None:
            continue
        want = (B, Hq, S) if name == "lse" else tuple(k.shape) if name in ("v", "dk", "dv") else tuple(q.shape)
        if tuple(t.shape) != want:
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {want}")
    return B, S, Hq, k.shape[2], D


def _docs(cu_seqlens):
    if cu_seqlens is None:
        return None, 0
    return _ptr(cu_seqlens, torch.int32, "cu_seqlens"), cu_seqlens.numel() - 1


def ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, num_docs=0):
    return int(load().ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, num_docs))


def ie_attn_bwd_fast_workspace_bytes(B, S, Hq, Hkv, D, num_docs=0, causal=True):
    return int(load().ie_attn_bwd_fast_workspace_bytes(B, S, Hq, Hkv, D, num_docs, int(bool(causal))))


def ie_attn_fwd(q, k, v, o, lse, cu_seqlens, scale, causal, stream=None):
    """o[B,S,Hq,D] bf16 and lse[B,Hq,S] fp32 are overwritten; all tensors live on the GPU."""
    B, S, Hq, Hkv, D = _shape(q, k, v=v, o=o, lse=lse)
    cu, nd = _docs(cu_seqlens)
    bf = torch.bfloat16
    rc = load().ie_attn_fwd(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"), _ptr(o, bf, "o"),
                            _ptr(lse, torch.float32, "lse"), cu, nd, B, S, Hq, Hkv, D, float(scale),
                            int(bool(causal)), _stream(stream))
    if rc != 0:
        _raise(rc)


BWD_DELTA, BWD_DQ, BWD_DKDV, BWD_ALL = 1, 2, 4, 7
BWD_STORED_DS = 16


def ie_attn_bwd(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace, stream=None, stored_ds=False):
    """dq, dk, dv are overwritten; `workspace` is a uint8 GPU tensor of ie_attn_bwd_workspace_bytes(...), or of
    ie_attn_bwd_fast_workspace_bytes(...) with `stored_ds`."""
    ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace, BWD_ALL, stream, stored_ds)


def ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace, phases, stream=None,
                       stored_ds=False):
    """Selected kernels of the backward pass (bit mask of BWD_DELTA, BWD_DQ, BWD_DKDV); `stored_ds` adds the flag
    that selects the path which keeps dS in the workspace."""
    B, S, Hq, Hkv, D = _shape(q, k, v=v, o=o, dout=dout, lse=lse, dq=dq, dk=dk, dv=dv)
    cu, nd = _docs(cu_seqlens)
    bf = torch.bfloat16
    ws = _ptr(workspace, torch.uint8, "workspace")
    rc = load().ie_attn_bwd_phases(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"), _ptr(o, bf, "o"),
                            _ptr(dout, bf, "dout"), _ptr(lse, torch.float32, "lse"), _ptr(dq, bf, "dq"),
                            _ptr(dk, bf, "dk"), _ptr(dv, bf, "dv"), cu, nd, B, S, Hq, Hkv, D, float(scale),
                            int(bool(causal)), ws, workspace.numel() if workspace is not None else 0,
                            int(phases) | (BWD_STORED_DS if stored_ds else 0), _stream(stream))
    if rc != 0:
        _raise(rc)


def ie_attn_bwd_static(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, stream=None):
    """ie_attn_bwd with the workspace in the library's own device array (no workspace argument, nothing allocated)."""
    B, S, Hq, Hkv, D = _shape(q, k, v=v, o=o, dout=dout, lse=lse, dq=dq, dk=dk, dv=dv)
    cu, nd = _docs(cu_seqlens)
    bf = torch.bfloat16
    rc = load().ie_attn_bwd_static(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"), _ptr(o, bf, "o"),
                                   _ptr(dout, bf, "dout"), _ptr(lse, torch.float32, "lse"), _ptr(dq, bf, "dq"),
                                   _ptr(dk, bf, "dk"), _ptr(dv, bf, "dv"), cu, nd, B, S, Hq, Hkv, D, float(scale),
                                   int(bool(causal)), _stream(stream))
    if rc != 0:
        _raise(rc)


def _sp_sizes(B, Sl, Hq, Hkv, D, P):
    _check_heads(Hq, Hkv, P)
    return B * Sl * (Hq + 2 * Hkv) * D, (B, P * Sl, Hq // P, D), (B, Hq // P, P * Sl)


def ie_attn_fwd_sp(xqkv, o, lse, B, Sl, Hq, Hkv, D, P, scale, causal, stream=None):
    """ie_attn_fwd on the received exchange buffer `xqkv` (layout of ie_sp.h); o [B,P*Sl,Hq/P,D], lse [B,Hq/P,P*Sl]."""
    n, o_shape, lse_shape = _sp_sizes(B, Sl, Hq, Hkv, D, P)
    if tuple(o.shape) != o_shape or tuple(lse.shape) != lse_shape:
        raise ValueError(f"o / lse must have shapes {o_shape} / {lse_shape}")
    rc = load().ie_attn_fwd_sp(_buf(xqkv, n, "xqkv"), _ptr(o, torch.bfloat16, "o"), _ptr(lse, torch.float32, "lse"),
                               B, Sl, Hq, Hkv, D, P, float(scale), int(bool(causal)), _stream(stream))
    if rc != 0:
        _raise(rc)


def ie_attn_bwd_sp(xqkv, o, dout, lse, dxqkv, B, Sl, Hq, Hkv, D, P, scale, causal, workspace, stream=None):
    """ie_attn_bwd on the received exchange buffer; dq | dk | dv go to `dxqkv` in the layout the returning exchange sends."""
    n, o_shape, lse_shape = _sp_sizes(B, Sl, Hq, Hkv, D, P)
    if tuple(o.shape) != o_shape or tuple(dout.shape) != o_shape or tuple(lse.shape) != lse_shape:
        raise ValueError(f"o, dout / lse must have shapes {o_shape} / {lse_shape}")
    bf = torch.bfloat16
    rc = load().ie_attn_bwd_sp(_buf(xqkv, n, "xqkv"), _ptr(o, bf, "o"), _ptr(dout, bf, "dout"), _ptr(lse, torch.float32, "lse"),
                               _buf(dxqkv, n, "dxqkv"), B, Sl, Hq, Hkv, D, P, float(scale), int(bool(causal)),
                               _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    if rc != 0:
        _raise(rc)


# -- conveniences that only allocate outputs (torch owns the memory) --------------------

def attn_fwd(q, k, v, scale, causal=True, cu_seqlens=None):
    B, S, Hq, Hkv, D = _shape(q, k)
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device=q.device)
    ie_attn_fwd(q, k, v, o, lse, cu_seqlens, scale, causal)
    return o, lse


def alloc_bwd_workspace(q, k, cu_seqlens=None, fast=False, causal=True):
    """`fast`: with room for dS where the shape has that path (ie_attn_bwd_fast_workspace_bytes)."""
    B, S, Hq, Hkv, D = _shape(q, k)
    nd = 0 if cu_seqlens is None else cu_seqlens.numel() - 1
    size = (ie_attn_bwd_fast_workspace_bytes(B, S, Hq, Hkv, D, nd, causal) if fast
            else ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, nd))
    return torch.empty(size, dtype=torch.uint8, device=q.device)


def attn_bwd(q, k, v, o, dout, lse, scale, causal=True, cu_seqlens=None, workspace=None, stored_ds=False):
    if workspace is None:
        workspace = alloc_bwd_workspace(q, k, cu_seqlens, fast=stored_ds, causal=causal)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ie_attn_bwd(q, k, v, o, dout, lse, dq, dk, dv, cu_seqlens, scale, causal, workspace, stored_ds=stored_ds)
    return dq, dk, dv


# -- re-layouts either side of the sequence-parallel all-to-alls (include/ie_sp.h) ---------------------
# Tensors are contiguous GPU tensors of any 2-byte dtype (bf16, or int16 bit patterns) and any shape with
# the right number of elements; the layouts are those of the header.

def _buf(t, numel, what):
    if not t.is_cuda or t.element_size() != 2 or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous GPU tensor of a 2-byte dtype")
    if t.numel() != numel:
        raise ValueError(f"{what} has {t.numel()} elements, expected {numel}")
    return t.data_ptr()


def _sp_call(name, ptrs, shape, stream):
    rc = getattr(load(), name)(*ptrs, *shape, _stream(stream))
    if rc != 0:
        _raise(rc)


def _check_heads(Hq, Hkv, P):
    if P < 1 or Hq % P or Hkv % P:
        raise ValueError("the head counts must be multiples of P")


def ie_sp_pack_qkv(qkv_local, xqkv, B, Sl, Hq, Hkv, D, P, stream=None):
    _check_heads(Hq, Hkv, P)
    n = B * Sl * (Hq + 2 * Hkv) * D
    _sp_call("ie_sp_pack_qkv", (_buf(qkv_local, n, "qkv_local"), _buf(xqkv, n, "xqkv")), (B, Sl, Hq, Hkv, D, P), stream)


def ie_sp_unpack_dqkv(xqkv, dqkv_local, B, Sl, Hq, Hkv, D, P, stream=None):
    _check_heads(Hq, Hkv, P)
    n = B * Sl * (Hq + 2 * Hkv) * D
    _sp_call("ie_sp_unpack_dqkv", (_buf(xqkv, n, "xqkv"), _buf(dqkv_local, n, "dqkv_local")), (B, Sl, Hq, Hkv, D, P), stream)


def ie_sp_unpack_qkv(xqkv, q, k, v, B, Sl, Hq, Hkv, D, P, stream=None):
    _check_heads(Hq, Hkv, P)
    nq, nk = B * Sl * Hq * D, B * Sl * Hkv * D
    _sp_call("ie_sp_unpack_qkv", (_buf(xqkv, nq + 2 * nk, "xqkv"), _buf(q, nq, "q"), _buf(k, nk, "k"), _buf(v, nk, "v")),
             (B, Sl, Hq, Hkv, D, P), stream)


def ie_sp_pack_dqkv(dq, dk, dv, xqkv, B, Sl, Hq, Hkv, D, P, stream=None):
    _check_heads(Hq, Hkv, P)
    nq, nk = B * Sl * Hq * D, B * Sl * Hkv * D
    _sp_call("ie_sp_pack_dqkv", (_buf(dq, nq, "dq"), _buf(dk, nk, "dk"), _buf(dv, nk, "dv"), _buf(xqkv, nq + 2 * nk, "xqkv")),
             (B, Sl, Hq, Hkv, D, P), stream)


def _sp_o(name, src, dst, B, Sl, Hq, D, P, stream):
    _check_heads(Hq, Hq, P)
    n = B * Sl * Hq * D
    _sp_call(name, (_buf(src, n, "source"), _buf(dst, n, "destination")), (B, Sl, Hq, D, P), stream)


def ie_sp_pack_o(o, xo, B, Sl, Hq, D, P, stream=None):
    _sp_o("ie_sp_pack_o", o, xo, B, Sl, Hq, D, P, stream)


def ie_sp_unpack_o(xo, o_local, B, Sl, Hq, D, P, stream=None):
    _sp_o("ie_sp_unpack_o", xo, o_local, B, Sl, Hq, D, P, stream)


def ie_sp_pack_do(dout_local, xo, B, Sl, Hq, D, P, stream=None):
    _sp_o("ie_sp_pack_do", dout_local, xo, B, Sl, Hq, D, P, stream)


def ie_sp_unpack_do(xo, dout, B, Sl, Hq, D, P, stream=None):
    _sp_o("ie_sp_unpack_do", xo, dout, B, Sl, Hq, D, P, stream)


# -- linear modules (include/ie_linear.h) ---------------------------------------------------------------

def _mat(t, rows, cols, what):
    if not t.is_cuda or t.dtype != torch.bfloat16 or not t.is_contiguous() or tuple(t.shape) != (rows, cols):
        raise ValueError(f"{what} must be a contiguous bf16 GPU tensor of shape ({rows}, {cols})")
    return t.data_ptr()


def ie_linear_fwd(x, w, y, stream=None):
    """y[M,N] = x[M,K] w[N,K]^T"""
    (M, K), N = x.shape, w.shape[0]
    rc = load().ie_linear_fwd(_mat(x, M, K, "x"), _mat(w, N, K, "w"), _mat(y, M, N, "y"), M, N, K, _stream(stream))
    if rc != 0:
        _raise(rc)


def ie_linear_bwd_input(dy, w, dx, stream=None):
    """dx[M,K] = dy[M,N] w[N,K]"""
    (M, N), K = dy.shape, w.shape[1]
    rc = load().ie_linear_bwd_input(_mat(dy, M, N, "dy"), _mat(w, N, K, "w"), _mat(dx, M, K, "dx"), M, N, K, _stream(stream))
    if rc != 0:
        _raise(rc)


def ie_linear_bwd_weight(dy, x, dw, stream=None):
    """dw[N,K] = dy[M,N]^T x[M,K]"""
    (M, N), K = dy.shape, x.shape[1]
    rc = load().ie_linear_bwd_weight(_mat(dy, M, N, "dy"), _mat(x, M, K, "x"), _mat(dw, N, K, "dw"), M, N, K, _stream(stream))
    if rc != 0:
        _raise(rc)
