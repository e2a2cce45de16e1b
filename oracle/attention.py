"""Python face of the fp64 CPU oracle (oracle/attention_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  Nothing on the product path may import it, and it
imports nothing from the product package.

Arrays are numpy float64, C-contiguous.  q, o, dout, dq: [B, S, Hq, D]; k, v, dk,
dv: [B, S, Hkv, D]; lse: [B, Hq, S].  The arithmetic (exact softmax attention of the
Transformer layer the paper runs per GPU over the full sequence, Sec. 2.1/2.4, and
its analytic gradients) lives in the C file; this module only marshals arguments.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain -O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-mavx2", "-mfma", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        i64, i32, f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_double
        shape = [ip, i32, i64, i64, i32, i32, i32, f64, i32, i64, i64]
        lib.ora_attn_fwd.argtypes = [dp] * 5 + shape
        lib.ora_attn_bwd_dq.argtypes = [dp] * 7 + shape
        lib.ora_attn_bwd_dkdv.argtypes = [dp] * 8 + shape
        for f in (lib.ora_attn_fwd, lib.ora_attn_bwd_dq, lib.ora_attn_bwd_dkdv, lib.ora_num_threads):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    return int(_load().ora_num_threads())


def _p(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"], "oracle arrays must be contiguous float64"
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _cu(cu_seqlens):
    if cu_seqlens is None:
        return None, 0, None
    cu = np.ascontiguousarray(np.asarray(cu_seqlens, dtype=np.int32))
    return cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(cu) - 1, cu


def _dims(q, k):
    B, S, Hq, D = q.shape
    assert k.shape[0] == B and k.shape[1] == S and k.shape[3] == D
    return B, S, Hq, k.shape[2], D


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def attn_fwd(q, k, v, scale, causal=True, cu_seqlens=None, rows=None, out=None):
    """lse and o for token rows `rows` = (begin, end) (default: all).  Returns (o, lse);
    rows outside the range keep whatever `out` = (o, lse) held (zeros if not given)."""
    B, S, Hq, Hkv, D = _dims(q, k)
    o, lse = out if out is not None else (np.zeros_like(q), np.zeros((B, Hq, S), dtype=np.float64))
    r0, r1 = (0, S) if rows is None else rows
    cup, nd, keep = _cu(cu_seqlens)
    rc = _load().ora_attn_fwd(_p(q), _p(k), _p(v), _p(o), _p(lse), cup, nd, B, S, Hq, Hkv, D,
                              float(scale), int(bool(causal)), r0, r1)
    _check(rc, "fwd")
    return o, lse


def attn_bwd_dq(q, k, v, o, dout, lse, scale, causal=True, cu_seqlens=None, rows=None, out=None):
    """dq for token rows `rows`; o and lse must hold the forward results of those rows."""
    B, S, Hq, Hkv, D = _dims(q, k)
    dq = out if out is not None else np.zeros_like(q)
    r0, r1 = (0, S) if rows is None else rows
    cup, nd, keep = _cu(cu_seqlens)
    rc = _load().ora_attn_bwd_dq(_p(q), _p(k), _p(v), _p(o), _p(dout), _p(lse), _p(dq), cup, nd, B, S, Hq, Hkv, D,
                                 float(scale), int(bool(causal)), r0, r1)
    _check(rc, "bwd_dq")
    return dq


def attn_bwd_dkdv(q, k, v, o, dout, lse, scale, causal=True, cu_seqlens=None, cols=None, out=None):
    """dk, dv for key tokens `cols`; o and lse must hold the forward results of every row that sees them."""
    B, S, Hq, Hkv, D = _dims(q, k)
    dk, dv = out if out is not None else (np.zeros_like(k), np.zeros_like(v))
    c0, c1 = (0, S) if cols is None else cols
    cup, nd, keep = _cu(cu_seqlens)
    rc = _load().ora_attn_bwd_dkdv(_p(q), _p(k), _p(v), _p(o), _p(dout), _p(lse), _p(dk), _p(dv), cup, nd,
                                   B, S, Hq, Hkv, D, float(scale), int(bool(causal)), c0, c1)
    _check(rc, "bwd_dkdv")
    return dk, dv


def attn_fwd_bwd(q, k, v, dout, scale, causal=True, cu_seqlens=None):
    """All three passes over the whole input.  Returns (o, lse, dq, dk, dv)."""
    o, lse = attn_fwd(q, k, v, scale, causal, cu_seqlens)
    dq = attn_bwd_dq(q, k, v, o, dout, lse, scale, causal, cu_seqlens)
    dk, dv = attn_bwd_dkdv(q, k, v, o, dout, lse, scale, causal, cu_seqlens)
    return o, lse, dq, dk, dv


def rows_needed_for_cols(S, cols, causal=True, cu_seqlens=None):
    """Token range whose forward results pass 3 needs for key columns `cols`."""
    c0, c1 = cols
    if cu_seqlens is None:
        return (c0 if causal else 0, S)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    # document of the first and last requested column (skip empty documents)
    first = int(np.searchsorted(cu, c0, side="right") - 1)
    last = int(np.searchsorted(cu, c1 - 1, side="right") - 1)
    return (c0 if causal else int(cu[first]), int(cu[last + 1]))
