"""CPU oracle of the local re-layouts either side of the sequence-parallel all-to-all.

TEST INFRASTRUCTURE ONLY: imported by tests/ and by the cpu_baseline leg of bench.py.  Nothing on
the product path may import it, and it imports nothing from the product package.

With sequence parallelism of degree P every module but attention holds S/P tokens of all heads and
attention holds all S tokens of heads/P heads; two all-to-alls per layer and direction change
between the two (Sec. 2.4 "SP-2", Sec. 3.2.2 "Sequence Parallelism").  An all-to-all moves P equal
contiguous chunks, chunk p to and from peer p, so each exchange needs a permutation before it
("pack") and one after it ("unpack").  Each function below is that permutation written as numpy
reshape / transpose / concatenate on arrays of 16-bit patterns (any dtype works; nothing is
computed), in the index notation of the layouts:

  qkv_local  [B][ q:[Sl][Hq][D] | k:[Sl][Hkv][D] | v:[Sl][Hkv][D] ]
  xqkv       [P][B][ q:[Sl][Hq/P][D] | k:[Sl][Hkv/P][D] | v:[Sl][Hkv/P][D] ]
  q (o, dout, dq) [B][P*Sl][Hq/P][D],  k, v (dk, dv) [B][P*Sl][Hkv/P][D]
  xo         [P][B][Sl][Hq/P][D]
  o_local (dout_local) [B][Sl][Hq][D]

All inputs and outputs are flat (1-D) arrays, as the buffers are on the device.
"""
import numpy as np


def _planes_of_qkv_local(qkv_local, B, Sl, Hq, Hkv, D):
    per_b = qkv_local.reshape(B, Sl * (Hq + 2 * Hkv) * D)
    nq, nk = Sl * Hq * D, Sl * Hkv * D
    q = per_b[:, :nq].reshape(B, Sl, Hq, D)
    k = per_b[:, nq:nq + nk].reshape(B, Sl, Hkv, D)
    v = per_b[:, nq + nk:].reshape(B, Sl, Hkv, D)
    return q, k, v


def _planes_of_xqkv(xqkv, B, Sl, Hq, Hkv, D, P):
    per_pb = xqkv.reshape(P, B, Sl * (Hq + 2 * Hkv) // P * D)
    nq, nk = Sl * (Hq // P) * D, Sl * (Hkv // P) * D
    q = per_pb[:, :, :nq].reshape(P, B, Sl, Hq // P, D)
    k = per_pb[:, :, nq:nq + nk].reshape(P, B, Sl, Hkv // P, D)
    v = per_pb[:, :, nq + nk:].reshape(P, B, Sl, Hkv // P, D)
    return q, k, v


def _concat_planes(q, k, v, lead):
    """[lead..., plane] x 3 -> flat [lead...][q | k | v]"""
    n = int(np.prod(lead))
    return np.concatenate([q.reshape(n, -1), k.reshape(n, -1), v.reshape(n, -1)], axis=1).reshape(-1)


def pack_qkv(qkv_local, B, Sl, Hq, Hkv, D, P):
    """xqkv[p][b][t][s][hl][:] = qkv_local[b][t][s][p*Hl_t + hl][:]  (Sec. 2.4 "SP-2")."""
    out = []
    for plane, H in zip(_planes_of_qkv_local(qkv_local, B, Sl, Hq, Hkv, D), (Hq, Hkv, Hkv)):
        x = plane.reshape(B, Sl, P, H // P, D)          # head = p*Hl + hl
        out.append(x.transpose(2, 0, 1, 3, 4))          # [P][B][Sl][Hl][D]
    return _concat_planes(*out, lead=(P, B))


def unpack_qkv(xqkv, B, Sl, Hq, Hkv, D, P):
    """t[b][p*Sl + s][hl][:] = xqkv[p][b][t][s][hl][:]; returns flat q, k, v."""
    out = []
    for plane in _planes_of_xqkv(xqkv, B, Sl, Hq, Hkv, D, P):
        x = plane.transpose(1, 0, 2, 3, 4)              # [B][P][Sl][Hl][D]; token = p*Sl + s
        out.append(np.ascontiguousarray(x).reshape(-1))
    return tuple(out)


def pack_o(o, B, Sl, Hq, D, P):
    """xo[p][b][s][hl][:] = o[b][p*Sl + s][hl][:]."""
    x = o.reshape(B, P, Sl, Hq // P, D)
    return np.ascontiguousarray(x.transpose(1, 0, 2, 3, 4)).reshape(-1)


def unpack_o(xo, B, Sl, Hq, D, P):
    """o_local[b][s][p*Hql + hl][:] = xo[p][b][s][hl][:]."""
    x = xo.reshape(P, B, Sl, Hq // P, D)
    return np.ascontiguousarray(x.transpose(1, 2, 0, 3, 4)).reshape(-1)   # [B][Sl][P][Hql][D]


def pack_do(dout_local, B, Sl, Hq, D, P):
    """xo[p][b][s][hl][:] = dout_local[b][s][p*Hql + hl][:]  (inverse of unpack_o)."""
    x = dout_local.reshape(B, Sl, P, Hq // P, D)
    return np.ascontiguousarray(x.transpose(2, 0, 1, 3, 4)).reshape(-1)


def unpack_do(xo, B, Sl, Hq, D, P):
    """dout[b][p*Sl + s][hl][:] = xo[p][b][s][hl][:]  (inverse of pack_o)."""
    x = xo.reshape(P, B, Sl, Hq // P, D)
    return np.ascontiguousarray(x.transpose(1, 0, 2, 3, 4)).reshape(-1)


def pack_dqkv(dq, dk, dv, B, Sl, Hq, Hkv, D, P):
    """xqkv[p][b][t][s][hl][:] = dt[b][p*Sl + s][hl][:]  (inverse of unpack_qkv)."""
    out = []
    for g, H in zip((dq, dk, dv), (Hq, Hkv, Hkv)):
        x = g.reshape(B, P, Sl, H // P, D)
        out.append(x.transpose(1, 0, 2, 3, 4))          # [P][B][Sl][Hl][D]
    return _concat_planes(*out, lead=(P, B))


def unpack_dqkv(xqkv, B, Sl, Hq, Hkv, D, P):
    """dqkv_local[b][t][s][p*Hl_t + hl][:] = xqkv[p][b][t][s][hl][:]  (inverse of pack_qkv)."""
    out = []
    for plane in _planes_of_xqkv(xqkv, B, Sl, Hq, Hkv, D, P):
        out.append(plane.transpose(1, 2, 0, 3, 4))      # [B][Sl][P][Hl][D]
    return _concat_planes(*out, lead=(B,))
