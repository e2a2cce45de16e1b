"""Pins of the permute oracle (oracle/sp_permute.py) to what the paper fixes about the two
sequence-parallel all-to-alls (Sec. 2.4 "SP-2", Sec. 3.2.2 "Sequence Parallelism"):

  - after pack -> all-to-all -> unpack every GPU holds the COMPLETE sequence of Q, K and V for its
    subset of the heads, and after attention the second exchange re-partitions the result along
    the sequence: checked by simulating all P ranks with the textbook all-to-all (rank r's chunk p
    becomes rank p's chunk r), written out here, on tensors whose every element is a unique tag;
  - an all-to-all needs P equal contiguous chunks and chunk p must hold exactly what peer p needs;
  - the backward exchanges carry gradients the other way, so their permutations are the inverses.

Shapes use pairwise different B, P, Sl, Hq/P, Hkv/P and D so that any swapped pair of axes changes
the result.
"""
import itertools

import numpy as np
import pytest

from oracle import sp_permute as sp

SHAPES = [  # B, Sl, Hq, Hkv, D, P
    (2, 5, 12, 12, 8, 3),
    (3, 7, 8, 4, 16, 2),     # grouped-query: fewer kv heads than q heads
    (1, 4, 6, 6, 8, 6),      # one head per peer
    (2, 3, 4, 2, 8, 1),      # no sequence parallelism
]


def all_to_all(send):
    """send[r] = rank r's flat send buffer of P equal chunks; returns recv with recv[r] chunk p = send[p] chunk r."""
    P = len(send)
    chunks = [np.split(s, P) for s in send]
    return [np.concatenate([chunks[p][r] for p in range(P)]) for r in range(P)]


def tagged(*shape):
    return np.arange(int(np.prod(shape)), dtype=np.int64).reshape(shape)


def local_qkv(Qg, Kg, Vg, r, Sl):
    """Rank r's fused projection output: its sequence slice of all heads, [B][q | k | v]."""
    B = Qg.shape[0]
    sl = slice(r * Sl, (r + 1) * Sl)
    return np.concatenate([Qg[:, sl].reshape(B, -1), Kg[:, sl].reshape(B, -1), Vg[:, sl].reshape(B, -1)], axis=1).reshape(-1)


@pytest.mark.parametrize("B,Sl,Hq,Hkv,D,P", SHAPES)
def test_first_exchange_gives_every_rank_the_full_sequence_of_its_heads(B, Sl, Hq, Hkv, D, P):
    S = P * Sl
    Qg, Kg, Vg = tagged(B, S, Hq, D), 10**7 + tagged(B, S, Hkv, D), 2 * 10**7 + tagged(B, S, Hkv, D)
    send = [sp.pack_qkv(local_qkv(Qg, Kg, Vg, r, Sl), B, Sl, Hq, Hkv, D, P) for r in range(P)]
    assert all(s.size == send[0].size and s.size % P == 0 for s in send)
    recv = all_to_all(send)
    for r in range(P):
        q, k, v = sp.unpack_qkv(recv[r], B, Sl, Hq, Hkv, D, P)
        hq, hk = Hq // P, Hkv // P
        np.testing.assert_array_equal(q.reshape(B, S, hq, D), Qg[:, :, r * hq:(r + 1) * hq])
        np.testing.assert_array_equal(k.reshape(B, S, hk, D), Kg[:, :, r * hk:(r + 1) * hk])
        np.testing.assert_array_equal(v.reshape(B, S, hk, D), Vg[:, :, r * hk:(r + 1) * hk])


@pytest.mark.parametrize("B,Sl,Hq,Hkv,D,P", SHAPES)
def test_second_exchange_repartitions_along_the_sequence(B, Sl, Hq, Hkv, D, P):
    S, hq = P * Sl, Hq // P
    Og = tagged(B, S, Hq, D)
    send = [sp.pack_o(np.ascontiguousarray(Og[:, :, r * hq:(r + 1) * hq]).reshape(-1), B, Sl, Hq, D, P) for r in range(P)]
    recv = all_to_all(send)
    for r in range(P):
        o_local = sp.unpack_o(recv[r], B, Sl, Hq, D, P)
        np.testing.assert_array_equal(o_local.reshape(B, Sl, Hq, D), Og[:, r * Sl:(r + 1) * Sl])


@pytest.mark.parametrize("B,Sl,Hq,Hkv,D,P", SHAPES)
def test_backward_exchanges_carry_gradients_the_other_way(B, Sl, Hq, Hkv, D, P):
    S, hq, hk = P * Sl, Hq // P, Hkv // P
    dOg = tagged(B, S, Hq, D)
    send = [sp.pack_do(np.ascontiguousarray(dOg[:, r * Sl:(r + 1) * Sl]).reshape(-1), B, Sl, Hq, D, P) for r in range(P)]
    recv = all_to_all(send)
    for r in range(P):
        dout = sp.unpack_do(recv[r], B, Sl, Hq, D, P)
        np.testing.assert_array_equal(dout.reshape(B, S, hq, D), dOg[:, :, r * hq:(r + 1) * hq])
    dQg, dKg, dVg = tagged(B, S, Hq, D), 10**7 + tagged(B, S, Hkv, D), 2 * 10**7 + tagged(B, S, Hkv, D)
    flat = lambda x: np.ascontiguousarray(x).reshape(-1)
    send = [sp.pack_dqkv(flat(dQg[:, :, r * hq:(r + 1) * hq]), flat(dKg[:, :, r * hk:(r + 1) * hk]),
                         flat(dVg[:, :, r * hk:(r + 1) * hk]), B, Sl, Hq, Hkv, D, P) for r in range(P)]
    recv = all_to_all(send)
    for r in range(P):
        got = sp.unpack_dqkv(recv[r], B, Sl, Hq, Hkv, D, P)
        np.testing.assert_array_equal(got, local_qkv(dQg, dKg, dVg, r, Sl))


@pytest.mark.parametrize("B,Sl,Hq,Hkv,D,P", SHAPES)
def test_chunk_p_holds_exactly_what_peer_p_needs(B, Sl, Hq, Hkv, D, P):
    """Send chunk p of the first exchange = head group p of the local slice (as a set; the order inside
    a chunk is the library's choice); send chunk p of the second = sequence slice p of the local heads."""
    Ql, Kl, Vl = tagged(B, Sl, Hq, D), 10**7 + tagged(B, Sl, Hkv, D), 2 * 10**7 + tagged(B, Sl, Hkv, D)
    x = sp.pack_qkv(local_qkv(Ql, Kl, Vl, 0, Sl), B, Sl, Hq, Hkv, D, P)
    hq, hk = Hq // P, Hkv // P
    for p, chunk in enumerate(np.split(x, P)):
        want = np.concatenate([Ql[:, :, p * hq:(p + 1) * hq].reshape(-1), Kl[:, :, p * hk:(p + 1) * hk].reshape(-1),
                               Vl[:, :, p * hk:(p + 1) * hk].reshape(-1)])
        np.testing.assert_array_equal(np.sort(chunk), np.sort(want))
    o = tagged(B, P * Sl, hq, D)
    for p, chunk in enumerate(np.split(sp.pack_o(o.reshape(-1), B, Sl, Hq, D, P), P)):
        np.testing.assert_array_equal(np.sort(chunk), np.sort(o[:, p * Sl:(p + 1) * Sl].reshape(-1)))


@pytest.mark.parametrize("B,Sl,Hq,Hkv,D,P", SHAPES)
def test_backward_permutations_invert_the_forward_ones(B, Sl, Hq, Hkv, D, P):
    rng = np.random.default_rng(5)
    n_qkv, n_o = B * Sl * (Hq + 2 * Hkv) * D, B * Sl * Hq * D
    x = rng.integers(0, 65536, n_qkv).astype(np.uint16)
    np.testing.assert_array_equal(sp.unpack_dqkv(sp.pack_qkv(x, B, Sl, Hq, Hkv, D, P), B, Sl, Hq, Hkv, D, P), x)
    np.testing.assert_array_equal(sp.pack_dqkv(*sp.unpack_qkv(x, B, Sl, Hq, Hkv, D, P), B, Sl, Hq, Hkv, D, P), x)
    y = rng.integers(0, 65536, n_o).astype(np.uint16)
    np.testing.assert_array_equal(sp.unpack_do(sp.pack_o(y, B, Sl, Hq, D, P), B, Sl, Hq, D, P), y)
    np.testing.assert_array_equal(sp.pack_do(sp.unpack_o(y, B, Sl, Hq, D, P), B, Sl, Hq, D, P), y)


def test_index_formulas_by_brute_force():
    """Every element, one at a time, by the index formulas of the layouts (plain loops)."""
    B, Sl, Hq, Hkv, D, P = 2, 3, 4, 2, 8, 2
    H = (Hq, Hkv, Hkv)
    Hl = tuple(h // P for h in H)
    n_local = Sl * sum(H) * D
    base_local = (0, Sl * Hq * D, Sl * (Hq + Hkv) * D)
    n_x = Sl * sum(Hl) * D
    base_x = (0, Sl * Hl[0] * D, Sl * (Hl[0] + Hl[1]) * D)
    qkv = np.arange(B * n_local, dtype=np.int64)
    x = sp.pack_qkv(qkv, B, Sl, Hq, Hkv, D, P)
    q, k, v = sp.unpack_qkv(x, B, Sl, Hq, Hkv, D, P)   # as if received: chunk p = sequence slice p
    planes = (q, k, v)
    back = sp.unpack_dqkv(x, B, Sl, Hq, Hkv, D, P)
    for p, b, t, s, d in itertools.product(range(P), range(B), range(3), range(Sl), range(D)):
        for hl in range(Hl[t]):
            xi = (p * B + b) * n_x + base_x[t] + (s * Hl[t] + hl) * D + d
            li = b * n_local + base_local[t] + (s * H[t] + p * Hl[t] + hl) * D + d
            assert x[xi] == qkv[li]
            assert back[li] == x[xi]
            assert planes[t][((b * P * Sl + p * Sl + s) * Hl[t] + hl) * D + d] == x[xi]
    o = np.arange(B * P * Sl * Hl[0] * D, dtype=np.int64)
    xo = sp.pack_o(o, B, Sl, Hq, D, P)
    o_local = sp.unpack_o(xo, B, Sl, Hq, D, P)
    for p, b, s, hl, d in itertools.product(range(P), range(B), range(Sl), range(Hl[0]), range(D)):
        xi = (((p * B + b) * Sl + s) * Hl[0] + hl) * D + d
        assert xo[xi] == o[((b * P * Sl + p * Sl + s) * Hl[0] + hl) * D + d]
        assert o_local[((b * Sl + s) * Hq + p * Hl[0] + hl) * D + d] == xo[xi]


def test_exchange_volumes_match_the_paper():
    """Per layer and direction the first exchange moves 6bSH bytes over the group and the second 2bSH
    (Sec. 3.2.2, with H the hidden size and 2-byte elements): per GPU that is 1/P of it."""
    B, Sl, Hq, D, P = 2, 8, 4, 8, 2
    S, hidden = P * Sl, Hq * D
    x = sp.pack_qkv(np.zeros(B * Sl * 3 * Hq * D, np.uint16), B, Sl, Hq, Hq, D, P)
    assert x.nbytes * P == 6 * B * S * hidden
    xo = sp.pack_o(np.zeros(B * S * (Hq // P) * D, np.uint16), B, Sl, Hq, D, P)
    assert xo.nbytes * P == 2 * B * S * hidden
