"""Pins of the fp64 oracle against what the definition of softmax attention fixes.

The paper prints no numeric example of attention (it names the fused kernel only,
Sec. 2.1), so every pin comes from mathematics: closed forms, invariants, special
cases that reduce to a library routine, and finite differences.  None of them calls
the oracle to produce its own expected value.
"""
import math

import numpy as np
import pytest
import torch


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def torch_reference(q, k, v, dout, scale, causal, cu=None):
    """Library route: dense masked softmax(QK^T) V with autograd, fp64, one [S,S] matrix per head."""
    B, S, Hq, D = q.shape
    Hkv = k.shape[2]
    Q = torch.tensor(q, requires_grad=True)
    K = torch.tensor(k, requires_grad=True)
    V = torch.tensor(v, requires_grad=True)
    rep = Hq // Hkv
    Kh = K.repeat_interleave(rep, dim=2).permute(0, 2, 1, 3)
    Vh = V.repeat_interleave(rep, dim=2).permute(0, 2, 1, 3)
    Qh = Q.permute(0, 2, 1, 3)
    doc = torch.zeros(S, dtype=torch.long)
    if cu is not None:
        for t in range(len(cu) - 1):
            doc[cu[t]:cu[t + 1]] = t
    allowed = doc[:, None] == doc[None, :]
    if causal:
        allowed &= torch.tril(torch.ones(S, S, dtype=torch.bool))
    scores = torch.einsum("bhid,bhjd->bhij", Qh, Kh) * scale
    scores = scores.masked_fill(~allowed, float("-inf"))
    lse = torch.logsumexp(scores, dim=-1)
    O = torch.einsum("bhij,bhjd->bhid", torch.softmax(scores, dim=-1), Vh).permute(0, 2, 1, 3)
    O.backward(torch.tensor(dout))
    return O.detach().numpy(), lse.detach().numpy(), Q.grad.numpy(), K.grad.numpy(), V.grad.numpy()


# ---------------------------------------------------------------- closed forms

def test_hand_worked_two_token_case(oracle):
    # S=2, D=1, scale=1, causal.  Row 1: s = [0, ln 3] -> p = [1/4, 3/4], LSE = ln 4.
    q = np.array([2.0, 1.0]).reshape(1, 2, 1, 1)
    k = np.array([0.0, math.log(3.0)]).reshape(1, 2, 1, 1)
    v = np.array([1.0, 5.0]).reshape(1, 2, 1, 1)
    do = np.array([7.0, 1.0]).reshape(1, 2, 1, 1)
    o, lse, dq, dk, dv = oracle.attn_fwd_bwd(q, k, v, do, 1.0, True)
    assert o.ravel() == pytest.approx([1.0, 4.0], abs=1e-14)
    assert lse.ravel() == pytest.approx([0.0, math.log(4.0)], abs=1e-14)
    # row 0 sees only itself: p=1, ds=0.  row 1: Delta=4, dp=[1,5], ds=[-3/4, 3/4]
    assert dq.ravel() == pytest.approx([0.0, 0.75 * math.log(3.0)], abs=1e-14)
    assert dk.ravel() == pytest.approx([-0.75, 0.75], abs=1e-14)
    assert dv.ravel() == pytest.approx([7.0 + 0.25, 0.75], abs=1e-14)
    # non-causal: row 0 (q=2) now also sees key 1: s=[0, 2 ln 3] -> p=[1/10, 9/10]
    o, lse = oracle.attn_fwd(q, k, v, 1.0, causal=False)
    assert o.ravel() == pytest.approx([0.1 + 4.5, 4.0], abs=1e-14)
    assert lse.ravel() == pytest.approx([math.log(10.0), math.log(4.0)], abs=1e-14)


def test_scale_enters_scores_and_gradients(oracle):
    # one query, two keys, D=2, scale=0.5: s = 0.5*[q.k0, q.k1]
    q = np.array([[2.0, 0.0], [2.0, 2.0]]).reshape(1, 2, 1, 2)
    k = np.array([[0.0, 1.0], [math.log(2.0), 0.0]]).reshape(1, 2, 1, 2)
    v = np.array([[1.0, 0.0], [0.0, 1.0]]).reshape(1, 2, 1, 2)
    do = np.array([[0.0, 0.0], [1.0, 0.0]]).reshape(1, 2, 1, 2)
    # row 1: s0 = 0.5*(2*0+2*1)=1, s1 = 0.5*(2 ln2) = ln 2 -> weights e : 2
    o, lse, dq, dk, dv = oracle.attn_fwd_bwd(q, k, v, do, 0.5, True)
    Z = math.e + 2.0
    p0, p1 = math.e / Z, 2.0 / Z
    assert o[0, 1, 0] == pytest.approx([p0, p1], abs=1e-14)
    assert lse[0, 0, 1] == pytest.approx(math.log(Z), abs=1e-14)
    delta = p0
    ds0, ds1 = p0 * (1.0 - delta), p1 * (0.0 - delta)
    assert dq[0, 1, 0] == pytest.approx([0.5 * ds1 * math.log(2.0), 0.5 * ds0], abs=1e-14)
    assert dk[0, 0, 0] == pytest.approx([0.5 * ds0 * 2.0, 0.5 * ds0 * 2.0], abs=1e-14)
    assert dk[0, 1, 0] == pytest.approx([0.5 * ds1 * 2.0, 0.5 * ds1 * 2.0], abs=1e-14)
    assert dv[0, 0, 0] == pytest.approx([p0, 0.0], abs=1e-14)
    assert dv[0, 1, 0] == pytest.approx([p1, 0.0], abs=1e-14)


def test_constant_value_rows_return_the_constant(oracle):
    B, S, H, D = 2, 97, 3, 16
    q, k = rand((B, S, H, D), 1), rand((B, S, H, D), 2)
    c = rand((D,), 3)
    v = np.broadcast_to(c, (B, S, H, D)).copy()
    for causal in (True, False):
        o, _ = oracle.attn_fwd(q, k, v, 0.3, causal)
        assert np.abs(o - c).max() < 1e-14


def test_zero_query_gives_running_mean_and_log_count(oracle):
    B, S, H, D = 1, 64, 2, 8
    q = np.zeros((B, S, H, D))
    k, v, do = rand((B, S, H, D), 4), rand((B, S, H, D), 5), rand((B, S, H, D), 6)
    o, lse, dq, dk, dv = oracle.attn_fwd_bwd(q, k, v, do, 0.7, True)
    counts = np.arange(1, S + 1, dtype=np.float64)
    mean = np.cumsum(v, axis=1) / counts[None, :, None, None]
    assert np.abs(o - mean).max() < 1e-13
    assert np.abs(lse - np.log(counts)[None, None, :]).max() < 1e-13
    assert np.abs(dk).max() == 0.0          # dk = scale * sum ds * q with q = 0
    # dv_j = sum_{i>=j} dO_i / (i+1)
    w = do / counts[None, :, None, None]
    expect_dv = np.flip(np.cumsum(np.flip(w, axis=1), axis=1), axis=1)
    assert np.abs(dv - expect_dv).max() < 1e-13
    # zero keys instead: dq must vanish
    o, lse, dq, dk, dv = oracle.attn_fwd_bwd(rand((B, S, H, D), 7), np.zeros((B, S, H, D)), v, do, 0.7, True)
    assert np.abs(dq).max() == 0.0
    assert np.abs(lse - np.log(counts)[None, None, :]).max() < 1e-13


def test_first_row_of_each_document(oracle):
    S, H, D = 50, 2, 4
    cu = np.array([0, 7, 7, 30, 50], dtype=np.int32)   # includes an empty document
    q, k, v = rand((1, S, H, D), 8), rand((1, S, H, D), 9), rand((1, S, H, D), 10)
    o, lse = oracle.attn_fwd(q, k, v, 0.5, True, cu)
    for a in (0, 7, 30):
        assert np.abs(o[0, a] - v[0, a]).max() < 1e-15
        assert np.abs(lse[0, :, a] - 0.5 * (q[0, a] * k[0, a]).sum(-1)).max() < 1e-14


def test_huge_margin_is_one_hot_and_stable(oracle):
    S, D = 33, 4
    e = np.zeros(D); e[1] = 1.0
    q = np.broadcast_to(e, (1, S, 1, D)).copy()
    k = np.zeros((1, S, 1, D))
    k[0, :, 0, 1] = 1000.0 * np.arange(S)            # score of key j is 1000*j: last visible key wins
    v = rand((1, S, 1, D), 11)
    o, lse = oracle.attn_fwd(q, k, v, 1.0, True)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    assert np.abs(o - v).max() < 1e-300 + 1e-15      # row i attends to key i only
    assert np.abs(lse[0, 0] - 1000.0 * np.arange(S)).max() < 1e-9
    o, _ = oracle.attn_fwd(q, k, v, 1.0, False)
    assert np.abs(o - v[:, -1:]).max() < 1e-15       # non-causal: everyone picks the last key


# ---------------------------------------------------------------- structure

def test_packed_equals_per_document(oracle):
    H, Hkv, D = 4, 2, 8
    lens = [5, 1, 0, 19, 40, 3]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    S = int(cu[-1])
    q, do = rand((1, S, H, D), 12), rand((1, S, H, D), 13)
    k, v = rand((1, S, Hkv, D), 14), rand((1, S, Hkv, D), 15)
    for causal in (True, False):
        packed = oracle.attn_fwd_bwd(q, k, v, do, 0.4, causal, cu)
        for a, e in zip(cu[:-1], cu[1:]):
            if e == a:
                continue
            sl = slice(int(a), int(e))
            single = oracle.attn_fwd_bwd(*(np.ascontiguousarray(x[:, sl]) for x in (q, k, v, do)), 0.4, causal)
            for name, pk, sg in zip("o lse dq dk dv".split(), packed, single):
                pk = pk[:, :, sl] if name == "lse" else pk[:, sl]
                assert np.array_equal(pk, sg), name


def test_gqa_equals_replicated_mha(oracle):
    S, Hq, Hkv, D = 37, 8, 2, 8
    q, do = rand((1, S, Hq, D), 16), rand((1, S, Hq, D), 17)
    k, v = rand((1, S, Hkv, D), 18), rand((1, S, Hkv, D), 19)
    g = oracle.attn_fwd_bwd(q, k, v, do, 0.35, True)
    rep = Hq // Hkv
    kk, vv = np.repeat(k, rep, axis=2), np.repeat(v, rep, axis=2)
    m = oracle.attn_fwd_bwd(q, kk, vv, do, 0.35, True)
    assert np.abs(g[0] - m[0]).max() < 1e-14 and np.abs(g[1] - m[1]).max() < 1e-14
    assert np.abs(g[2] - m[2]).max() < 1e-13
    assert np.abs(g[3] - m[3].reshape(1, S, Hkv, rep, D).sum(3)).max() < 1e-13
    assert np.abs(g[4] - m[4].reshape(1, S, Hkv, rep, D).sum(3)).max() < 1e-13


def test_row_and_column_ranges_match_full_run(oracle):
    S, Hq, Hkv, D = 96, 4, 2, 8
    cu = np.array([0, 10, 50, 96], dtype=np.int32)
    q, do = rand((1, S, Hq, D), 20), rand((1, S, Hq, D), 21)
    k, v = rand((1, S, Hkv, D), 22), rand((1, S, Hkv, D), 23)
    for cuarg in (None, cu):
        o, lse, dq, dk, dv = oracle.attn_fwd_bwd(q, k, v, do, 0.3, True, cuarg)
        rows = (41, 60)
        o2, lse2 = oracle.attn_fwd(q, k, v, 0.3, True, cuarg, rows=rows)
        assert np.array_equal(o2[:, 41:60], o[:, 41:60]) and np.array_equal(lse2[:, :, 41:60], lse[:, :, 41:60])
        assert np.abs(o2[:, :41]).max() == 0 and np.abs(o2[:, 60:]).max() == 0
        dq2 = oracle.attn_bwd_dq(q, k, v, o2, do, lse2, 0.3, True, cuarg, rows=rows)
        assert np.array_equal(dq2[:, 41:60], dq[:, 41:60])
        cols = (44, 49)
        need = oracle.rows_needed_for_cols(S, cols, True, cuarg)
        assert need == ((44, 96) if cuarg is None else (44, 50))
        o3, lse3 = oracle.attn_fwd(q, k, v, 0.3, True, cuarg, rows=need)
        dk3, dv3 = oracle.attn_bwd_dkdv(q, k, v, o3, do, lse3, 0.3, True, cuarg, cols=cols)
        assert np.array_equal(dk3[:, 44:49], dk[:, 44:49]) and np.array_equal(dv3[:, 44:49], dv[:, 44:49])


# ---------------------------------------------------------------- library route

@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("packed", [False, True])
def test_against_library_softmax_and_autograd(oracle, causal, packed):
    S, Hq, Hkv, D = 83, 6, 2, 16
    B = 1 if packed else 2
    cu = np.array([0, 9, 9, 40, 83], dtype=np.int32) if packed else None
    q, do = rand((B, S, Hq, D), 24), rand((B, S, Hq, D), 25)
    k, v = rand((B, S, Hkv, D), 26), rand((B, S, Hkv, D), 27)
    got = oracle.attn_fwd_bwd(q, k, v, do, 0.25, causal, cu)
    ref = torch_reference(q, k, v, do, 0.25, causal, cu)
    for name, g, r in zip("o lse dq dk dv".split(), got, ref):
        assert np.abs(g - r).max() < 1e-12, name


# ---------------------------------------------------------------- gradients by finite differences

@pytest.mark.parametrize("causal,packed,Hq,Hkv", [(True, False, 1, 1), (False, False, 2, 1), (True, True, 4, 2)])
def test_gradients_by_central_differences(oracle, causal, packed, Hq, Hkv):
    S, D, scale, h = 11, 5, 0.6, 1e-5
    cu = np.array([0, 4, 11], dtype=np.int32) if packed else None
    q, do = rand((1, S, Hq, D), 28), rand((1, S, Hq, D), 29)
    k, v = rand((1, S, Hkv, D), 30), rand((1, S, Hkv, D), 31)
    _, _, dq, dk, dv = oracle.attn_fwd_bwd(q, k, v, do, scale, causal, cu)

    def loss(q_, k_, v_):
        o, _ = oracle.attn_fwd(q_, k_, v_, scale, causal, cu)
        return float((o * do).sum())

    for which, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[which]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[which]
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * h)
        err = np.abs(num - grad).max() / max(1.0, np.abs(grad).max())
        assert err < 1e-8, (which, err)


# ---------------------------------------------------------------- invariants of the gradients

def test_gradient_invariants(oracle):
    S, Hq, Hkv, D = 120, 4, 2, 16
    cu = np.array([0, 33, 120], dtype=np.int32)
    q, do = rand((1, S, Hq, D), 32), rand((1, S, Hq, D), 33)
    k, v = rand((1, S, Hkv, D), 34), rand((1, S, Hkv, D), 35)
    o, lse, dq, dk, dv = oracle.attn_fwd_bwd(q, k, v, do, 0.2, True, cu)
    # softmax is invariant to adding a constant vector to all keys of a document: sum_j dk_j = 0 per document
    for a, e in ((0, 33), (33, 120)):
        assert np.abs(dk[0, a:e].sum(0)).max() < 1e-12
    rep = Hq // Hkv
    for g in range(Hkv):
        hs = slice(g * rep, (g + 1) * rep)
        # scores depend on q.k only: <q,dq> over the group equals <k,dk>
        assert abs((q[0, :, hs] * dq[0, :, hs]).sum() - (k[0, :, g] * dk[0, :, g]).sum()) < 1e-11
        # o is linear in v: <v,dv> = <o,dO>
        assert abs((v[0, :, g] * dv[0, :, g]).sum() - (o[0, :, hs] * do[0, :, hs]).sum()) < 1e-11


def test_bad_arguments_are_rejected(oracle):
    q = rand((1, 8, 3, 4), 36)
    k = rand((1, 8, 2, 4), 37)
    with pytest.raises(ValueError):
        oracle.attn_fwd(q, k, k, 1.0)                       # Hq % Hkv != 0
    q = rand((1, 8, 2, 4), 38)
    with pytest.raises(ValueError):
        oracle.attn_fwd(q, k, k, 1.0, True, np.array([0, 5, 7]))   # cu does not end at S
