"""GPU parity of the backward path that stores dS (selected with IE_BWD_STORED_DS and a workspace of
ie_attn_bwd_fast_workspace_bytes; dense
input with D = 128 and S a multiple of 128, causal or not):
element by element against the fp64 oracle to the same bar as the recomputing path, dK and dV bit-equal to the
recomputing path's (the same kernel arithmetic, plus stores), and the errors for shapes without that path or a
workspace that is too small for it."""
import numpy as np
import pytest

from parity_util import compare_all, randn_bf16, to64

pytestmark = pytest.mark.gpu


def run_both(q, k, v, do, scale, causal=True):
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    qd, kd, vd, dod = (x.to(dev) for x in (q, k, v, do))
    o, lse = binding.attn_fwd(qd, kd, vd, scale, causal, None)
    plain = binding.attn_bwd(qd, kd, vd, o, dod, lse, scale, causal, None)
    ws = binding.alloc_bwd_workspace(qd, kd, None, fast=True, causal=causal)
    ws.fill_(0xFF)   # (bf16 NaN patterns: an element of dS the kernels do not write would show)
    stored = binding.attn_bwd(qd, kd, vd, o, dod, lse, scale, causal, None, workspace=ws, stored_ds=True)
    torch.cuda.synchronize()
    return o, lse, plain, stored, ws


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("B,S,Hq,Hkv", [(1, 128, 1, 1), (1, 384, 2, 2), (2, 640, 4, 2), (1, 2048, 8, 8), (1, 1152, 16, 2)])
def test_stored_ds_path_against_oracle(oracle, B, S, Hq, Hkv, causal):
    import torch
    from paper_2401_09149_amd import binding
    D = 128
    scale = D ** -0.5
    q, do = (randn_bf16((B, S, Hq, D), 700 + S + i) for i in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), 710 + S + i) for i in range(2))
    fast = binding.ie_attn_bwd_fast_workspace_bytes(B, S, Hq, Hkv, D, 0, causal)
    base = binding.ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, 0)
    assert fast == base + (B * Hq * S * (S + 128) if causal else 2 * B * Hq * S * S)
    print("case stored dS", (B, S, Hq, Hkv, causal), flush=True)
    o, lse, plain, stored, _ = run_both(q, k, v, do, scale, causal)
    ref = oracle.attn_fwd_bwd(to64(q), to64(k), to64(v), to64(do), scale, causal, None)
    compare_all((o, lse) + tuple(stored), ref, f"stored dS B{B} S{S} Hq{Hq} Hkv{Hkv} causal{int(causal)}")
    assert torch.equal(plain[1], stored[1]) and torch.equal(plain[2], stored[2])   # dk, dv: same arithmetic
    # dq: the same bf16 dS summed in another order
    d = (plain[0].float() - stored[0].float()).abs().max().item()
    assert d <= 2 ** -6 * max(1.0, plain[0].float().abs().max().item()), d


def test_phases_on_the_stored_ds_path_and_reproducibility():
    import torch
    from paper_2401_09149_amd import binding
    B, S, Hq, Hkv, D = 1, 1024, 8, 4, 128
    dev = "cuda:0"
    scale = D ** -0.5
    q, do = (randn_bf16((B, S, Hq, D), 760 + i).to(dev) for i in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), 770 + i).to(dev) for i in range(2))
    o, lse = binding.attn_fwd(q, k, v, scale, True, None)
    ws = binding.alloc_bwd_workspace(q, k, None, fast=True)
    first = binding.attn_bwd(q, k, v, o, do, lse, scale, True, None, workspace=ws, stored_ds=True)
    again = binding.attn_bwd(q, k, v, o, do, lse, scale, True, None, workspace=ws, stored_ds=True)
    dq, dk, dv = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
    ws2 = binding.alloc_bwd_workspace(q, k, None, fast=True)
    for phase in (binding.BWD_DELTA, binding.BWD_DKDV, binding.BWD_DQ):
        binding.ie_attn_bwd_phases(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws2, phase, stored_ds=True)
    torch.cuda.synchronize()
    for a, b, c in zip(first, again, (dq, dk, dv)):
        assert torch.equal(a, b) and torch.equal(a, c)


@pytest.mark.parametrize("S,D,causal", [(300, 128, True), (512, 64, True), (300, 128, False)])
def test_path_is_chosen_by_the_flag_not_by_the_workspace_size(S, D, causal):
    """A larger workspace changes nothing by itself; asking for the stored-dS path on a shape that has none is an
    error, and so is asking for it with a workspace that has no room for dS."""
    import torch
    from paper_2401_09149_amd import binding
    B, Hq, Hkv = 1, 2, 2
    assert (binding.ie_attn_bwd_fast_workspace_bytes(B, S, Hq, Hkv, D, 0, causal)
            == binding.ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, 0))
    assert (binding.ie_attn_bwd_fast_workspace_bytes(B, 512, Hq, Hkv, 128, 3, True)
            == binding.ie_attn_bwd_workspace_bytes(B, 512, Hq, Hkv, 128, 3))
    dev = "cuda:0"
    scale = D ** -0.5
    q, k, v, do = (randn_bf16((B, S, Hq, D), 780 + i).to(dev) for i in range(4))
    o, lse = binding.attn_fwd(q, k, v, scale, causal, None)
    plain = binding.attn_bwd(q, k, v, o, do, lse, scale, causal, None)
    big = torch.empty(binding.ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, 0) + (64 << 20), dtype=torch.uint8, device=dev)
    other = binding.attn_bwd(q, k, v, o, do, lse, scale, causal, None, workspace=big)
    torch.cuda.synchronize()
    for a, b in zip(plain, other):
        assert torch.equal(a, b)
    with pytest.raises(binding.IeAttnError) as err:
        binding.attn_bwd(q, k, v, o, do, lse, scale, causal, None, workspace=big, stored_ds=True)
    assert err.value.code == -3


def test_large_workspace_alone_does_not_store_ds():
    """On a shape that has the stored-dS path, a workspace with room for dS but no flag takes the recomputing path
    and leaves the extra bytes untouched; the flag with a small workspace is IE_ERR_WORKSPACE."""
    import torch
    from paper_2401_09149_amd import binding
    B, S, Hq, Hkv, D = 1, 512, 2, 2, 128
    dev = "cuda:0"
    scale = D ** -0.5
    q, k, v, do = (randn_bf16((B, S, Hq, D), 785 + i).to(dev) for i in range(4))
    o, lse = binding.attn_fwd(q, k, v, scale, True, None)
    small = binding.ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, 0)
    ws = binding.alloc_bwd_workspace(q, k, None, fast=True)
    assert ws.numel() > small
    ws.fill_(0xA5)
    got = binding.attn_bwd(q, k, v, o, do, lse, scale, True, None, workspace=ws)
    plain = binding.attn_bwd(q, k, v, o, do, lse, scale, True, None)
    torch.cuda.synchronize()
    assert bool((ws[small:] == 0xA5).all())
    for a, b in zip(got, plain):
        assert torch.equal(a, b)
    with pytest.raises(binding.IeAttnError) as err:
        binding.attn_bwd(q, k, v, o, do, lse, scale, True, None, workspace=ws[:small], stored_ds=True)
    assert err.value.code == -4


def test_autograd_wrapper_with_a_shared_workspace():
    import torch
    from paper_2401_09149_amd import binding
    from paper_2401_09149_amd.autograd import attention
    dev = "cuda:0"
    B, S, Hq, Hkv, D = 1, 768, 4, 2, 128
    q, do = (randn_bf16((B, S, Hq, D), 791 + j).to(dev) for j in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), 793 + j).to(dev) for j in range(2))
    scale = D ** -0.5
    o_ref, lse_ref = binding.attn_fwd(q, k, v, scale, True, None)
    ws = binding.alloc_bwd_workspace(q, k, None, fast=True)
    ref = binding.attn_bwd(q, k, v, o_ref, do, lse_ref, scale, True, None, workspace=ws, stored_ds=True)
    for _ in range(2):   # two "layers" sharing the workspace, one after the other
        qg, kg, vg = (t.clone().requires_grad_(True) for t in (q, k, v))
        attention(qg, kg, vg, workspace=ws, stored_ds=True).backward(do)
        for got, want in zip((qg.grad, kg.grad, vg.grad), ref):
            assert torch.equal(got, want)
