"""The attention calls that read q, k, v from the received sequence-parallel exchange buffer and write dq, dk, dv
into the one to be sent (ie_attn_fwd_sp / ie_attn_bwd_sp) against the unfused sequence: ie_sp_unpack_qkv ->
ie_attn_fwd / ie_attn_bwd -> ie_sp_pack_dqkv, on the same buffer.  The same kernels do the same arithmetic on the same
values in the same order, only the addresses differ, so every output must be bit-identical."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,Sl,Hq,Hkv,D,P,causal", [
    (1, 256, 8, 8, 128, 4, True),      # one tile per chunk in the forward
    (2, 512, 8, 4, 128, 2, True),      # batch entries interleaved with peers, GQA widths
    (1, 1024, 4, 4, 128, 4, False),    # not causal
    (2, 256, 4, 2, 64, 2, True),       # head dimension 64 (the other forward kernel)
    (1, 2048, 16, 16, 128, 8, True),   # two local heads, eight peers
    (1, 8192, 32, 32, 128, 4, True),   # the paper's own plan for 7B at 32K (s_sp = 4: 8 heads per GPU), full size
])
def test_fused_calls_equal_unpack_attention_pack(B, Sl, Hq, Hkv, D, P, causal):
    from paper_2401_09149_amd import binding
    try:
        for rows in ((256, 128) if D == 128 else (0,)):   # both sizes of the forward's and dQ's work items
            binding.ie_attn_set_tile_rows(rows)
            _fused_against_unfused(B, Sl, Hq, Hkv, D, P, causal)
    finally:
        binding.ie_attn_set_tile_rows(0)


def _fused_against_unfused(B, Sl, Hq, Hkv, D, P, causal):
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    Hql, Hkvl, S = Hq // P, Hkv // P, P * Sl
    n = B * Sl * (Hq + 2 * Hkv) * D
    gen = torch.Generator(device="cpu").manual_seed(5000 + Sl + Hq + D + P)
    xqkv = torch.randn(n, generator=gen, dtype=torch.float32).to(torch.bfloat16).to(dev)
    dout = torch.randn((B, S, Hql, D), generator=gen, dtype=torch.float32).to(torch.bfloat16).to(dev)
    scale = D ** -0.5
    print("case fused sp", (B, Sl, Hq, Hkv, D, P, causal), flush=True)
    # unfused: re-layout, attention, re-layout
    q = torch.empty((B, S, Hql, D), dtype=torch.bfloat16, device=dev)
    k, v = (torch.empty((B, S, Hkvl, D), dtype=torch.bfloat16, device=dev) for _ in range(2))
    binding.ie_sp_unpack_qkv(xqkv, q, k, v, B, Sl, Hq, Hkv, D, P)
    o, lse = binding.attn_fwd(q, k, v, scale, causal, None)
    dq, dk, dv = binding.attn_bwd(q, k, v, o, dout, lse, scale, causal, None)
    want = torch.empty_like(xqkv)
    binding.ie_sp_pack_dqkv(dq, dk, dv, want, B, Sl, Hq, Hkv, D, P)
    # fused
    o2 = torch.full_like(o, float("nan"))
    lse2 = torch.full_like(lse, float("nan"))
    binding.ie_attn_fwd_sp(xqkv, o2, lse2, B, Sl, Hq, Hkv, D, P, scale, causal)
    got = torch.full_like(xqkv, float("nan"))
    ws = torch.empty(binding.ie_attn_bwd_workspace_bytes(B, S, Hql, Hkvl, D, 0), dtype=torch.uint8, device=dev)
    binding.ie_attn_bwd_sp(xqkv, o2, dout, lse2, got, B, Sl, Hq, Hkv, D, P, scale, causal, ws)
    torch.cuda.synchronize()
    assert torch.equal(o2, o) and torch.equal(lse2, lse)
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))


def test_fused_calls_reject_chunks_the_kernels_cannot_split():
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    for Sl in (128, 384):   # too short for a forward tile / not a power of two
        B, Hq, Hkv, D, P = 1, 4, 4, 128, 2
        x = torch.zeros(B * Sl * (Hq + 2 * Hkv) * D, dtype=torch.bfloat16, device=dev)
        o = torch.empty((B, P * Sl, Hq // P, D), dtype=torch.bfloat16, device=dev)
        lse = torch.empty((B, Hq // P, P * Sl), dtype=torch.float32, device=dev)
        with pytest.raises(binding.IeAttnError) as err:
            binding.ie_attn_fwd_sp(x, o, lse, B, Sl, Hq, Hkv, D, P, 0.1, True)
        assert err.value.code == -3
