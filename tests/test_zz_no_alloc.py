"""ie_attn_bwd_static (the backward entry point that takes no workspace and allocates nothing: its workspace is a
device array inside the library) against ie_attn_bwd on the same inputs, through the C ABI: the same kernels on the
same operands, so the results must be bit-identical; two calls in a row, the second on a smaller input (the array
then still holds the first call's values beyond what the second one writes)."""
import pytest

from parity_util import randn_bf16

pytestmark = pytest.mark.gpu


def _case(B, S, Hq, Hkv, D, seed, cu=None):
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    scale = D ** -0.5
    q, do = (randn_bf16((B, S, Hq, D), seed + i).to(dev) for i in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), seed + 2 + i).to(dev) for i in range(2))
    cud = None if cu is None else torch.tensor(cu, dtype=torch.int32, device=dev)
    o, lse = binding.attn_fwd(q, k, v, scale, True, cud)
    want = binding.attn_bwd(q, k, v, o, do, lse, scale, True, cud)
    got = [torch.full_like(t, float("nan")) for t in want]
    torch.cuda.synchronize()
    return (q, k, v, o, do, lse, cud, scale), want, got


def test_static_workspace_entry_point_matches_ie_attn_bwd():
    import torch
    from paper_2401_09149_amd import binding
    big = _case(1, 2048, 8, 4, 128, 4100)
    small = _case(2, 300, 4, 4, 128, 4200)
    packed = _case(1, 1000, 2, 1, 64, 4300, cu=[0, 130, 130, 700, 1000])
    print("static entry point: 3 calls in a row on one stream", flush=True)
    for (q, k, v, o, do, lse, cud, scale), _, got in (big, small, packed):
        binding.ie_attn_bwd_static(q, k, v, o, do, lse, got[0], got[1], got[2], cud, scale, True)
    torch.cuda.synchronize()
    for name, (_, want, got) in (("big", big), ("small", small), ("packed", packed)):
        for a, b in zip(got, want):
            assert torch.equal(a, b), name


def test_static_workspace_entry_point_rejects_sizes_beyond_its_array():
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    B, S, H, D = 1, (1 << 21) // 2 + 128, 2, 64          # B*Hq*S just over the limit; never launched
    q = torch.empty((B, S, H, D), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((B, H, S), dtype=torch.float32, device=dev)
    with pytest.raises(binding.IeAttnError) as err:
        binding.ie_attn_bwd_static(q, q, q, q, q, lse, q, q, q, None, 0.125, True)
    assert err.value.code == -4
