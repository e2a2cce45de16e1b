"""Bit-exact parity of the eight re-layout kernels (include/ie_sp.h) with the numpy oracle, through the
C ABI, on random 16-bit patterns.  Every output buffer is pre-filled with a sentinel pattern, so an element
the kernel failed to write shows up as a mismatch (each function is a bijection of its buffers)."""
import numpy as np
import pytest
import torch

from oracle import sp_permute as sp
from paper_2401_09149_amd import binding, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(x):
    return torch.from_numpy(x).to(DEV)


def out(n):
    return torch.full((n,), 0x7A5A, dtype=torch.int16, device=DEV)


def same(got, want, what):
    got = got.cpu().numpy()
    assert got.shape == want.shape
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, f"{what}: {bad.size} of {want.size} elements differ, first at {bad[:4]}"


def check_all(B, Sl, Hq, Hkv, D, P, seed):
    shape_qkv, shape_o = (B, Sl, Hq, Hkv, D, P), (B, Sl, Hq, D, P)
    nq, nk = B * Sl * Hq * D, B * Sl * Hkv * D
    n = nq + 2 * nk
    a = workloads.make_bit_patterns(n, seed).numpy()
    ad = dev(a)
    # first exchange, forward and backward
    x = out(n)
    binding.ie_sp_pack_qkv(ad, x, *shape_qkv)
    same(x, sp.pack_qkv(a, *shape_qkv), "pack_qkv")
    q, k, v = out(nq), out(nk), out(nk)
    binding.ie_sp_unpack_qkv(ad, q, k, v, *shape_qkv)
    for g, w, name in zip((q, k, v), sp.unpack_qkv(a, *shape_qkv), "qkv"):
        same(g, w, "unpack_qkv " + name)
    x = out(n)
    binding.ie_sp_pack_dqkv(ad[:nq], ad[nq:nq + nk], ad[nq + nk:], x, *shape_qkv)
    same(x, sp.pack_dqkv(a[:nq], a[nq:nq + nk], a[nq + nk:], *shape_qkv), "pack_dqkv")
    x = out(n)
    binding.ie_sp_unpack_dqkv(ad, x, *shape_qkv)
    same(x, sp.unpack_dqkv(a, *shape_qkv), "unpack_dqkv")
    # second exchange
    for name in ("pack_o", "unpack_o", "pack_do", "unpack_do"):
        y = out(nq)
        getattr(binding, "ie_sp_" + name)(ad[:nq], y, *shape_o)
        same(y, getattr(sp, name)(a[:nq], *shape_o), name)


SMALL = [  # B, Sl, Hq, Hkv, D, P
    (1, 1, 1, 1, 8, 1),          # one token, one 16-byte run
    (2, 96, 8, 4, 64, 4),
    (3, 257, 12, 12, 64, 3),     # ragged tail of the token tiles; run of 4*64 elements = 32 units
    (1, 1000, 6, 3, 8, 3),       # runs of 2 and 1 units: many runs per wave
    (2, 37, 9, 3, 24, 3),        # 9 units per run (does not divide the workgroup size)
    (1, 5, 64, 64, 512, 1),      # 4096 units per run: one run per workgroup tile
    (1, 3, 160, 32, 512, 2),     # 5120 units per run: a run longer than a tile
    (5, 129, 4, 4, 128, 4),      # one head per peer, B > P
    (1, 4096, 16, 2, 128, 2),    # grouped-query planes of different width in one launch
]


@pytest.mark.parametrize("B,Sl,Hq,Hkv,D,P", SMALL)
def test_small_and_ragged_shapes(B, Sl, Hq, Hkv, D, P):
    print(f"case B{B} Sl{Sl} Hq{Hq} Hkv{Hkv} D{D} P{P}", flush=True)
    check_all(B, Sl, Hq, Hkv, D, P, seed=7 * B + Sl)
    torch.cuda.synchronize()


@pytest.mark.parametrize("cfg", workloads.SP_CONFIGS, ids=lambda c: c.name)
def test_plan_shapes_at_full_size(cfg):
    print(f"case {cfg.name}", flush=True)
    check_all(cfg.B, cfg.Sl, cfg.Hq, cfg.Hkv, cfg.D, cfg.P, cfg.seed)
    torch.cuda.synchronize()


def test_buffer_beyond_2_to_31_elements():
    """Offsets are 64-bit: a fused buffer of 2.4e9 elements (4.8 GB), first exchange only."""
    B, Sl, Hq, Hkv, D, P = 1, 98304, 64, 64, 128, 8
    shape = (B, Sl, Hq, Hkv, D, P)
    nq = B * Sl * Hq * D
    n = 3 * nq
    assert n > 2 ** 31
    print("case large", n, flush=True)
    a = workloads.make_bit_patterns(n, 99).numpy()
    ad = dev(a)
    x = out(n)
    binding.ie_sp_pack_qkv(ad, x, *shape)
    same(x, sp.pack_qkv(a, *shape), "pack_qkv")
    del x
    q, k, v = out(nq), out(nq), out(nq)
    binding.ie_sp_unpack_qkv(ad, q, k, v, *shape)
    for g, w, name in zip((q, k, v), sp.unpack_qkv(a, *shape), "qkv"):
        same(g, w, "unpack_qkv " + name)


def test_misaligned_and_overlong_arguments_are_rejected_on_device_tensors():
    a = out(2 * 8 * 64 + 8)
    with pytest.raises(binding.IeAttnError) as e:
        binding.ie_sp_pack_o(a[4:4 + 1024], a[:1024].clone(), 1, 2, 8, 64, 2)   # 8-byte aligned only
    assert e.value.code == -6
    with pytest.raises(ValueError):
        binding.ie_sp_pack_o(a, a.clone(), 1, 2, 8, 64, 2)                      # wrong element count
