"""Parity of the linear-module kernels (include/ie_linear.h) with the fp64 oracle, through the C ABI.

Tolerance (written out here): the kernel accumulates bf16 x bf16 products (exact in fp32) in fp32 and rounds
once to bf16.  Rounding to bf16 is at most 2^-9 relative; fp32 accumulation of R terms of magnitude ~1 adds
an error that grows like R * 2^-24 (about 1e-3 at R = 22016, the longest contraction of the paper's
models).  With N(0,1) inputs |result| ~ sqrt(R), so:  |got - ref| <= 2^-8 |ref| + 2e-3 * sqrt(R / 1024) + 1e-3."""
import math

import numpy as np
import pytest
import torch

from oracle import linear as lin
from paper_2401_09149_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def randn_bf16(shape, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16)


def f64(t):
    return t.to("cpu", torch.float32).numpy().astype(np.float64)


def close(got, ref, R, what):
    got = f64(got)
    tol = 2.0 ** -8 * np.abs(ref) + 2e-3 * math.sqrt(R / 1024.0) + 1e-3
    bad = np.abs(got - ref) > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {ref.size} outside tolerance, worst {np.abs(got - ref).max():.3e}"


def run_all(M, N, K, seed, which=("fwd", "dx", "dw")):
    x, w, dy = randn_bf16((M, K), seed), randn_bf16((N, K), seed + 1), randn_bf16((M, N), seed + 2)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    sentinel = lambda *s: torch.full(s, float("nan"), dtype=torch.bfloat16, device=DEV)
    if "fwd" in which:
        y = sentinel(M, N)
        binding.ie_linear_fwd(xd, wd, y)
        close(y, lin.linear_fwd(f64(x), f64(w)), K, f"y M{M} N{N} K{K}")
    if "dx" in which:
        dx = sentinel(M, K)
        binding.ie_linear_bwd_input(dyd, wd, dx)
        close(dx, lin.linear_bwd_input(f64(dy), f64(w)), N, f"dx M{M} N{N} K{K}")
    if "dw" in which:
        dw = sentinel(N, K)
        binding.ie_linear_bwd_weight(dyd, xd, dw)
        close(dw, lin.linear_bwd_weight(f64(dy), f64(x)), M, f"dw M{M} N{N} K{K}")


@pytest.mark.parametrize("M,N,K", [
    (64, 64, 64),        # one partial tile, one contraction step
    (256, 256, 256),     # exactly one tile
    (512, 768, 320),     # several tiles, odd number of contraction steps
    (320, 1088, 576),    # ragged tiles in both output dimensions (multiples of 64)
    (2112, 520, 1024),   # 9 row tiles: the panel order wraps; N a multiple of 8 only (fwd and dw need N % 8)
])
def test_small_shapes_all_three_products(M, N, K):
    print(f"case M{M} N{N} K{K}", flush=True)
    which = ["fwd", "dw"] if N % 64 else ["fwd", "dx", "dw"]
    run_all(M, N, K, seed=M + N + K, which=which)


def test_ragged_token_count_forward_and_dx():
    """M is arbitrary where it is not contracted (y and dx): 1000 tokens, and a single one."""
    run_all(1000, 320, 256, seed=5, which=("fwd", "dx"))
    run_all(1, 128, 64, seed=6, which=("fwd", "dx"))


def test_output_columns_that_are_multiples_of_8_only():
    run_all(128, 72, 128, seed=7, which=("fwd",))        # y rows of 72
    run_all(128, 128, 200, seed=8, which=("dx", "dw"))   # dx and dw rows of 200


@pytest.mark.parametrize("M,N,K", [(8192, 12288, 4096), (16384, 22016, 8192)])
def test_paper_shapes_sampled(M, N, K):
    """7B QKV projection at one GPU's 8192 tokens (hidden 4096), and the 65B gate/up projection whose output is the
    (16384, 22016) activation of the appendix on memory fragmentation (hidden 8192; Table 2): whole outputs against
    the oracle would take minutes of float64 matmul, so 64 sampled rows of each output are compared."""
    x, w, dy = randn_bf16((M, K), 21), randn_bf16((N, K), 22), randn_bf16((M, N), 23)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    dw = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    binding.ie_linear_fwd(xd, wd, y)
    binding.ie_linear_bwd_input(dyd, wd, dx)
    binding.ie_linear_bwd_weight(dyd, xd, dw)
    rng = np.random.default_rng(3)
    rows = np.sort(rng.choice(M, 64, replace=False))
    close(y[rows], lin.linear_fwd(f64(x[rows]), f64(w)), K, "y rows")
    close(dx[rows], lin.linear_bwd_input(f64(dy[rows]), f64(w)), N, "dx rows")
    nrows = np.sort(rng.choice(N, 64, replace=False))
    close(dw[nrows], lin.linear_bwd_weight(f64(dy[:, nrows]), f64(x)), M, "dw rows")


def test_autograd_layer_slice_runs_end_to_end():
    """QKV projection -> attention -> output projection through the autograd wrappers, against torch on the same
    bf16 operands (a composition check; each kernel has its own parity test against its oracle)."""
    from paper_2401_09149_amd.autograd import attention, linear
    B, S, H, heads = 1, 512, 256, 2
    D = H // heads
    x = randn_bf16((B, S, H), 31).to(DEV).requires_grad_(True)
    wqkv = (randn_bf16((3 * H, H), 32) * 0.06).to(torch.bfloat16).to(DEV).requires_grad_(True)
    wo = (randn_bf16((H, H), 33) * 0.06).to(torch.bfloat16).to(DEV).requires_grad_(True)
    dy = randn_bf16((B, S, H), 34).to(DEV)

    def layer(lin, att):
        qkv = lin(x, wqkv).reshape(B, S, 3, heads, D)
        o = att(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2])
        return lin(o.reshape(B, S, H), wo)

    def ref_att(q, k, v):
        qf, kf, vf = (t.float().transpose(1, 2) for t in (q, k, v))
        s = qf @ kf.transpose(-1, -2) * D ** -0.5
        s = s.masked_fill(torch.triu(torch.ones(S, S, dtype=torch.bool, device=DEV), 1), float("-inf"))
        return (torch.softmax(s, -1) @ vf).transpose(1, 2).to(torch.bfloat16)

    y = layer(linear, attention)
    y.backward(dy)
    got = [y.detach().float()] + [t.grad.float() for t in (x, wqkv, wo)]
    for t in (x, wqkv, wo):
        t.grad = None
    yr = layer(lambda a, w: (a.float() @ w.float().t()).to(torch.bfloat16), ref_att)
    yr.backward(dy)
    want = [yr.detach().float()] + [t.grad.float() for t in (x, wqkv, wo)]
    for name, g, r in zip(("y", "dx", "dwqkv", "dwo"), got, want):
        rel = (g - r).norm() / r.norm()
        print(name, float(rel), flush=True)
        assert rel < 2e-2, (name, float(rel))
