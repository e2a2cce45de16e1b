"""GPU parity on seeded random shapes: batch, length, head counts, head dimension, mask and packing drawn from a
fixed generator, every case element by element against the fp64 oracle.  Shapes that have the stored-dS backward
path (dense, causal, D = 128, S a multiple of 128) run both backward paths."""
import numpy as np
import pytest

from parity_util import compare_all, randn_bf16, run_gpu, to64

pytestmark = pytest.mark.gpu


def draw_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.integers(1, 4))
        Hq = Hkv * int(rng.choice([1, 2, 4]))
        causal = bool(rng.integers(0, 4) > 0)
        packed = bool(rng.integers(0, 3) == 0)
        if packed:
            B = 1
            ndocs = int(rng.integers(1, 9))
            lens = [int(x) for x in rng.choice([0, 1, 17, 64, 127, 128, 129, 200, 300, 513], size=ndocs)]
            if sum(lens) == 0:
                lens[0] = 33
            cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            S = int(cu[-1])
        else:
            B = int(rng.integers(1, 4))
            cu = None
            S = int(rng.integers(1, 1400))
            if i % 3 == 0:   # every third dense case on a multiple of 128: the shapes the stored-dS path takes
                S = 128 * int(rng.integers(1, 11))
        cases.append((i, B, S, Hq, Hkv, D, causal, cu))
    return cases


CASES = draw_cases(48, seed=20240117)


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"{c[0]}-B{c[1]}S{c[2]}Hq{c[3]}Hkv{c[4]}D{c[5]}{'c' if c[6] else 'n'}{'p' if c[7] is not None else 'd'}")
def test_random_shape(oracle, case):
    import torch
    from paper_2401_09149_amd import binding
    i, B, S, Hq, Hkv, D, causal, cu = case
    scale = D ** -0.5
    q, do = (randn_bf16((B, S, Hq, D), 5000 + 10 * i + j) for j in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), 5002 + 10 * i + j) for j in range(2))
    print("random case", case[:7], None if cu is None else cu.tolist(), flush=True)
    got = run_gpu(q, k, v, do, scale, causal, cu)
    ref = oracle.attn_fwd_bwd(to64(q), to64(k), to64(v), to64(do), scale, causal, cu)
    compare_all(got, ref, f"random {i}")
    nd = 0 if cu is None else len(cu) - 1
    if binding.ie_attn_bwd_fast_workspace_bytes(B, S, Hq, Hkv, D, nd, causal) > binding.ie_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, nd):
        dev = "cuda:0"
        qd, kd, vd, dod = (x.to(dev) for x in (q, k, v, do))
        ws = binding.alloc_bwd_workspace(qd, kd, None, fast=True, causal=causal)
        stored = binding.attn_bwd(qd, kd, vd, got[0], dod, got[1], scale, causal, None, workspace=ws, stored_ds=True)
        torch.cuda.synchronize()
        compare_all(got[:2] + tuple(stored), ref, f"random {i}, stored dS")
        assert torch.equal(stored[1], got[3]) and torch.equal(stored[2], got[4])
