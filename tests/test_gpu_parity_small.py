"""GPU parity, element by element against the fp64 oracle, at sizes the oracle finishes in
seconds: several tiles plus ragged tails, both head dims, GQA, batches, packed documents
(including empty and one-token documents), non-causal, and the degenerate S = 1."""
import numpy as np
import pytest

from parity_util import compare_all, randn_bf16, run_gpu, to64

pytestmark = pytest.mark.gpu


def case(oracle, B, S, Hq, Hkv, D, causal=True, cu=None, seed=0, scale=None, grad_abs_tol=None):
    scale = D ** -0.5 if scale is None else scale
    q = randn_bf16((B, S, Hq, D), seed)
    k = randn_bf16((B, S, Hkv, D), seed + 1)
    v = randn_bf16((B, S, Hkv, D), seed + 2)
    do = randn_bf16((B, S, Hq, D), seed + 3)
    label = f"B{B} S{S} Hq{Hq} Hkv{Hkv} D{D} causal{int(causal)} docs{None if cu is None else len(cu) - 1}"
    print("case", label, flush=True)
    got = run_gpu(q, k, v, do, scale, causal, cu)
    ref = oracle.attn_fwd_bwd(to64(q), to64(k), to64(v), to64(do), scale, causal, cu)
    return compare_all(got, ref, label, **({} if grad_abs_tol is None else {"grad_abs_tol": grad_abs_tol}))


def test_config0_tiny(oracle):
    from paper_2401_09149_amd import workloads as W
    cfg = W.CONFIGS[0]
    q, k, v, do = W.make_inputs(cfg)
    got = run_gpu(q, k, v, do, cfg.scale, cfg.causal, None)
    ref = oracle.attn_fwd_bwd(to64(q), to64(k), to64(v), to64(do), cfg.scale, cfg.causal)
    compare_all(got, ref, cfg.name)


@pytest.mark.parametrize("S", [1, 2, 31, 64, 65, 127, 128, 129, 300, 1000])
def test_ragged_lengths_d128(oracle, S):
    case(oracle, 1, S, 2, 2, 128, seed=10 + S)


@pytest.mark.parametrize("S", [1, 63, 200, 777])
def test_ragged_lengths_d64(oracle, S):
    case(oracle, 1, S, 3, 3, 64, seed=20 + S)


def test_several_tiles_d128(oracle):
    case(oracle, 1, 2048 + 77, 2, 2, 128, seed=31)


def test_batch_and_gqa(oracle):
    case(oracle, 2, 700, 8, 2, 128, seed=41)
    case(oracle, 3, 333, 4, 1, 64, seed=42)


@pytest.mark.parametrize("D", [64, 128])
def test_non_causal(oracle, D):
    case(oracle, 2, 515, 4, 2, D, causal=False, seed=51)


@pytest.mark.parametrize("causal", [True, False])
def test_packed_documents(oracle, causal):
    lens = [1, 0, 130, 5, 64, 0, 0, 257, 128, 1, 700, 3]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    case(oracle, 1, int(cu[-1]), 4, 2, 128, causal=causal, cu=cu, seed=61)


def test_packed_many_documents(oracle):
    # more documents than threads in a workgroup: exercises the multi-round document search
    rng = np.random.default_rng(7)
    lens = rng.integers(0, 9, size=700)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    case(oracle, 1, int(cu[-1]), 2, 2, 64, cu=cu, seed=71)


def test_packed_single_document_equals_dense(oracle):
    S = 640
    cu = np.array([0, S], dtype=np.int32)
    case(oracle, 1, S, 2, 1, 128, cu=cu, seed=81)


def test_large_scores_stay_finite(oracle):
    # scale 4x the usual: rows become nearly one-hot, exercising max subtraction and rescaling.
    # dq and dk carry the factor `scale`, so their absolute bar (stated for scale = 1/sqrt(D))
    # is widened by the same factor 4; the relative bar is unchanged.
    case(oracle, 1, 513, 2, 2, 128, seed=91, scale=4 * 128 ** -0.5, grad_abs_tol=4 * 5e-2)


def test_error_codes_on_device_tensors():
    import torch
    from paper_2401_09149_amd import binding
    q = torch.zeros((1, 16, 2, 96), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(binding.IeAttnError) as e:
        binding.attn_fwd(q, q, q, 0.1)
    assert e.value.code == -3
