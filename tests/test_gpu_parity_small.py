"""GPU parity, element by element against the fp64 oracle, at sizes the oracle finishes in
seconds: several tiles plus ragged tails, both head dims, GQA, batches, packed documents
(including empty and one-token documents), non-causal, and the degenerate S = 1."""
import numpy as np
import pytest

from parity_util import compare_all, randn_bf16, run_gpu, to64

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def persistent_kernels():
    """At head dimension 128 the library would pick the kernels with 128-row work items for most shapes of this file
    (short sequences); the tests that call it directly are about the 256-row persistent kernels and their work queues,
    so those are fixed here.  `case` runs both item sizes itself."""
    from paper_2401_09149_amd import binding
    binding.ie_attn_set_tile_rows(256)
    yield
    binding.ie_attn_set_tile_rows(0)


def case(oracle, B, S, Hq, Hkv, D, causal=True, cu=None, seed=0, scale=None, grad_abs_tol=None):
    scale = D ** -0.5 if scale is None else scale
    q = randn_bf16((B, S, Hq, D), seed)
    k = randn_bf16((B, S, Hkv, D), seed + 1)
    v = randn_bf16((B, S, Hkv, D), seed + 2)
    do = randn_bf16((B, S, Hq, D), seed + 3)
    label = f"B{B} S{S} Hq{Hq} Hkv{Hkv} D{D} causal{int(causal)} docs{None if cu is None else len(cu) - 1}"
    print("case", label, flush=True)
    from paper_2401_09149_amd import binding
    ref = oracle.attn_fwd_bwd(to64(q), to64(k), to64(v), to64(do), scale, causal, cu)
    kw = {} if grad_abs_tol is None else {"grad_abs_tol": grad_abs_tol}
    # head dimension 128 has kernels with 256-row and with 128-row work items, chosen by shape: both are held to the bar
    report = None
    try:
        for rows in ((256, 128) if D == 128 else (0,)):
            binding.ie_attn_set_tile_rows(rows)
            report = compare_all(run_gpu(q, k, v, do, scale, causal, cu), ref, f"{label} rows{rows}", **kw)
    finally:
        binding.ie_attn_set_tile_rows(0)
    return report


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


@pytest.mark.parametrize("S", [255, 256, 257, 384, 385, 511, 512, 769])
def test_lengths_around_the_256_row_tile_d128(oracle, S):
    # the head-dim-128 forward works on 256-query tiles and 128-key stages: lengths on and next to
    # their multiples, so that waves with no unmasked tile, one, and several all occur
    case(oracle, 1, S, 1, 1, 128, seed=100 + S)


@pytest.mark.parametrize("S", [512, 640])
def test_non_causal_whole_tiles_d128(oracle, S):
    # every key tile is complete and unmasked for every wave: the hand-sequenced path alone
    case(oracle, 1, S, 2, 1, 128, causal=False, seed=110 + S)


def test_packed_lengths_around_tiles(oracle):
    lens = [256, 255, 257, 512, 1, 384, 129]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    case(oracle, 1, int(cu[-1]), 2, 2, 128, cu=cu, seed=121)


def test_late_outlier_keys_move_the_reference(oracle):
    # Two keys far into the sequence, the second larger than the first, carry scores far above
    # everything before them for the rows that point their way: the softmax reference of those
    # rows has to move in the middle of the unmasked tiles, twice.  Magnitudes grow with the
    # outliers (dq and dk carry k and q), hence the wider absolute bar; the relative bar stands.
    B, S, H, D = 1, 1300, 2, 128
    q = randn_bf16((B, S, H, D), 131)
    k = randn_bf16((B, S, H, D), 132).float()
    k[:, 700] *= 12.0
    k[:, 1000] *= 30.0
    k = k.to(q.dtype)
    v = randn_bf16((B, S, H, D), 133)
    do = randn_bf16((B, S, H, D), 134)
    scale = D ** -0.5
    from paper_2401_09149_amd import binding
    ref = oracle.attn_fwd_bwd(to64(q), to64(k), to64(v), to64(do), scale, True, None)
    for rows in (256, 128):
        binding.ie_attn_set_tile_rows(rows)
        compare_all(run_gpu(q, k, v, do, scale, True, None), ref, f"late outliers rows{rows}", grad_abs_tol=30 * 5e-2)


def test_backward_is_bitwise_reproducible_and_phases_compose():
    import torch
    from paper_2401_09149_amd import binding
    B, S, Hq, Hkv, D = 2, 900, 4, 2, 128
    dev = "cuda:0"
    q, do = (randn_bf16((B, S, Hq, D), 141 + i).to(dev) for i in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), 143 + i).to(dev) for i in range(2))
    scale = D ** -0.5
    o, lse = binding.attn_fwd(q, k, v, scale, True, None)
    o2, lse2 = binding.attn_fwd(q, k, v, scale, True, None)
    assert torch.equal(o, o2) and torch.equal(lse, lse2)
    first = binding.attn_bwd(q, k, v, o, do, lse, scale, True, None)
    again = binding.attn_bwd(q, k, v, o, do, lse, scale, True, None)
    for a, b in zip(first, again):
        assert torch.equal(a, b)
    # the three phases one call at a time, sharing the workspace, give the same bits
    dq, dk, dv = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
    ws = binding.alloc_bwd_workspace(q, k, None)
    for phase in (binding.BWD_DELTA, binding.BWD_DQ, binding.BWD_DKDV):
        binding.ie_attn_bwd_phases(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws, phase)
    torch.cuda.synchronize()
    for a, b in zip(first, (dq, dk, dv)):
        assert torch.equal(a, b)
    for bad in (0, 8, 15):
        with pytest.raises(binding.IeAttnError) as e:
            binding.ie_attn_bwd_phases(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws, bad)
        assert e.value.code == -3


def test_overlapping_launches_on_two_streams_and_many_launches_in_a_row():
    """The persistent kernels draw their items from per-launch counters (backward: in the caller's workspace;
    forward: one of a fixed number of slots, handed out again when its last launch has completed or sits on
    the same stream): launches that overlap on two streams must not disturb each other, and many more launches
    than slots in a row on one stream, with nothing completed in between, must all give the right result."""
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    D, scale = 128, 128 ** -0.5
    shapes = [(1, 4096, 8, 8), (2, 1500, 4, 2)]   # (B, S, Hq, Hkv): eight work lists / a single list
    data = []
    for i, (B, S, Hq, Hkv) in enumerate(shapes):
        q, do = (randn_bf16((B, S, Hq, D), 151 + 10 * i + j).to(dev) for j in range(2))
        k, v = (randn_bf16((B, S, Hkv, D), 153 + 10 * i + j).to(dev) for j in range(2))
        o, lse = binding.attn_fwd(q, k, v, scale, True, None)
        grads = binding.attn_bwd(q, k, v, o, do, lse, scale, True, None)
        data.append((q, k, v, do, o, lse, grads))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    results = [[], []]
    for rep in range(3):
        for i, (q, k, v, do, o, lse, _) in enumerate(data):
            with torch.cuda.stream(streams[i]):
                o2, lse2 = binding.attn_fwd(q, k, v, scale, True, None)
                results[i].append((o2, lse2) + tuple(binding.attn_bwd(q, k, v, o2, do, lse2, scale, True, None)))
    torch.cuda.synchronize()
    for i, (q, k, v, do, o, lse, grads) in enumerate(data):
        for got in results[i]:
            for a, b in zip(got, (o, lse) + tuple(grads)):
                assert torch.equal(a, b)
    q, k, v, do, o, lse, grads = data[0]
    o3, lse3 = torch.empty_like(o), torch.empty_like(lse)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = binding.alloc_bwd_workspace(q, k, None)
    for _ in range(300):   # more forward launches in flight than the pool has slots
        binding.ie_attn_fwd(q, k, v, o3, lse3, None, scale, True)
        binding.ie_attn_bwd(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws)
    for t in (o3, lse3, dq, dk, dv):
        t.fill_(float("nan"))
    binding.ie_attn_fwd(q, k, v, o3, lse3, None, scale, True)
    binding.ie_attn_bwd(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws)
    torch.cuda.synchronize()
    assert torch.equal(o3, o) and torch.equal(lse3, lse)
    for got, want in zip((dq, dk, dv), grads):
        assert torch.equal(got, want)


def test_forward_never_shares_a_work_queue_slot():
    """More forward launches in flight on DIFFERENT streams than the library has work-queue slots (256): every call
    either succeeds, and then its result is right, or fails with IE_ERR_BUSY before launching anything; no call
    silently shares counters with a launch that is still running.  Afterwards the slots come back."""
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    B, S, Hq, Hkv, D = 1, 32768, 16, 16, 128          # about 4 ms per launch: the first ones are still running
    scale = D ** -0.5                                  # when the 257th is issued
    q, k, v = (randn_bf16((B, S, H, D), 171 + j).to(dev) for j, H in enumerate((Hq, Hkv, Hkv)))
    o_ref, lse_ref = binding.attn_fwd(q, k, v, scale, True, None)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(300)]
    # (all launches write the same values to one pair of buffers: a launch that went wrong leaves its mark all the same)
    o = torch.empty_like(o_ref)
    lse = torch.empty_like(lse_ref)
    accepted = busy = 0
    for st in streams:
        try:
            binding.ie_attn_fwd(q, k, v, o, lse, None, scale, True, stream=st)
            accepted += 1
        except binding.IeAttnError as e:
            assert e.code == -7, e
            busy += 1
    torch.cuda.synchronize()
    print(f"  {accepted} launches accepted, {busy} refused with IE_ERR_BUSY", flush=True)
    assert accepted >= 256
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    o, lse = binding.attn_fwd(q, k, v, scale, True, None)   # everything has completed: slots are free again
    torch.cuda.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)


def test_autograd_wrapper_gives_the_same_gradients():
    import torch
    from paper_2401_09149_amd import binding
    from paper_2401_09149_amd.autograd import attention
    dev = "cuda:0"
    B, S, Hq, Hkv, D = 2, 700, 4, 2, 128
    q, do = (randn_bf16((B, S, Hq, D), 171 + j).to(dev) for j in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), 173 + j).to(dev) for j in range(2))
    scale = D ** -0.5
    o_ref, lse_ref = binding.attn_fwd(q, k, v, scale, True, None)
    ref = binding.attn_bwd(q, k, v, o_ref, do, lse_ref, scale, True, None)
    qg, kg, vg = (t.clone().requires_grad_(True) for t in (q, k, v))
    o = attention(qg, kg, vg)
    assert torch.equal(o, o_ref)
    o.backward(do)
    for got, want in zip((qg.grad, kg.grad, vg.grad), ref):
        assert torch.equal(got, want)
    # activation recomputation: the backward pass runs the forward kernel again; same bits
    qr, kr, vr = (t.clone().requires_grad_(True) for t in (q, k, v))
    o2 = attention(qr, kr, vr, recompute=True)
    assert torch.equal(o2, o_ref)
    o2.backward(do)
    for got, want in zip((qr.grad, kr.grad, vr.grad), ref):
        assert torch.equal(got, want)


def test_error_codes_on_device_tensors():
    import torch
    from paper_2401_09149_amd import binding
    q = torch.zeros((1, 16, 2, 96), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(binding.IeAttnError) as e:
        binding.attn_fwd(q, q, q, 0.1)
    assert e.value.code == -3


def test_forward_and_backward_can_be_captured_in_a_graph_and_replayed():
    """The library only launches kernels on the caller's stream (no allocation, no memset, no synchronisation), so a
    step can be captured into a graph.  Replays, with eager work and synchronisation between them and with new input
    values each time, must give the bits of the eager calls; both backward paths."""
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    B, S, Hq, Hkv, D = 1, 1024, 4, 2, 128
    scale = D ** -0.5
    q, do = (randn_bf16((B, S, Hq, D), 901 + j).to(dev) for j in range(2))
    k, v = (randn_bf16((B, S, Hkv, D), 903 + j).to(dev) for j in range(2))
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device=dev)
    for fast in (False, True):
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = binding.alloc_bwd_workspace(q, k, None, fast=fast)

        def step():
            binding.ie_attn_fwd(q, k, v, o, lse, None, scale, True)
            binding.ie_attn_bwd(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws, stored_ds=fast)

        step()   # eager once: one-time set-up (occupancy queries) happens outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for trial in range(3):
            q.copy_(randn_bf16((B, S, Hq, D), 910 + trial).to(dev))   # new values in the captured buffers
            step()
            torch.cuda.synchronize()
            want = [t.clone() for t in (o, lse, dq, dk, dv)]
            for t in (o, lse, dq, dk, dv):
                t.zero_()
            graph.replay()
            torch.cuda.synchronize()
            for got, ref in zip((o, lse, dq, dk, dv), want):
                assert torch.equal(got, ref), (fast, trial)


_PIN_ALL_SLOTS = r"""
import sys
import torch
sys.path.insert(0, {root!r})
from paper_2401_09149_amd import binding
dev = "cuda:0"
B, S, H, D = 1, 512, 2, 128
binding.ie_attn_set_tile_rows(256)
g = torch.Generator().manual_seed(77)
q, k, v = (torch.randn((B, S, H, D), generator=g).to(torch.bfloat16).to(dev) for _ in range(3))
scale = D ** -0.5
o_ref, lse_ref = binding.attn_fwd(q, k, v, scale, True, None)
torch.cuda.synchronize()
outs = [(torch.empty_like(o_ref), torch.empty_like(lse_ref)) for _ in range(260)]
codes = []
graph = torch.cuda.CUDAGraph()
with torch.cuda.graph(graph):
    for o, lse in outs:
        try:
            binding.ie_attn_fwd(q, k, v, o, lse, None, scale, True)
            codes.append(0)
        except binding.IeAttnError as e:
            codes.append(e.code)
graph.replay()
torch.cuda.synchronize()
ok = sum(c == 0 for c in codes)
assert ok == 256, codes.count(0)                       # one slot per captured call, for good
assert all(c == -7 for c in codes[256:]), codes[256:]  # the others: IE_ERR_BUSY, nothing launched, the capture intact
for (o, lse), c in zip(outs, codes):
    if c == 0:
        assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
try:
    binding.attn_fwd(q, k, v, scale, True, None)        # eager calls find no slot either from now on
    raise SystemExit("an eager call got a slot that a captured graph holds")
except binding.IeAttnError as e:
    assert e.code == -7
binding.ie_attn_set_tile_rows(128)                      # the 128-row forward needs no slot
o2, lse2 = binding.attn_fwd(q, k, v, scale, True, None)
torch.cuda.synchronize()
assert (o2.float() - o_ref.float()).abs().max() < 2e-2
print("pinned", ok)
"""


def test_captured_forward_calls_pin_their_slots_and_the_rest_get_ie_err_busy():
    """A forward call recorded under stream capture keeps its work-queue slot for the life of the process (the host
    cannot see a graph's replays).  With all 256 slots held that way every further call of the 256-row forward must
    fail with IE_ERR_BUSY before launching anything, under capture and eagerly, and the graph must still replay
    correctly.  Run in a process of its own, which it leaves without slots."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", _PIN_ALL_SLOTS.format(root=root)], capture_output=True, text=True, timeout=280)
    print(r.stdout[-2000:], r.stderr[-2000:], flush=True)
    assert r.returncode == 0 and "pinned 256" in r.stdout


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(oracle, seed):
    """Shapes, head groupings, masks and document splits drawn from a seeded generator: whatever combination of ragged
    tiles, empty and one-token documents, batches and head groups comes up, every element against the oracle."""
    rng = np.random.default_rng(9000 + seed)
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    Hq = Hkv * int(rng.choice([1, 2, 4]))
    causal = bool(rng.integers(0, 2))
    if rng.integers(0, 3) == 0:   # packed documents, B = 1
        lens = rng.integers(0, 400, size=int(rng.integers(1, 9)))
        lens[rng.integers(0, len(lens))] += 1   # at least one token
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        case(oracle, 1, int(cu[-1]), Hq, Hkv, D, causal=causal, cu=cu, seed=9100 + seed)
    else:
        B = int(rng.choice([1, 2, 3]))
        S = int(rng.integers(1, 900))
        case(oracle, B, S, Hq, Hkv, D, causal=causal, seed=9100 + seed)
