#!/usr/bin/env python3
"""Benchmark of the attention hot path on one MI355X.

A step is one pass of the whole path (forward, then backward: delta, dK/dV, dQ) over one
batch of seeded synthetic input that is already resident in HBM.  The backward pass gets the
O(S) workspace of ie_attn_bwd_workspace_bytes; the optional path that keeps dS in B*Hq*S*(S+128) bytes more
is timed beside it and reported under bwd.other_path (--stored-ds swaps the two).  The workload is the
7B-class layer with all heads on one GPU: B=1, S=32768, Hq=Hkv=32, D=128, causal, bf16.
FLOP convention: forward = 4*S^2*D*Hq / 2 (causal halving), backward = 2.5x forward.

Prints ONE JSON line.  `value` is fwd+bwd TFLOP/s; `roofline` describes the kernel that
takes the most time, measured live with events on the launch stream; `cpu_baseline` times
the fp64 oracle on the host cores on a bounded sample of the same inputs.  After the timed
steps, `sp_permute` reports the re-layout kernels that sit either side of attention under
sequence parallelism (HBM-bound copies, GB/s against the HBM peak) and `linear` the linear modules of
the same layer (MFMA-bound); neither is part of `value`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA: 256 CU x 4 SIMD x 1024 FLOP/clk x 2.4 GHz = 2516.6
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def event_ms(fn, iters):
    import torch
    start = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    stop = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    for i in range(iters):
        start[i].record()
        fn()
        stop[i].record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in zip(start, stop))
    return sum(ts) / len(ts), ts[0], ts[len(ts) // 2]


def tile_efficiency(cfg, cu_np, bq=256, bk=128):
    """Credited (query, key) pairs (L^2/2 per document) over the pairs the forward's tiles cover:
    every launched (bq-query tile, bk-key tile) counted in full, masked part included."""
    import numpy as np
    lens = [cfg.S] if cu_np is None else [int(x) for x in np.diff(cu_np)]
    credited = executed = 0.0
    for L in lens:
        credited += L * L / 2.0 if cfg.causal else float(L) * L
        for t in range((L + bq - 1) // bq):
            nk = min(bq * (t + 1), L) if cfg.causal else L
            executed += float(bq) * bk * ((nk + bk - 1) // bk)
    return credited / executed if executed else None


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` (fetch + write), from the committed rocprofv3 counter summary
    of this workload, or None when no summary has been recorded."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.json")
    try:
        with open(path) as f:
            return json.load(f)["bytes_per_launch"].get(kernel)
    except (OSError, ValueError, KeyError):
        return None


def cpu_baseline(cfg, cu_np, q, k, v, dout, prefix, heads):
    """fp64 oracle, all three passes, on the causal prefix [0, prefix) of the first `heads` heads."""
    import numpy as np
    import torch
    from oracle import attention as ora
    from paper_2401_09149_amd import workloads as W
    ora.build()
    sl = lambda t, hcount: np.ascontiguousarray(
        t[:, :prefix, :hcount].to("cpu", torch.float32).numpy().astype(np.float64))
    kv_heads = max(1, heads * cfg.Hkv // cfg.Hq)
    q64, k64, v64, do64 = sl(q, heads), sl(k, kv_heads), sl(v, kv_heads), sl(dout, heads)
    t0 = time.perf_counter()
    ora.attn_fwd_bwd(q64, k64, v64, do64, cfg.scale, True)
    dt = time.perf_counter() - t0
    flop = 3.5 * 2.0 * float(prefix) ** 2 * cfg.D * heads
    full = 3.5 * W.fwd_flops(cfg, cu_np)
    return {
        "value": flop / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": ora.num_threads(),
        "kind": "oracle",
        "seconds": dt,
        # extrapolated, not measured: the sample's time scaled by the FLOP ratio (per head and, for a shorter prefix, by length^2)
        "extrapolated_full_config_seconds": dt * full / flop,
        "sample": f"fp64 oracle fwd+bwd (3 passes) on tokens [0,{prefix}) of q heads 0..{heads - 1} of the same "
                  f"seeded inputs (a self-contained causal prefix), same FLOP convention",
    }


def sp_permute_bench(cfg, iters, with_cpu, profiled_with):
    """The eight re-layout kernels either side of the two sequence-parallel all-to-alls, on one GPU's buffers of a
    plan of the paper; each launch reads its tensor once and writes it once (2 bytes of traffic per tensor byte).
    Buffers rotate through a ring larger than the last-level cache, so every launch streams from and to HBM."""
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    ring = 6
    n, nq = cfg.n_qkv, cfg.n_o
    nk = (n - nq) // 2
    new = lambda m: [torch.empty(m, dtype=torch.int16, device=dev) for _ in range(ring)]
    A, X, Q, K, V, Y = new(n), new(n), new(nq), new(nk), new(nk), new(nq)
    for t in A + Q + K + V:
        t.random_(-32768, 32767)
    sq, so = (cfg.B, cfg.Sl, cfg.Hq, cfg.Hkv, cfg.D, cfg.P), (cfg.B, cfg.Sl, cfg.Hq, cfg.D, cfg.P)
    calls = {
        "pack_qkv": (lambda i: binding.ie_sp_pack_qkv(A[i], X[i], *sq), n),
        "unpack_qkv": (lambda i: binding.ie_sp_unpack_qkv(A[i], Q[i], K[i], V[i], *sq), n),
        "pack_o": (lambda i: binding.ie_sp_pack_o(Q[i], Y[i], *so), nq),
        "unpack_o": (lambda i: binding.ie_sp_unpack_o(Q[i], Y[i], *so), nq),
        "pack_do": (lambda i: binding.ie_sp_pack_do(Q[i], Y[i], *so), nq),
        "unpack_do": (lambda i: binding.ie_sp_unpack_do(Q[i], Y[i], *so), nq),
        "pack_dqkv": (lambda i: binding.ie_sp_pack_dqkv(Q[i], K[i], V[i], X[i], *sq), n),
        "unpack_dqkv": (lambda i: binding.ie_sp_unpack_dqkv(A[i], X[i], *sq), n),
    }
    res, total_bytes, total_ms = {}, 0.0, 0.0
    for name, (fn, elems) in calls.items():
        for i in range(ring):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fn(i % ring)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        res[name] = {"us": ms * 1e3, "GBps": 4.0 * elems / ms / 1e6}
        total_bytes += 4.0 * elems
        total_ms += ms
    achieved = total_bytes / total_ms / 1e6
    out = {"workload": cfg.name, "B": cfg.B, "Sl": cfg.Sl, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "D": cfg.D, "P": cfg.P,
           "dtype": "u16", "kernel": "sp_permute_kernel", "per_call": res,
           # ie_attn_fwd_sp / ie_attn_bwd_sp read and write the exchange buffers themselves: these two calls drop out of a layer
           "us_saved_by_fused_attention_calls": res["unpack_qkv"]["us"] + res["pack_dqkv"]["us"],
           "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                        "traffic": measured_traffic(profiled_with, "sp_permute_kernel"),
                        "algorithmic_bytes": total_bytes / len(calls),
                        "note": "all eight calls of one layer (forward and backward): bytes moved / time; traffic and "
                                "algorithmic_bytes are means per launch over the eight calls"}}
    if with_cpu:
        from oracle import sp_permute as ora
        a = A[0].cpu().numpy()
        t0 = time.perf_counter()
        x = ora.pack_qkv(a, *sq)
        ora.unpack_qkv(x, *sq)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2 * 4.0 * n / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle", "seconds": dt,
                               "sample": "numpy oracle, pack_qkv then unpack_qkv of the same buffer size"}
    return out


def linear_bench(iters, with_cpu, profiled_with):
    """The linear modules of one 7B layer (hidden 4096, MLP 11008; Table 2) applied to one GPU's 8192 tokens of the
    paper's 32K plan (s_sp = 4): forward, input gradient and weight gradient of the QKV, output, gate/up and down
    projections.  FLOP = 2 M N K per product.  torch.matmul (the vendor library) on the same operands is timed
    beside it as context."""
    import torch
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    M = 8192
    modules = [("qkv", 12288, 4096), ("out", 4096, 4096), ("gate_up", 22016, 4096), ("down", 4096, 11008)]
    gen = torch.Generator(device=dev)
    gen.manual_seed(3000)
    mk = lambda *shape: torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    per, flop_total, ms_total, lib_ms_total = {}, 0.0, 0.0, 0.0
    for name, N, K in modules:
        x, w, dy = mk(M, K), mk(N, K), mk(M, N)
        y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
        ours = [timed(lambda: binding.ie_linear_fwd(x, w, y)), timed(lambda: binding.ie_linear_bwd_input(dy, w, dx)),
                timed(lambda: binding.ie_linear_bwd_weight(dy, x, dw))]
        lib = [timed(lambda: torch.matmul(x, w.t(), out=y)), timed(lambda: torch.matmul(dy, w, out=dx)),
               timed(lambda: torch.matmul(dy.t(), x, out=dw))]
        flop = 2.0 * M * N * K
        per[name] = {"N": N, "K": K, "tflops": [flop / t / 1e9 for t in ours], "library_tflops": [flop / t / 1e9 for t in lib]}
        flop_total += 3 * flop
        ms_total += sum(ours)
        lib_ms_total += sum(lib)
        del x, w, dy, y, dx, dw
    # the 65B gate/up projection whose output is the (16384, 22016) activation of the appendix on memory fragmentation
    M2, N2, K2 = 16384, 22016, 8192
    x, w, dy = mk(M2, K2), mk(N2, K2), mk(M2, N2)
    y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
    ours = [timed(lambda: binding.ie_linear_fwd(x, w, y)), timed(lambda: binding.ie_linear_bwd_input(dy, w, dx)),
            timed(lambda: binding.ie_linear_bwd_weight(dy, x, dw))]
    lib = [timed(lambda: torch.matmul(x, w.t(), out=y)), timed(lambda: torch.matmul(dy, w, out=dx)),
           timed(lambda: torch.matmul(dy.t(), x, out=dw))]
    flop2 = 2.0 * M2 * N2 * K2
    big = {"M": M2, "N": N2, "K": K2, "tflops": [flop2 / t / 1e9 for t in ours], "library_tflops": [flop2 / t / 1e9 for t in lib]}
    del x, w, dy, y, dx, dw
    achieved = flop_total / ms_total / 1e9
    out = {"workload": "7b_linear_m8192", "M": M, "dtype": "bf16", "kernel": "linear_gemm_kernel",
           "order": ["fwd", "bwd_input", "bwd_weight"], "per_module": per, "ms_per_layer": ms_total,
           "library_ms_per_layer": lib_ms_total, "gate_up_65b_m16384": big,
           "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(profiled_with, "linear_gemm_kernel"),
                        "note": "all twelve products of one layer: FLOP / time; traffic: HBM bytes per launch, mean over the three instantiations' means"}}
    if with_cpu:
        import numpy as np
        from oracle import linear as ora
        rows, N, K = 256, 12288, 4096
        x64 = np.random.default_rng(1).standard_normal((rows, K))
        w64 = np.random.default_rng(2).standard_normal((N, K))
        t0 = time.perf_counter()
        ora.linear_fwd(x64, w64)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * rows * N * K / dt / 1e12, "unit": "TFLOP/s", "cores": os.cpu_count(), "kind": "oracle",
                               "seconds": dt, "sample": f"fp64 oracle (numpy matmul), forward of the QKV projection on {rows} tokens"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1, help="index into the workload table (default: the headline config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-prefix", type=int, default=32768)
    ap.add_argument("--cpu-heads", type=int, default=1)
    ap.add_argument("--sp-config", type=int, default=1, help="index into the re-layout workload table; -1 skips that part")
    ap.add_argument("--no-linear", action="store_true", help="skip the linear-module part")
    ap.add_argument("--stored-ds", action="store_true",
                    help="time the optional backward path that keeps dS in a B*Hq*S*(S+128)-byte workspace as the step's backward "
                         "(default: the O(S)-workspace path; the other one is reported under bwd.other_path)")
    ap.add_argument("--no-other-path", action="store_true", help="do not time the other backward path beside the step's own")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling the profiler's FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2401_09149_amd import binding, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    binding.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config]
    cu_np = W.make_cu_seqlens(cfg)
    cu = None if cu_np is None else torch.tensor(cu_np, dtype=torch.int32, device=dev)
    q, k, v, dout = W.make_inputs(cfg, device=dev)
    o = torch.empty_like(q)
    lse = torch.empty((cfg.B, cfg.Hq, cfg.S), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    nd = 0 if cu is None else cu.numel() - 1
    small_bytes = binding.ie_attn_bwd_workspace_bytes(cfg.B, cfg.S, cfg.Hq, cfg.Hkv, cfg.D, nd)
    ds_bytes = binding.ie_attn_bwd_fast_workspace_bytes(cfg.B, cfg.S, cfg.Hq, cfg.Hkv, cfg.D, nd, cfg.causal)
    has_ds_path = ds_bytes > small_bytes
    stored_ds = args.stored_ds and has_ds_path
    ws = binding.alloc_bwd_workspace(q, k, cu, fast=stored_ds, causal=cfg.causal)

    def fwd():
        binding.ie_attn_fwd(q, k, v, o, lse, cu, cfg.scale, cfg.causal)

    def bwd(phases=binding.BWD_ALL):
        binding.ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu, cfg.scale, cfg.causal, ws, phases, stored_ds=stored_ds)

    def step():
        fwd()
        bwd()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)     # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # Per-kernel durations, events on the launch stream (torch's current stream).
    it = max(3, min(args.steps, 10))
    fwd_ms, fwd_min, fwd_med = event_ms(fwd, it)
    bwd_ms, bwd_min, bwd_med = event_ms(bwd, it)
    delta_ms, _, _ = event_ms(lambda: bwd(binding.BWD_DELTA), it)
    dkdv_ms, _, _ = event_ms(lambda: bwd(binding.BWD_DKDV), it)
    dq_ms, _, _ = event_ms(lambda: bwd(binding.BWD_DQ), it)   # (with a stored dS: reads what the dK/dV phase just left)

    # the other backward path, for comparison; not part of `value`
    other = None
    if has_ds_path and not args.no_other_path and (stored_ds or ds_bytes <= 64e9):
        ws_o = binding.alloc_bwd_workspace(q, k, cu, fast=not stored_ds, causal=cfg.causal)
        bwd_o = lambda ph=binding.BWD_ALL: binding.ie_attn_bwd_phases(q, k, v, o, dout, lse, dq, dk, dv, cu, cfg.scale,
                                                                      cfg.causal, ws_o, ph, stored_ds=not stored_ds)
        bwd_o()
        o_ms, _, _ = event_ms(bwd_o, it)
        o_dkdv, _, _ = event_ms(lambda: bwd_o(binding.BWD_DKDV), it)
        o_dq, _, _ = event_ms(lambda: bwd_o(binding.BWD_DQ), it)
        other = {"path": "recompute" if stored_ds else "stored_ds", "ms": o_ms, "dq_ms": o_dq, "dkdv_ms": o_dkdv,
                 "tflops": W.bwd_flops(cfg, cu_np) / (o_ms * 1e-3) / 1e12, "workspace_bytes": ws_o.numel()}
        del ws_o

    delta_bytes = 2.0 * cfg.B * cfg.S * cfg.Hq * cfg.D * 2 + 3.0 * cfg.B * cfg.S * cfg.Hq * 4
    f_fwd = W.fwd_flops(cfg, cu_np)
    f_bwd = W.bwd_flops(cfg, cu_np)
    value = (f_fwd + f_bwd) / (ms_per_step * 1e-3) / 1e12
    fwd_tflops = f_fwd / (fwd_ms * 1e-3) / 1e12
    bwd_tflops = f_bwd / (bwd_ms * 1e-3) / 1e12

    # Roofline of the kernel that takes the most time.  Matrix FLOP each kernel executes per
    # visible (query, key) pair and query head: forward 4D (S, PV); dK/dV kernel 8D (S, dP, dV,
    # dK); dQ kernel 6D (S, dP recomputed, dQ), of which only the dQ product (2D) is not
    # already counted in the dK/dV kernel.  Pairs are counted as L^2/2 per document.
    # With a stored dS the dQ kernel is one product (2D) and bound by reading dS: 2 bytes per
    # pair of the block triangle, B*Hq*S*(S+128) in all, plus K once per query tile from L2.
    pairs = f_fwd / (4.0 * cfg.D)   # = B * Hq * sum L^2 / 2
    kernels = {
        ("attn_fwd_wide_kernel" if cfg.D == 128 else "attn_fwd_kernel"): (fwd_ms, 4.0 * cfg.D * pairs),
        ("attn_bwd_dkdv_kernel_store_ds" if stored_ds else "attn_bwd_dkdv_kernel"): (dkdv_ms, 8.0 * cfg.D * pairs),
    }
    if stored_ds:
        kernels["attn_bwd_dq_from_ds_kernel"] = (dq_ms, float(cfg.B) * cfg.Hq * cfg.S * (cfg.S + 128))   # bytes
    else:
        kernels["attn_bwd_dq_kernel"] = (dq_ms, 6.0 * cfg.D * pairs)
    dom = max(kernels, key=lambda n: kernels[n][0])
    dom_ms, dom_work = kernels[dom]
    if dom == "attn_bwd_dq_from_ds_kernel":
        achieved = dom_work / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": measured_traffic(cfg.name, dom), "ms": dom_ms}
    else:
        achieved = dom_work / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(cfg.name, dom), "ms": dom_ms}

    out = {
        "metric": "causal attention fwd+bwd TFLOPS and % of bf16 MFMA peak, 1 MI355X, S=32K D=128",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "S": cfg.S, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "D": cfg.D,
                   "causal": cfg.causal, "packed_docs": None if cu_np is None else len(cu_np) - 1, "seed": cfg.seed},
        "frac_of_peak": value / PEAK_BF16_TFLOPS,
        "fwd": {"ms": fwd_ms, "ms_min": fwd_min, "ms_median": fwd_med, "tflops": fwd_tflops, "frac_of_peak": fwd_tflops / PEAK_BF16_TFLOPS},
        "bwd": {"ms": bwd_ms, "ms_min": bwd_min, "ms_median": bwd_med, "tflops": bwd_tflops, "frac_of_peak": bwd_tflops / PEAK_BF16_TFLOPS,
                "delta_ms": delta_ms, "dq_ms": dq_ms, "dkdv_ms": dkdv_ms,
                # the HBM-bound preprocessing kernel: o and dO read once, two fp32 planes written, lse read
                "delta_GBps": delta_bytes / delta_ms / 1e6, "delta_frac_of_hbm_peak": delta_bytes / delta_ms / 1e6 / PEAK_HBM_GBS,
                "path": "stored_ds" if stored_ds else "recompute", "workspace_bytes": ws.numel(), "other_path": other},
        "peak_tflops": PEAK_BF16_TFLOPS,
        "fwd_tile_efficiency": tile_efficiency(cfg, cu_np) if cfg.D == 128 else tile_efficiency(cfg, cu_np, 128, 64),
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        prefix = min(args.cpu_prefix, cfg.S if cu_np is None else int(cu_np[1]))
        out["cpu_baseline"] = cpu_baseline(cfg, cu_np, q, k, v, dout, prefix, min(args.cpu_heads, cfg.Hq))
    if args.sp_config >= 0:
        del q, k, v, dout, o, lse, dq, dk, dv, ws
        out["sp_permute"] = sp_permute_bench(W.SP_CONFIGS[args.sp_config], 4 * it, not args.no_cpu_baseline, cfg.name)
    if not args.no_linear:
        if args.sp_config < 0:
            del q, k, v, dout, o, lse, dq, dk, dv, ws
        out["linear"] = linear_bench(it, not args.no_cpu_baseline, cfg.name)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
