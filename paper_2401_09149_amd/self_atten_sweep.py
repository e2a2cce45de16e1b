"""Times the attention kernels over the per-GPU shapes of the paper's own parallel plans.

The paper's computation profiler measures `self-atten(b, S, H, D/s_sp)` on a single GPU for the
shapes its planner considers (Sec. 4.2 "Computation Profiler"); this is that sweep for the plans
the paper lists as its own choice ("Our Work" rows of Appendix Tables 4-7): micro-batch b, all S
tokens, heads/s_sp heads of dimension 128 (Table 2: 32, 40, 48 and 64 heads).  Inputs are N(0,1)
rounded to bf16, drawn on the device (timing only; parity is the tests' business).  The backward pass is
timed twice: with the small workspace (dQ recomputes S, P, dP) and, where B*Hq*S*(S+128) bytes more fit the
limit given by --ds-limit-gb, with the workspace that lets the dK/dV kernel store dS.

    python -m paper_2401_09149_amd.self_atten_sweep [--iters 5] [--out profiles/self_atten_sweep.md] [--json table.json]

The JSON table (one record per shape: b, S, heads, head_dim, fwd_ms, bwd_ms, bwd_stored_ds_ms) is what
planner.ProfiledCompute reads in place of its analytic attention rate.
"""
import argparse
import sys

# model -> (heads, {sequence length: (micro-batch b, s_sp)}), "Our Work" rows of Appendix Tables 4-7
PLANS = {
    "7B": (32, {4096: (2, 1), 8192: (1, 1), 16384: (1, 2), 32768: (1, 4), 65536: (1, 8), 131072: (1, 16), 262144: (1, 32)}),
    "13B": (40, {4096: (1, 1), 8192: (8, 8), 16384: (1, 4), 32768: (1, 8), 65536: (1, 8), 131072: (1, 4), 262144: (1, 8)}),
    "30B": (48, {4096: (1, 2), 8192: (1, 4), 16384: (1, 8), 32768: (1, 8), 65536: (1, 16), 131072: (1, 8), 262144: (1, 8)}),
    "65B": (64, {4096: (1, 2), 8192: (1, 8), 16384: (1, 2), 32768: (1, 4), 65536: (1, 8), 131072: (1, 8), 262144: (1, 8)}),
}
HEAD_DIM = 128
PEAK_BF16_TFLOPS = 2500.0


def shapes():
    for model, (heads, plans) in PLANS.items():
        for S, (b, s_sp) in plans.items():
            assert heads % s_sp == 0
            yield model, S, b, s_sp, heads // s_sp


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--out", default=None, help="also write the table (markdown) to this file")
    ap.add_argument("--json", default=None, help="also write the measurements as a JSON table for planner.ProfiledCompute")
    ap.add_argument("--ds-limit-gb", type=float, default=160.0, help="largest workspace for the stored-dS backward path")
    args = ap.parse_args()
    import torch
    from . import binding
    if not torch.cuda.is_available():
        print("self_atten_sweep: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    binding.load()
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    D = HEAD_DIM
    scale = D ** -0.5
    lines = ["| model | S | b | s_sp | heads/GPU | fwd ms | fwd TFLOP/s | bwd ms | bwd TFLOP/s | bwd ms, stored dS | workspace GB | fwd+bwd % of 2.5 PFLOP/s (faster bwd) |",
             "|---|---|---|---|---|---|---|---|---|---|---|---|"]
    records = []
    for model, S, b, s_sp, H in shapes():
        mk = lambda: torch.randn((b, S, H, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        q, k, v, do = mk(), mk(), mk(), mk()
        o = torch.empty_like(q)
        lse = torch.empty((b, H, S), dtype=torch.float32, device=dev)
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = binding.alloc_bwd_workspace(q, k, None)
        fwd = lambda: binding.ie_attn_fwd(q, k, v, o, lse, None, scale, True)
        bwd = lambda: binding.ie_attn_bwd_phases(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws, binding.BWD_ALL)
        bwd_ds = lambda: binding.ie_attn_bwd_phases(q, k, v, o, do, lse, dq, dk, dv, None, scale, True, ws, binding.BWD_ALL,
                                                    stored_ds=True)

        def timed(fn):
            for _ in range(2):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.iters

        f_ms, b_ms = timed(fwd), timed(bwd)
        big = binding.ie_attn_bwd_fast_workspace_bytes(b, S, H, H, D, 0, True)
        s_ms = None
        if ws.numel() < big <= args.ds_limit_gb * 1e9:
            del ws
            ws = torch.empty(big, dtype=torch.uint8, device=dev)
            s_ms = timed(bwd_ds)
        flop_f = 2.0 * b * H * float(S) ** 2 * D   # 4 S^2 D H / 2 (causal halving); backward = 2.5x
        tf_f, tf_b = flop_f / f_ms / 1e9, 2.5 * flop_f / b_ms / 1e9
        both = 3.5 * flop_f / (f_ms + min(b_ms, s_ms or b_ms)) / 1e9
        line = (f"| {model} | {S} | {b} | {s_sp} | {H} | {f_ms:.3f} | {tf_f:.0f} | {b_ms:.3f} | {tf_b:.0f} | "
                f"{'—' if s_ms is None else format(s_ms, '.3f')} | {'—' if s_ms is None else format(big / 1e9, '.1f')} | "
                f"{100 * both / PEAK_BF16_TFLOPS:.1f} |")
        print(line, flush=True)
        lines.append(line)
        records.append({"model": model, "b": b, "S": S, "s_sp": s_sp, "heads": H, "head_dim": D, "fwd_ms": f_ms, "bwd_ms": b_ms,
                        "bwd_stored_ds_ms": s_ms, "stored_ds_workspace_bytes": big if s_ms is not None else None})
        del q, k, v, do, o, lse, dq, dk, dv, ws
    if args.json:
        import json
        with open(args.json, "w") as f:
            json.dump({"kernel": "ie_attn_fwd / ie_attn_bwd, causal, bf16", "iters": args.iters, "records": records}, f, indent=1)
            f.write("\n")
    if args.out:
        with open(args.out, "w") as f:
            f.write("# self-atten(b, S, H, D/s_sp) on one MI355X over the paper's own plans (Appendix Tables 4-7, \"Our Work\")\n\n")
            f.write(f"command: `python -m paper_2401_09149_amd.self_atten_sweep --iters {args.iters} --out <this file>`\n\n")
            f.write("causal, head dimension 128, bf16; FLOP convention: forward 4·S²·D·H/2, backward 2.5×\n\n")
            f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
