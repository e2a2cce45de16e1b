"""Shader cycles per MFMA and the shader clock of the two hand-sequenced kernels, read in-kernel.

The kernels carry cycle counters under -DIE_EXP_TIMING (per workgroup or wave: shader cycles via the
cycle counter, elapsed time via the constant 100 MHz counter, time spent in barriers); such a build
writes them into an output buffer INSTEAD of results (the forward into lse, the dK/dV kernel into
dq), so it is only good for this report.  What-if builds delete part of the forward's work
(-DIE_EXP_W_NOSM: no softmax arithmetic, _NOLDS: no LDS reads, _NOCOPY: no global->LDS copies):
their results are wrong by construction and only their cycle counts mean something.

    python -m paper_2401_09149_amd.cycle_report --build      # here, no GPU needed: builds _variants/
    python -m paper_2401_09149_amd.cycle_report              # on the GPU: prints the report
"""
import argparse
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
VARIANTS = {
    "timing": ["-DIE_EXP_TIMING"],
    "timing_nosm": ["-DIE_EXP_TIMING", "-DIE_EXP_W_NOSM"],
    "timing_nolds": ["-DIE_EXP_TIMING", "-DIE_EXP_W_NOLDS"],
    "timing_nocopy": ["-DIE_EXP_TIMING", "-DIE_EXP_W_NOCOPY"],
    "timing_bare": ["-DIE_EXP_TIMING", "-DIE_EXP_W_NOSM", "-DIE_EXP_W_NOLDS", "-DIE_EXP_W_NOCOPY"],
}


def lib_path(name):
    return os.path.join(HERE, "_variants", f"libie_attn_{name}.so")


def measure(which):
    """Runs in a process whose IE_ATTN_LIB points at a timing build."""
    import time
    import torch
    from . import binding, workloads as W
    cfg = W.CONFIGS[1]
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    mk = lambda h: torch.randn((cfg.B, cfg.S, h, cfg.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q, k, v, do = mk(cfg.Hq), mk(cfg.Hkv), mk(cfg.Hkv), mk(cfg.Hq)
    o = torch.empty_like(q)
    lse = torch.zeros((cfg.B, cfg.Hq, cfg.S), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.zeros_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = binding.alloc_bwd_workspace(q, k, None, fast=(which == "dkdv_ds"))   # dkdv_ds: the variant that stores dS
    fwd = lambda: binding.ie_attn_fwd(q, k, v, o, lse, None, cfg.scale, True)
    bwd = lambda ph: binding.ie_attn_bwd_phases(q, k, v, o, do, lse, dq, dk, dv, None, cfg.scale, True, ws, ph)

    def timed(fn, warm=100, iters=20):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / iters

    if which == "fwd":
        ms = timed(fwd)
        n = (cfg.S // 256) * cfg.Hq * 4   # waves
        d = lse.view(torch.int64).flatten()[: n * 8].cpu().numpy().reshape(n, 8).astype(float)
        cyc, wall, nkt, nfast, tsync, tfast = (d[:, i] for i in range(6))
        ghz = cyc.sum() / wall.sum() * 0.1
        per_simd = lambda c: c.sum() / 1024 / ghz * 1e-6   # ms of one SIMD's time (one wave per SIMD, 1024 SIMDs)
        print(f"forward: {ms:.3f} ms, shader clock {ghz:.3f} GHz, "
              f"{tfast.sum() / (nfast.sum() * 128):.1f} cycles per MFMA in the hand-sequenced tiles "
              f"({int(nfast.sum())} of {int(nkt.sum())} wave-tiles), {tsync.sum() / nkt.sum():.0f} cycles per tile at the barrier; "
              f"per SIMD {per_simd(tfast):.3f} ms in hand-sequenced tiles, {per_simd(cyc - tfast):.3f} ms in prologue, masked tiles "
              f"and epilogue ({(cyc - tfast).mean():.0f} cycles per workgroup), {ms - per_simd(cyc):.3f} ms idle (launch gaps, tail)")
    else:
        fwd()
        bwd(binding.BWD_DELTA)
        ms = timed(lambda: bwd(binding.BWD_DKDV))
        n = (cfg.S // 128) * cfg.Hkv      # workgroups
        d = dq.view(torch.int64).flatten()[: n * 8].cpu().numpy().reshape(n, 8).astype(float)
        tot, tf, nf, tg, ts, steps, tready = (d[:, i] for i in range(7))
        clock = tot.sum() / 256 / (ms * 1e-3) / 1e9   # one workgroup per CU at a time, 256 CUs, all busy
        print(f"dK/dV{' with dS stores' if which == 'dkdv_ds' else ''}: {ms:.3f} ms, shader clock about {clock:.2f} GHz (sum of workgroup cycles / 256 CUs / time), "
              f"{tf.sum() / nf.sum() / 128:.1f} cycles per MFMA in the hand-sequenced tiles ({int(nf.sum())} of {int(steps.sum())} steps), "
              f"{ts.sum() / steps.sum():.0f} cycles per step at the barrier; per workgroup {tf.mean():.0f} cycles in hand-sequenced "
              f"tiles, {tg.mean():.0f} in masked tiles, {ts.mean():.0f} at barriers, {tready.mean():.0f} waiting for K/V and the first stage, "
              f"{(tot - tf - tg - ts - tready).mean():.0f} in the rest (descriptor arithmetic between steps, flush of the last tile, the counters themselves)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true", help="build the instrumented variants (hipcc, no GPU needed) and exit")
    ap.add_argument("--measure", default=None, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.build:
        from . import build as B
        for name, flags in VARIANTS.items():
            print(B.build_variant(name, flags))
        return
    if args.measure:
        measure(args.measure)
        return
    for name in VARIANTS:
        if not os.path.exists(lib_path(name)):
            print(f"cycle_report: {lib_path(name)} is missing; run with --build first", file=sys.stderr)
            sys.exit(1)
    runs = [("timing", "fwd"), ("timing", "dkdv"), ("timing", "dkdv_ds"), ("timing_nosm", "fwd"), ("timing_nolds", "fwd"), ("timing_nocopy", "fwd"), ("timing_bare", "fwd")]
    for name, which in runs:
        env = dict(os.environ, IE_ATTN_LIB=lib_path(name))
        label = {"timing": "as built", "timing_nosm": "no softmax arithmetic", "timing_nolds": "no LDS reads",
                 "timing_nocopy": "no global->LDS copies", "timing_bare": "MFMAs and barriers only"}[name]
        print(f"[{label}] ", end="", flush=True)
        r = subprocess.run([sys.executable, "-m", "paper_2401_09149_amd.cycle_report", "--measure", which], env=env,
                           capture_output=True, text=True, cwd=os.path.dirname(HERE))
        print(r.stdout.strip() or r.stderr.strip()[-400:], flush=True)


if __name__ == "__main__":
    main()
