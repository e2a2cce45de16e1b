"""Shared helpers for the GPU parity tests: run the HIP path through the C ABI and the fp64
oracle on the same bf16 bit patterns, and compare to the stated tolerances."""
import numpy as np
import torch

# Tolerances of the parity bar (bf16 inputs, fp32 accumulation, bf16 outputs).
TOL_O = 2e-2          # max |O - O_ref|
TOL_LSE = 1e-3        # max |LSE - LSE_ref|
TOL_GRAD_ABS = 5e-2   # max abs error of dQ, dK, dV
TOL_GRAD_REL = 1e-2   # relative Frobenius error of dQ, dK, dV


def randn_bf16(shape, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16)


def to64(t):
    return np.ascontiguousarray(t.detach().to("cpu", torch.float32).numpy().astype(np.float64))


def run_gpu(q, k, v, dout, scale, causal, cu):
    """Forward then backward through the C ABI.  Inputs are CPU bf16 tensors."""
    from paper_2401_09149_amd import binding
    dev = "cuda:0"
    qd, kd, vd, dod = (x.to(dev) for x in (q, k, v, dout))
    cud = None if cu is None else torch.tensor(np.asarray(cu), dtype=torch.int32, device=dev)
    o, lse = binding.attn_fwd(qd, kd, vd, scale, causal, cud)
    dq, dk, dv = binding.attn_bwd(qd, kd, vd, o, dod, lse, scale, causal, cud)
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


# Below this RMS magnitude a reference gradient counts as zero: with a single visible key
# dS = P (dP - delta) vanishes identically, the fp64 reference is rounding noise, and the fp32
# path leaves the difference of two sums of D products of O(1) terms (about 1e-7 each); a
# relative error against that is meaningless.  The absolute bar applies regardless.
REL_FLOOR_RMS = 1e-4


def grad_errors(got, ref):
    d = got - ref
    floor = REL_FLOOR_RMS * np.sqrt(ref.size)
    return float(np.abs(d).max()), float(np.linalg.norm(d) / max(np.linalg.norm(ref), floor))


def compare_all(got, ref, label="", grad_abs_tol=TOL_GRAD_ABS):
    """got: GPU tensors (o, lse, dq, dk, dv); ref: oracle fp64 arrays in the same order."""
    o, lse, dq, dk, dv = (to64(x) for x in got)
    ro, rlse, rdq, rdk, rdv = ref
    report = {
        "o_max": float(np.abs(o - ro).max()),
        "lse_max": float(np.abs(lse - rlse).max()),
    }
    for name, g, r in (("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        report[name + "_max"], report[name + "_rel"] = grad_errors(g, r)
    print(label, {k_: f"{v_:.2e}" for k_, v_ in report.items()}, flush=True)
    assert np.isfinite(o).all() and np.isfinite(lse).all() and np.isfinite(dq).all()
    assert np.isfinite(dk).all() and np.isfinite(dv).all()
    assert report["o_max"] <= TOL_O, report
    assert report["lse_max"] <= TOL_LSE, report
    for name in ("dq", "dk", "dv"):
        assert report[name + "_max"] <= grad_abs_tol, report
        assert report[name + "_rel"] <= TOL_GRAD_REL, report
    return report
