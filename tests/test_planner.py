"""Pins of the planner slice (paper_2401_09149_amd/planner.py) to what the paper prints: Table 2 (model sizes),
the memory and communication equations of Sec. 3.2, the constraints of Sec. 4.5, and the paper's own plans
(Appendix Tables 4-7, tests/golden/paper_plans.csv): each of them must satisfy every constraint and fit the
80 GB GPUs it was run on.  The search is checked against an independent brute-force enumeration."""
import itertools
import os

import pytest

from paper_2401_09149_amd import planner as pl

HERE = os.path.dirname(os.path.abspath(__file__))
N, B_TOKENS, CAP = 128, 2 ** 22, 80e9     # Sec. 5.1: 128 GPUs of 80 GB; Sec. 5.2: global batch of 4M tokens = the plans' b * S * n * s_dp


def paper_plans():
    out = []
    for line in open(os.path.join(HERE, "golden", "paper_plans.csv")):
        if line.startswith("#"):
            continue
        f = line.strip().split(",")
        n, b, pp, dp, tp, sp, ps, oss, a = map(int, f[2:])
        out.append((f[0], int(f[1]), pl.Plan(b, n, a, pp, dp, tp, sp, ps, oss, oss)))   # s_gs is not tabulated: {1, s_oss}
    return out


def test_table3_model_sizes():
    """Psi = 12 H^2 + 2 H per layer; L Psi + 2 V H parameters give the models their names."""
    assert pl.MODELS["7B"].psi == 12 * 4096 ** 2 + 2 * 4096
    for name, lo, hi in (("7B", 6.5e9, 7.5e9), ("13B", 12.5e9, 14e9), ("30B", 27e9, 31e9), ("65B", 63e9, 67e9)):
        m = pl.MODELS[name]
        assert lo < m.L * m.psi + 2 * m.V * m.H < hi


def test_every_plan_of_the_paper_is_feasible_and_fits():
    plans = paper_plans()
    assert len(plans) == 28
    for name, S, plan in plans:
        model = pl.MODELS[name]
        assert pl.violated_constraints(plan, model, N, B_TOKENS, S) == [], (name, S)
        mem = pl.memory_bytes(plan, model, S)
        assert mem["total"] < CAP, (name, S, mem)
        assert mem["total"] > 0.2 * CAP        # and none of them leaves the GPU nearly empty


def test_memory_equations():
    m = pl.MODELS["7B"]
    base = pl.Plan(b=1, n=4, a=0, s_pp=1, s_dp=128, s_tp=1, s_sp=1, s_ps=1, s_gs=1, s_oss=1)
    S = 32768
    mem = pl.memory_bytes(base, m, S)
    # Table 2: P and G take 2 bytes per parameter, OS 6; activations 34 b S H per layer without recomputation
    assert mem["P"] == 2 * m.L * m.psi and mem["G"] == mem["P"] and mem["OS"] == 3 * mem["P"]
    assert mem["ACT"] == 34 * S * m.H * m.L
    rec = pl.memory_bytes(pl.Plan(1, 4, 1, 1, 128, 1, 1, 1, 1, 1), m, S)
    assert rec["ACT"] == 2 * S * m.H * m.L                     # a = 1: only the layer boundaries are kept
    sp = pl.memory_bytes(pl.Plan(1, 4, 0, 1, 32, 1, 4, 2, 4, 4), m, S)
    assert sp["ACT"] == mem["ACT"] / 4                          # sequence parallelism divides activations by s_sp
    assert sp["P"] == mem["P"] / 2 and sp["G"] == mem["G"] / 8 and sp["OS"] == mem["OS"] / 8   # s_ps, s_ps s_gs, s_ps s_oss
    pp = pl.memory_bytes(pl.Plan(1, 2, 0, 4, 32, 1, 1, 1, 1, 1), m, S)
    assert pp["P"] == mem["P"] / 4 and pp["ACT"] == 2 * mem["ACT"] / 4    # min(s_pp, n) micro-batches in flight
    # the summary equation read literally (G / s_gs, OS / s_oss, equal weights) would not fit the paper's own plan
    name, S65, plan = [x for x in paper_plans() if x[0] == "65B" and x[1] == 262144][0]
    m65 = pl.MODELS["65B"]
    literal = 2 * m65.L * m65.psi / (plan.s_pp * plan.s_tp) * (1 / plan.s_ps + 1 / plan.s_gs + 1 / plan.s_oss)
    assert literal > CAP > pl.memory_bytes(plan, m65, S65)["total"]


class UnitBandwidth:
    """w = 1 byte/s for every operation: tau is the volume, so the counts and sizes of the equations show."""
    def tau(self, op, v, p, span):
        return 0.0 if p <= 1 else float(v)


def test_communication_volumes_of_the_equations():
    m = pl.MODELS["7B"]
    S, n = 32768, 4
    bSH = S * m.H
    sp = pl.comm_time_layer(pl.Plan(1, n, 0, 1, 32, 1, 4, 1, 1, 1), m, S, N, UnitBandwidth())
    assert sp["sp"] == 2 * n * 6 * bSH + 2 * n * 2 * bSH       # two all-to-alls of 6bSH and 2bSH bytes, forward and backward
    assert "tp" not in sp and "ps" not in sp and "gs" not in sp
    tp = pl.comm_time_layer(pl.Plan(1, n, 0, 1, 32, 4, 4, 1, 1, 1), m, S, N, UnitBandwidth())
    assert tp["tp"] == (2 * n + 3 * n) * 2 * bSH               # 2n reduce-scatters and 3n all-gathers of 2bSH bytes
    ps = pl.comm_time_layer(pl.Plan(1, n, 0, 1, 32, 1, 4, 2, 4, 4), m, S, N, UnitBandwidth())
    assert ps["ps"] == 3 * n * 2 * m.psi                       # 2n all-gathers + n reduce-scatters of 2 Psi bytes
    assert ps["oss"] == 2 * (2 * m.psi / 2)                    # reduce-scatter + all-reduce of 2 Psi / s_ps
    assert ps["gs"] == (n - 1) * (2 * m.psi / 2)


def test_each_constraint_can_be_violated_alone():
    m, S = pl.MODELS["7B"], 32768
    ok = pl.Plan(1, 4, 0, 1, 32, 1, 4, 2, 4, 4)
    assert pl.violated_constraints(ok, m, N, B_TOKENS, S) == []
    change = lambda **kw: pl.Plan(**{**ok.__dict__, **kw})
    assert pl.violated_constraints(change(n=2), m, N, B_TOKENS, S) == ["global_batch"]
    assert "gpu_count" in pl.violated_constraints(change(s_dp=16, n=8), m, N, B_TOKENS, S)
    assert pl.violated_constraints(change(s_tp=2), m, N, B_TOKENS, S) == ["tp_is_1_or_sp"]
    assert pl.violated_constraints(change(s_ps=3), m, N, B_TOKENS, S) == ["ps_divides", "oss_divides"]
    assert pl.violated_constraints(change(s_oss=128, s_gs=128), m, N, B_TOKENS, S) == ["oss_divides"]
    assert pl.violated_constraints(change(s_gs=2), m, N, B_TOKENS, S) == ["gs_is_1_or_oss"]
    m40 = pl.MODELS["13B"]                                      # 40 heads are not divisible by 16
    assert pl.violated_constraints(pl.Plan(1, 16, 0, 1, 8, 1, 16, 1, 1, 1), m40, N, B_TOKENS, S) == ["heads_divisible"]


def test_step_time_formula():
    """(n + s_pp - 1) (T_other + ceil(L / s_pp) R max(VPro, UPro)) + T_update, with constant stand-ins."""
    m, S = pl.MODELS["7B"], 4096

    class FixedCompute:
        def layer_time(self, model, plan, S):
            return 0.010

    class NoComm:
        def tau(self, op, v, p, span):
            return 0.0

    plan = pl.Plan(1, 8, 0, 4, 32, 1, 1, 1, 1, 1)
    t = pl.step_time(plan, m, S, N, NoComm(), FixedCompute(), R=1.25, t_other=0.002)
    assert t == pytest.approx((8 + 4 - 1) * (0.002 + 8 * 1.25 * 0.010))


def test_search_equals_brute_force_on_a_small_problem():
    m = pl.Model("tiny", H=512, L=4, heads=8, V=1000)
    S, n_gpus, batch, cap = 2048, 8, 2 ** 15, 0.5e9
    got = pl.search(m, S, n_gpus, batch, cap, top=10)
    assert 1 <= len(got) <= 10 and got == sorted(got)
    bw, comp = pl.SyntheticBandwidth(), pl.AnalyticCompute()
    every = []
    r = range(1, 17)
    for b, n, a, pp, dp, sp, ps, oss in itertools.product(r, r, (0, 1), (1, 2, 4, 8), (1, 2, 4, 8), (1, 2, 4, 8), (1, 2, 4, 8), (1, 2, 4, 8)):
        for tp in {1, sp}:
            for gs in {1, oss}:
                plan = pl.Plan(b, n, a, pp, dp, tp, sp, ps, gs, oss)
                if pl.violated_constraints(plan, m, n_gpus, batch, S) or pl.memory_bytes(plan, m, S)["total"] > cap:
                    continue
                every.append((pl.step_time(plan, m, S, n_gpus, bw, comp), plan))
    every.sort()
    assert [t for t, _ in got] == pytest.approx([t for t, _ in every[:len(got)]])
    assert got[0][1] == every[0][1]


def test_long_sequences_need_sequence_parallelism():
    """7B at 256K on 80 GB GPUs: without sequence (or tensor) parallelism and recomputation off nothing fits, and the
    fastest feasible plans split the sequence at least 8 ways, as every system in the paper's Table 4 does."""
    m, S = pl.MODELS["7B"], 262144
    assert pl.memory_bytes(pl.Plan(1, 4, 0, 1, 4, 1, 1, 128, 1, 1), m, S)["ACT"] > 10 * CAP
    best = pl.search(m, S, N, B_TOKENS, CAP, top=10, max_b=2)
    assert len(best) == 10
    assert all(plan.s_sp >= 8 for _, plan in best)


@pytest.mark.gpu
def test_measured_layer_time_on_the_gpu_is_close_to_the_analytic_stand_in():
    """UPro on the device: one 7B layer at 32K with s_sp = 4 (8 heads and 8192 tokens per GPU)."""
    m, S = pl.MODELS["7B"], 32768
    plan = pl.Plan(1, 4, 0, 1, 32, 1, 4, 2, 4, 4)
    measured = pl.measured_compute(m, S, s_sp=4)
    analytic = pl.AnalyticCompute().layer_time(m, plan, S)
    print(f"measured {measured * 1e3:.2f} ms, analytic {analytic * 1e3:.2f} ms", flush=True)
    assert 0.6 * analytic < measured < 1.6 * analytic


def test_profiled_compute_looks_up_and_scales():
    """A measured table replaces the analytic attention rate: exact shapes are looked up, others scale by
    b * heads * S^2 from the nearest measured shape, and the linear part stays analytic."""
    table = {"records": [
        {"b": 1, "S": 32768, "heads": 8, "fwd_ms": 2.0, "bwd_ms": 6.0, "bwd_stored_ds_ms": 5.0},
        {"b": 1, "S": 65536, "heads": 4, "fwd_ms": 4.0, "bwd_ms": 12.0, "bwd_stored_ds_ms": None},
    ]}
    assert pl.ProfiledCompute(table).attention_times(1, 32768, 8) == (2.0e-3, 6.0e-3)   # default: the O(S) path
    pc = pl.ProfiledCompute(table, stored_ds=True)
    assert pc.attention_times(1, 32768, 8) == (2.0e-3, 5.0e-3)
    assert pc.attention_times(1, 65536, 4) == (4.0e-3, 12.0e-3)          # no stored-dS time: the recomputing one
    f, b = pc.attention_times(1, 32768, 10)                               # 1.25 times the work of the first record
    assert abs(f - 2.5e-3) < 1e-12 and abs(b - 6.25e-3) < 1e-12
    m = pl.MODELS["7B"]
    plan = pl.Plan(b=1, n=1, a=0, s_pp=1, s_dp=1, s_tp=1, s_sp=4, s_ps=1, s_gs=1, s_oss=1)
    lin = 2.0 * 32768 * m.psi / 4 / pc.linear
    assert abs(pc.layer_time(m, plan, 32768) - (2.0e-3 + 5.0e-3 + 3 * lin)) < 1e-12
    plan_a = pl.Plan(b=1, n=1, a=1, s_pp=1, s_dp=1, s_tp=1, s_sp=4, s_ps=1, s_gs=1, s_oss=1)
    assert abs(pc.layer_time(m, plan_a, 32768) - (2 * (2.0e-3 + lin) + 5.0e-3 + 2 * lin)) < 1e-12
    # the stored-dS time comes with its memory: the workspace is charged to the plan
    assert pc.attention_workspace_bytes(1, 32768, 8) == 8 * 8 * 32768 + 8 * 32768 * (32768 + 128)
    assert pc.attention_workspace_bytes(1, 65536, 4) == 8 * 4 * 65536                   # no stored-dS time in the table
    assert pl.ProfiledCompute(table).attention_workspace_bytes(1, 32768, 8) == 8 * 8 * 32768
    mem = pl.memory_bytes(plan, m, 32768, compute=pc)
    assert mem["attn_workspace"] == pc.attention_workspace_bytes(1, 32768, 8)
    assert mem["total"] == pl.memory_bytes(plan, m, 32768)["total"] + mem["attn_workspace"]
    # usable by the search in place of the analytic model
    best = pl.search(m, 32768, 32, 4 * 2 ** 20, 80e9, compute=pc, top=3)
    assert best and all(t > 0 for t, _ in best)
