"""Strategy-planner slice: the paper's memory model, communication model, constraints and plan search,
as host arithmetic (no GPU needed; the per-layer computation times can come from the kernels of this
package measured on the GPU, see measured_compute()).

An execution plan is S = [b, n, a, s_pp, s_dp, s_tp, s_sp, s_ps, s_gs, s_oss] (Sec. 3, "Search Space"):
micro-batch size and number, activation recomputation, pipeline / data / tensor / sequence parallel sizes
and the sharding factors of parameters, gradients and optimizer states.  This module has
  - the constraints of the integer program of Sec. 4.5 ("Execution Simulator") and of Sec. 3.2.3,
  - the memory model of Sec. 3.2 (activations, pipeline factor, P / G / OS sharding),
  - the per-layer communication time of Sec. 3.2 (tensor parallelism, sequence parallelism, parameter,
    gradient and optimizer-state sharding) over tau(o, v, p) = v / w(o, v, p) (Sec. 3.2.1),
  - the step time T_fwd_bwd = (n + s_pp - 1) (T_other + ceil(L / s_pp) OPro) with
    OPro = R max(VPro, UPro) (Sec. 4.2, Sec. 4.5), and
  - the exhaustive search of Appendix "Solution Algorithm" that keeps the ten fastest feasible plans.

Readings where the paper is at odds with itself (each is pinned by a test):
  * The summary equation for M_tf divides G and OS by s_gs and s_oss only and weighs P, G and OS alike;
    the text of Sec. 3.2.3 divides G by s_ps * s_gs and OS by s_ps * s_oss, and Table 2 gives OS three times
    the bytes of P.  The text and the table are followed (with the summary equation the paper's own plan for
    65B at 256K would need 130 GB of an 80 GB GPU).
  * "When a = 1 ... 2bSH ... Conversely, if a = 1 ... 34bSH": the second is a = 0, as in the equation
    M_ACT = sum (2bSH + 32bSH (1 - a)).
  * GPU-count constraint: s_dp * s_sp * s_pp = N (s_tp is either 1 or equal to s_sp, Sec. 3.2.3 Config-1/2).
  * Pipeline: the first stage keeps min(s_pp, n) micro-batches of activations (Sec. 3.2.2).
What the paper leaves to profiling on its own cluster (the bandwidth table w, T_other, M_other, the slowdown
R) are parameters here; SyntheticBandwidth is a stand-in with the shape of the paper's Figure 5, not data.
"""
import heapq
import itertools
import math
from dataclasses import dataclass


@dataclass(frozen=True)
class Model:
    """Table 2: hidden size, layers, attention heads, vocabulary."""
    name: str
    H: int
    L: int
    heads: int
    V: int = 100_000

    @property
    def psi(self):
        """Parameters of one Transformer layer (Table 2)."""
        return 12 * self.H * self.H + 2 * self.H


MODELS = {m.name: m for m in (Model("7B", 4096, 32, 32), Model("13B", 5120, 40, 40), Model("30B", 6144, 60, 48),
                              Model("65B", 8192, 80, 64))}


@dataclass(frozen=True, order=True)
class Plan:
    b: int
    n: int
    a: int
    s_pp: int
    s_dp: int
    s_tp: int
    s_sp: int
    s_ps: int
    s_gs: int
    s_oss: int


def violated_constraints(plan, model, N, B_tokens, S):
    """Names of the constraints `plan` breaks (empty list: feasible apart from memory).  Sec. 4.5, Eq. (3)-(8);
    Sec. 3.2.3 (ranges of the sharding factors, Config-1/2); Sec. 5.4 (heads divisible by s_sp)."""
    p, bad = plan, []
    if min(p.b, p.n, p.s_pp, p.s_dp, p.s_tp, p.s_sp, p.s_ps, p.s_gs, p.s_oss) < 1 or p.a not in (0, 1):
        return ["positive"]
    if p.b * S * p.n * p.s_dp != B_tokens:
        bad.append("global_batch")
    if p.s_dp * p.s_sp * p.s_pp != N:
        bad.append("gpu_count")
    if p.s_tp not in (1, p.s_sp):
        bad.append("tp_is_1_or_sp")
    if N % (p.s_ps * p.s_pp * p.s_tp) != 0:
        bad.append("ps_divides")
    if N % (p.s_ps * p.s_oss * p.s_pp * p.s_tp) != 0:
        bad.append("oss_divides")
    if p.s_gs not in (1, p.s_oss):
        bad.append("gs_is_1_or_oss")
    if model.heads % p.s_sp != 0:
        bad.append("heads_divisible")
    if p.s_pp > model.L:
        bad.append("stages_le_layers")
    return bad


def memory_bytes(plan, model, S, other_bytes=0.0, compute=None):
    """GPU memory of the Transformer layers (Sec. 3.2) plus `other_bytes` (head, embedding, buffers: profiled in
    the paper, a parameter here) plus the workspace of the attention backward path whose time `compute` reports
    (one layer's worth: it is live during one layer's backward pass and shared by all layers).  Returns the parts
    and their total."""
    p = plan
    states = model.L * model.psi / (p.s_pp * p.s_tp)          # parameters held per GPU before sharding
    P = 2.0 * states / p.s_ps
    G = 2.0 * states / (p.s_ps * p.s_gs)
    OS = 6.0 * states / (p.s_ps * p.s_oss)
    per_layer = p.b * S * model.H * (2 + 32 * (1 - p.a))       # bytes, one micro-batch, one layer
    ACT = min(p.s_pp, p.n) * model.L * per_layer / (p.s_pp * p.s_sp)
    ws = 0.0
    if compute is not None and hasattr(compute, "attention_workspace_bytes"):
        ws = float(compute.attention_workspace_bytes(p.b, S, max(1, model.heads // max(p.s_sp, p.s_tp))))
    return {"P": P, "G": G, "OS": OS, "ACT": ACT, "other": float(other_bytes), "attn_workspace": ws,
            "total": P + G + OS + ACT + other_bytes + ws}


class SyntheticBandwidth:
    """Effective bandwidth w(o, v, p) in bytes/s: rises with the message size and saturates, lower across nodes
    than inside one, lower for more participants (the shape of the paper's Figure 5).  A stand-in for the table
    the paper profiles on its cluster."""

    def __init__(self, intra=200e9, inter=40e9, half_size=8e6, gpus_per_node=8):
        self.intra, self.inter, self.half, self.gpn = intra, inter, half_size, gpus_per_node

    def w(self, op, v, p, span):
        """`span`: GPUs the group's ranks are spread over counting the groups placed inside it (decides intra/inter)."""
        peak = self.intra if span <= self.gpn else self.inter
        algo = {"all-reduce": 0.5, "all-gather": 1.0, "reduce-scatter": 1.0, "all-to-all": 1.0}[op]
        return peak * algo * (p - 1) / p * v / (v + self.half) if p > 1 else float("inf")

    def tau(self, op, v, p, span):
        return 0.0 if p <= 1 or v <= 0 else v / self.w(op, v, p, span)


def comm_time_layer(plan, model, S, N, bw):
    """Communication time of one layer over a step, by cause (Sec. 3.2.2, 3.2.3).  Placement follows the paper's
    takeaways: the tensor/sequence group sits on the fewest nodes, the parameter-sharding group next."""
    p, H, psi = plan, model.H, model.psi
    bSH = p.b * S * H
    span_sp = p.s_sp
    span_ps = p.s_sp * p.s_ps if p.s_tp == 1 else p.s_tp * p.s_ps
    t = {}
    if p.s_tp > 1:    # Megatron-style: all-gather / reduce-scatter of activations (Config-1)
        t["tp"] = 2 * p.n * bw.tau("reduce-scatter", 2 * bSH, p.s_tp, span_sp) + 3 * p.n * bw.tau("all-gather", 2 * bSH, p.s_tp, span_sp)
    elif p.s_sp > 1:  # two all-to-alls per layer and direction: 6bSH and 2bSH bytes
        t["sp"] = 2 * p.n * bw.tau("all-to-all", 6 * bSH, p.s_sp, span_sp) + 2 * p.n * bw.tau("all-to-all", 2 * bSH, p.s_sp, span_sp)
    shard = 2.0 * psi / p.s_tp
    if p.s_ps > 1:
        t["ps"] = 2 * p.n * bw.tau("all-gather", shard, p.s_ps, span_ps) + p.n * bw.tau("reduce-scatter", shard, p.s_ps, span_ps)
    replicas = N // (p.s_pp * p.s_tp * p.s_ps)                 # GPUs that hold the same parameter shard
    t["oss"] = bw.tau("reduce-scatter", shard / p.s_ps, p.s_oss, N) + bw.tau("all-reduce", shard / p.s_ps, replicas, N)
    if p.s_gs > 1:
        t["gs"] = (p.n - 1) * bw.tau("all-reduce", shard / p.s_ps, replicas, N)
    return t


class AnalyticCompute:
    """UPro stand-in: forward + backward time of one layer for one micro-batch from sustained rates
    (FLOP/s) of the attention and linear kernels.  Attention: 4 S^2 H / 2 FLOP forward with the causal half,
    backward 2.5x; linear: 24 S H^2 FLOP forward (Psi ~ 12 H^2 weights), backward 2x; with a = 1 the forward is
    run once more (Sec. 3.2).  Both are divided over the s_sp (or s_tp) GPUs of the group."""

    def __init__(self, attn_flops=0.95e15, linear_flops=1.15e15):
        self.attn, self.linear = attn_flops, linear_flops

    def layer_time(self, model, plan, S):
        g = max(plan.s_sp, plan.s_tp)
        attn_fwd = 2.0 * plan.b * S * S * model.H / g
        lin_fwd = 2.0 * plan.b * S * model.psi / g
        fwd = attn_fwd / self.attn + lin_fwd / self.linear
        bwd = 2.5 * attn_fwd / self.attn + 2.0 * lin_fwd / self.linear
        return fwd * (1 + plan.a) + bwd


class ProfiledCompute(AnalyticCompute):
    """UPro with a measured attention table (Sec. 4.2: self-atten(b, S, H, D / s_sp) is profiled on one GPU and the
    simulator looks the times up): `table` is the JSON that `self_atten_sweep --json` writes.  A shape that was
    measured is looked up; any other falls back to the measured shape with the nearest FLOP count, scaled by the ratio
    of FLOP counts (attention time is proportional to b * heads * S^2 once the chip is full).  The linear modules stay
    analytic.  `stored_ds`: use the backward time of the path that keeps dS in a workspace of b * heads * S * (S + 128)
    bytes where the table has one; `attention_workspace_bytes` then reports those bytes and `memory_bytes` charges them.
    Off by default: the fused kernel is in the paper's design because it keeps attention memory O(S) (Sec. 3.2)."""

    def __init__(self, table, linear_flops=1.15e15, stored_ds=False):
        super().__init__(linear_flops=linear_flops)
        import json
        if isinstance(table, str):
            with open(table) as f:
                table = json.load(f)
        self.records, self.stored = {}, {}
        for r in table["records"]:
            use_ds = bool(stored_ds and r.get("bwd_stored_ds_ms"))
            bwd = r["bwd_stored_ds_ms"] if use_ds else r["bwd_ms"]
            self.records[(r["b"], r["S"], r["heads"])] = (r["fwd_ms"] * 1e-3, bwd * 1e-3)
            self.stored[(r["b"], r["S"], r["heads"])] = use_ds
        if not self.records:
            raise ValueError("empty attention table")

    def _nearest(self, b, S, heads):
        want = float(b) * heads * S * S
        return min(self.records, key=lambda k: abs(math.log(want / (float(k[0]) * k[2] * k[1] * k[1]))))

    def attention_workspace_bytes(self, b, S, heads):
        """Bytes of backward workspace behind the time attention_times reports: two [b, heads, S] fp32 planes, plus
        dS (bf16, the lower block triangle: b * heads * S * (S + 128) bytes) where the stored-dS time is used."""
        key = (b, S, heads) if (b, S, heads) in self.records else self._nearest(b, S, heads)
        small = 8.0 * b * heads * S
        return small + (float(b) * heads * S * (S + 128) if self.stored[key] else 0.0)

    def attention_times(self, b, S, heads):
        """(forward, backward) seconds of self-atten(b, S, heads) on one GPU."""
        hit = self.records.get((b, S, heads))
        if hit:
            return hit
        want = float(b) * heads * S * S
        key = self._nearest(b, S, heads)
        f, bw_ = self.records[key]
        ratio = want / (float(key[0]) * key[2] * key[1] * key[1])
        return f * ratio, bw_ * ratio

    def layer_time(self, model, plan, S):
        g = max(plan.s_sp, plan.s_tp)
        lin_fwd = 2.0 * plan.b * S * model.psi / g / self.linear
        a_fwd, a_bwd = self.attention_times(plan.b, S, max(1, model.heads // g))
        return (a_fwd + lin_fwd) * (1 + plan.a) + a_bwd + 2.0 * lin_fwd


def step_time(plan, model, S, N, bw, compute, R=1.3, t_other=0.0):
    """T_fwd_bwd + T_update (Sec. 4.5).  The sharding traffic of the optimizer step is T_update; everything else
    overlaps with computation at the cost of the slowdown R (OPro, Sec. 4.2)."""
    c = comm_time_layer(plan, model, S, N, bw)
    layers = math.ceil(model.L / plan.s_pp)
    per_micro_comm = (sum(v for k, v in c.items() if k != "oss")) / plan.n
    opro = R * max(per_micro_comm, compute.layer_time(model, plan, S))
    t_fwd_bwd = (plan.n + plan.s_pp - 1) * (t_other + layers * opro)
    return t_fwd_bwd + layers * c["oss"]


def _powers_of_two(limit):
    x = 1
    while x <= limit:
        yield x
        x *= 2


def candidate_plans(model, S, N, B_tokens):
    """The loops of the search algorithm (Appendix "Solution Algorithm"), with the divisibility constraints used
    to skip values that cannot pass."""
    for s_pp in (d for d in range(1, N + 1) if N % d == 0 and d <= model.L):
        for s_sp in _powers_of_two(N // s_pp):
            if (N // s_pp) % s_sp or model.heads % s_sp:
                continue
            s_dp = N // (s_pp * s_sp)
            if B_tokens % (S * s_dp):
                continue
            per_group = B_tokens // (S * s_dp)                # micro-batch size x number
            for s_tp in {1, s_sp}:
                for b in (d for d in range(1, per_group + 1) if per_group % d == 0):
                    n = per_group // b
                    room = N // (s_pp * s_tp)
                    for s_ps in (d for d in range(1, room + 1) if room % d == 0):
                        for s_oss in (d for d in range(1, room // s_ps + 1) if (room // s_ps) % d == 0):
                            for s_gs in {1, s_oss}:
                                for a in (0, 1):
                                    yield Plan(b, n, a, s_pp, s_dp, s_tp, s_sp, s_ps, s_gs, s_oss)


def search(model, S, N, B_tokens, capacity_bytes, bw=None, compute=None, top=10, R=1.3, other_bytes=0.0, max_b=None):
    """The `top` fastest plans that satisfy every constraint and fit in memory: list of (seconds, Plan)."""
    bw = bw or SyntheticBandwidth()
    compute = compute or AnalyticCompute()
    best = []   # max-heap on time through negation
    for i, plan in enumerate(candidate_plans(model, S, N, B_tokens)):
        if max_b is not None and plan.b > max_b:
            continue
        if violated_constraints(plan, model, N, B_tokens, S):
            continue
        if memory_bytes(plan, model, S, other_bytes, compute)["total"] > capacity_bytes:
            continue
        t = step_time(plan, model, S, N, bw, compute, R)
        if len(best) < top:
            heapq.heappush(best, (-t, i, plan))
        elif t < -best[0][0]:
            heapq.heapreplace(best, (-t, i, plan))
    return sorted((-t, plan) for t, _, plan in best)


def measured_compute(model, S, s_sp, b=1, iters=3):
    """UPro on the GPU (Sec. 4.2): times self-atten(b, S, heads / s_sp, head dim) and the twelve linear products of a
    layer on (b * S / s_sp, H) with the kernels of this package; returns seconds of forward + backward for one layer and
    one micro-batch.  Needs a GPU."""
    import torch
    from . import binding
    dev = "cuda:0"
    hd = model.H // model.heads
    heads = model.heads // s_sp
    mk = lambda *shape: torch.randn(shape, device=dev, dtype=torch.float32).to(torch.bfloat16)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e-3

    q, k, v, do = (mk(b, S, heads, hd) for _ in range(4))
    total = timed(lambda: binding.attn_fwd(q, k, v, hd ** -0.5, True))
    o, lse = binding.attn_fwd(q, k, v, hd ** -0.5, True)
    total += timed(lambda: binding.attn_bwd(q, k, v, o, do, lse, hd ** -0.5, True))
    del q, k, v, do, o, lse
    M = b * S // s_sp
    ffn = ((8 * model.H // 3 + 255) // 256) * 256   # LLaMA MLP width, rounded up to a multiple of 256
    for N_, K_ in ((3 * model.H, model.H), (model.H, model.H), (2 * ffn, model.H), (model.H, ffn)):
        x, w, dy = mk(M, K_), mk(N_, K_), mk(M, N_)
        y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
        total += timed(lambda: binding.ie_linear_fwd(x, w, y))
        total += timed(lambda: binding.ie_linear_bwd_input(dy, w, dx))
        total += timed(lambda: binding.ie_linear_bwd_weight(dy, x, dw))
        del x, w, dy, y, dx, dw
    return total
